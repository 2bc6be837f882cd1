// Shared device-side types and small helpers for the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define RS_WAVE 64
#define RS_BLOCK_TOKENS 16

// Prompt boundaries passed by value to kernels (no host->device copy on the launch path).
struct SeqInfo {
    int32_t n_req;
    int32_t cu[65];     // cu[0..n_req]
    int32_t start[64];  // position of each prompt's first row (0: a whole prompt; a multiple of 16: a later chunk of it)
};

// Rotary table entry: cos and sin of pos * base^(-2i/hd), formed in float64 on the host.
struct CosSin {
    float c, s;
};

__device__ __forceinline__ bf16x8 ld_bf16x8(const bf16_t *p) { return *(const bf16x8 *)p; }
// streaming read: data that is used once (decode weights, cached K/V) should not displace the other
// side's working set from the shared caches
__device__ __forceinline__ bf16x8 ld_bf16x8_stream(const bf16_t *p) {
    return __builtin_nontemporal_load((const bf16x8 *)p);
}
__device__ __forceinline__ void st_bf16x8(bf16_t *p, bf16x8 v) { *(bf16x8 *)p = v; }
__device__ __forceinline__ bf16x8 zero_bf16x8() {
    bf16x8 z;
#pragma unroll
    for (int i = 0; i < 8; ++i) z[i] = (bf16_t)0.0f;
    return z;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Fragment-packed layout of a GEMM operand X[M][K] (the GEMM inputs h, attn and act of both
// sides, and the library's copies of the weight matrices): [K/16 k blocks][Mt row tiles of 32]
// [64 lanes][8].  The 16 bytes that lane (h*32 + r) of a 32x32x16 MFMA operand needs for row
// 32*t + r and k in [16*kb + 8*h, +8) sit in lane order, so a wave-wide fragment load is one
// contiguous 1 KB read, and the (rows x 32 k) slab of a GEMM tile is two contiguous runs instead
// of one 64-byte piece per 2K-byte-strided row (which crowds a few memory channels).
// Element offset of the 8-element chunk holding (m, k):
__host__ __device__ __forceinline__ size_t packed_offset(int m, int k, int Mt) {
    return ((size_t)(k >> 4) * Mt + (m >> 5)) * 512 + (size_t)((((k >> 3) & 1) << 5) + (m & 31)) * 8;
}
// Row tiles of a packed activation matrix of M rows: at least the two tiles the skinny kernel reads.
__host__ __device__ __forceinline__ int packed_mt(int M) { return M <= 64 ? 2 : (M + 31) >> 5; }

// K pool layout inside one (block, kv head): [hd/32][4][16][8] = (32-wide dim group s, 8-wide
// sub-chunk kh, permuted token row, 8 dims).  A 16x16x32 MFMA row operand for dim group s is then
// one contiguous 1 KB (lane = kh*16 + row), and the token order 0-3, 8-11, 4-7, 12-15 (bits 2 and
// 3 of the slot swapped) makes each of the two score tiles of the decode kernel read whole 128-byte
// lines.  Element offset of the 8-dim chunk holding (token slot t, dim d) within the block/head:
__host__ __device__ __forceinline__ int kpool_chunk_offset(int t, int d) {
    const int prow = (t & 3) | ((t & 8) >> 1) | ((t & 4) << 1);
    return (((d >> 5) * 4 + ((d >> 3) & 3)) * 16 + prow) * 8;
}
