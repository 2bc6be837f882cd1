// RMSNorm and rotary-embedding + paged KV write kernels (bandwidth-trivial steps of the layer).
#include <algorithm>

#include "kernels.h"

// ---------------------------------------------------------------------------------------------
// RMSNorm.  The output feeds a GEMM and is written in the fragment-packed operand layout, where
// the 16-byte chunks of 8 consecutive rows (same k) are 128 contiguous bytes: a 256-thread
// workgroup therefore takes R rows, 256/R threads per row, so that neighbouring threads complete
// whole lines.  R = 8 for large M; R = 1 (one row per workgroup) when M is small and parallelism
// matters more than write coalescing.  A row's reduction tree depends on d and R only, and R on M
// only.
// ---------------------------------------------------------------------------------------------
template <int R, int NC>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const bf16_t *__restrict__ x,
                                                      const bf16_t *__restrict__ g,
                                                      bf16_t *__restrict__ out, int M, int d, float eps, int Mt) {
    constexpr int TPR = 256 / R;   // threads per row
    __shared__ float red[256 / 64][R];
    const int tid = threadIdx.x;
    const int r = tid % R, t = tid / R;
    const int row = blockIdx.x * R + r;
    const bool valid = row < M;
    const bf16_t *xr = x + (size_t)(valid ? row : M - 1) * d;
    const int nchunk = d >> 3;
    // the thread's chunks t, t + TPR, ... stay in registers between the two passes (NC of them at most:
    // the launcher picks NC >= nchunk / TPR); all loads are in flight at once
    bf16x8 xv[NC];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = t + i * TPR;
        xv[i] = c < nchunk ? ld_bf16x8(xr + c * 8) : zero_bf16x8();
    }
    // the gains do not depend on the sum: fetched now, behind the row's own loads, not after the barrier
    bf16x8 gv[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = t + i * TPR;
        gv[i] = c < nchunk ? ld_bf16x8(g + c * 8) : zero_bf16x8();
    }
#pragma unroll
    for (int i = 0; i < NC; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float f = (float)xv[i][e];
            ss += f * f;
        }
    // lanes with the same (lane % R) hold the same row: butterfly over the other lane bits, then the 4 waves
#pragma unroll
    for (int o = 32; o >= R; o >>= 1) ss += __shfl_xor(ss, o, 64);
    if ((tid & 63) < R) red[tid >> 6][tid & 63] = ss;
    __syncthreads();
    const float tot = (red[0][r] + red[1][r]) + (red[2][r] + red[3][r]);
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    if (!valid) return;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = t + i * TPR;
        if (c >= nchunk) break;
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (bf16_t)((float)xv[i][e] * inv * (float)gv[i][e]);
        st_bf16x8(out + packed_offset(row, c * 8, Mt), o);
    }
}

void launch_rmsnorm(hipStream_t st, const bf16_t *x, const bf16_t *g, bf16_t *out, int M, int d, float eps) {
    if (M <= 0) return;
    const int nchunk = d >> 3, Mt = packed_mt(M);
    // R and NC are functions of (M, d) only
    if (M >= 512 && nchunk <= 16 * 32)
        hipLaunchKernelGGL((rmsnorm_kernel<8, 16>), dim3((M + 7) / 8), dim3(256), 0, st, x, g, out, M, d, eps, Mt);
    else if (M >= 512 && nchunk <= 32 * 32)
        hipLaunchKernelGGL((rmsnorm_kernel<8, 32>), dim3((M + 7) / 8), dim3(256), 0, st, x, g, out, M, d, eps, Mt);
    else if (nchunk <= 8 * 256)
        hipLaunchKernelGGL((rmsnorm_kernel<1, 8>), dim3(M), dim3(256), 0, st, x, g, out, M, d, eps, Mt);
    else
        hipLaunchKernelGGL((rmsnorm_kernel<1, 32>), dim3(M), dim3(256), 0, st, x, g, out, M, d, eps, Mt);
}

// ---------------------------------------------------------------------------------------------
// RoPE on q (in place) and k, then K -> pool[blk][kvh] in the dim-group / permuted-row chunk order
// of kpool_chunk_offset, V -> pool[blk][kvh][:][slot].
// One workgroup per token row; work items of 8 elements are spread over the 256 threads.
// A block id outside the pool, or a position outside the rotary table, is never dereferenced:
// the item is skipped and the error flag raised.
//
// The V pool is transposed ([dim][slot]), so a single token touches one 2-byte element in each of
// Hkv*hd different 32-byte sectors.  A decode row has no choice; a prompt does: workgroups past the
// first M of a prefill launch each take one 16-token block of one prompt, gather its V values
// token by token (a wave reads 256 contiguous bytes per token) and write whole [dim][16] rows, so
// that a wave's stores cover one contiguous span.  The token-row workgroups of a prefill launch
// then leave V alone.  The last, partly filled block of a prompt is written element by element:
// its other slots belong to tokens that decode appends later and are not touched.
// (Giving the block workgroups the block's K as well -- rotated there, 16 lanes writing the 256 contiguous
// bytes of a chunk's 16 slots -- measured slower, 21 -> 26 us at 2048 tokens: the few block workgroups
// become the long pole while the many token-row workgroups, which hide their scattered K stores well, idle.)
// ---------------------------------------------------------------------------------------------
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

static __device__ void v_block_write(const RopeKvArgs &a, int vb) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // prompt and block within it
    int req = 0, first = 0;
    for (;; ++req) {
        if (req >= a.seq.n_req) return;
        const int nb = (a.seq.cu[req + 1] - a.seq.cu[req] + RS_BLOCK_TOKENS - 1) / RS_BLOCK_TOKENS;
        if (vb < first + nb) break;
        first += nb;
    }
    const int bi = vb - first;
    const int b0 = a.seq.start[req] / RS_BLOCK_TOKENS;                   // a chunk starts on a block boundary
    const int len = min(a.seq.cu[req + 1] - a.seq.cu[req], a.max_pos - a.seq.start[req]);   // rows past the table are flagged by their own workgroup
    const int nvalid = min(len - bi * RS_BLOCK_TOKENS, RS_BLOCK_TOKENS);
    if (nvalid <= 0 || b0 + bi >= a.max_blk) return;
    const int blk = a.tables[(size_t)req * a.max_blk + b0 + bi];
    if ((unsigned)blk >= (unsigned)a.n_blocks) return;                   // flagged by the token rows
    const int hd = a.hd, nqkv = (a.Hq + 2 * a.Hkv) * hd;
    const bf16_t *row0 = a.qkv + (size_t)(a.seq.cu[req] + bi * RS_BLOCK_TOKENS) * nqkv + (a.Hq + a.Hkv) * hd;
    for (int kvh = wave; kvh < a.Hkv; kvh += 4)
        for (int dp = lane; dp < (hd >> 1); dp += 64) {
            uint32_t w[RS_BLOCK_TOKENS];
#pragma unroll
            for (int t = 0; t < RS_BLOCK_TOKENS; ++t)
                w[t] = t < nvalid ? *(const uint32_t *)(row0 + (size_t)t * nqkv + kvh * hd + 2 * dp) : 0u;
            bf16_t *dst = a.v_pool + (((size_t)blk * a.Hkv + kvh) * hd + 2 * dp) * RS_BLOCK_TOKENS;
            if (nvalid == RS_BLOCK_TOKENS) {
                uint32_t ev[8], od[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    ev[j] = (w[2 * j] & 0xffffu) | (w[2 * j + 1] << 16);
                    od[j] = (w[2 * j] >> 16) | (w[2 * j + 1] & 0xffff0000u);
                }
                u32x4_t *d4 = (u32x4_t *)dst;
                d4[0] = u32x4_t{ev[0], ev[1], ev[2], ev[3]};
                d4[1] = u32x4_t{ev[4], ev[5], ev[6], ev[7]};
                d4[2] = u32x4_t{od[0], od[1], od[2], od[3]};
                d4[3] = u32x4_t{od[4], od[5], od[6], od[7]};
            } else {
                uint16_t *d2 = (uint16_t *)dst;
#pragma unroll
                for (int t = 0; t < RS_BLOCK_TOKENS; ++t)
                    if (t < nvalid) {
                        d2[t] = (uint16_t)(w[t] & 0xffffu);
                        d2[RS_BLOCK_TOKENS + t] = (uint16_t)(w[t] >> 16);
                    }
            }
        }
}

__global__ __launch_bounds__(256) void rope_kvwrite_kernel(RopeKvArgs a) {
    if ((int)blockIdx.x >= a.M) {
        v_block_write(a, (int)blockIdx.x - a.M);
        return;
    }
    const int row = blockIdx.x;
    const int tid = threadIdx.x;
    int req, pos;
    if (a.ctx_lens) {
        req = row;
        pos = a.ctx_lens[row];
    } else {
        req = 0;
        while (req + 1 < a.seq.n_req && row >= a.seq.cu[req + 1]) ++req;
        pos = a.seq.start[req] + row - a.seq.cu[req];
    }
    if (pos < 0 || pos >= a.max_pos) {
        if (tid == 0) atomicOr(a.err_flag, 1);
        return;
    }
    const int bi = pos / RS_BLOCK_TOKENS, slot = pos % RS_BLOCK_TOKENS;
    int blk = -1;
    if (bi < a.max_blk) blk = a.tables[(size_t)req * a.max_blk + bi];
    const bool blk_ok = (unsigned)blk < (unsigned)a.n_blocks;
    if (!blk_ok && tid == 0) atomicOr(a.err_flag, 2);

    const int hd = a.hd, half = hd >> 1;
    const int cph = half >> 3;  // 8-element chunks per half head
    const int nqkv = (a.Hq + 2 * a.Hkv) * hd;
    bf16_t *rowp = a.qkv + (size_t)row * nqkv;
    const CosSin *tab = a.table + (size_t)pos * half;

    const int n_rot = (a.Hq + a.Hkv) * cph;
    for (int it = tid; it < n_rot; it += 256) {
        const int head = it / cph, c = it % cph;
        bf16_t *hp = rowp + head * hd;
        bf16x8 lo = ld_bf16x8(hp + c * 8);
        bf16x8 hi = ld_bf16x8(hp + half + c * 8);
        bf16x8 olo, ohi;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            CosSin cs = tab[c * 8 + i];
            float x0 = (float)lo[i], x1 = (float)hi[i];
            olo[i] = (bf16_t)(x0 * cs.c - x1 * cs.s);
            ohi[i] = (bf16_t)(x1 * cs.c + x0 * cs.s);
        }
        if (head < a.Hq) {
            st_bf16x8(hp + c * 8, olo);
            st_bf16x8(hp + half + c * 8, ohi);
        } else if (blk_ok) {
            const int kvh = head - a.Hq;
            bf16_t *dst = a.k_pool + ((size_t)blk * a.Hkv + kvh) * RS_BLOCK_TOKENS * hd;
            st_bf16x8(dst + kpool_chunk_offset(slot, c * 8), olo);
            st_bf16x8(dst + kpool_chunk_offset(slot, half + c * 8), ohi);
        }
    }
    if (blk_ok && a.ctx_lens) {
        const int n_v = a.Hkv * (hd >> 3);
        const bf16_t *vrow = rowp + (a.Hq + a.Hkv) * hd;
        for (int it = tid; it < n_v; it += 256) {
            const int kvh = it / (hd >> 3), c = it % (hd >> 3);
            bf16x8 v = ld_bf16x8(vrow + kvh * hd + c * 8);
            bf16_t *dst = a.v_pool + (((size_t)blk * a.Hkv + kvh) * hd + c * 8) * RS_BLOCK_TOKENS + slot;
#pragma unroll
            for (int i = 0; i < 8; ++i) dst[i * RS_BLOCK_TOKENS] = v[i];
        }
    }
}

void launch_rope_kvwrite(hipStream_t st, const RopeKvArgs &a) {
    if (a.M <= 0) return;
    int v_blocks = 0;   // prefill: one more workgroup per 16-token block of each prompt
    if (!a.ctx_lens)
        for (int r = 0; r < a.seq.n_req; ++r)
            v_blocks += (a.seq.cu[r + 1] - a.seq.cu[r] + RS_BLOCK_TOKENS - 1) / RS_BLOCK_TOKENS;
    hipLaunchKernelGGL(rope_kvwrite_kernel, dim3(a.M + v_blocks), dim3(256), 0, st, a);
}

// ---------------------------------------------------------------------------------------------
// CU probe: every workgroup reads the hardware-id registers, spins briefly so that workgroups
// spread over all CUs the queue may use, and bumps the bin of the CU it ran on.
// HW_ID (register 4): cu_id bits 11:8, sh_id bit 12, se_id bits 15:13.  XCC_ID (register 20):
// bits 3:0.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void cu_probe_kernel(int32_t *hist) {
    const uint32_t hw = __builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));
    const uint32_t xcc = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));
    const uint64_t t0 = wall_clock64();
    while (wall_clock64() - t0 < 2000) {  // ~20 us at 100 MHz
    }
    if (threadIdx.x == 0) {
        const uint32_t cu = (hw >> 8) & 15, sh = (hw >> 12) & 1, se = (hw >> 13) & 7;
        atomicAdd(&hist[((xcc & 15) << 8) | (se << 5) | (sh << 4) | cu], 1);
    }
}

void launch_cu_probe(hipStream_t st, int32_t *hist, int n_workgroups) {
    hipLaunchKernelGGL(cu_probe_kernel, dim3(n_workgroups), dim3(64), 0, st, hist);
}

// ---------------------------------------------------------------------------------------------
// Streaming read: grid-stride 16-byte loads, 8 in flight per thread; measures the read bandwidth
// a CU partition can pull.  The XOR fold is compared with a value it cannot take for all-equal
// input words, so nothing is stored.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4_t *__restrict__ src, u32x4_t *sink, size_t n16) {
    size_t i = (size_t)blockIdx.x * 2048 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 2048;
    u32x4_t acc = {0, 0, 0, 0};
    for (; i + 256 * 7 < n16; i += stride) {
        u32x4_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(&src[i + 256 * u]);   // streamed: read once
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u && sink) sink[0] = acc;
}

void launch_stream_read(hipStream_t st, const void *src, size_t bytes, int n_workgroups) {
    hipLaunchKernelGGL(stream_read_kernel, dim3(n_workgroups), dim3(256), 0, st, (const u32x4_t *)src, (u32x4_t *)nullptr,
                       bytes / 16);
}

// ---------------------------------------------------------------------------------------------
// Zero fill by kernel: a memset node recorded into a captured graph is not something a caller's
// graph should contain, a kernel node is fine.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fill_zero_kernel(u32x4_t *dst, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = u32x4_t{0, 0, 0, 0};
}

void launch_fill_zero(hipStream_t st, void *dst, size_t bytes) {
    const size_t n16 = bytes / 16;
    if (!n16) return;
    const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 1024);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(256), 0, st, (u32x4_t *)dst, n16);
}

// ---------------------------------------------------------------------------------------------
// Matrix-core probe: what the chip sustains when nothing but MFMAs is issued.  Every wave keeps 8
// independent 32x32x16 bf16 accumulator tiles in registers and issues MFMAs back to back, operands
// never leave registers; 2 workgroups of 4 waves per compute unit.  2 * 32 * 32 * 16 flop per MFMA.
// The operands are pseudo-random values in +-[0.5, 1) with random mantissas, a different pair per
// accumulator: the clock the chip holds under matrix load depends on how many bits toggle, and constant
// or few-valued operands let it clock far higher than any real GEMM's data does.
// The published peak assumes the nominal clock; under this load the chip clocks lower, and no GEMM
// can beat what this loop reaches on the same partition.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void mfma_probe_kernel(float *sink, int iters) {
    bf16x8 a[8], b[8];
    uint32_t x = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        typedef uint32_t u32x4p __attribute__((ext_vector_type(4)));
        u32x4p wa, wb;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x ^= x << 13; x ^= x >> 17; x ^= x << 5;
            wa[i] = (x & 0x807f807fu) | 0x3f003f00u;   // sign and mantissa random, exponent of 0.5
            x ^= x << 13; x ^= x >> 17; x ^= x << 5;
            wb[i] = (x & 0x807f807fu) | 0x3f003f00u;
        }
        a[j] = __builtin_bit_cast(bf16x8, wa);
        b[j] = __builtin_bit_cast(bf16x8, wb);
    }
    f32x16 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[j], acc[j], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) t += acc[j][e];
    if (t == -1.0f) sink[0] = t;   // keeps the loop alive; sink is a valid float whether or not this ever fires
}

double launch_mfma_probe(hipStream_t st, float *sink, int n_workgroups, int iters) {
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(n_workgroups), dim3(256), 0, st, sink, iters);
    return (double)n_workgroups * 4 * (double)iters * 8 * 32768.0;
}

// An empty kernel: used once per new pair of masked streams to make the runtime set up whatever two
// concurrently active queues need, inside the set-up call instead of inside the first overlapping layer call.
__global__ void noop_kernel() {}
void launch_noop(hipStream_t st) { hipLaunchKernelGGL(noop_kernel, dim3(1), dim3(64), 0, st); }
