// Attention kernels over the paged KV cache (gfx950, bf16 MFMA, fp32 softmax).
//
// Pool layouts (one layer):  K [n_blocks][Hkv][hd/32][4][16][8] (see kpool_chunk_offset)
// V [n_blocks][Hkv][hd][16], so one (block, kv head) is a contiguous 16*hd*2-byte run in each
// pool, a K fragment of the MFMA "row x k" operand is one contiguous 1 KB, and V, being token-
// minor, feeds the operand whose contraction index is the token without any transpose.
//
// Both kernels evaluate S^T = K Q^T and O^T = V^T P^T, so that a lane owns one query column:
// the running maximum and sum of the online softmax are per-lane scalars.
#include <type_traits>

#include "kernels.h"

#define NEG_INF (-__builtin_huge_valf())
#define PREFILL_TAB_LDS 2048   // block ids of a prompt kept in LDS by the prefill kernel (32K tokens)

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// =============================================================================================
// Decode: one query token per request, keys gathered through the block table.
// Workgroup = (512-token chunk, kv head, request); its 4 waves take 128 tokens (8 blocks) each,
// two blocks per iteration.  The G = Hq/Hkv query heads that share the kv head are the (zero
// padded) 16 columns of the MFMA tiles, so every K/V byte is fetched once per kv head, straight
// from the pools into MFMA fragments with 16-byte loads (no LDS staging).
// The chunking depends on the context length only, never on the launch's CU share.
//
// Measured alternatives that were no better (Llama-3-8B shape, batch 64, contexts U[512,4096]; whole chip /
// 128-CU partition / partition beside a prefill pass; this kernel: 110 / 144 / 172 us):
//   * a persistent launch whose waves are independent workers on 128-token items, the next item's block ids
//     and first K/V loads in flight while an item is computed, items dealt round-robin: 126 / 156 / 171 us
//     (no round trip is exposed any more, yet nothing is gained: the kernel is not bound by the start-up of
//     its workgroups); the same with a device-side item counter: 200 us on any partition (12 500
//     single-address atomics serialise at about 16 ns each);
//   * the kv heads of one (request, chunk) on ONE XCD instead of eight: 7-10 % slower everywhere.
// What the measurements fit: a compute unit sustains a bounded number of outstanding lines, so its rate is
// that bound over the memory latency of the access pattern -- 47 GB/s for a linear stream, 34 GB/s for
// these 4 KB pieces of shuffled 32 KB blocks (38 GB/s with consecutive block ids), on a 128-CU partition.
//
// Row permutation: the two 16x16 score tiles of an iteration do not hold "block 0" and "block 1"
// but, with h = lane>>4, tile A row 4h+i <- token 8(h&1)+i of block h>>1 and tile B row 4h+i <-
// token 8(h&1)+4+i of block h>>1.  A lane's 4+4 score registers are then 8 consecutive tokens of
// one block, exactly the contraction slice k' = 8h..8h+7 that lane supplies to the 16x16x32 P V
// product, and the matching V fragment V[block h>>1][d][8(h&1)..+8] is one 16-byte load.
// =============================================================================================
template <int HD>
__global__ __launch_bounds__(256, 2) void decode_attn_kernel(DecodeAttnArgs a) {
    constexpr int KS = HD / 32;  // 16x16x32 steps over head_dim for S^T
    constexpr int DT = HD / 16;  // 16-row tiles of O^T
    extern __shared__ float smem_dec[];   // [4][HD][G] partial outputs, then [4][G] max, [4][G] sum

    // kv head fastest: consecutive workgroup ids are dealt to the 8 XCDs in turn, and every kv head
    // carries the same work, whereas chunk c only exists for contexts longer than c chunks.  With the chunk
    // index slowest the workgroups that have nothing to do (chunks past a request's context) gather at
    // the end of the grid instead of following each request: on a CU partition that measured 5 % faster
    // (128 CUs: 160 -> 152 us), on the whole chip 2 % slower, so the launcher chooses by partition size.
    // (Consecutive ids go to the 8 XCDs in turn, so the kv heads of one block are read through 8 different L2s
    // at about the same time; putting them on ONE XCD instead measured 7-10 % slower on every partition.)
    const int hk = blockIdx.x;
    const int b = a.chunk_major ? blockIdx.y : blockIdx.z, chunk = a.chunk_major ? blockIdx.z : blockIdx.y;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c16 = lane & 15, h = lane >> 4;
    const int G = a.Hq / a.Hkv;
    float *s_o = smem_dec;
    float *s_m = smem_dec + 4 * HD * G;
    float *s_l = s_m + 4 * G;

    int n_keys = a.ctx_lens[b] + 1;
    if (n_keys < 1 || n_keys > a.max_ctx) {
        if (tid == 0 && chunk == 0 && hk == 0) atomicOr(a.err_flag, 8);
        if (n_keys < 1) return;
        n_keys = a.max_ctx;
    }
    if (chunk * RS_DECODE_CHUNK >= n_keys) return;

    constexpr int WT = RS_DECODE_CHUNK / 4;   // tokens per wave
    const int t0 = chunk * RS_DECODE_CHUNK + wave * WT;
    const int t1 = min(t0 + WT, n_keys);
    // the wave's (up to) WT/16 block ids, fetched once: lane i holds the id of block i of the range
    int my_blk = -1;
    {
        const int nb = t1 > t0 ? (t1 - t0 + 15) >> 4 : 0;
        if (lane < nb) {
            my_blk = a.tables[(size_t)b * a.max_blk + (t0 >> 4) + lane];
            if ((unsigned)my_blk >= (unsigned)a.n_blocks) {
                atomicOr(a.err_flag, 2);
                my_blk = -1;
            }
        }
    }

    bf16x8 qf[KS];
    {
        const bf16_t *qp = a.q + (size_t)b * a.q_stride + (size_t)(hk * G + c16) * HD;
#pragma unroll
        for (int s = 0; s < KS; ++s) qf[s] = (c16 < G) ? ld_bf16x8(qp + 32 * s + 8 * h) : zero_bf16x8();
    }

    float m_run = NEG_INF, l_run = 0.f;
    f32x4 o[DT];
#pragma unroll
    for (int i = 0; i < DT; ++i) o[i] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // K operand: MFMA row c16 = 4 hr + ir comes from block (hr>>1), token 8(hr&1)+ir (+4 for tile
    // B): in the pool's permuted row order these are rows c16&7 (tile A) and 8 + (c16&7) (tile B)
    const bool k_second = (c16 >> 3) != 0;   // this lane's K rows come from the iteration's second block
    const bool v_second = (h >> 1) != 0;     // this lane's V slice comes from the second block
    const size_t k_lane = (size_t)(h * 16 + (c16 & 7)) * 8;
    const size_t v_lane = (size_t)c16 * 16 + 8 * (h & 1);
    const size_t blk_stride = (size_t)a.Hkv * 16 * HD;
    const bf16_t *k_head = a.k_pool + (size_t)hk * 16 * HD;
    const bf16_t *v_head = a.v_pool + (size_t)hk * 16 * HD;
    const float sc = a.scale_log2;

    // Two register buffers of one iteration's K and V fragments (32 tokens, 16 KB per wave): the loads
    // of iteration it+1 are issued before iteration it is computed, so the wave always has bytes in
    // flight.  The number of iterations is wave-uniform; each count gets its own straight-line copy
    // of the schedule, which keeps the compiler's wait counts exact (a load issued under a branch
    // would force a wait for everything at the join).
    bf16x8 kA[2][KS], kB[2][KS], vf[2][DT];
    auto issue = [&](int it, int buf) {
        // the iteration's two block ids as wave-uniform scalars; blocks that are missing (past the
        // context, or rejected) read block 0: valid memory whose contents are masked out in compute()
        const int b0 = __builtin_amdgcn_readlane(my_blk, 2 * it);
        const int b1 = __builtin_amdgcn_readlane(my_blk, 2 * it + 1);
        const size_t o0 = (size_t)max(b0, 0) * blk_stride, o1 = (size_t)max(b1, 0) * blk_stride;
        const bf16_t *kp = k_head + (k_second ? o1 : o0) + k_lane;
        const bf16_t *vp = v_head + (v_second ? o1 : o0) + v_lane;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            kA[buf][s] = ld_bf16x8_stream(kp + 512 * s);
            kB[buf][s] = ld_bf16x8_stream(kp + 512 * s + 64);
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) vf[buf][dt] = ld_bf16x8_stream(vp + dt * 256);
    };
    auto compute = [&](int it, int buf) {
        const int base = t0 + 32 * it;
        const int b0 = __builtin_amdgcn_readlane(my_blk, 2 * it);
        const int b1 = __builtin_amdgcn_readlane(my_blk, 2 * it + 1);
        const bool full = base + 32 <= n_keys && b0 >= 0 && b1 >= 0;   // uniform: every token valid
        f32x4 sA = {0.f, 0.f, 0.f, 0.f}, sB = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            sA = mfma16(kA[buf][s], qf[s], sA);
            sB = mfma16(kB[buf][s], qf[s], sB);
        }
        // this lane's 8 scores are tokens tok0 .. tok0+7 (A: +0..3, B: +4..7) of its V block
        if (!full) {
            const int tok0 = base + 16 * (h >> 1) + 8 * (h & 1);
            const int nv = ((v_second ? b1 : b0) >= 0) ? min(max(n_keys - tok0, 0), 8) : 0;   // valid tokens
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (i >= nv) sA[i] = NEG_INF;
                if (4 + i >= nv) sB[i] = NEG_INF;
            }
            // zero V of invalid tokens so that 0 * garbage cannot produce NaN: dword j holds tokens 2j, 2j+1
            uint32_t msk[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) msk[j] = nv >= 2 * j + 2 ? 0xffffffffu : (nv == 2 * j + 1 ? 0x0000ffffu : 0u);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
                u32x4v raw = __builtin_bit_cast(u32x4v, vf[buf][dt]);
#pragma unroll
                for (int j = 0; j < 4; ++j) raw[j] &= msk[j];
                vf[buf][dt] = __builtin_bit_cast(bf16x8, raw);
            }
        }
        float m_tile = fmaxf(fmaxf(fmaxf(sA[0], sA[1]), fmaxf(sA[2], sA[3])), fmaxf(fmaxf(sB[0], sB[1]), fmaxf(sB[2], sB[3])));
        m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 16, 64));
        m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32, 64));
        const float m_new = fmaxf(m_run, m_tile);            // running maximum of RAW scores
        const float m_safe = (m_new == NEG_INF) ? 0.f : m_new;
        const float ms = m_safe * sc;
        bf16x8 pf;
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float pa = __builtin_amdgcn_exp2f(fmaf(sA[i], sc, -ms)), pb = __builtin_amdgcn_exp2f(fmaf(sB[i], sc, -ms));
            psum += pa + pb;
            pf[i] = (bf16_t)pa;
            pf[4 + i] = (bf16_t)pb;
        }
        if (__any(m_new != m_run)) {
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_safe) * sc);
            l_run *= alpha;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) o[dt] = o[dt] * alpha;
            m_run = m_new;
        }
        l_run += psum;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt] = mfma16(vf[buf][dt], pf, o[dt]);
    };
    auto run = [&](auto ntag) {
        constexpr int N = decltype(ntag)::value;
        issue(0, 0);
#pragma unroll
        for (int it = 0; it < N; ++it) {
            if (it + 1 < N) issue(it + 1, (it + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);   // the next iteration's loads go out before this one's arithmetic
            compute(it, it & 1);
        }
    };
    static_assert(WT / 32 == 4, "one schedule per iteration count below");
    const int nit = t1 > t0 ? (t1 - t0 + 31) >> 5 : 0;   // wave-uniform
    switch (nit) {
        case 1: run(std::integral_constant<int, 1>{}); break;
        case 2: run(std::integral_constant<int, 2>{}); break;
        case 3: run(std::integral_constant<int, 3>{}); break;
        case 4: run(std::integral_constant<int, 4>{}); break;
        default: break;
    }
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);

    // combine the 4 waves (fixed order) and emit the chunk's partial result
    if (c16 < G) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i = 0; i < 4; ++i) s_o[(wave * HD + 16 * dt + 4 * h + i) * G + c16] = o[dt][i];
        if (h == 0) {
            s_m[wave * G + c16] = m_run;
            s_l[wave * G + c16] = l_run;
        }
    }
    __syncthreads();
    for (int idx = tid; idx < G * HD; idx += 256) {
        const int gg = idx % G, d = idx / G;   // consecutive threads read consecutive words of s_o: no bank conflicts
        const float mx = fmaxf(fmaxf(s_m[gg], s_m[G + gg]), fmaxf(s_m[2 * G + gg], s_m[3 * G + gg]));
        const float ms = (mx == NEG_INF) ? 0.f : mx;
        float acc = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float e = __builtin_amdgcn_exp2f((s_m[w * G + gg] - ms) * a.scale_log2);
            acc += s_o[(w * HD + d) * G + gg] * e;
            l += s_l[w * G + gg] * e;
        }
        const size_t pi = ((size_t)b * a.Hq + hk * G + gg) * a.n_chunks + chunk;
        a.part_o[pi * HD + d] = acc;
        if (d == 0) {
            a.part_ml[pi * 2] = mx;
            a.part_ml[pi * 2 + 1] = l;
        }
    }
}

// Merges the per-chunk partial results of one (request, query head) in chunk order.
template <int HD>
__global__ __launch_bounds__(HD) void decode_combine_kernel(DecodeAttnArgs a) {
    const int hq = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
    int n_keys = a.ctx_lens[b] + 1;
    const int col = hq * HD + d;
    bf16_t *op = a.out + packed_offset(a.out_row0 + b, col, a.out_Mt ? a.out_Mt : packed_mt(a.B)) + (col & 7);   // feeds the output projection
    if (n_keys < 1) {
        *op = (bf16_t)0.f;
        return;
    }
    if (n_keys > a.max_ctx) n_keys = a.max_ctx;
    const int nch = (n_keys + RS_DECODE_CHUNK - 1) / RS_DECODE_CHUNK;
    const size_t p0 = ((size_t)b * a.Hq + hq) * a.n_chunks;
    float mx = NEG_INF;
    for (int c = 0; c < nch; ++c) mx = fmaxf(mx, a.part_ml[(p0 + c) * 2]);
    const float ms = (mx == NEG_INF) ? 0.f : mx;
    float acc = 0.f, l = 0.f;
    for (int c = 0; c < nch; ++c) {
        const float e = exp2f((a.part_ml[(p0 + c) * 2] - ms) * a.scale_log2);   // maxima are raw scores
        acc += a.part_o[(p0 + c) * HD + d] * e;
        l += a.part_ml[(p0 + c) * 2 + 1] * e;
    }
    *op = (bf16_t)(l > 0.f ? acc / l : 0.f);
}

void launch_decode_attention(hipStream_t st, const DecodeAttnArgs &a) {
    if (a.B <= 0) return;
    dim3 grid(a.Hkv, a.chunk_major ? a.B : a.n_chunks, a.chunk_major ? a.n_chunks : a.B);
    dim3 cgrid(a.Hq, a.B);
    const int G = a.Hq / a.Hkv;
    const size_t lds = (size_t)(4 * a.hd * G + 8 * G) * sizeof(float);   // <= 33 KB at G = 16
    if (a.hd == 128) {
        hipLaunchKernelGGL(decode_attn_kernel<128>, grid, dim3(256), lds, st, a);
        hipLaunchKernelGGL(decode_combine_kernel<128>, cgrid, dim3(128), 0, st, a);
    } else {
        hipLaunchKernelGGL(decode_attn_kernel<64>, grid, dim3(256), lds, st, a);
        hipLaunchKernelGGL(decode_combine_kernel<64>, cgrid, dim3(64), 0, st, a);
    }
}

// =============================================================================================
// Prefill: causal attention of whole prompts, reading the K/V the same layer call has just
// written to the pools.  A workgroup owns one query head and a PAIR of 128-query tiles of one
// prompt, tile n-1-p then tile p, so that every workgroup does the same amount of causal work.
// Wave w owns 32 query rows of the tile; keys are consumed 64 (= 4 blocks) at a time through two
// LDS buffers: the next key tile's global loads are in flight while the current one is multiplied,
// one barrier per key tile.  The prompt's block ids are copied to LDS once, so a key tile costs one
// memory round trip (pool) instead of two chained ones (table, then pool).
// The K tile sits in LDS as its four blocks in the pool's own order and the V tile as [block][8-token half][dim]:
// the 16 lanes of a fragment read are then 16 consecutive 16-byte chunks (no bank conflicts, no swizzle), every
// read address is a per-lane base plus a constant, and a whole tile comes in by LDS-DMA (global -> LDS, no
// staging registers, no LDS stores).
//
// What bounds it on long prompts: every wave reads the whole 32 KB K/V tile from LDS for its 32 queries, one
// kilobyte of LDS reads per MFMA, which with four matrix cores per CU is the LDS's whole bandwidth (128 bytes
// per cycle); and per score there are about as many vector cycles (scale, exponential at quarter rate, sum,
// maximum, conversion) as matrix cycles.  Two workgroups per CU (two waves per SIMD) overlap the two kinds of
// work as far as the LDS allows.  Measured alternative, dropped: two 32-query strips per wave (each K and V
// fragment feeds two MFMAs: half the LDS reads), which needs both strips' accumulators (128 registers) and so
// leaves one wave per SIMD; bit-identical results, but 1.4-1.8x SLOWER at every size (16384 tokens: 3.48
// against 2.44 ms on the whole chip) although strip 1's exponentials were placed under strip 0's P V MFMAs:
// with a single wave per SIMD every dependent chain of the softmax (running maximum, half-wave exchanges, the
// rescale decision) is exposed, and what the second wave hides here for nothing would have to be software
// pipelined by hand across key tiles.
// =============================================================================================
template <int HD>
__global__ __launch_bounds__(256, 2) void prefill_attn_kernel(PrefillAttnArgs a) {
    constexpr int CPR = HD / 8;   // 16-byte chunks per K row
    constexpr int KS = HD / 16;   // 32x32x16 steps over head_dim
    constexpr int DT = HD / 32;   // 32-row tiles of O^T
    constexpr int NKC = (64 * CPR) / 256, NVC = (HD * 8) / 256;  // chunks per thread per tile
    extern __shared__ __attribute__((aligned(1024))) bf16_t smem_attn[];
    bf16_t *Ks = smem_attn;                 // [2][64 * HD]
    bf16_t *Vs = smem_attn + 2 * 64 * HD;   // [2][HD * 64]
    int32_t *s_tab = (int32_t *)(smem_attn + 4 * 64 * HD);   // [PREFILL_TAB_LDS] block ids of this prompt

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c32 = lane & 31, h = lane >> 5;

    // (request, pair) of this workgroup
    int pr = blockIdx.x, req = 0, nt = 0;
    for (;; ++req) {
        nt = (a.seq.cu[req + 1] - a.seq.cu[req] + 127) >> 7;
        const int np = (nt + 1) >> 1;
        if (pr < np || req + 1 >= a.seq.n_req) break;
        pr -= np;
    }
    if (pr >= ((nt + 1) >> 1)) return;
    const int row0 = a.seq.cu[req];
    const int len = a.seq.cu[req + 1] - row0;
    // a later chunk of a prompt: its first row sits at position `prior`, and the positions before it are keys too
    // (read from the cache like the chunk's own); key positions below are absolute, query rows relative to the chunk
    const int prior = a.seq.start[req];
    const int tot = prior + len;
    const int hq = blockIdx.y;
    const int G = a.Hq / a.Hkv;
    const int hk = hq / G;
    const int32_t *tab = a.tables + (size_t)req * a.max_blk;
    const float sc = a.scale_log2;
    const int n_blk = (tot + 15) >> 4;
    for (int i = tid; i < min(n_blk, PREFILL_TAB_LDS); i += 256) s_tab[i] = tab[i];
    // (two separate loads: a pointer chosen between the LDS copy and the table would become a generic-address
    // load, which waits for every outstanding LDS and global access)
    auto block_of = [&](int bi) {
        int b = s_tab[min(bi, PREFILL_TAB_LDS - 1)];
        if (bi >= PREFILL_TAB_LDS) {
            int g = tab[bi];
            asm volatile("" : "+v"(g));   // pins the global load to this branch: the two loads must not be merged
            b = g;
        }
        return b;
    };

    // K tile in LDS: the four blocks one after the other, each in the pool's own order (element offset of row r, 16-byte column cc)
    auto klds = [](int r, int cc) { return (r >> 4) * (16 * HD) + kpool_chunk_offset(r & 15, cc * 8); };

    // this thread's chunks of a key tile on the checked path: K chunk j = (row c/CPR, 16-byte column c%CPR),
    // V chunk j = (dim c>>3, block (c&7)>>1, 8-token half c&1), c = tid + 256 j
    // V tile in LDS: per block the 8-token halves apart, [block][half][dim][8 tokens]: the 16 lanes of a fragment read
    // (16 dims, one half) are 16 consecutive 16-byte chunks
    auto vlds = [](int blk, int half, int d) { return blk * (16 * HD) + half * (8 * HD) + d * 8; };
    // Brings key tile [kv0, kv0 + 64) into LDS buffer buf (nobody reads that buffer before the next barrier).
    auto load_tile = [&](int kv0, int buf) {
        bf16_t *ks = Ks + buf * 64 * HD;
        bf16_t *vs = Vs + buf * HD * 64;
        if (HD == 128 && kv0 + 64 <= tot && (kv0 >> 4) + 4 <= PREFILL_TAB_LDS) {
            const int b0 = kv0 >> 4;
            int blk[4];
            bool ok = true;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                blk[j] = __builtin_amdgcn_readfirstlane(s_tab[b0 + j]);
                ok = ok && (unsigned)blk[j] < (unsigned)a.n_blocks;
            }
            if (ok) {   // uniform; a tile with a bad block id takes the checked path below, which reports it
                // Whole tile by LDS-DMA (global -> LDS, 16 bytes per lane, lane l's bytes land at the window's
                // base + 16 l; no registers): wave w copies block w.  K keeps the pool's order (4 KB straight);
                // V's 16-byte chunk (dim d, half) goes to [half][d], so a lane fetches chunk (64 i + l, half).
                const int w = __builtin_amdgcn_readfirstlane(wave);
                const int bw = w == 0 ? blk[0] : w == 1 ? blk[1] : w == 2 ? blk[2] : blk[3];
                const size_t head = ((size_t)bw * a.Hkv + hk) * 16 * HD;
                const bf16_t *ksrc = a.k_pool + head + lane * 8;
                const bf16_t *vsrc = a.v_pool + head + lane * 16;
                bf16_t *kdst = ks + w * (16 * HD), *vdst = vs + w * (16 * HD);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(ksrc + j * 512),
                                                     (__attribute__((address_space(3))) void *)(kdst + j * 512), 16, 0, 0);
#pragma unroll
                for (int j = 0; j < 4; ++j)   // j = 2 * half + i
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void *)(vsrc + (j & 1) * (64 * 16) + (j >> 1) * 8),
                        (__attribute__((address_space(3))) void *)(vdst + (j >> 1) * (8 * HD) + (j & 1) * 512), 16, 0, 0);
                return;
            }
        }
        // checked path (a ragged last tile, a bad block id, head_dim 64): through registers
        bf16x8 rk[NKC], rv[NVC];
#pragma unroll
        for (int j = 0; j < NKC; ++j) {
            const int c = tid + 256 * j;
            const int r = c / CPR, cc = c % CPR;
            const int tok = kv0 + r;
            bf16x8 v = zero_bf16x8();
            if ((tok & ~15) < tot) {
                const int blk = block_of(tok >> 4);
                if ((unsigned)blk < (unsigned)a.n_blocks)
                    v = ld_bf16x8(a.k_pool + ((size_t)blk * a.Hkv + hk) * 16 * HD + kpool_chunk_offset(tok & 15, cc * 8));
                else if (cc == 0 && (tok & 15) == 0)
                    atomicOr(a.err_flag, 2);
            }
            rk[j] = v;
        }
#pragma unroll
        for (int j = 0; j < NVC; ++j) {
            const int c = tid + 256 * j;
            const int d = c >> 3, cc = c & 7;
            const int tok0 = kv0 + (cc >> 1) * 16 + (cc & 1) * 8;
            bf16x8 v = zero_bf16x8();
            if (tok0 < tot) {
                const int blk = block_of(tok0 >> 4);
                if ((unsigned)blk < (unsigned)a.n_blocks) {
                    v = ld_bf16x8(a.v_pool + (((size_t)blk * a.Hkv + hk) * HD + d) * 16 + (cc & 1) * 8);
                    if (tok0 + 8 > tot) {  // zero V past the prompt: 0 * garbage must not be NaN
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            if (tok0 + i >= tot) v[i] = (bf16_t)0.f;
                    }
                }
            }
            rv[j] = v;
        }
#pragma unroll
        for (int j = 0; j < NKC; ++j) {
            const int c = tid + 256 * j;
            *(bf16x8 *)&ks[klds(c / CPR, c % CPR)] = rk[j];
        }
#pragma unroll
        for (int j = 0; j < NVC; ++j) {
            const int c = tid + 256 * j;
            *(bf16x8 *)&vs[vlds((c & 7) >> 1, c & 1, c >> 3)] = rv[j];
        }
    };

    for (int which = 0; which < 2; ++which) {
        const int tile = which == 0 ? nt - 1 - pr : pr;   // the heavier tile first
        if (which == 1 && tile == nt - 1 - pr) break;
        const int q0 = tile * 128;
        const int q_local = q0 + wave * 32 + c32;
        const bool q_valid = q_local < len;
        const int q_row = q_valid ? q_local : len - 1;
        const int q_pos = prior + q_row;   // absolute position: the causal bound
        bf16x8 qf[KS];
        {
            const bf16_t *qp = a.q + (size_t)(row0 + q_row) * a.q_stride + (size_t)hq * HD + 8 * h;
#pragma unroll
            for (int s = 0; s < KS; ++s) qf[s] = ld_bf16x8(qp + 16 * s);
        }
        const int wave_q_min = prior + q0 + wave * 32;
        const int wave_q_max = min(wave_q_min + 31, tot - 1);
        const int kv_end = prior + min(q0 + 128, len);
        const int n_kv_tiles = (kv_end + 63) >> 6;

        float m_run = NEG_INF, l_run = 0.f;   // running max of raw scores, running sum
        f32x16 o[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;

        __syncthreads();   // s_tab visible; the previous tile's last reads done before buffer 0 is refilled
        load_tile(0, 0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the LDS-DMA loads have landed
        __syncthreads();
        for (int kt = 0; kt < n_kv_tiles; ++kt) {
            const int kv0 = kt * 64;
            const bool more = kt + 1 < n_kv_tiles;
            if (more) load_tile(kv0 + 64, (kt + 1) & 1);
            if (kv0 <= wave_q_max) {
                const bf16_t *ks = Ks + (kt & 1) * 64 * HD;
                const bf16_t *vs = Vs + (kt & 1) * HD * 64;
                f32x16 st[2];
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                    for (int i = 0; i < 16; ++i) st[t2][i] = 0.f;
                {
                    // K fragment i = (key half i & 1, head_dim step i >> 1), read four fragments ahead of its MFMA; the
                    // two score tiles alternate, each still summed over the steps in order
                    constexpr int NQK = 2 * KS, R = 4;
                    auto kread = [&](int i) { return *(const bf16x8 *)&ks[klds(32 * (i & 1) + c32, 2 * (i >> 1) + h)]; };
                    bf16x8 kf[R];
#pragma unroll
                    for (int i = 0; i < R; ++i) kf[i] = kread(i);
#pragma unroll
                    for (int i = 0; i < NQK; ++i) {
                        st[i & 1] = mfma32(kf[i % R], qf[i >> 1], st[i & 1]);
                        __builtin_amdgcn_sched_barrier(0);
                        if (i + R < NQK) kf[i % R] = kread(i + R);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                if (kv0 + 63 > wave_q_min) {   // only tiles that touch the diagonal need the mask
#pragma unroll
                    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const int key = kv0 + 32 * t2 + (i >> 2) * 8 + 4 * h + (i & 3);
                            if (key > q_pos) st[t2][i] = NEG_INF;
                        }
                }
                float m_tile = NEG_INF;
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                    for (int i = 0; i < 16; ++i) m_tile = fmaxf(m_tile, st[t2][i]);
                {   // the other half-wave holds the rest of this query column: one swap gives each lane both maxima
                    const uint32_t mb = __builtin_bit_cast(uint32_t, m_tile);
                    const auto sw = __builtin_amdgcn_permlane32_swap(mb, mb, false, false);
                    m_tile = fmaxf(__builtin_bit_cast(float, (uint32_t)sw[0]), __builtin_bit_cast(float, (uint32_t)sw[1]));
                }
                const float m_new = fmaxf(m_run, m_tile);
                const float m_safe = (m_new == NEG_INF) ? 0.f : m_new;
                const float ms = m_safe * sc;
                float psum = 0.f;
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float p = __builtin_amdgcn_exp2f(fmaf(st[t2][i], sc, -ms));
                        st[t2][i] = p;
                        psum += p;
                    }
                if (__any(m_new != m_run)) {   // the maximum rarely moves after the first tiles
                    const float alpha = __builtin_amdgcn_exp2f((m_run - m_safe) * sc);
                    l_run *= alpha;
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) o[dt] = o[dt] * alpha;
                    m_run = m_new;
                }
                l_run += psum;
                // V fragments are read one block (DT fragments) ahead of their MFMAs
                bf16x8 vfr[2][DT];
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) vfr[0][dt] = *(const bf16x8 *)&vs[vlds(0, h, 32 * dt + c32)];
#pragma unroll
                for (int blk4 = 0; blk4 < 4; ++blk4) {  // one 16-token block per MFMA step
                    // The score registers give lane half h the block's tokens 4h..4h+3 and 8+4h..8+4h+3.  The two
                    // half-waves (same query column) trade their middle pieces, h = 0 then holds tokens 0-7 and
                    // h = 1 tokens 8-15: the contraction slices of V's own layout, 16 bytes per (dim, half).
                    bf16x8 pf;
#pragma unroll
                    for (int t = 0; t < 8; ++t) pf[t] = (bf16_t)st[blk4 >> 1][8 * (blk4 & 1) + t];
                    typedef uint32_t u32x4p __attribute__((ext_vector_type(4)));
                    u32x4p pr4 = __builtin_bit_cast(u32x4p, pf);
#pragma unroll
                    for (int u = 0; u < 2; ++u) {   // upper half-wave of word u <-> lower half-wave of word u + 2
                        const auto sw = __builtin_amdgcn_permlane32_swap(pr4[u], pr4[u + 2], false, false);
                        pr4[u] = sw[0];
                        pr4[u + 2] = sw[1];
                    }
                    pf = __builtin_bit_cast(bf16x8, pr4);
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        if (blk4 + 1 < 4) vfr[(blk4 + 1) & 1][dt] = *(const bf16x8 *)&vs[vlds(blk4 + 1, h, 32 * dt + c32)];
                        o[dt] = mfma32(vfr[blk4 & 1][dt], pf, o[dt]);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the LDS-DMA loads have landed
            __syncthreads();
        }
        l_run += __shfl_xor(l_run, 32, 64);
        if (q_valid) {
            const float inv = 1.0f / l_run;
            // the output feeds the output projection: fragment-packed operand layout
            const int Mt = a.Mt_out ? a.Mt_out : packed_mt(a.seq.cu[a.seq.n_req]);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    bf16x4 v;
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = (bf16_t)(o[dt][4 * j + i] * inv);
                    const int col = hq * HD + 32 * dt + 8 * j + 4 * h;
                    *(bf16x4 *)(a.out + packed_offset(row0 + q_local, col, Mt) + (col & 7)) = v;
                }
        }
    }
}

void launch_prefill_attention(hipStream_t st, const PrefillAttnArgs &a) {
    int pairs = 0;
    for (int r = 0; r < a.seq.n_req; ++r) pairs += ((a.seq.cu[r + 1] - a.seq.cu[r] + 127) / 128 + 1) / 2;
    if (pairs <= 0) return;
    dim3 grid(pairs, a.Hq);
    if (a.hd == 128) {
        constexpr int lds = 4 * 64 * 128 * 2 + PREFILL_TAB_LDS * 4;
        static bool set = false;
        if (!set) {
            (void)hipFuncSetAttribute((const void *)prefill_attn_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            set = true;
        }
        hipLaunchKernelGGL(prefill_attn_kernel<128>, grid, dim3(256), lds, st, a);
    } else {
        hipLaunchKernelGGL(prefill_attn_kernel<64>, grid, dim3(256), 4 * 64 * 64 * 2 + PREFILL_TAB_LDS * 4, st, a);
    }
}

void attention_kernels_init() {
    (void)hipFuncSetAttribute((const void *)prefill_attn_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              4 * 64 * 128 * 2 + PREFILL_TAB_LDS * 4);
}

