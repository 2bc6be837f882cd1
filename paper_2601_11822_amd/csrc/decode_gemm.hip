// Decode-side projections (at most 64 rows): weight-streaming GEMMs with the RMSNorm folded in.
//
// A decode step multiplies a few rows by every weight of the layer once (paper section 2.1: decode is
// bound by reading weights and cache, not by arithmetic), so each of the four projections is a stream of
// its matrix through the matrix cores at the rate the partition's memory path allows, and everything
// around that stream is overhead to be removed:
//
//   * RMSNorm needs a whole row before it can scale an element, which would cost a kernel of its own in
//     front of the QKV and the gate/up projection.  But the row's scale is one scalar: with
//     s = 1/sqrt(mean(x^2) + eps),  RMSNorm(x; g) W^T = s * ((x . g) W^T).  The streaming kernel therefore
//     reads the hidden state x row-major as it is, multiplies by the gain while it stages the rows in LDS,
//     and adds up the squares of the part of each row it sees; the per-slice sums of squares go out
//     beside the partial products, and the consumer of the partial products (the rotary/KV epilogue, the
//     SwiGLU epilogue) forms s and applies it.  No normalised copy of x is ever written.
//   * The 4 waves of a workgroup take different weight rows over the SAME K slice, so the slice's
//     activation rows are fetched once per workgroup into LDS (double buffered, 16 k-blocks at a time)
//     and every wave's vector memory path carries weights only: each wave keeps PD one-kilobyte weight
//     fragments in flight in a register ring that is refilled right after the MFMAs that free a slot.
//   * K is cut into S slices so that every compute unit of a partition holds several workgroups; S and
//     the tile counts follow from (N, K) alone, and the slices are added in slice order by the epilogue,
//     so results do not depend on the CU share.  Loads past a slice's end re-read its last k-block
//     (cache hits), so the ring's wait counts stay static without fetching a byte of another slice.
#include <algorithm>

#include "kernels.h"

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// z * sigmoid(z); the reciprocal is the hardware's one-instruction approximation (1 ulp): an IEEE division costs
// ten more vector instructions per element of a 256x256 epilogue, for digits far below the bf16 the result is rounded to
__device__ __forceinline__ float silu_f(float z) { return z * __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }

#define DS_CH 16   // k-blocks per activation chunk: two 32 KB slabs in LDS

// ACT 0: activations fragment-packed (two 32-row tiles per k-block), as the attention merge and the SwiGLU
//        epilogue write them.
// ACT 1: activations row-major [M][K]; multiplied by gain[K] while staged; sums of squares written out.
// PAIR : RT == 2 and the wave's two tiles are row tile f of Wp (gate) and of Wp2 (up); else RT tiles of Wp.
// PSPLIT: RT == 1 and the pair is spread over waves: waves 0-1 take gate tiles 2x, 2x+1 of Wp, waves 2-3 the matching
//         up tiles of Wp2 (half as many features per workgroup as PAIR, the same sums and the same output columns).
template <int ACT, int RT, bool PAIR, int PD, bool PSPLIT = false>
__global__ __launch_bounds__(256, 2) void dstream_kernel(DGemmArgs a, int kb_per_wg, int Nv) {
    constexpr int CH = DS_CH;
    // An activation piece is stored 8 steps after its load was issued, right behind a weight fragment that is
    // consumed PD steps after ITS issue: with PD == 8 the two are due together and the in-order wait counts cost
    // nothing; a deeper ring would make every piece wait for weights that are not needed yet (measured: 2x slower).
    // Taking the pieces out of these waves altogether -- one or two extra waves per workgroup that only stage the
    // next slab, the four streaming waves with a ring of 16 (128 KB of weights in flight per workgroup) -- gave the
    // same results and was slower on all 256 CUs (QKV 20.2 -> 23.9 us, gate/up 42.6 -> 50.4, output/down 21.3 -> 22.3)
    // and no faster beside a prefill pass on 128: depth in flight is not what bounds this stream.
    static_assert(CH % PD == 0, "ring slots are static inside an unrolled chunk");
    static_assert(!PAIR || RT == 2, "a pair is a gate tile and an up tile");
    static_assert(!PSPLIT || (RT == 1 && !PAIR), "a split pair is one tile per wave");
    extern __shared__ __attribute__((aligned(1024))) bf16_t slab[];   // [2][CH][2 row tiles][64 lanes][8]
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c32 = lane & 31, h = lane >> 5;
    const int M = a.M, K = a.K;
    const int kb_begin = blockIdx.y * kb_per_wg;
    const int kb_end = kb_begin + kb_per_wg - 1;     // loads past the slice re-read its last k-block
    const int nchunks = kb_per_wg / CH;
    const int Nt = ((a.N + 63) / 64) * 2;
    const size_t wstride = (size_t)Nt * 512;
    const bf16_t *w[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        if (PAIR)
            w[t] = (t ? a.Wp2 : a.Wp) + (size_t)min(4 * (int)blockIdx.x + wave, Nt - 1) * 512 + lane * 8;
        else if (PSPLIT)
            w[t] = (wave >= 2 ? a.Wp2 : a.Wp) + (size_t)min(2 * (int)blockIdx.x + (wave & 1), Nt - 1) * 512 + lane * 8;
        else
            w[t] = a.Wp + (size_t)min((4 * (int)blockIdx.x + wave) * RT + t, Nt - 1) * 512 + lane * 8;
    }

    f32x16 acc[RT][2];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // ---- activation pieces: a chunk's slab is 32 pieces of 1 KB; wave w brings 8 of them per chunk
    // ACT 0: piece q = 8 wave + j is (k-block q/2, row tile q%2) of the packed matrix: one contiguous kilobyte.
    // ACT 1: piece j of wave w is rows 8j..8j+7 x the chunk's 16-byte columns 8w..8w+7 (lane l: row 8j + l%8,
    //        column 8w + l/8): eight 128-byte runs of eight rows, stored to the fragment order
    //        ((k-block*2 + row tile)*64 + half*32 + row%32).
    float ssq[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) ssq[j] = 0.f;
    const int k8 = 8 * wave + (lane >> 3);            // ACT 1: this lane's 16-byte column inside a chunk
    auto x_addr = [&](int chunk, int j) -> const bf16_t * {
        if (ACT == 0) {
            const int q = 8 * wave + j;
            const size_t kb = (size_t)min(kb_begin + chunk * CH + (q >> 1), kb_end);
            return a.A_packed + kb * 1024 + (q & 1) * 512 + lane * 8;
        } else {
            const int m = min(8 * j + (lane & 7), M - 1);
            const int ch = min(chunk, nchunks - 1);
            return a.X_rows + (size_t)m * K + (size_t)(kb_begin + ch * CH) * 16 + k8 * 8;
        }
    };
    auto g_addr = [&](int chunk) -> const bf16_t * {
        const int ch = min(chunk, nchunks - 1);
        return a.gain + (size_t)(kb_begin + ch * CH) * 16 + k8 * 8;
    };
    auto x_store = [&](bf16_t *dst_slab, int j, bf16x8 xv, bf16x8 gv, bool count) {
        if (ACT == 0) {
            *(bf16x8 *)&dst_slab[(8 * wave + j) * 512 + lane * 8] = xv;
        } else {
            const int m = 8 * j + (lane & 7);
            bf16x8 hv;
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float f = m < M ? (float)xv[e] : 0.f;
                s += f * f;
                hv[e] = (bf16_t)(f * (float)gv[e]);
            }
            if (count) ssq[j] += s;
            *(bf16x8 *)&dst_slab[(((k8 >> 1) * 2 + (m >> 5)) * 64 + (k8 & 1) * 32 + (m & 31)) * 8] = hv;
        }
    };
    {   // chunk 0's slab, up front
        bf16x8 t[8], g = zero_bf16x8();
        if (ACT == 1) g = ld_bf16x8(g_addr(0));
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = ld_bf16x8(x_addr(0, j));
#pragma unroll
        for (int j = 0; j < 8; ++j) x_store(slab, j, t[j], g, true);
    }
    bf16x8 rw[PD][RT], rxs[8], rg = zero_bf16x8();
    auto load_w = [&](int p, int step) {
        const size_t kb = (size_t)min(kb_begin + step, kb_end);
#pragma unroll
        for (int t = 0; t < RT; ++t) rw[p][t] = ld_bf16x8_stream(w[t] + kb * wstride);
    };
#pragma unroll
    for (int p = 0; p < PD; ++p) load_w(p, p);
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

    for (int c = 0; c < nchunks; ++c) {
        const bf16_t *cur = slab + (c & 1) * (CH * 1024) + lane * 8;
        bf16_t *nxt = slab + ((c + 1) & 1) * (CH * 1024);
        const bool more = c + 1 < nchunks;
#pragma unroll
        for (int s = 0; s < CH; ++s) {
            const int p = s % PD;
            const bf16x8 x0 = *(const bf16x8 *)&cur[(2 * s) * 512], x1 = *(const bf16x8 *)&cur[(2 * s + 1) * 512];
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                acc[t][0] = mfma32(rw[p][t], x0, acc[t][0]);
                acc[t][1] = mfma32(rw[p][t], x1, acc[t][1]);
            }
            // the piece of the next slab that was fetched eight steps ago
            if (s >= 8) x_store(nxt, s - 8, rxs[s - 8], rg, more);
            load_w(p, c * CH + s + PD);
            if (s < 8) {
                if (ACT == 1 && s == 0) rg = ld_bf16x8(g_addr(c + 1));
                rxs[s] = ld_bf16x8(x_addr(c + 1, s));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // every wave has read slab c and written its pieces of slab c+1; the weight loads stay in flight
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }
    // each wave owns its rows: partial tile straight from the accumulators
#pragma unroll
    for (int tn = 0; tn < RT; ++tn)
#pragma unroll
        for (int tm = 0; tm < 2; ++tm) {
            const int m = 32 * tm + c32;
            if (m >= M) continue;
            // virtual columns: 64 per feature tile of a pair (32 gate, then 32 up), else the weight rows themselves
            const int col = PSPLIT ? (2 * (int)blockIdx.x + (wave & 1)) * 64 + 32 * (wave >> 1)
                                   : (int)blockIdx.x * (128 * RT) + wave * (32 * RT) + 32 * tn;
            float *dst = a.part + ((size_t)blockIdx.y * M + m) * Nv + col;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x4 v = {acc[tn][tm][4 * j], acc[tn][tm][4 * j + 1], acc[tn][tm][4 * j + 2], acc[tn][tm][4 * j + 3]};
                *(f32x4 *)(dst + 8 * j + 4 * h) = v;
            }
        }
    if (ACT == 1 && blockIdx.x == 0) {
        // sums of squares of the slice: lanes with the same l%8 hold the same row, then the 4 waves in wave order
        float *red = (float *)slab;   // free since the last barrier
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float v = ssq[j];
            v += __shfl_xor(v, 8, 64);
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            if (lane < 8) red[wave * 64 + 8 * j + lane] = v;
        }
        __syncthreads();
        if (tid < 64) a.ssq_part[blockIdx.y * 64 + tid] = ((red[tid] + red[64 + tid]) + red[128 + tid]) + red[192 + tid];
    }
}

// ---------------------------------------------------------------------------------------------
// The schedule of a projection: a function of (N, K, pair) alone.
// ---------------------------------------------------------------------------------------------
bool dgemm_applies(int N, int K) { return K >= 256 && K % 256 == 0 && N >= 128 && N % 4 == 0; }

DGemmPlan dgemm_plan(int N, int K, bool pair) {
    DGemmPlan p{};
    p.pair = pair;
    // a workgroup's 4 waves take two 32-row weight tiles each: 256 rows, or 128 gate rows and their up rows
    p.cols = pair ? (N + 127) / 128 : (N + 255) / 256;
    p.Nv = p.cols * 256;
    const int Kb = K / 16;
    // K slices: as many as keep the launch within about one workgroup per compute unit of a half-chip partition
    // (128) with at least 32 k-blocks (two chunks) per slice, in whole chunks.  (A wide gate/up pair was split
    // once more before, for the whole chip's sake: 2 % slower on a 128-CU partition; the whole chip now gets its
    // workgroups from the half-height forms of the launcher instead, which leave the sums as they are.)  Measured on the Llama-3-8B shapes: on a partition the stream is bound by what one compute unit can
    // pull, so one large workgroup per unit beats two half-sized ones (the activation rows are staged once
    // instead of twice); on the whole chip more, smaller workgroups win a little -- this is the better compromise.
    const int cap = 128;
    int S = 1;
    for (int s = 2; s <= 64; ++s)
        if (Kb % (s * DS_CH) == 0 && Kb / s >= 2 * DS_CH && p.cols * s <= cap) S = s;
    p.S = S;
    p.kb_per_wg = Kb / S;
    return p;
}

size_t dgemm_partial_elems(int M, int N, int K, bool pair) {
    const DGemmPlan p = dgemm_plan(N, K, pair);
    return (size_t)p.S * (size_t)M * (size_t)p.Nv;
}

// `narrow`: workgroups of 128 weight rows (one tile per wave) instead of 256, twice as many of them; for a gate/up
// pair, 64 features per workgroup (two gate tiles and their two up tiles, one per wave) instead of 128.
// The K slices and the order of every sum are those of the plan, so the
// results are the same bits; only the number of compute units that have a workgroup changes.  The caller picks the
// form per projection with dgemm_prefers_half_height: on the whole chip the plan's 96-128 workgroups leave too many
// units idle (Llama-3-8B decode step alone on 256 CUs 0.243 -> 0.2325 ms with half-height workgroups), on a 128-CU
// partition one large workgroup per unit is the faster shape (0.2914 against 0.2992 ms), and where the full-height
// count fills the units badly (128 workgroups on 96 units: two rounds, the second a third full) the half-height
// form's three shorter rounds win (decode step on 96 CUs 0.402 -> 0.393 ms, on 192 CUs 0.265 -> 0.261 ms).
// Which of the two forms a side of `cus` compute units launches: rounds of workgroups (one per unit) times what a
// workgroup moves.  A full-height workgroup streams its weights plus a quarter as many activation bytes (64 rows
// against 256), a half-height one half the weights and the same activations: 0.6 of the bytes.
bool dgemm_prefers_half_height(const DGemmPlan &p, int cus) {
    if (cus <= 0) return false;
    const int wgs = p.cols * p.S;
    const double full = (double)((wgs + cus - 1) / cus), half = 0.6 * (double)((2 * wgs + cus - 1) / cus);
    return half < full;
}

void launch_dgemm_partials(hipStream_t st, const DGemmArgs &a, const DGemmPlan &p, bool narrow) {
    constexpr int lds = 2 * DS_CH * 2048;
    const dim3 grid(p.cols, p.S), grid_narrow(2 * p.cols, p.S), block(256);
    const bool rows = a.X_rows != nullptr;
    if (p.pair && narrow) {
        if (rows) hipLaunchKernelGGL((dstream_kernel<1, 1, false, 8, true>), grid_narrow, block, lds, st, a, p.kb_per_wg, p.Nv);
        else hipLaunchKernelGGL((dstream_kernel<0, 1, false, 8, true>), grid_narrow, block, lds, st, a, p.kb_per_wg, p.Nv);
    } else if (p.pair) {
        if (rows) hipLaunchKernelGGL((dstream_kernel<1, 2, true, 8>), grid, block, lds, st, a, p.kb_per_wg, p.Nv);
        else hipLaunchKernelGGL((dstream_kernel<0, 2, true, 8>), grid, block, lds, st, a, p.kb_per_wg, p.Nv);
    } else if (narrow) {
        if (rows) hipLaunchKernelGGL((dstream_kernel<1, 1, false, 8>), grid_narrow, block, lds, st, a, p.kb_per_wg, p.Nv);
        else hipLaunchKernelGGL((dstream_kernel<0, 1, false, 8>), grid_narrow, block, lds, st, a, p.kb_per_wg, p.Nv);
    } else {
        if (rows) hipLaunchKernelGGL((dstream_kernel<1, 2, false, 8>), grid, block, lds, st, a, p.kb_per_wg, p.Nv);
        else hipLaunchKernelGGL((dstream_kernel<0, 2, false, 8>), grid, block, lds, st, a, p.kb_per_wg, p.Nv);
    }
}

// ---------------------------------------------------------------------------------------------
// Epilogues: the K slices are added in slice order; where the projection's input was an RMSNorm, the
// row's scale is formed here from the slices' sums of squares (in slice order) and applied first.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float row_scale(const float *ssq_part, int S_ssq, int m, int d, float eps) {
    float t = 0.f;
    for (int s = 0; s < S_ssq; ++s) t += ssq_part[s * 64 + m];
    return 1.0f / sqrtf(t / (float)d + eps);
}

// One thread per 4 output columns.  RESIDUAL: out = resid + sum (row-major).  SWIGLU: out = silu(s g) * (s u),
// fragment-packed for the down projection (gate and up of a feature sit 32 virtual columns apart).
template <int EPI>
__global__ __launch_bounds__(256) void dgemm_epilogue_kernel(DEpiArgs a) {
    const int M = a.M, N = a.N;
    const int groups = N >> 2;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * groups) return;
    const int m = idx / groups, n = (idx % groups) * 4;
    bf16x4 v;
    if (EPI == EPI_SWIGLU) {
        const int col = (n >> 5) * 64 + (n & 31);
        f32x4 g = {0.f, 0.f, 0.f, 0.f}, u = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < a.S; ++s) {
            const float *p = a.part + ((size_t)s * M + m) * a.Nv + col;
            g += *(const f32x4 *)p;
            u += *(const f32x4 *)(p + 32);
        }
        const float sc = a.ssq_part ? row_scale(a.ssq_part, a.S_ssq, m, a.d, a.eps) : 1.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = (bf16_t)(silu_f(g[i] * sc) * (u[i] * sc));
        *(bf16x4 *)(a.out + packed_offset(m, n, packed_mt(M)) + (n & 7)) = v;
    } else {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < a.S; ++s) acc += *(const f32x4 *)(a.part + ((size_t)s * M + m) * a.Nv + n);
        const bf16x4 r = *(const bf16x4 *)(a.resid + (size_t)m * N + n);
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = (bf16_t)(acc[i] + (float)r[i]);
        *(bf16x4 *)(a.out + (size_t)m * N + n) = v;
    }
}

void launch_dgemm_epilogue(hipStream_t st, const DEpiArgs &a, int epi) {
    const int blocks = (a.M * (a.N / 4) + 255) / 256;
    if (epi == EPI_SWIGLU) hipLaunchKernelGGL(dgemm_epilogue_kernel<EPI_SWIGLU>, dim3(blocks), dim3(256), 0, st, a);
    else hipLaunchKernelGGL(dgemm_epilogue_kernel<EPI_RESIDUAL>, dim3(blocks), dim3(256), 0, st, a);
}

// QKV epilogue of a decode step: sums the K slices, applies the first RMSNorm's row scale, rotates q and k
// at the row's position (rotate-half pairs (i, i + hd/2), angles from the host-built table), stores q | k | v
// as bf16 rows for the attention kernel, and appends k and v to the paged cache through the block table:
// K in the pool's fragment order (kpool_chunk_offset), V token-minor.  One thread owns 4 dims of a pair's
// lower half and the matching 4 of the upper half.  A position outside the rotary table or a block id
// outside the pool is never used as an index: the row's cache write is skipped and the error word raised.
template <int HD>
__global__ __launch_bounds__(256) void qkv_rope_epilogue_kernel(QkvEpiArgs a) {
    constexpr int TPH = HD / 8;           // threads per head
    constexpr int HPW = 256 / TPH;        // heads per workgroup
    const int m = blockIdx.x, tid = threadIdx.x;
    const int head = blockIdx.y * HPW + tid / TPH;
    const int n_heads = a.Hq + 2 * a.Hkv;
    if (head >= n_heads) return;
    const int i0 = (tid % TPH) * 4, half = HD / 2;
    const int pos = a.ctx_lens[m];
    const bool pos_ok = pos >= 0 && pos < a.max_pos;
    if (!pos_ok && tid == 0 && blockIdx.y == 0) atomicOr(a.err_flag, 1);
    f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < a.S; ++s) {
        const float *p = a.part + ((size_t)s * a.M + m) * a.Nv + head * HD + i0;
        lo += *(const f32x4 *)p;
        hi += *(const f32x4 *)(p + half);
    }
    const float sc = row_scale(a.ssq_part, a.S, m, a.d, a.eps);
    lo *= sc;
    hi *= sc;
    bf16x4 olo, ohi;
    if (head < a.Hq + a.Hkv) {
        if (!pos_ok) return;
        const CosSin *tab = a.table + (size_t)pos * half + i0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const CosSin cs = tab[i];
            olo[i] = (bf16_t)(lo[i] * cs.c - hi[i] * cs.s);
            ohi[i] = (bf16_t)(hi[i] * cs.c + lo[i] * cs.s);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            olo[i] = (bf16_t)lo[i];
            ohi[i] = (bf16_t)hi[i];
        }
    }
    bf16_t *row = a.qkv + (size_t)m * (n_heads * HD) + head * HD;
    *(bf16x4 *)(row + i0) = olo;
    *(bf16x4 *)(row + half + i0) = ohi;
    if (head < a.Hq || !pos_ok) return;
    const int bi = pos / RS_BLOCK_TOKENS, slot = pos % RS_BLOCK_TOKENS;
    int blk = -1;
    if (bi < a.max_blk) blk = a.tables[(size_t)m * a.max_blk + bi];
    if ((unsigned)blk >= (unsigned)a.n_blocks) {
        if (tid % TPH == 0 && head == a.Hq) atomicOr(a.err_flag, 2);
        return;
    }
    if (head < a.Hq + a.Hkv) {
        bf16_t *dst = a.k_pool + ((size_t)blk * a.Hkv + (head - a.Hq)) * RS_BLOCK_TOKENS * HD;
        *(bf16x4 *)(dst + kpool_chunk_offset(slot, i0 & ~7) + (i0 & 7)) = olo;
        *(bf16x4 *)(dst + kpool_chunk_offset(slot, (half + i0) & ~7) + (i0 & 7)) = ohi;
    } else {
        bf16_t *dst = a.v_pool + ((size_t)blk * a.Hkv + (head - a.Hq - a.Hkv)) * HD * RS_BLOCK_TOKENS + slot;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dst[(i0 + i) * RS_BLOCK_TOKENS] = olo[i];
            dst[(half + i0 + i) * RS_BLOCK_TOKENS] = ohi[i];
        }
    }
}

void launch_qkv_rope_epilogue(hipStream_t st, const QkvEpiArgs &a) {
    const int n_heads = a.Hq + 2 * a.Hkv;
    if (a.hd == 128) {
        hipLaunchKernelGGL(qkv_rope_epilogue_kernel<128>, dim3(a.M, (n_heads + 15) / 16), dim3(256), 0, st, a);
    } else {
        hipLaunchKernelGGL(qkv_rope_epilogue_kernel<64>, dim3(a.M, (n_heads + 31) / 32), dim3(256), 0, st, a);
    }
}

void decode_gemm_kernels_init() {
    auto set = [](const void *f) { (void)hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * DS_CH * 2048); };
    set((const void *)dstream_kernel<0, 2, false, 8>);
    set((const void *)dstream_kernel<1, 2, false, 8>);
    set((const void *)dstream_kernel<0, 2, true, 8>);
    set((const void *)dstream_kernel<1, 2, true, 8>);
    set((const void *)dstream_kernel<0, 1, false, 8>);
    set((const void *)dstream_kernel<1, 1, false, 8>);
    set((const void *)dstream_kernel<0, 1, false, 8, true>);
    set((const void *)dstream_kernel<1, 1, false, 8, true>);
}
