// bf16 GEMMs out = epi(A[M,K] * W[N,K]^T) on the gfx950 matrix cores (fp32 accumulation).
//
// A lane's 8-element MFMA fragment is 8 consecutive k of one row: one 16-byte chunk, and the unit
// of the fragment-packed operand layout (packed_offset) that the activations are always stored in.
// The weight tile is the MFMA "row" operand and the activation tile the "column" operand:
// a lane then owns 4 consecutive output columns of one output row, which makes the epilogues
// (residual add, SwiGLU, bf16 pack) plain per-lane code with 8-byte stores.
#include <algorithm>
#include <type_traits>

#include "kernels.h"

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// z * sigmoid(z); the reciprocal is the hardware's one-instruction approximation (1 ulp): an IEEE division costs
// ten more vector instructions per element of a 256x256 epilogue, for digits far below the bf16 the result is rounded to
__device__ __forceinline__ float silu_f(float z) { return z * __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }
// 4 consecutive output columns (n % 4 == 0) of row m
__device__ __forceinline__ void store_out4(const GemmArgs &a, int m, int n, bf16x4 v) {
    bf16_t *dst = a.out_packed ? a.out + packed_offset(m, n, packed_mt(a.M)) + (n & 7) : a.out + (size_t)m * a.N + n;
    *(bf16x4 *)dst = v;
}

// ---------------------------------------------------------------------------------------------
// Tiled kernel: BM x BN output tile per 256-thread workgroup (2x2 waves), BK = 64, operands
// (fragment-packed A, row-major W) staged global -> registers -> LDS (16-byte chunks, chunk index XOR (row>>1)&7 against bank
// conflicts on the 64-bank LDS), next tile's global loads in flight during the MFMAs.  Every tail (M, N, K) is
// handled by predicated zero-filled loads and predicated stores.
//
// SwiGLU: the B tile interleaves 32 gate rows with the 32 matching up rows, so gate and up of
// one output element sit in the same lane and register index of neighbouring accumulators.
// ---------------------------------------------------------------------------------------------
template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(GemmArgs a) {
    constexpr int BK = 64;
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int CA = BM / 32, CB = BN / 32;  // 16-byte chunks per thread per tile
    __shared__ __attribute__((aligned(16))) bf16_t As[BM * BK];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[BN * BK];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int c32 = lane & 31, h = lane >> 5;
    const int M = a.M, N = a.N, K = a.K;
    const int bm = blockIdx.y * BM;
    const int nb = blockIdx.x;

    // global row pointers of this thread's chunks
    const bf16_t *pa[CA];
    const bf16_t *pb[CB];
    const int cc = tid & 7;  // chunk column (same for all of a thread's chunks)
    const int Mt = packed_mt(M);
#pragma unroll
    for (int j = 0; j < CA; ++j) {
        const int r = (tid >> 3) + 32 * j;
        const int m = bm + r;
        pa[j] = (m < M) ? a.A + packed_offset(m, cc * 8, Mt) : nullptr;   // chunk (m, k0 + 8cc) for k0 = 0
    }
    const size_t a_kmul = (size_t)Mt * 32;   // a step of 64 in k is 4 k blocks of Mt KB
#pragma unroll
    for (int j = 0; j < CB; ++j) {
        const int r = (tid >> 3) + 32 * j;  // row of the B tile
        if (EPI == EPI_SWIGLU) {
            const int t = r >> 5;
            const int f = nb * (BN / 2) + (t >> 1) * 32 + (r & 31);
            pb[j] = (f < N) ? ((t & 1) ? a.W2 : a.W) + (size_t)f * K + cc * 8 : nullptr;
        } else {
            const int n = nb * BN + r;
            pb[j] = (n < N) ? a.W + (size_t)n * K + cc * 8 : nullptr;
        }
    }

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    bf16x8 ra[CA], rb[CB];
    auto gload = [&](int k0) {
        const bool kin = k0 + cc * 8 < K;
#pragma unroll
        for (int j = 0; j < CA; ++j) ra[j] = (kin && pa[j]) ? ld_bf16x8(pa[j] + k0 * a_kmul) : zero_bf16x8();
#pragma unroll
        for (int j = 0; j < CB; ++j) rb[j] = (kin && pb[j]) ? ld_bf16x8(pb[j] + k0) : zero_bf16x8();
    };
    gload(0);
    for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
        for (int j = 0; j < CA; ++j) {
            const int r = (tid >> 3) + 32 * j;
            *(bf16x8 *)&As[r * BK + ((cc ^ ((r >> 1) & 7)) << 3)] = ra[j];
        }
#pragma unroll
        for (int j = 0; j < CB; ++j) {
            const int r = (tid >> 3) + 32 * j;
            *(bf16x8 *)&Bs[r * BK + ((cc ^ ((r >> 1) & 7)) << 3)] = rb[j];
        }
        __syncthreads();
        if (k0 + BK < K) gload(k0 + BK);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            bf16x8 wf[TN], xf[TM];
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int r = wn * WN + 32 * tn + c32;
                wf[tn] = *(const bf16x8 *)&Bs[r * BK + (((2 * s + h) ^ ((r >> 1) & 7)) << 3)];
            }
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const int r = wm * WM + 32 * tm + c32;
                xf[tm] = *(const bf16x8 *)&As[r * BK + (((2 * s + h) ^ ((r >> 1) & 7)) << 3)];
            }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = mfma32(wf[tn], xf[tm], acc[tn][tm]);
        }
        __syncthreads();
    }

    // epilogue: lane owns row m, columns n0 + 8j + 4h + (0..3)
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int m = bm + wm * WM + 32 * tm + c32;
        if (m >= M) continue;
        if (EPI == EPI_SWIGLU) {
#pragma unroll
            for (int p = 0; p < TN / 2; ++p)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int f = nb * (BN / 2) + (wn * (TN / 2) + p) * 32 + 8 * j + 4 * h;
                    if (f >= N) continue;
                    bf16x4 v;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        v[i] = (bf16_t)(silu_f(acc[2 * p][tm][4 * j + i]) * acc[2 * p + 1][tm][4 * j + i]);
                    store_out4(a, m, f, v);
                }
        } else {
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int n = nb * BN + wn * WN + 32 * tn + 8 * j + 4 * h;
                    if (n >= N) continue;
                    bf16x4 v;
                    if (EPI == EPI_RESIDUAL) {
                        const bf16x4 r = *(const bf16x4 *)(a.resid + (size_t)m * N + n);
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] = (bf16_t)(acc[tn][tm][4 * j + i] + (float)r[i]);
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] = (bf16_t)acc[tn][tm][4 * j + i];
                    }
                    store_out4(a, m, n, v);
                }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Direct kernel (K % 32 == 0): same tiling and epilogues as the tiled kernel, but both operands
// are read in the fragment-packed layout (activations as their producers wrote them, weights from
// the library's packed copies) and go global -> LDS with the 16-byte LDS-DMA load (no register
// staging) through a ring of NS LDS stages of BK = 32, so that a K tile is requested NS-1 tiles
// (several microseconds of MFMA work) before it is consumed: HBM latency is covered although only
// one wave runs per SIMD.
//
// A wave-wide load moves one 1 KB fragment block (32 rows x 16 k), lane l fetching and storing
// chunk l: the slab of a K tile is BM/32 + BN/32 contiguous kilobytes per k block, which spreads
// over the memory channels (a row-major operand would give one 64-byte piece per 2K-byte-strided
// row, crowding a few channels: the DMA fill rate of this tile walk measured 13 TB/s row-major
// and 22 TB/s packed).  In LDS a block keeps the lane order, so a fragment read is 64 consecutive
// 16-byte chunks: conflict free without a swizzle.  Row tiles past M or N are clamped to the last
// tile (their results are never stored); K tiles past the end re-fetch the last tile into a stage
// nobody reads, which keeps the loop body branch free.
//
// Per K tile (two MFMA steps, one barrier): the loads of tile kt+NS-1 trickle out between the
// MFMAs; step 0 reads the step-1 fragments; step 1 waits until tile kt+1 has landed (vmcnt counts
// the younger loads that may still fly), meets the other waves at the barrier and reads tile
// kt+1's step-0 fragments.  In both steps the first MFMA is issued before the reads, so a wait
// in front of a step is already satisfied and the barrier never sits between idle matrix cores.
//
// One wave runs per SIMD, so every instruction issued between two MFMAs that takes longer than the
// MFMA itself (32 cycles) leaves the matrix core idle.  The loop therefore issues at most one fragment
// read and one load between two MFMAs, and a load costs three instructions: the slab bases of the K
// tile being fetched are uniform (scalar registers, advanced by a constant per K tile with scalar
// adds), each load's lane offset inside the slab is loop invariant, and the wave index is a compile-time
// constant of the loop copy a wave runs, so the LDS address of a load is scalar too (no lane read-back).
// ---------------------------------------------------------------------------------------------
// One output tile: rows [bm, bm + BM), column tile nb (of width BN; BN/2 output columns for SwiGLU).
// PARTIAL: the tile covers K tiles [kt0, kt0 + nk_part) only and stores its raw float32 sums to
// part[z][m][n] (row stride N), for an epilogue pass that adds the slices in order.
// LDS stages of the 256x256 tile's ring (32 KB each): a K tile is requested three tiles ahead.  A fifth stage (the
// whole 160 KB of a compute unit) measured the same, alone and beside a bandwidth-bound kernel on the other
// partition: what that neighbour costs is not memory latency the ring could cover.
#define RS_NS_FULL 4
template <int BM, int BN, int EPI, int NS, int NW, bool PARTIAL = false>
__device__ __forceinline__ void gemm_direct_tile(const GemmArgs &a, const int bm, const int nb, bf16_t *smem,
                                                 const int kt0 = 0, const int nk_part = 0, float *part = nullptr, const int z = 0) {
    constexpr int BK = 32;
    constexpr int WGN = NW / 2;                      // waves: 2 along M x NW/2 along N
    constexpr int WM = BM / 2, WN = BN / WGN;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int TA = BM / 32, TB = BN / 32;        // 32-row blocks per k block of the tile
    constexpr int LA = 2 * TA / NW, LB = 2 * TB / NW;   // wave-wide loads per wave per stage
    constexpr int STAGE = (BM + BN) * BK;            // elements per stage: [2][TA] A blocks, then [2][TB] B blocks
    constexpr int D = NS - 1;                        // prefetch distance in K tiles
    static_assert(TN + TM + 1 <= TN * TM, "a step must have a slot per fragment read");

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WGN, wn = wave % WGN;
    const int c32 = lane & 31, h = lane >> 5;
    const int M = a.M, N = a.N, K = a.K;
    const int Mt = packed_mt(M), Nt = ((N + 63) / 64) * 2;   // row tiles per k block of A and of the weights

    const bf16_t *wp = a.Wp, *wp2 = a.Wp2;
    if (a.tile_expert) {   // grouped: this 128-row tile multiplies one expert's matrices, or is not in use
        const int e = a.tile_expert[bm >> 7];
        if (e < 0) return;
        wp += (size_t)e * a.expert_stride;
        if (EPI == EPI_SWIGLU) wp2 += (size_t)e * a.expert_stride;
    }
    const size_t ksa = (size_t)Mt * 1024, ksb = (size_t)Nt * 1024;   // elements per K tile (2 k blocks)
    const int nk = PARTIAL ? nk_part : K / BK;

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    constexpr int SL = 2 * TN * TM, LT = LA + LB, SP = SL / LT;
    auto k_loop = [&](auto wtag) {
        constexpr int W = decltype(wtag)::value;
        constexpr int CWM = W / WGN, CWN = W % WGN;
        // The LT loads of a K tile are spread evenly over its SL MFMA slots, and wave w places its own w
        // quarter-spacings later than wave 0: the lock-stepped waves never queue behind one another at the
        // CU's one memory pipeline.
        constexpr int SHIFT = (W * SP) / NW;
        // loads of the current iteration already issued when the barrier of slot SL/2 is reached
        constexpr int EARLY = ((SL / 2 - 1 - SHIFT) / SP) + 1;
        // byte offsets of this wave's loads inside a K tile's slab: the slab bases are uniform and advance by a
        // constant per K tile, so a load costs its own instruction and the LDS address register, nothing else
        uint32_t oa[LA], ob[LB];
#pragma unroll
        for (int j = 0; j < LA; ++j) {
            const int q = W * LA + j, s = q / TA, t = q % TA;
            oa[j] = (uint32_t)(((s * Mt + min((bm >> 5) + t, Mt - 1)) * 512 + lane * 8) * 2);
        }
#pragma unroll
        for (int j = 0; j < LB; ++j) {
            const int q = W * LB + j, s = q / TB, t = q % TB;
            if (EPI == EPI_SWIGLU)   // blocks alternate: 32 gate rows, the 32 matching up rows
                ob[j] = (uint32_t)(((s * Nt + min(nb * (TB / 2) + (t >> 1), Nt - 1)) * 512 + lane * 8) * 2);
            else
                ob[j] = (uint32_t)(((s * Nt + min(nb * TB + t, Nt - 1)) * 512 + lane * 8) * 2);
        }
        const char *ga = (const char *)(a.A + (size_t)kt0 * ksa);
        const char *gb = (const char *)(wp + (size_t)kt0 * ksb);
        const char *gb2 = EPI == EPI_SWIGLU ? (const char *)(wp2 + (size_t)kt0 * ksb) : nullptr;
        int fetch_kt = 0;   // the K tile the slab bases point at
        auto advance = [&]() {   // to the next K tile, staying on the last one (its re-fetches land in a stage nobody reads)
            const size_t in = fetch_kt + 1 < nk ? 1 : 0;
            ga += in * ksa * 2;
            gb += in * ksb * 2;
            if (EPI == EPI_SWIGLU) gb2 += in * ksb * 2;
            ++fetch_kt;
        };
        // loads [j0, j1) of the LA + LB wave-wide loads that bring the K tile at the slab bases into the stage at
        // element offset so
        auto issue = [&](int so, int j0, int j1) {
            bf16_t *sa = smem + so;
            bf16_t *sb = sa + BM * BK;
#pragma unroll
            for (int j = 0; j < LA + LB; ++j) {
                if (j < j0 || j >= j1) continue;
                if (j < LA) {
                    const char *g = ga;
                    asm volatile("" : "+s"(g));   // the address is formed here, next to its load, not at the top of the K tile
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(g + oa[j]),
                                                     (__attribute__((address_space(3))) void *)(sa + (W * LA + j) * 512), 16, 0, 0);
                } else {
                    const bool up = EPI == EPI_SWIGLU && (((W * LB + j - LA) % TB) & 1);
                    const char *g = up ? gb2 : gb;
                    asm volatile("" : "+s"(g));
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(g + ob[j - LA]),
                                                     (__attribute__((address_space(3))) void *)(sb + (W * LB + j - LA) * 512), 16, 0, 0);
                }
            }
        };
        bf16x8 wf[2][TN], xf[2][TM];
        // fragment f (weights first, then activations) of step `step` of the K tile in the stage at element offset so
        auto read_frag = [&](int set, int so, int step, int f) {
            const bf16_t *sa = smem + so + lane * 8;
            const bf16_t *sb = sa + BM * BK;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                if (f == tn) wf[set][tn] = *(const bf16x8 *)&sb[(step * TB + CWN * TN + tn) * 512];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                if (f == TN + tm) xf[set][tm] = *(const bf16x8 *)&sa[(step * TA + CWM * TM + tm) * 512];
        };
        // prologue: K tiles 0 .. D-1 into stages 0 .. D-1
#pragma unroll
        for (int i = 0; i < D; ++i) {
            issue(i * STAGE, 0, LA + LB);
            advance();
        }
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((D - 1) * (LA + LB)) : "memory");
#pragma unroll
        for (int f = 0; f < TN + TM; ++f) read_frag(0, 0, 0, f);

        // One K tile = SL MFMA slots (two steps of TN x TM); its loads fill the stage before its own (tile kt + D).
        // The fragment reads and the loads are placed one per slot between the MFMAs.
        int so_cur = 0;   // element offset of the stage that holds K tile kt (uniform)
        for (int kt = 0; kt < nk; ++kt) {
            const int so_ld = so_cur == 0 ? (NS - 1) * STAGE : so_cur - STAGE;
            const int so_nxt = so_cur == (NS - 1) * STAGE ? 0 : so_cur + STAGE;
#pragma unroll
            for (int sl = 0; sl < SL; ++sl) {
                const int step = sl / (TN * TM), tn = (sl % (TN * TM)) / TM, tm = sl % TM;
                if (sl == SL / 2)
                    // tile kt+1 has landed once only the younger loads are outstanding; this wave's
                    // LDS reads are complete before it tells the others so at the barrier
                    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"((D - 2) * LT + EARLY) : "memory");
                acc[tn][tm] = mfma32(wf[step][tn], xf[step][tm], acc[tn][tm]);
                __builtin_amdgcn_sched_barrier(0);
                if (sl >= 1 && sl < 1 + TN + TM) read_frag(1, so_cur, 1, sl - 1);
                if (sl >= SL / 2 + 1 && sl < SL / 2 + 1 + TN + TM) read_frag(0, so_nxt, 0, sl - SL / 2 - 1);
                if (sl >= SHIFT && (sl - SHIFT) % SP == 0 && (sl - SHIFT) / SP < LT)
                    issue(so_ld, (sl - SHIFT) / SP, (sl - SHIFT) / SP + 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            advance();
            so_cur = so_nxt;
        }
    };
    switch (__builtin_amdgcn_readfirstlane(wave)) {
        case 0: k_loop(std::integral_constant<int, 0>{}); break;
        case 1: k_loop(std::integral_constant<int, 1>{}); break;
        case 2: k_loop(std::integral_constant<int, 2>{}); break;
        case 3: k_loop(std::integral_constant<int, 3>{}); break;
        case 4: k_loop(std::integral_constant<int, 4 % NW>{}); break;
        case 5: k_loop(std::integral_constant<int, 5 % NW>{}); break;
        case 6: k_loop(std::integral_constant<int, 6 % NW>{}); break;
        default: k_loop(std::integral_constant<int, 7 % NW>{}); break;
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");

    if (PARTIAL) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int m = bm + wm * WM + 32 * tm + c32;
            if (m >= M) continue;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int n = nb * BN + wn * WN + 32 * tn + 8 * j + 4 * h;
                    if (n >= N) continue;
                    f32x4 v = {acc[tn][tm][4 * j], acc[tn][tm][4 * j + 1], acc[tn][tm][4 * j + 2], acc[tn][tm][4 * j + 3]};
                    *(f32x4 *)(part + ((size_t)z * M + m) * N + n) = v;
                }
        }
        return;
    }
    // Output addresses without a branch per store: the 4 columns c0 + 32q + 8j + 4h (c0 a multiple of 32) of row m
    // sit at row_term(m) + col_term(c0, h) + (2q + j/2) * S16 + (j%2) * S8 in either layout, where a step of 16 columns
    // is S16 = Mt*512 elements in the fragment-packed layout and 16 row-major, a step of 8 columns 256 or 8.
    const bool packed = a.out_packed;
    const size_t S16 = packed ? (size_t)packed_mt(a.M) * 512 : 16;
    const int S8 = packed ? 256 : 8;
    const int c0 = EPI == EPI_SWIGLU ? nb * (BN / 2) + wn * (TN / 2) * 32 : nb * BN + wn * WN;
    constexpr int NQ = EPI == EPI_SWIGLU ? TN / 2 : TN;
    const size_t col_term = (packed ? (size_t)(c0 >> 4) * S16 : (size_t)c0) + 4 * h;
    const bool whole = c0 + 32 * NQ <= N;     // wave-uniform: no column of this wave's tile is past the edge
    auto rows = [&](auto checked) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int m = bm + wm * WM + 32 * tm + c32;
            if (m >= M) continue;
            bf16_t *dst = a.out + (packed ? (size_t)(m >> 5) * 512 + (size_t)(m & 31) * 8 : (size_t)m * N) + col_term;
            const bf16_t *res = EPI == EPI_RESIDUAL ? a.resid + (size_t)m * N + c0 + 4 * h : nullptr;
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (decltype(checked)::value && c0 + 32 * q + 8 * j + 4 * h >= N) continue;
                    bf16x4 v;
                    if (EPI == EPI_SWIGLU) {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            v[i] = (bf16_t)(silu_f(acc[2 * q][tm][4 * j + i]) * acc[2 * q + 1][tm][4 * j + i]);
                    } else if (EPI == EPI_RESIDUAL) {
                        const bf16x4 r = *(const bf16x4 *)(res + 32 * q + 8 * j);
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] = (bf16_t)(acc[q][tm][4 * j + i] + (float)r[i]);
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] = (bf16_t)acc[q][tm][4 * j + i];
                    }
                    *(bf16x4 *)(dst + (size_t)(2 * q + (j >> 1)) * S16 + (j & 1) * S8) = v;
                }
        }
    };
    if (whole) rows(std::false_type{});
    else rows(std::true_type{});
}

// Order of the output tiles: super columns of four column tiles, inside one the row tiles four at a time, a
// 4 x 4 block column by column.  Tiles that run at the same time on an XCD (16 on half the chip, 32 on the whole
// chip) then share four weight slabs and four or eight activation slabs, whatever the number of row tiles: with
// plain column-major order an XCD's set was all rows of one or two columns, and each round re-read the whole
// activation matrix.
__device__ __forceinline__ void tile_rc(int t, int m_tiles, int n_tiles, int &r, int &c) {
    constexpr int CW = 4, RH = 4;
    const int per_sc = CW * m_tiles;
    const int sc = t / per_sc, c0 = sc * CW;
    const int w = min(CW, n_tiles - c0);      // the last super column may be narrower
    const int u = t - sc * per_sc;
    const int rb = u / (RH * w), r0 = rb * RH;
    const int hgt = min(RH, m_tiles - r0);    // the last row block may be lower
    const int v = u - rb * (RH * w);
    r = r0 + v % hgt;
    c = c0 + v / hgt;
}

// The flat workgroup id is remapped so that the workgroups resident on one XCD (ids congruent
// mod 8) own a contiguous run of tiles in that order, served by that XCD's L2.
template <int BM, int BN, int EPI, int NS, int NW>
__global__ __launch_bounds__(64 * NW) void gemm_direct_kernel(GemmArgs a, int m_tiles, int n_tiles) {
    extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];
    const int total = m_tiles * n_tiles;
    const int per_xcd = (total + 7) >> 3;
    const int t = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (t >= total) return;
    int r, c;
    tile_rc(t, m_tiles, n_tiles, r, c);
    gemm_direct_tile<BM, BN, EPI, NS, NW>(a, r * BM, c, smem);
}

// Whole rounds of 256x256 tiles, then a last half round: when the 256x256 tiles do not divide by
// the number of compute units, the first n_full workgroups (a multiple of the unit count) take
// whole tiles and the remaining tiles are cut into their two 128-row halves, one workgroup each,
// which are dispatched last.  The arithmetic of an output element does not depend on the tile
// that holds it, so the schedule may follow the size of the partition.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_direct_mixed_kernel(GemmArgs a, int m_tiles, int n_full, int n_half) {
    extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];
    const int id = blockIdx.x;
    const int n_tiles = (n_full + (n_half >> 1)) / m_tiles;   // column tiles
    if (id < n_full) {
        const int t = (id & 7) * (n_full >> 3) + (id >> 3);          // n_full is a multiple of 8
        int r, c;
        tile_rc(t, m_tiles, n_tiles, r, c);
        gemm_direct_tile<256, 256, EPI, RS_NS_FULL, 4>(a, r * 256, c, smem);
    } else {
        const int j = id - n_full;
        const int u = (j & 7) * ((n_half + 7) >> 3) + (j >> 3);
        if (u >= n_half) return;
        const int t = n_full + (u >> 1);
        int r, c;
        tile_rc(t, m_tiles, n_tiles, r, c);
        const int bm = r * 256 + (u & 1) * 128;
        if (bm >= a.M) return;
        gemm_direct_tile<128, 256, EPI, 5, 4>(a, bm, c, smem);
    }
}

// Few output tiles and a long K (the projections back to d_model at a few hundred rows): the K range is
// cut into S slices, one workgroup per (tile, slice), and skinny_epilogue_kernel adds the slices in order
// and applies the epilogue.  S follows from (M, N, K) alone, so results do not depend on the CU share.
__global__ __launch_bounds__(256) void gemm_direct_splitk_kernel(GemmArgs a, int m_tiles, int n_tiles, int nk_per, float *part) {
    extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];
    const int tiles = m_tiles * n_tiles;
    const int z = blockIdx.x / tiles, t = blockIdx.x % tiles;
    const int nk_total = a.K / 32;
    const int kt0 = z * nk_per;
    gemm_direct_tile<128, 256, EPI_STORE, 5, 4, true>(a, (t % m_tiles) * 128, t / m_tiles, smem, kt0, min(nk_per, nk_total - kt0), part, z);
}

static inline int direct_splits(int M, int N, int K) {
    const long tiles = (long)((M + 127) / 128) * ((N + 255) / 256);
    const int nk = K / 32;
    int S = 1;
    // until about half of a whole chip's compute units have a workgroup; at least 16 K tiles per slice
    while (tiles * S * 2 <= 256 && S < 8 && nk / (S * 2) >= 16) S *= 2;
    return S;
}
size_t direct_partial_elems(int M, int N, int K) { return (size_t)direct_splits(M, N, K) * (size_t)M * (size_t)N; }

template <int EPI>
__global__ __launch_bounds__(256) void skinny_epilogue_kernel(GemmArgs a, const float *__restrict__ part, int S, int Nv);

static void launch_direct_splitk(hipStream_t st, const GemmArgs &a, int S) {
    const int m_tiles = (a.M + 127) / 128, n_tiles = (a.N + 255) / 256;
    const int nk_total = a.K / 32, nk_per = (nk_total + S - 1) / S;
    constexpr int lds = 5 * (128 + 256) * 32 * 2;
    hipLaunchKernelGGL(gemm_direct_splitk_kernel, dim3(m_tiles * n_tiles * S), dim3(256), lds, st, a, m_tiles, n_tiles, nk_per, a.partials);
    const int eblocks = (a.M * (a.N / 4) + 255) / 256;
    if (a.epi == EPI_RESIDUAL)
        hipLaunchKernelGGL(skinny_epilogue_kernel<EPI_RESIDUAL>, dim3(eblocks), dim3(256), 0, st, a, a.partials, S, a.N);
    else
        hipLaunchKernelGGL(skinny_epilogue_kernel<EPI_STORE>, dim3(eblocks), dim3(256), 0, st, a, a.partials, S, a.N);
}

// Main pass of the large-tile kernel only, whole K in one slice: part[m][n] (row stride N) holds the float32
// sums.  False (nothing launched) when the shape is not one the kernel takes.
bool launch_gemm_direct_partials(hipStream_t st, const GemmArgs &a, float *part) {
    if (!(a.K % 32 == 0 && a.K >= 32 && a.Wp && a.M >= 1 && a.N >= 1024 && a.N % 4 == 0)) return false;
    const int m_tiles = (a.M + 127) / 128, n_tiles = (a.N + 255) / 256;
    constexpr int lds = 5 * (128 + 256) * 32 * 2;
    hipLaunchKernelGGL(gemm_direct_splitk_kernel, dim3(m_tiles * n_tiles), dim3(256), lds, st, a, m_tiles, n_tiles, a.K / 32, part);
    return true;
}

template <int EPI>
static void launch_direct_mixed_epi(hipStream_t st, const GemmArgs &a, int m_tiles, int n_full, int n_half) {
    constexpr int lds = RS_NS_FULL * 512 * 32 * 2;   // the larger of the two rings
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void *)gemm_direct_mixed_kernel<EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_set = true;
    }
    const int grid = n_full + ((n_half + 7) / 8) * 8;
    hipLaunchKernelGGL((gemm_direct_mixed_kernel<EPI>), dim3(grid), dim3(256), lds, st, a, m_tiles, n_full, n_half);
}

template <int BM, int BN, int EPI, int NS, int NW>
static void launch_direct_epi(hipStream_t st, const GemmArgs &a) {
    const int m_tiles = (a.M + BM - 1) / BM;
    const int n_tiles = (EPI == EPI_SWIGLU) ? (a.N + BN / 2 - 1) / (BN / 2) : (a.N + BN - 1) / BN;
    const int total = m_tiles * n_tiles;
    const int grid = ((total + 7) / 8) * 8;
    constexpr int lds = NS * (BM + BN) * 32 * 2;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void *)gemm_direct_kernel<BM, BN, EPI, NS, NW>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_set = true;
    }
    hipLaunchKernelGGL((gemm_direct_kernel<BM, BN, EPI, NS, NW>), dim3(grid), dim3(64 * NW), lds, st, a, m_tiles, n_tiles);
}

template <int BM, int BN, int NS, int NW>
static void launch_direct(hipStream_t st, const GemmArgs &a) {
    switch (a.epi) {
        case EPI_STORE: launch_direct_epi<BM, BN, EPI_STORE, NS, NW>(st, a); break;
        case EPI_RESIDUAL: launch_direct_epi<BM, BN, EPI_RESIDUAL, NS, NW>(st, a); break;
        default: launch_direct_epi<BM, BN, EPI_SWIGLU, NS, NW>(st, a); break;
    }
}

// Grouped GEMM (one weight matrix per 128-row tile, tile_expert[]).  The work list that follows the tile
// table (tile_expert[n] = number of units, then one code per unit: 2 * tile + 1 for two neighbouring tiles of
// one expert taken as one 256x256 tile, the cheaper shape per row, 2 * tile for a single 128x256 tile) names
// the tiles in use, so the workgroups with work come first in every column tile and the rest leave at once.
// The arithmetic of an output element does not depend on the tile that holds it.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_grouped_kernel(GemmArgs a, int n_tiles) {
    extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];
    const int n128 = a.M >> 7;   // most units there can be
    const int total = n128 * n_tiles;
    const int per_xcd = (total + 7) >> 3;
    const int t = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (t >= total) return;
    const int u = t % n128, nb = t / n128;
    const int32_t *units = a.tile_expert + n128;
    if (u >= __builtin_amdgcn_readfirstlane(units[0])) return;
    const int code = __builtin_amdgcn_readfirstlane(units[1 + u]);
    if (code & 1) gemm_direct_tile<256, 256, EPI, RS_NS_FULL, 4>(a, (code >> 1) * 128, nb, smem);
    else gemm_direct_tile<128, 256, EPI, 5, 4>(a, (code >> 1) * 128, nb, smem);
}

template <int EPI>
static void launch_grouped_epi(hipStream_t st, const GemmArgs &a) {
    const int n_tiles = (EPI == EPI_SWIGLU) ? (a.N + 127) / 128 : (a.N + 255) / 256;
    const int grid = (((a.M >> 7) * n_tiles + 7) / 8) * 8;
    hipLaunchKernelGGL((gemm_grouped_kernel<EPI>), dim3(grid), dim3(256), RS_NS_FULL * 32768, st, a, n_tiles);
}

bool launch_gemm_grouped(hipStream_t st, const GemmArgs &a) {
    if (!(a.K % 32 == 0 && a.K >= 32 && a.Wp && a.N >= 1024 && a.M % 128 == 0 && a.tile_expert)) return false;
    if (a.epi == EPI_SWIGLU) launch_grouped_epi<EPI_SWIGLU>(st, a);
    else if (a.epi == EPI_STORE) launch_grouped_epi<EPI_STORE>(st, a);
    else return false;
    return true;
}

template <int BM, int BN>
static void launch_tiled(hipStream_t st, const GemmArgs &a) {
    const int n_virtual = (a.epi == EPI_SWIGLU) ? 2 * a.N : a.N;
    // SwiGLU tiles hold BN/2 output columns, padded per 32-column group
    dim3 grid(a.epi == EPI_SWIGLU ? (a.N + BN / 2 - 1) / (BN / 2) : (n_virtual + BN - 1) / BN,
              (a.M + BM - 1) / BM);
    switch (a.epi) {
        case EPI_STORE:
            hipLaunchKernelGGL((gemm_tiled_kernel<BM, BN, EPI_STORE>), grid, dim3(256), 0, st, a);
            break;
        case EPI_RESIDUAL:
            hipLaunchKernelGGL((gemm_tiled_kernel<BM, BN, EPI_RESIDUAL>), grid, dim3(256), 0, st, a);
            break;
        default:
            hipLaunchKernelGGL((gemm_tiled_kernel<BM, BN, EPI_SWIGLU>), grid, dim3(256), 0, st, a);
            break;
    }
}

// Tile shapes of the direct kernel and their cost per tile relative to a 256x256 tile (area over
// measured relative efficiency).  The schedule with the fewest weighted rounds on the partition's
// compute units wins; the arithmetic of an output element is the same in all of them.
bool launch_gemm_tiled(hipStream_t st, const GemmArgs &a) {
    if (a.M <= 0 || a.N <= 0) return true;
    const bool aligned = (a.K % 32 == 0) && a.K >= 32;
    if (aligned && a.Wp && a.M > 64 && a.N >= 1024) {
        if (a.epi != EPI_SWIGLU && a.partials && a.N % 4 == 0) {
            const int S = direct_splits(a.M, a.N, a.K);
            if (S > 1 && direct_partial_elems(a.M, a.N, a.K) <= a.partial_cap) {
                launch_direct_splitk(st, a, S);
                return true;
            }
        }
        const int cus = a.cus > 0 ? a.cus : 256;
        const int nv = a.epi == EPI_SWIGLU ? 2 * a.N : a.N;
        const int mt256 = (a.M + 255) / 256, mt128 = (a.M + 127) / 128;
        const long t_full = (long)mt256 * ((nv + 255) / 256), t_half = (long)mt128 * ((nv + 255) / 256);
        const long t_192 = (long)mt256 * ((a.N + 191) / 192);
        auto rounds = [&](long t) { return (double)((t + cus - 1) / cus); };
        constexpr double C_HALF = 0.59, C_192 = 0.79;
        const double cost_full = rounds(t_full), cost_half = rounds(t_half) * C_HALF;
        const double cost_192 = a.epi == EPI_SWIGLU ? 1e30 : rounds(t_192) * C_192;
        const int n_full = (int)(t_full / cus) * cus, rest = (int)t_full - n_full;
        const bool mixed_ok = n_full > 0 && n_full % 8 == 0 && rest > 0 && 2 * rest <= cus;
        const double cost_mixed = mixed_ok ? n_full / cus + C_HALF : 1e30;
        const double best = std::min(std::min(cost_full, cost_mixed), std::min(cost_half, cost_192));
        if (best == cost_full) {
            launch_direct<256, 256, RS_NS_FULL, 4>(st, a);   // RS_NS_FULL x 32 KB of LDS
        } else if (best == cost_mixed) {
            switch (a.epi) {
                case EPI_STORE: launch_direct_mixed_epi<EPI_STORE>(st, a, mt256, n_full, 2 * rest); break;
                case EPI_RESIDUAL: launch_direct_mixed_epi<EPI_RESIDUAL>(st, a, mt256, n_full, 2 * rest); break;
                default: launch_direct_mixed_epi<EPI_SWIGLU>(st, a, mt256, n_full, 2 * rest); break;
            }
        } else if (best == cost_192) {
            if (a.epi == EPI_STORE) launch_direct_epi<256, 192, EPI_STORE, 4, 4>(st, a);   // 4 x 28 KB
            else launch_direct_epi<256, 192, EPI_RESIDUAL, 4, 4>(st, a);
        } else {
            launch_direct<128, 256, 5, 4>(st, a);   // 5 x 24 KB of LDS
        }
    } else {
        // the generic kernel reads the caller's row-major matrices: refuse when they have been released
        if (!a.W || (a.epi == EPI_SWIGLU && !a.W2)) return false;
        if (a.M >= 1024 && a.N >= 1024) launch_tiled<256, 256>(st, a);
        else launch_tiled<128, 128>(st, a);
    }
    return true;
}

// ---------------------------------------------------------------------------------------------
// Skinny kernel (M <= 64): bandwidth bound, so built for bytes in flight.  Both operands arrive in
// MFMA fragment order -- the activations fragment-packed by their producer, the weights repacked
// once when they are set -- so every load is one contiguous 1 KB per wave straight into the
// registers that feed the matrix core: no LDS staging, and since only register loads are
// outstanding they complete in order and the compiler's own wait counts are exact.
//
// Packed weights: [ceil(K/16) k blocks][ceil(N/64)*2 row tiles of 32][64 lanes][8], zero padded;
// lane h*32 + r of block (kb, t) holds W[32t + r][16kb + 8h .. +8).  k-block major: the waves of
// all workgroups advance through K together, so at any moment the chip reads a few contiguous
// regions that spread evenly over the memory channels (row-tile-major streams would all sit at
// the same offset within their 2^n-spaced rows and crowd the same channels).
//
// Workgroup = 64 (virtual) weight rows x one K slice; its 4 waves split the slice.  Each wave keeps
// PD k-blocks (4 KB each: two weight and two activation fragments) in flight in a register ring;
// two workgroups fit a CU, i.e. 8 waves x 32 KB in flight per CU.  Loads past the wave's range
// re-fetch the last block (cache hits, never used), which keeps the ring's wait counts static.
// The 4 waves are summed in wave order through LDS; the S slices of K are summed in slice order
// by the epilogue kernel.  S depends on (N, K) only, so results never depend on the CU share.
// ---------------------------------------------------------------------------------------------
// RT = 32-row weight tiles per workgroup (and per wave: the 4 waves split K, not rows)
#define RS_SKINNY_RT 2
static inline int skinny_virtual_n(int N, int epi) {
    constexpr int VT = 32 * RS_SKINNY_RT;   // virtual rows per workgroup; SwiGLU: half gate, half up
    return epi == EPI_SWIGLU ? ((N + VT / 2 - 1) / (VT / 2)) * VT : ((N + VT - 1) / VT) * VT;
}
static inline int skinny_kblocks(int K) { return (K + 15) / 16; }
static inline int skinny_splits(int N, int K, int epi) {
    const int tiles = skinny_virtual_n(N, epi) / (32 * RS_SKINNY_RT);
    const int Kb = skinny_kblocks(K);
    int S = 1;
    // enough workgroups for one per CU and more, but at least 8 k-blocks per wave
    while (tiles * S < RS_SKINNY_TARGET_WGS && S < 16 && Kb / (2 * S) >= 32) S *= 2;
    return S;
}
static inline int skinny_kb_per_wg(int K, int S) {
    const int per = (skinny_kblocks(K) + S - 1) / S;
    return ((per + 3) / 4) * 4;  // 4 waves
}
static inline int shared_virtual_n(int N, int epi);
static inline int shared_splits(int N, int K, int epi);
size_t skinny_partial_elems(int M, int N, int K, int epi) {
    const size_t plain = (size_t)skinny_splits(N, K, epi) * (size_t)M * (size_t)skinny_virtual_n(N, epi);
    const size_t shared = (size_t)shared_splits(N, K, epi) * (size_t)M * (size_t)shared_virtual_n(N, epi);
    return std::max(plain, shared);
}
size_t packed_weight_elems(int N, int K) {
    return (size_t)((N + 63) / 64) * 2 * (size_t)skinny_kblocks(K) * 512;
}

// One thread per 16-byte chunk of the packed matrix.
__global__ __launch_bounds__(256) void pack_weights_kernel(const bf16_t *__restrict__ W, bf16_t *__restrict__ Wp,
                                                           int N, int K, int Kb, long n_chunks) {
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n_chunks) return;
    const int lane = (int)(idx & 63);
    const long blk = idx >> 6;
    const int Nt = ((N + 63) / 64) * 2;
    const int t = (int)(blk % Nt), kb = (int)(blk / Nt);
    const int row = 32 * t + (lane & 31), k0 = 16 * kb + 8 * (lane >> 5);
    bf16x8 v = zero_bf16x8();
    if (row < N) {
        if (k0 + 8 <= K) {
            v = ld_bf16x8(W + (size_t)row * K + k0);
        } else {
            for (int i = 0; i < 8; ++i)
                if (k0 + i < K) v[i] = W[(size_t)row * K + k0 + i];
        }
    }
    st_bf16x8(Wp + idx * 8, v);
}

void launch_pack_weights(hipStream_t st, const bf16_t *W, bf16_t *Wp, int N, int K) {
    const long n_chunks = (long)(packed_weight_elems(N, K) / 8);
    hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)((n_chunks + 255) / 256)), dim3(256), 0, st, W, Wp, N, K,
                       skinny_kblocks(K), n_chunks);
}

template <int EPI, int RT, int PD>
__global__ __launch_bounds__(256, RT <= 2 ? 2 : 1) void gemm_skinny_kernel(GemmArgs a, float *__restrict__ part,
                                                          int kb_per_wg, int Kb, int Nv) {
    // RT * 32 KB: the waves' accumulators for the in-order reduction, [wave][tile][lane][16]
    extern __shared__ __attribute__((aligned(1024))) float red[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c32 = lane & 31, h = lane >> 5;
    const int M = a.M;
    const int kbw = kb_per_wg >> 2;
    const int kb0 = __builtin_amdgcn_readfirstlane(blockIdx.y * kb_per_wg + wave * kbw);
    const int nsteps = max(min(kb0 + kbw, Kb) - kb0, 0);
    const int kb_last = Kb - 1;

    // the workgroup's RT row tiles in the packed matrices.  SwiGLU: virtual tile t is gate (t even) or
    // up (t odd) tile RT/2 * blockIdx.x + t/2, so gate and up of a feature sit 32 virtual columns apart
    const int Nt = ((a.N + 63) / 64) * 2;
    const size_t wstride = (size_t)Nt * 512, tstride = 512;   // elements per k block / per row tile
    const bf16_t *w[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        if (EPI == EPI_SWIGLU)
            w[t] = ((t & 1) ? a.Wp2 : a.Wp) + (size_t)min((RT / 2) * (int)blockIdx.x + (t >> 1), Nt - 1) * tstride + lane * 8;
        else
            w[t] = a.Wp + (size_t)min(RT * (int)blockIdx.x + t, Nt - 1) * tstride + lane * 8;
    }
    const bf16_t *x = a.A + lane * 8;

    f32x16 acc[RT][2];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    bf16x8 rw[PD][RT], rx[PD][2];
    auto load = [&](int p, int step) {
        const size_t kb = (size_t)min(kb0 + step, kb_last);
#pragma unroll
        for (int t = 0; t < RT; ++t) rw[p][t] = ld_bf16x8_stream(w[t] + kb * wstride);
        rx[p][0] = ld_bf16x8(x + kb * 1024);
        rx[p][1] = ld_bf16x8(x + kb * 1024 + 512);
    };
#pragma unroll
    for (int p = 0; p < PD; ++p) load(p, p);
    auto step = [&](int p) {
#pragma unroll
        for (int t = 0; t < RT; ++t) {
            acc[t][0] = mfma32(rw[p][t], rx[p][0], acc[t][0]);
            acc[t][1] = mfma32(rw[p][t], rx[p][1], acc[t][1]);
        }
    };
    // whole rings: branch free, so the wait in front of each step is "all but the PD-1 younger steps"
    int i = 0;
    for (; i + PD <= nsteps; i += PD) {
#pragma unroll
        for (int p = 0; p < PD; ++p) {
            step(p);
            load(p, i + p + PD);
            __builtin_amdgcn_sched_barrier(0);   // refill the ring slot at once: keeps the bytes in flight level
        }
    }
    // the last, partial ring is already in flight
    const int rem = nsteps - i;
#pragma unroll
    for (int p = 0; p < PD; ++p)
        if (p < rem) step(p);
    // in-order reduction of the 4 waves
#pragma unroll
    for (int tn = 0; tn < RT; ++tn)
#pragma unroll
        for (int tm = 0; tm < 2; ++tm)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x4 v = {acc[tn][tm][4 * j], acc[tn][tm][4 * j + 1], acc[tn][tm][4 * j + 2], acc[tn][tm][4 * j + 3]};
                *(f32x4 *)&red[(((wave * (2 * RT) + tn * 2 + tm) * 4 + j) * 64 + lane) * 4] = v;   // lanes 16 bytes apart: no bank conflicts
            }
    __syncthreads();
    // wave w finishes tiles w, w + 4, ...: sum of the 4 waves in wave order
#pragma unroll
    for (int q = 0; q < (2 * RT) / 4; ++q) {
        const int tile = wave + 4 * q, tn = tile >> 1, tm = tile & 1;
        const int m = 32 * tm + c32;
        if (m < M) {
            float *dst = part + ((size_t)blockIdx.y * M + m) * Nv + blockIdx.x * (32 * RT) + 32 * tn;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x4 v = *(const f32x4 *)&red[(((0 * (2 * RT) + tile) * 4 + j) * 64 + lane) * 4];
#pragma unroll
                for (int ww = 1; ww < 4; ++ww) v += *(const f32x4 *)&red[(((ww * (2 * RT) + tile) * 4 + j) * 64 + lane) * 4];
                *(f32x4 *)(dst + 8 * j + 4 * h) = v;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Skinny kernel, shared activations (used for the wide gate/up matrix).  A CU moves about 55 GB/s
// through its vector memory path whether the bytes come from HBM or from L2 (measured: the plain
// weight stream of gemm_skinny_kernel reaches 50 GB/s per CU, and 30 once every wave also fetches
// its own activation fragments, which are as many bytes as the weights).  Here the 4 waves of a
// workgroup take different rows over the SAME K slice, so the slice's activation k-blocks are
// fetched once per workgroup into LDS (a quarter of the bytes) and read from there:
//   * K is cut into chunks of CH k-blocks; the chunk's activations (CH x 2 KB) sit in one of two
//     LDS slabs; while chunk c is computed each wave fetches its 8 pieces of chunk c+1's slab, one
//     per step, through the same register ring as its weights (so all loads stay register loads,
//     in order, exact wait counts) and stores them to the other slab when their ring slot comes
//     up; one barrier per chunk (s_barrier after lgkmcnt(0): the weight ring is NOT drained);
//   * no K split inside the workgroup, hence no LDS reduction: each wave writes its own 64 x 64
//     partial tile; K is split S ways across workgroups, summed in slice order by the epilogue
//     kernel as before (S depends on the shape only).
// ---------------------------------------------------------------------------------------------
#define RS_SHARED_CH 16
static inline bool skinny_shared_applies(const GemmArgs &a) {
    if (skinny_kblocks(a.K) % (4 * RS_SHARED_CH) != 0 || a.N < 4096) return false;
    return a.epi == EPI_SWIGLU || (a.epi == EPI_RESIDUAL && a.K >= 8192);   // wide, or long enough in K to split 8 ways
}
static inline int shared_virtual_n(int N, int epi) {
    return epi == EPI_SWIGLU ? ((N + 127) / 128) * 256 : ((N + 255) / 256) * 256;
}
static inline int shared_splits(int N, int K, int epi) {
    const int tiles = shared_virtual_n(N, epi) / 256;
    const int Kb = skinny_kblocks(K);
    int S = 1;
    while (tiles * S < 224 && S < 16 && Kb % (2 * S * RS_SHARED_CH) == 0 && Kb / (2 * S) >= 4 * RS_SHARED_CH) S *= 2;
    return S;
}

template <int EPI, int CH>
__global__ __launch_bounds__(256, 2) void gemm_skinny_shared_kernel(GemmArgs a, float *__restrict__ part, int kb_per_wg,
                                                                     int Kb, int Nv) {
    constexpr int PD = 8;                      // ring depth; divides CH, so ring slots are static in the unrolled chunk
    static_assert(CH % PD == 0 && CH * 2 == 32, "4 waves x 8 pieces fill one slab");
    extern __shared__ __attribute__((aligned(1024))) bf16_t slab[];   // [2][CH][2 token tiles][64 lanes][8]
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c32 = lane & 31, h = lane >> 5;
    const int M = a.M;
    const int kb_begin = blockIdx.y * kb_per_wg;
    const int nchunks = kb_per_wg / CH;
    const int kb_last = Kb - 1;
    const int Nt = ((a.N + 63) / 64) * 2;
    const size_t wstride = (size_t)Nt * 512;
    const bf16_t *w0, *w1;
    if (EPI == EPI_SWIGLU) {   // wave w: gate tile and up tile of feature tile 4 * blockIdx.x + w
        const int f = min(4 * (int)blockIdx.x + wave, Nt - 1);
        w0 = a.Wp + (size_t)f * 512 + lane * 8;
        w1 = a.Wp2 + (size_t)f * 512 + lane * 8;
    } else {
        w0 = a.Wp + (size_t)min(8 * (int)blockIdx.x + 2 * wave, Nt - 1) * 512 + lane * 8;
        w1 = a.Wp + (size_t)min(8 * (int)blockIdx.x + 2 * wave + 1, Nt - 1) * 512 + lane * 8;
    }
    const bf16_t *x = a.A + lane * 8;

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // piece q (0..31) of a chunk's slab = 1 KB = (k-block q/2, token tile q%2); wave w fetches pieces 8w .. 8w+7
    auto x_piece = [&](int chunk, int j) {
        const int q = 8 * wave + j;
        const size_t kb = (size_t)min(kb_begin + chunk * CH + (q >> 1), kb_last);
        return ld_bf16x8(x + kb * 1024 + (q & 1) * 512);
    };
    // chunk 0's slab, up front
    {
        bf16x8 t[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = x_piece(0, j);
#pragma unroll
        for (int j = 0; j < 8; ++j) *(bf16x8 *)&slab[(8 * wave + j) * 512 + lane * 8] = t[j];
    }
    bf16x8 rw0[PD], rw1[PD], rxs[PD];
    auto load_w = [&](int p, int step) {   // step counts k-blocks from kb_begin
        const size_t kb = (size_t)min(kb_begin + step, kb_last);
        rw0[p] = ld_bf16x8_stream(w0 + kb * wstride);
        rw1[p] = ld_bf16x8_stream(w1 + kb * wstride);
    };
#pragma unroll
    for (int p = 0; p < PD; ++p) load_w(p, p);
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

    for (int c = 0; c < nchunks; ++c) {
        const bf16_t *cur = slab + (c & 1) * (CH * 1024) + lane * 8;
        bf16_t *nxt = slab + ((c + 1) & 1) * (CH * 1024);
#pragma unroll
        for (int s = 0; s < CH; ++s) {
            const int p = s % PD;
            const bf16x8 x0 = *(const bf16x8 *)&cur[(2 * s) * 512], x1 = *(const bf16x8 *)&cur[(2 * s + 1) * 512];
            acc[0][0] = mfma32(rw0[p], x0, acc[0][0]);
            acc[0][1] = mfma32(rw0[p], x1, acc[0][1]);
            acc[1][0] = mfma32(rw1[p], x0, acc[1][0]);
            acc[1][1] = mfma32(rw1[p], x1, acc[1][1]);
            // the piece of the next slab that was fetched into this slot PD steps ago
            if (s >= PD && s - PD < 8) *(bf16x8 *)&nxt[(8 * wave + (s - PD)) * 512 + lane * 8] = rxs[p];
            load_w(p, c * CH + s + PD);
            if (s < 8) rxs[p] = x_piece(c + 1, s);
            __builtin_amdgcn_sched_barrier(0);
        }
        // every wave has read slab c and written its pieces of slab c+1; the weight loads stay in flight
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }
    // each wave owns its rows: partial tile straight from the accumulators
#pragma unroll
    for (int tn = 0; tn < 2; ++tn)
#pragma unroll
        for (int tm = 0; tm < 2; ++tm) {
            const int m = 32 * tm + c32;
            if (m >= M) continue;
            float *dst = part + ((size_t)blockIdx.y * M + m) * Nv + blockIdx.x * 256 + wave * 64 + 32 * tn;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x4 v = {acc[tn][tm][4 * j], acc[tn][tm][4 * j + 1], acc[tn][tm][4 * j + 2], acc[tn][tm][4 * j + 3]};
                *(f32x4 *)(dst + 8 * j + 4 * h) = v;
            }
        }
}

// Sums the K slices in order and applies the epilogue; one thread per 4 output columns.
template <int EPI>
__global__ __launch_bounds__(256) void skinny_epilogue_kernel(GemmArgs a, const float *__restrict__ part,
                                                              int S, int Nv) {
    const int M = a.M, N = a.N;
    const int groups = N >> 2;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * groups) return;
    const int m = idx / groups, n = (idx % groups) * 4;
    bf16x4 v;
    if (EPI == EPI_SWIGLU) {
        const int col = (n >> 5) * 64 + (n & 31);
        f32x4 g = {0.f, 0.f, 0.f, 0.f}, u = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < S; ++s) {
            const float *p = part + ((size_t)s * M + m) * Nv + col;
            g += *(const f32x4 *)p;
            u += *(const f32x4 *)(p + 32);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = (bf16_t)(silu_f(g[i]) * u[i]);
    } else {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < S; ++s) acc += *(const f32x4 *)(part + ((size_t)s * M + m) * Nv + n);
        if (EPI == EPI_RESIDUAL) {
            const bf16x4 r = *(const bf16x4 *)(a.resid + (size_t)m * N + n);
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = (bf16_t)(acc[i] + (float)r[i]);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = (bf16_t)acc[i];
        }
    }
    store_out4(a, m, n, v);
}

template <int EPI>
static void launch_skinny_epi(hipStream_t st, const GemmArgs &a, float *partials) {
    if (skinny_shared_applies(a)) {
        constexpr int CH = RS_SHARED_CH, lds = 2 * CH * 2048;
        const int Nv = shared_virtual_n(a.N, a.epi), S = shared_splits(a.N, a.K, a.epi);
        const int kbpw = skinny_kblocks(a.K) / S;
        hipLaunchKernelGGL((gemm_skinny_shared_kernel<EPI, CH>), dim3(Nv / 256, S), dim3(256), lds, st, a, partials, kbpw,
                           skinny_kblocks(a.K), Nv);
        hipLaunchKernelGGL(skinny_epilogue_kernel<EPI>, dim3((a.M * (a.N / 4) + 255) / 256), dim3(256), 0, st, a, partials, S, Nv);
        return;
    }
    constexpr int RT = RS_SKINNY_RT, PD = 10;   // (RT + 2) * PD loads per wave in flight; at most 63 can be outstanding (gemm_kernels_init uses the same pair)
    constexpr int lds = RT * 32768;
    const int Nv = skinny_virtual_n(a.N, a.epi);
    const int S = skinny_splits(a.N, a.K, a.epi);
    const int kbpw = skinny_kb_per_wg(a.K, S);
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void *)gemm_skinny_kernel<EPI, RT, PD>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_set = true;
    }
    const int eblocks = (a.M * (a.N / 4) + 255) / 256;
    hipLaunchKernelGGL((gemm_skinny_kernel<EPI, RT, PD>), dim3(Nv / (32 * RT), S), dim3(256), lds, st, a, partials, kbpw,
                       skinny_kblocks(a.K), Nv);
    hipLaunchKernelGGL(skinny_epilogue_kernel<EPI>, dim3(eblocks), dim3(256), 0, st, a, partials, S, Nv);
}

// Whether the partial-sum pass of a plain projection (M <= 64 rows) can take the shared-activation streaming kernel.
bool gemm_skinny_partials_shared(int N, int K) {
    return K % 16 == 0 && skinny_kblocks(K) % (4 * RS_SHARED_CH) == 0 && N >= 4096;
}

void launch_gemm_skinny_partials(hipStream_t st, const GemmArgs &a, float *partials, int *S_out, int *Nv_out) {
    if (gemm_skinny_partials_shared(a.N, a.K)) {
        constexpr int CH = RS_SHARED_CH;
        const int Nv = shared_virtual_n(a.N, EPI_STORE), S = shared_splits(a.N, a.K, EPI_STORE);
        *S_out = S;
        *Nv_out = Nv;
        if (a.M <= 0 || a.N <= 0) return;
        hipLaunchKernelGGL((gemm_skinny_shared_kernel<EPI_STORE, CH>), dim3(Nv / 256, S), dim3(256), 2 * CH * 2048, st, a, partials,
                           skinny_kblocks(a.K) / S, skinny_kblocks(a.K), Nv);
        return;
    }
    constexpr int RT = RS_SKINNY_RT, PD = 10;
    const int Nv = skinny_virtual_n(a.N, EPI_STORE), S = skinny_splits(a.N, a.K, EPI_STORE);
    *S_out = S;
    *Nv_out = Nv;
    if (a.M <= 0 || a.N <= 0) return;
    hipLaunchKernelGGL((gemm_skinny_kernel<EPI_STORE, RT, PD>), dim3(Nv / (32 * RT), S), dim3(256), RT * 32768, st, a, partials,
                       skinny_kb_per_wg(a.K, S), skinny_kblocks(a.K), Nv);
}

void launch_gemm_skinny(hipStream_t st, const GemmArgs &a, float *partials) {
    if (a.M <= 0 || a.N <= 0) return;
    // A residual projection too short in K for the shared-activation kernel (the attention output projection)
    // has few, short K ranges per wave in the streaming kernel; the K-sliced large-tile kernel serves it better
    // on a partition (8B layer, 64 rows: 27 -> 21 us on 128 CUs, equal on 256).  A function of the shape alone.
    if (a.epi == EPI_RESIDUAL && !skinny_shared_applies(a) && a.K % 32 == 0 && a.K >= 512 && a.Wp && a.N >= 1024 && a.N % 4 == 0 &&
        a.partials == partials && a.partial_cap > 0) {
        const int S = direct_splits(a.M, a.N, a.K);
        if (S > 1 && direct_partial_elems(a.M, a.N, a.K) <= a.partial_cap) {
            launch_direct_splitk(st, a, S);
            return;
        }
    }
    switch (a.epi) {
        case EPI_STORE: launch_skinny_epi<EPI_STORE>(st, a, partials); break;
        case EPI_RESIDUAL: launch_skinny_epi<EPI_RESIDUAL>(st, a, partials); break;
        default: launch_skinny_epi<EPI_SWIGLU>(st, a, partials); break;
    }
}

// Raises the dynamic-LDS limit of every kernel that needs more than the default, once, at context
// creation: nothing but launches is then left for a call that may run under stream capture.
void gemm_kernels_init() {
    auto set = [](const void *f, int lds) { (void)hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lds); };
    constexpr int RT = RS_SKINNY_RT, PD = 10;
    set((const void *)gemm_skinny_kernel<EPI_STORE, RT, PD>, RT * 32768);
    set((const void *)gemm_skinny_kernel<EPI_RESIDUAL, RT, PD>, RT * 32768);
    set((const void *)gemm_skinny_kernel<EPI_SWIGLU, RT, PD>, RT * 32768);
    set((const void *)gemm_skinny_shared_kernel<EPI_SWIGLU, RS_SHARED_CH>, 2 * RS_SHARED_CH * 2048);
    set((const void *)gemm_skinny_shared_kernel<EPI_STORE, RS_SHARED_CH>, 2 * RS_SHARED_CH * 2048);
    set((const void *)gemm_skinny_shared_kernel<EPI_RESIDUAL, RS_SHARED_CH>, 2 * RS_SHARED_CH * 2048);
    set((const void *)gemm_direct_splitk_kernel, 5 * (128 + 256) * 32 * 2);
    set((const void *)gemm_grouped_kernel<EPI_STORE>, RS_NS_FULL * 32768);
    set((const void *)gemm_grouped_kernel<EPI_SWIGLU>, RS_NS_FULL * 32768);
    set((const void *)gemm_direct_mixed_kernel<EPI_STORE>, RS_NS_FULL * 32768);
    set((const void *)gemm_direct_mixed_kernel<EPI_RESIDUAL>, RS_NS_FULL * 32768);
    set((const void *)gemm_direct_mixed_kernel<EPI_SWIGLU>, RS_NS_FULL * 32768);
    set((const void *)gemm_direct_kernel<256, 256, EPI_STORE, RS_NS_FULL, 4>, RS_NS_FULL * 32768);
    set((const void *)gemm_direct_kernel<256, 256, EPI_RESIDUAL, RS_NS_FULL, 4>, RS_NS_FULL * 32768);
    set((const void *)gemm_direct_kernel<256, 256, EPI_SWIGLU, RS_NS_FULL, 4>, RS_NS_FULL * 32768);
    set((const void *)gemm_direct_kernel<128, 256, EPI_STORE, 5, 4>, 122880);
    set((const void *)gemm_direct_kernel<128, 256, EPI_RESIDUAL, 5, 4>, 122880);
    set((const void *)gemm_direct_kernel<128, 256, EPI_SWIGLU, 5, 4>, 122880);
    set((const void *)gemm_direct_kernel<256, 192, EPI_STORE, 4, 4>, 114688);
    set((const void *)gemm_direct_kernel<256, 192, EPI_RESIDUAL, 4, 4>, 114688);
}

