// bf16 GEMMs out = epi(A[M,K] * W[N,K]^T) on the gfx950 matrix cores (fp32 accumulation).
//
// Both operands are K-contiguous, so a lane's 8-element MFMA fragment is one 16-byte load.
// The weight tile is the MFMA "row" operand and the activation tile the "column" operand:
// a lane then owns 4 consecutive output columns of one output row, which makes the epilogues
// (residual add, SwiGLU, bf16 pack) plain per-lane code with 8-byte stores.
#include <type_traits>

#include "kernels.h"

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

// ---------------------------------------------------------------------------------------------
// Tiled kernel: BM x BN output tile per 256-thread workgroup (2x2 waves), BK = 64, operands
// staged global -> registers -> LDS (16-byte chunks, chunk index XOR (row>>1)&7 against bank
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
#pragma unroll
    for (int j = 0; j < CA; ++j) {
        const int r = (tid >> 3) + 32 * j;
        const int m = bm + r;
        pa[j] = (m < M) ? a.A + (size_t)m * K + cc * 8 : nullptr;
    }
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
        for (int j = 0; j < CA; ++j) ra[j] = (kin && pa[j]) ? ld_bf16x8(pa[j] + k0) : zero_bf16x8();
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
                    *(bf16x4 *)(a.out + (size_t)m * N + f) = v;
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
                    *(bf16x4 *)(a.out + (size_t)m * N + n) = v;
                }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Direct kernel (K % 32 == 0): same tiling and epilogues as the tiled kernel, but the operand
// tiles go global -> LDS with the 16-byte LDS-DMA load (no register staging) through a ring of
// NS LDS stages of BK = 32, so that a K tile is requested NS-1 tiles (several microseconds of
// MFMA work) before it is consumed: HBM latency is covered although only one wave runs per SIMD.
//
// A wave-wide load fills 1 KB = 16 rows x 64 B.  The LDS has 64 four-byte banks, so four rows
// span the banks once; 16 lanes reading one logical 16-byte chunk of 16 consecutive rows are
// conflict free when the stored chunk index is chunk ^ ((row >> 2) & 3).  The swizzle is applied
// by permuting which global chunk each lane fetches.  Rows past M or N are clamped to the last
// valid row (their results are never stored); K tiles past the end re-fetch the last tile into a
// stage nobody reads, which keeps the loop body branch free.
//
// Per K tile (two MFMA steps, one barrier): the loads of tile kt+NS-1 trickle out between the
// MFMAs; step 0 reads the step-1 fragments; step 1 waits until tile kt+1 has landed (vmcnt counts
// the younger loads that may still fly), meets the other waves at the barrier and reads tile
// kt+1's step-0 fragments.  In both steps the first MFMAs are issued before the reads, so a wait
// in front of a step is already satisfied and the barrier never sits between idle matrix cores.
//
// The flat workgroup id is remapped so that the workgroups resident on one XCD (ids congruent
// mod 8) cover a compact block of tiles: all row tiles of a few column tiles, served by that
// XCD's L2.
// ---------------------------------------------------------------------------------------------
template <int BM, int BN, int EPI, int NS, int OCC>
__global__ __launch_bounds__(256, OCC) void gemm_direct_kernel(GemmArgs a, int m_tiles, int n_tiles) {
    constexpr int BK = 32;
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int LA = BM / 64, LB = BN / 64;        // wave-wide loads per wave per stage
    constexpr int STAGE = (BM + BN) * BK;            // elements per stage
    constexpr int D = NS - 1;                        // prefetch distance in K tiles
    extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int c32 = lane & 31, h = lane >> 5;
    const int M = a.M, N = a.N, K = a.K;

    // XCD-aware tile order: xcd = id % 8 owns a contiguous run of column-major tiles
    const int total = m_tiles * n_tiles;
    const int per_xcd = (total + 7) >> 3;
    const int t = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (t >= total) return;
    const int bm = (t % m_tiles) * BM;
    const int nb = t / m_tiles;

    const int lrow = lane >> 2;                                     // row within the 16-row group
    const int lchunk = ((lane & 3) ^ ((lane >> 4) & 3)) << 3;       // element offset of the fetched chunk
    const bf16_t *pa[LA];
    const bf16_t *pb[LB];
#pragma unroll
    for (int j = 0; j < LA; ++j) {
        const int r = (wave * LA + j) * 16 + lrow;
        pa[j] = a.A + (size_t)min(bm + r, M - 1) * K + lchunk;
    }
#pragma unroll
    for (int j = 0; j < LB; ++j) {
        const int r = (wave * LB + j) * 16 + lrow;
        if (EPI == EPI_SWIGLU) {
            const int tt = r >> 5;
            const int f = min(nb * (BN / 2) + (tt >> 1) * 32 + (r & 31), N - 1);
            pb[j] = ((tt & 1) ? a.W2 : a.W) + (size_t)f * K + lchunk;
        } else {
            pb[j] = a.W + (size_t)min(nb * BN + r, N - 1) * K + lchunk;
        }
    }
    const int nk = K / BK;
    // loads [j0, j1) of the LA + LB wave-wide loads that bring K tile kt into its stage
    auto issue = [&](int kt, int j0, int j1) {
        const int stage = kt % NS;
        const int k0 = min(kt, nk - 1) * BK;
        bf16_t *sa = smem + stage * STAGE;
        bf16_t *sb = sa + BM * BK;
#pragma unroll
        for (int j = 0; j < LA + LB; ++j) {
            if (j < j0 || j >= j1) continue;
            if (j < LA)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(pa[j] + k0),
                                                 (__attribute__((address_space(3))) void *)(sa + (wave * LA + j) * 512),
                                                 16, 0, 0);
            else
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(pb[j - LA] + k0),
                                                 (__attribute__((address_space(3))) void *)(sb + (wave * LB + j - LA) * 512),
                                                 16, 0, 0);
        }
    };

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int x3 = (c32 >> 2) & 3;
    const int a_row = (wm * WM + c32) * BK, b_row = (wn * WN + c32) * BK;
    bf16x8 wf[2][TN], xf[2][TM];
    auto read_frags = [&](int set, int kt, int step) {
        const bf16_t *sa = smem + (kt % NS) * STAGE;
        const bf16_t *sb = sa + BM * BK;
        const int co = ((2 * step + h) ^ x3) << 3;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) wf[set][tn] = *(const bf16x8 *)&sb[b_row + tn * 32 * BK + co];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) xf[set][tm] = *(const bf16x8 *)&sa[a_row + tm * 32 * BK + co];
    };
#pragma unroll
    for (int i = 0; i < D; ++i) issue(i, 0, LA + LB);
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((D - 1) * (LA + LB)) : "memory");
    read_frags(0, 0, 0);

    // One K tile = SL MFMA slots (two steps of TN x TM).  A load instruction holds up the
    // issuing wave while the CU's one memory pipeline takes it, and a wave that cannot issue
    // cannot feed its matrix core either; so the LT loads of the next tile are placed one at a
    // time, evenly between the MFMAs, and wave w places its loads w quarter-spacings later than
    // wave 0: the four lock-stepped waves never queue behind one another.
    constexpr int SL = 2 * TN * TM, LT = LA + LB, SP = SL / LT;
    auto k_loop = [&](auto wtag) {
        constexpr int W = decltype(wtag)::value;
        constexpr int SHIFT = (W * SP) / 4;
        // loads of the current iteration already issued when the barrier of slot SL/2 is reached
        constexpr int EARLY = ((SL / 2 - 1 - SHIFT) / SP) + 1;
        for (int kt = 0; kt < nk; ++kt) {
#pragma unroll
            for (int sl = 0; sl < SL; ++sl) {
                const int step = sl / (TN * TM), tn = (sl % (TN * TM)) / TM, tm = sl % TM;
                if (sl == SL / 2)
                    // tile kt+1 has landed once only the younger loads are outstanding; this wave's
                    // LDS reads are complete before it tells the others so at the barrier
                    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"((D - 2) * LT + EARLY) : "memory");
                acc[tn][tm] = mfma32(wf[step][tn], xf[step][tm], acc[tn][tm]);
                __builtin_amdgcn_sched_barrier(0);
                if (sl == TM - 1) read_frags(1, kt, 1);
                if (sl == SL / 2 + TM - 1) read_frags(0, kt + 1, 0);
                if (sl >= SHIFT && (sl - SHIFT) % SP == 0 && (sl - SHIFT) / SP < LT)
                    issue(kt + D, (sl - SHIFT) / SP, (sl - SHIFT) / SP + 1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    switch (__builtin_amdgcn_readfirstlane(wave)) {
        case 0: k_loop(std::integral_constant<int, 0>{}); break;
        case 1: k_loop(std::integral_constant<int, 1>{}); break;
        case 2: k_loop(std::integral_constant<int, 2>{}); break;
        default: k_loop(std::integral_constant<int, 3>{}); break;
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");

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
                    *(bf16x4 *)(a.out + (size_t)m * N + f) = v;
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
                    *(bf16x4 *)(a.out + (size_t)m * N + n) = v;
                }
        }
    }
}

template <int BM, int BN, int EPI, int NS, int OCC>
static void launch_direct_epi(hipStream_t st, const GemmArgs &a) {
    const int m_tiles = (a.M + BM - 1) / BM;
    const int n_tiles = (EPI == EPI_SWIGLU) ? (a.N + BN / 2 - 1) / (BN / 2) : (a.N + BN - 1) / BN;
    const int total = m_tiles * n_tiles;
    const int grid = ((total + 7) / 8) * 8;
    constexpr int lds = NS * (BM + BN) * 32 * 2;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void *)gemm_direct_kernel<BM, BN, EPI, NS, OCC>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_set = true;
    }
    hipLaunchKernelGGL((gemm_direct_kernel<BM, BN, EPI, NS, OCC>), dim3(grid), dim3(256), lds, st, a, m_tiles, n_tiles);
}

template <int BM, int BN, int NS, int OCC>
static void launch_direct(hipStream_t st, const GemmArgs &a) {
    switch (a.epi) {
        case EPI_STORE: launch_direct_epi<BM, BN, EPI_STORE, NS, OCC>(st, a); break;
        case EPI_RESIDUAL: launch_direct_epi<BM, BN, EPI_RESIDUAL, NS, OCC>(st, a); break;
        default: launch_direct_epi<BM, BN, EPI_SWIGLU, NS, OCC>(st, a); break;
    }
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

void launch_gemm_tiled(hipStream_t st, const GemmArgs &a) {
    if (a.M <= 0 || a.N <= 0) return;
    const bool aligned = (a.K % 32 == 0) && a.K >= 32;
    if (aligned && a.M >= 512 && a.N >= 1024) {
        // the tile grid is a function of the problem shape only
        const long tiles256 = (long)((a.M + 255) / 256) * ((a.epi == EPI_SWIGLU ? 2 * a.N : a.N) / 256);
        if (tiles256 >= 256)
            launch_direct<256, 256, 4, 1>(st, a);   // 4 x 32 KB of LDS
        else
            launch_direct<128, 256, 5, 1>(st, a);   // 5 x 24 KB of LDS
    } else if (a.M >= 1024 && a.N >= 1024) {
        launch_tiled<256, 256>(st, a);
    } else {
        launch_tiled<128, 128>(st, a);
    }
}

// ---------------------------------------------------------------------------------------------
// Skinny kernel (M <= 64): the weights are streamed once from HBM straight into MFMA fragments,
// no LDS staging.  Workgroup = 64 (virtual) weight rows x one K slice; its 4 waves split the
// slice and are summed in wave order through LDS; the S slices of K are summed in slice order
// by the epilogue kernel.  S depends on (N, K) only, so results never depend on the CU share.
// Within a 64-wide K window lane half h covers k in [32h, 32h+32): 64 contiguous bytes/lane.
// ---------------------------------------------------------------------------------------------
static inline int skinny_virtual_n(int N, int epi) {
    return epi == EPI_SWIGLU ? ((N + 31) / 32) * 64 : ((N + 63) / 64) * 64;
}
static inline int skinny_splits(int N, int K, int epi) {
    const int tiles = skinny_virtual_n(N, epi) / 64;
    int S = 1;
    while (tiles * S < 256 && S < 16 && (K + 2 * S - 1) / (2 * S) >= 256) S *= 2;
    return S;
}
static inline int skinny_k_per_wg(int K, int S) {
    const int per = (K + S - 1) / S;
    return ((per + 255) / 256) * 256;  // 4 waves x whole 64-wide windows
}
size_t skinny_partial_elems(int M, int N, int K, int epi) {
    return (size_t)skinny_splits(N, K, epi) * (size_t)M * (size_t)skinny_virtual_n(N, epi);
}

template <int EPI>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(GemmArgs a, float *__restrict__ part,
                                                          int k_per_wg, int Nv) {
    // 64 KB: per wave two 8 KB weight slabs [64 rows][64 k] (rows of 128 B, chunk ^= (row>>1)&7);
    // after the K loop the same bytes hold the waves' accumulators for the in-order reduction
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem_sk[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c32 = lane & 31, h = lane >> 5;
    const int M = a.M, N = a.N, K = a.K;
    const int kw = k_per_wg >> 2;
    const int kb = blockIdx.y * k_per_wg + wave * kw;
    const int ke = min(kb + kw, K);
    const int nsteps = ke > kb ? (ke - kb + 63) >> 6 : 0;
    bf16_t *slab = (bf16_t *)(smem_sk + wave * 16384);

    // weight rows fetched by this lane in each of the 8 wave-wide DMA loads of a slab
    const bf16_t *wrow[8];
    int wchunk[8];
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        const int row = 8 * g + (lane >> 3);
        wchunk[g] = ((lane & 7) ^ ((row >> 1) & 7)) << 3;   // k offset of the chunk this lane stores
        if (EPI == EPI_SWIGLU) {
            const int f = min((int)blockIdx.x * 32 + (row & 31), N - 1);
            wrow[g] = ((row >> 5) ? a.W2 : a.W) + (size_t)f * K;
        } else {
            wrow[g] = a.W + (size_t)min((int)blockIdx.x * 64 + row, N - 1) * K;
        }
    }
    auto issue_w = [&](int k0, int stage) {
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            // a chunk past K is replaced by the window's first chunk (finite data; X is zero there)
            const int ko = (k0 + wchunk[g] < K) ? wchunk[g] : 0;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(wrow[g] + k0 + ko),
                                             (__attribute__((address_space(3))) void *)(slab + stage * 4096 + g * 512),
                                             16, 0, 0);
        }
    };
    // activation fragments straight from the fragment-packed matrix: contiguous 1 KB per load
    auto load_x = [&](int k0, bf16x8 (&xf)[2][4]) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int kb16 = (k0 >> 4) + s;
            const bool kin = 16 * kb16 + 8 * h < K;
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
                xf[tm][s] = (kin && 32 * tm + c32 < M) ? ld_bf16x8(a.A + ((size_t)(kb16 * 2 + tm) * 64 + lane) * 8)
                                                       : zero_bf16x8();
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    bf16x8 xcur[2][4], xnext[2][4];
    if (nsteps > 0) {
        issue_w(kb, 0);
        load_x(kb, xcur);
    }
    const int x7 = (c32 >> 1) & 7;
    for (int i = 0; i < nsteps; ++i) {
        const bool more = i + 1 < nsteps;
        if (more) {
            issue_w(kb + 64 * (i + 1), (i + 1) & 1);
            load_x(kb + 64 * (i + 1), xnext);
            // LDS-DMA loads and register loads each complete in order, but not with respect to one
            // another: the younger (fast, L2-resident) activation loads may all be done while older
            // weight DMAs still fly.  "At most 8 outstanding" is the largest count that still implies
            // step i is complete: were a load of W(i) or X(i) pending, so were the 8 of its kind
            // from step i+1, i.e. 16 in total.
            asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        const bf16_t *sl = slab + (i & 1) * 4096;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            bf16x8 wf[2];
#pragma unroll
            for (int tn = 0; tn < 2; ++tn)
                wf[tn] = *(const bf16x8 *)&sl[(32 * tn + c32) * 64 + (((2 * s + h) ^ x7) << 3)];
#pragma unroll
            for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                for (int tm = 0; tm < 2; ++tm) acc[tn][tm] = mfma32(wf[tn], xcur[tm][s], acc[tn][tm]);
        }
        if (more) {
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int s = 0; s < 4; ++s) xcur[tm][s] = xnext[tm][s];
        }
    }
    // in-order reduction of the 4 waves; each wave first overwrites only its own slab bytes
    float *red = (float *)smem_sk;   // [wave][tile][lane][16]
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int tn = 0; tn < 2; ++tn)
#pragma unroll
        for (int tm = 0; tm < 2; ++tm)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x4 v = {acc[tn][tm][4 * j], acc[tn][tm][4 * j + 1], acc[tn][tm][4 * j + 2], acc[tn][tm][4 * j + 3]};
                *(f32x4 *)&red[((wave * 4 + tn * 2 + tm) * 64 + lane) * 16 + 4 * j] = v;
            }
    __syncthreads();
    // wave w finishes tile (tn, tm) = (w>>1, w&1): sum of the 4 waves in wave order
    const int tn = wave >> 1, tm = wave & 1;
    const int m = 32 * tm + c32;
    if (m < M) {
        float *dst = part + ((size_t)blockIdx.y * M + m) * Nv + blockIdx.x * 64 + 32 * tn;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f32x4 v = *(const f32x4 *)&red[((0 * 4 + wave) * 64 + lane) * 16 + 4 * j];
#pragma unroll
            for (int w = 1; w < 4; ++w) v += *(const f32x4 *)&red[((w * 4 + wave) * 64 + lane) * 16 + 4 * j];
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
    bf16_t *dst = a.out_packed ? a.out + packed_chunk_offset(m, n) + (n & 7) : a.out + (size_t)m * N + n;
    *(bf16x4 *)dst = v;
}

void launch_gemm_skinny(hipStream_t st, const GemmArgs &a, float *partials) {
    if (a.M <= 0 || a.N <= 0) return;
    const int Nv = skinny_virtual_n(a.N, a.epi);
    const int S = skinny_splits(a.N, a.K, a.epi);
    const int kpw = skinny_k_per_wg(a.K, S);
    dim3 grid(Nv / 64, S);
    const int eblocks = (a.M * (a.N / 4) + 255) / 256;
    switch (a.epi) {
        case EPI_STORE:
            hipLaunchKernelGGL(gemm_skinny_kernel<EPI_STORE>, grid, dim3(256), 65536, st, a, partials, kpw, Nv);
            hipLaunchKernelGGL(skinny_epilogue_kernel<EPI_STORE>, dim3(eblocks), dim3(256), 0, st, a, partials, S, Nv);
            break;
        case EPI_RESIDUAL:
            hipLaunchKernelGGL(gemm_skinny_kernel<EPI_RESIDUAL>, grid, dim3(256), 65536, st, a, partials, kpw, Nv);
            hipLaunchKernelGGL(skinny_epilogue_kernel<EPI_RESIDUAL>, dim3(eblocks), dim3(256), 0, st, a, partials, S, Nv);
            break;
        default:
            hipLaunchKernelGGL(gemm_skinny_kernel<EPI_SWIGLU>, grid, dim3(256), 65536, st, a, partials, kpw, Nv);
            hipLaunchKernelGGL(skinny_epilogue_kernel<EPI_SWIGLU>, dim3(eblocks), dim3(256), 0, st, a, partials, S, Nv);
            break;
    }
}
