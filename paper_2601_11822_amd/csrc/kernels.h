// Host-callable launchers of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.h"

// out[m,:] = x[m,:] * rsqrt(mean(x[m,:]^2) + eps) * g      (bf16 in, fp32 math, bf16 out)
// x is row-major [M][d]; `out` is written fragment-packed (packed_offset with packed_mt(M) row tiles).
void launch_rmsnorm(hipStream_t st, const bf16_t *x, const bf16_t *g, bf16_t *out, int M, int d, float eps);

struct RopeKvArgs {
    bf16_t *qkv;            // [M][nqkv]; q part rotated in place
    const CosSin *table;    // [max_pos][hd/2]
    bf16_t *k_pool;         // this layer: [n_blocks][Hkv][16][hd]
    bf16_t *v_pool;         // this layer: [n_blocks][Hkv][hd][16]
    const int32_t *tables;  // [n_req][max_blk]
    const int32_t *ctx_lens;  // decode: position of row m (and request = m); prefill: nullptr
    int32_t *err_flag;
    int M, Hq, Hkv, hd, max_blk, n_blocks, max_pos;
    SeqInfo seq;  // prefill only
};
void launch_rope_kvwrite(hipStream_t st, const RopeKvArgs &a);

struct PrefillAttnArgs {
    const bf16_t *q;  // [T][q_stride] (rotated)
    int q_stride;
    bf16_t *out;  // [T][Hq*hd], fragment-packed (packed_mt(T) row tiles)
    const bf16_t *k_pool, *v_pool;
    const int32_t *tables;
    int32_t *err_flag;
    int Hq, Hkv, hd, max_blk, n_blocks;
    float scale_log2;  // log2(e)/sqrt(hd)
    SeqInfo seq;       // seq.start[r] > 0: the rows are a later chunk of prompt r and also attend to its cached positions before them
    int Mt_out = 0;    // row tiles of the packed output matrix when it holds more rows than this call's (0: packed_mt of this call's rows)
};
void launch_prefill_attention(hipStream_t st, const PrefillAttnArgs &a);

struct DecodeAttnArgs {
    const bf16_t *q;  // [B][q_stride]
    int q_stride;
    bf16_t *out;  // [B][Hq*hd], fragment-packed (packed_mt(B) row tiles)
    const bf16_t *k_pool, *v_pool;
    const int32_t *tables;
    const int32_t *ctx_lens;
    int32_t *err_flag;
    float *part_o;   // [B][Hq][n_chunks][hd]
    float *part_ml;  // [B][Hq][n_chunks][2]
    int B, Hq, Hkv, hd, max_blk, n_blocks, max_ctx, n_chunks;
    float scale_log2;
    int chunk_major;   // order of the workgroups only (results do not depend on it): chunks slowest, else requests slowest
    int out_row0 = 0, out_Mt = 0;   // the packed output matrix holds other rows first / more row tiles (0: packed_mt(B))
};
#define RS_SKINNY_TARGET_WGS 384  // the skinny GEMM splits K until it has about this many workgroups
#define RS_DECODE_CHUNK 512  // tokens per workgroup of the decode attention
void launch_decode_attention(hipStream_t st, const DecodeAttnArgs &a);

enum GemmEpilogue { EPI_STORE = 0, EPI_RESIDUAL = 1, EPI_SWIGLU = 2 };

// out[M,N] = epi(A[M,K] * W[N,K]^T).  EPI_RESIDUAL adds resid[M,N].  EPI_SWIGLU:
// out[M,N] = silu(A*W^T) * (A*W2^T) with W, W2 both [N,K].
// A is always fragment-packed (packed_offset, packed_mt(M) row tiles).  W / W2 are the caller's
// row-major matrices (read by the tail-safe tiled kernel), Wp / Wp2 the library's fragment-packed
// copies of the same matrices (launch_pack_weights; read by the direct and the skinny kernels).
struct GemmArgs {
    const bf16_t *A;
    const bf16_t *W, *W2;
    const bf16_t *Wp, *Wp2;
    const bf16_t *resid;  // row-major [M][N]
    bf16_t *out;          // row-major [M][N], or fragment-packed when it feeds another GEMM
    int M, N, K;
    int epi;
    int out_packed = 0;
    int cus = 0;  // compute units of the launching stream's partition (0: the whole chip); scheduling only
    // float32 scratch for launch_gemm_tiled's K-sliced path (few tiles, long K); without it that path is not taken
    float *partials = nullptr;
    size_t partial_cap = 0;   // elements
    // grouped form (launch_gemm_grouped): the expert whose weights each 128-row tile multiplies (-1: skip the
    // tile), and the distance in elements between consecutive experts' packed matrices (Wp and Wp2 alike)
    const int32_t *tile_expert = nullptr;
    size_t expert_stride = 0;
};
// Upper bound of what the K-sliced path of launch_gemm_tiled needs, for any M: S * M * N <= this.
#define RS_DIRECT_PARTIAL_ELEMS ((size_t)10 << 20)
// false (nothing launched): the shape needs the generic kernel, which reads a.W / a.W2, and they are null
bool launch_gemm_tiled(hipStream_t st, const GemmArgs &a);

// Skinny variant for M <= 64 (decode): weight-streaming, deterministic split-K through
// `partials` (fp32, at least skinny_partial_elems(...) elements).  Reads A, Wp and Wp2.
size_t skinny_partial_elems(int M, int N, int K, int epi);
void launch_gemm_skinny(hipStream_t st, const GemmArgs &a, float *partials);
// Main pass only (a.epi must be EPI_STORE): leaves part[s][m][n], s < *S_out K-slices, row stride
// *Nv_out floats; the product's element (m, n) is the sum of its slices in slice order.
void launch_gemm_skinny_partials(hipStream_t st, const GemmArgs &a, float *partials, int *S_out, int *Nv_out);
// True where that pass streams the weights with the shared-activation kernel (about HBM rate for M <= 64 rows).
bool gemm_skinny_partials_shared(int N, int K);
bool launch_gemm_direct_partials(hipStream_t st, const GemmArgs &a, float *part);
size_t packed_weight_elems(int N, int K);
void launch_pack_weights(hipStream_t st, const bf16_t *W, bf16_t *Wp, int N, int K);

// ---- decode-side projections (decode_gemm.hip): at most 64 rows, weights streamed once, RMSNorm folded in ----
struct DGemmArgs {
    const bf16_t *A_packed;   // activations fragment-packed with two row tiles (packed_mt(M) == 2), or
    const bf16_t *X_rows;     // row-major [M][K] hidden state: multiplied by gain[K] on the way in, and
    const bf16_t *gain;       //   the sums of squares of each row over each K slice go to
    float *ssq_part;          //   ssq_part[slice][64]  (the epilogue turns them into the RMSNorm scale)
    const bf16_t *Wp, *Wp2;   // fragment-packed weights [N][K]; Wp2: the up matrix of a gate/up pair
    float *part;              // out: float32 partial products [S][M][Nv]
    int M, N, K;
};
struct DGemmPlan {
    bool pair;
    int cols, S, kb_per_wg, Nv;   // workgroups along N, K slices, k-blocks per slice, row stride of the partial products
};
// True if the streaming kernel takes this projection (K a multiple of 256, N a multiple of 4 and at least 128).
bool dgemm_applies(int N, int K);
DGemmPlan dgemm_plan(int N, int K, bool pair);
size_t dgemm_partial_elems(int M, int N, int K, bool pair);
// narrow: half-height workgroups, twice as many (same sums, same bits); dgemm_prefers_half_height says when, from the
// number of compute units the side owns
void launch_dgemm_partials(hipStream_t st, const DGemmArgs &a, const DGemmPlan &p, bool narrow);
bool dgemm_prefers_half_height(const DGemmPlan &p, int cus);
struct DEpiArgs {
    const float *part;        // [S][M][Nv]
    int S, Nv;
    const float *ssq_part;    // [S_ssq][64] or nullptr: no row scale
    int S_ssq, d;
    float eps;
    const bf16_t *resid;      // EPI_RESIDUAL: row-major [M][N]
    bf16_t *out;              // EPI_RESIDUAL: row-major [M][N]; EPI_SWIGLU: fragment-packed [M][N]
    int M, N;
};
void launch_dgemm_epilogue(hipStream_t st, const DEpiArgs &a, int epi);
struct QkvEpiArgs {
    const float *part;        // [S][M][Nv] partial q | k | v
    const float *ssq_part;    // [S][64]
    int S, Nv, d;
    float eps;
    bf16_t *qkv;              // out: [M][(Hq+2Hkv)*hd] with q and k rotated
    const CosSin *table;
    bf16_t *k_pool, *v_pool;  // this layer
    const int32_t *tables, *ctx_lens;
    int32_t *err_flag;
    int M, Hq, Hkv, hd, max_blk, n_blocks, max_pos;
};
void launch_qkv_rope_epilogue(hipStream_t st, const QkvEpiArgs &a);
void decode_gemm_kernels_init();

// Grouped GEMM over 128-row tiles that each belong to one expert: STORE or SWIGLU epilogue, a.M = the padded
// row capacity (a multiple of 128), a.expert_stride and a.tile_expert set, the latter followed by the work list
// that moe_plan_kernel writes behind the a.M / 128 tile entries.  Needs K % 32 == 0 and N >= 1024.
bool launch_gemm_grouped(hipStream_t st, const GemmArgs &a);

#define RS_MOE_MAX_EXPERTS 16
// Rows of the grouped (expert-major) layout that M rows with two experts each can need: every expert's segment
// is padded to whole 128-row tiles, and a segment of two or more tiles may be preceded by one idle tile so that
// it starts on a 256-row boundary.
static inline int moe_row_cap(int M, int E) { return ((2 * M + 255 * E + 127) / 128) * 128; }
struct MoeArgs {
    const bf16_t *h;        // normalised rows, fragment-packed with packed_mt(M) row tiles
    const bf16_t *router;   // [E][d] row-major
    int32_t *sel;           // [M][2] experts of each row
    float *wt;              // [M][2] their weights
    int32_t *pos;           // [M][2] grouped row of each assignment
    int32_t *src;           // [Mg_cap] source row of each grouped row, -1 for padding
    int32_t *tile_expert;   // [2 * (Mg_cap / 128) + 1]: expert of each tile, then the grouped GEMM's work list
    bf16_t *a_g;            // gathered rows, fragment-packed with Mg_cap / 32 row tiles
    const bf16_t *out_g;    // [Mg_cap][d] expert outputs, row-major
    const bf16_t *x1;       // [M][d]
    bf16_t *y;              // [M][d]
    int M, d, E, Mg_cap;
};
void launch_moe_route_and_gather(hipStream_t st, const MoeArgs &a);
void launch_moe_combine(hipStream_t st, const MoeArgs &a);

struct EmbedArgs {
    const int32_t *tokens;     // [n], or per-slot tokens when row_slot is given, or slot regions when slots is given
    const int32_t *row_slot;   // [n] or nullptr
    const bf16_t *table;       // [vocab][d]
    bf16_t *x;                 // [n][d] row-major
    int32_t *err_flag;
    int n, d, vocab;
    // several prompts (or a chunk of each, from position seq.start[q]) in one call: row r of prompt q (seq.cu
    // delimits them) is token tokens[slots[q] * slot_stride + seq.start[q] + (r - seq.cu[q])]
    const int32_t *slots = nullptr;
    int slot_stride = 0;
    SeqInfo seq{};
};
void launch_embed(hipStream_t st, const EmbedArgs &a);
// out[q][:] = x[seq.cu[q+1] - 1][:]: the last row of each prompt, for the LM head.
void launch_gather_last_rows(hipStream_t st, const bf16_t *x, bf16_t *out, int d, const SeqInfo &seq);

struct HeadArgmaxArgs {
    const float *part;         // [S][M][Nv] partial logits
    float *logits;             // [M][N] or nullptr
    int32_t *tokens;           // [M] or nullptr
    const int32_t *row_slot;   // [M] or nullptr
    int32_t *tok_by_slot;      // scattered copy of the tokens, or nullptr
    int S, M, N, Nv;
};
void launch_head_argmax(hipStream_t st, const HeadArgmaxArgs &a);

// Counts workgroups per physical CU: hist[(xcc << 8) | (se << 5) | (sh << 4) | cu] += 1.
void launch_cu_probe(hipStream_t st, int32_t *hist, int n_workgroups);

// Reads `bytes` (multiple of 16) once with coalesced 16-byte loads.
void launch_stream_read(hipStream_t st, const void *src, size_t bytes, int n_workgroups);

// Back-to-back register-only 32x32x16 bf16 MFMAs; returns the flops the launch performs.
double launch_mfma_probe(hipStream_t st, float *sink, int n_workgroups, int iters);

void launch_noop(hipStream_t st);

// Zeroes `bytes` (a multiple of 16) of device memory with a kernel (usable under stream capture).
void launch_fill_zero(hipStream_t st, void *dst, size_t bytes);

// Called once per context creation (see gemm.hip).
void gemm_kernels_init();
void attention_kernels_init();

