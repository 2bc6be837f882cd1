/*
 * CPU oracle for one Llama-style decoder layer with a paged KV cache.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition that the
 * GPU library is checked against.  It shares no code with the GPU path and the
 * product never calls it; only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg do.
 *
 * The paper (section 2.1) states what the two phases are: prefill evaluates the
 * whole prompt in parallel (large matrix products and causal self-attention)
 * and fills the KV cache; decode evaluates one new token per request, attending
 * over the accumulated cache.  Section 4.5.1 states that the cache is paged
 * (blocks allocated per request, addressed through a block table) and shared,
 * never copied, between the two phases.  The layer algebra itself is the
 * textbook Llama block; every step below is that definition written out:
 *
 *   h  = RMSNorm(x; g1)                 h = x / sqrt(mean(x^2) + eps) * g1
 *   q,k,v = h Wq^T, h Wk^T, h Wv^T      (Wqkv rows: all q heads, then k, then v)
 *   RoPE(q), RoPE(k) at the token's position, rotate-half pairing (i, i+hd/2)
 *   K/V of the token -> cache[block_table[req][pos/16]][pos%16][kv_head][:]
 *   o  = softmax(q K^T / sqrt(hd)) V    over keys j <= pos of the same request,
 *                                       query head hq uses kv head hq / (Hq/Hkv)
 *   x1 = x + o Wo^T
 *   h2 = RMSNorm(x1; g2)
 *   y  = x1 + (silu(h2 Wg^T) * (h2 Wu^T)) Wd^T        silu(z) = z / (1 + exp(-z))
 *
 * A prompt may also be evaluated in chunks (section 3.1: chunked prefill, the hybrid-batching baseline the
 * paper compares with): a chunk's tokens sit at positions start..start+len-1 and attend to every cached
 * position before them plus themselves; orc_prefill_chunk_layer reads all keys back through the block table.
 * Pinned by: chunked == whole prefill rows == float64 dense rows (tests/test_oracle_pins.py).
 *
 * Arithmetic is float32 (the precision the task fixes for the oracle); the
 * rotary angles are formed in float64 and their cos/sin rounded to float32.
 * Matrix products accumulate k = 0..K-1 in order for every output element.
 * Inputs arrive as bfloat16 bit patterns and are widened exactly.
 * Weights are [out_features][in_features].
 *
 * OpenMP spreads independent rows over the host cores; nothing else is blocked,
 * fused or reordered.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_ERR_ARG (-1)
#define ORC_ERR_BLOCK (-4)

/* exact widening of a bfloat16 bit pattern */
static inline float bf16_widen(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

void orc_bf16_to_f32(const uint16_t *in, float *out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = bf16_widen(in[i]);
}

/* out[k][n] = w[n][k]: a plain copy into [in][out] order so that the product
 * below can walk outputs contiguously while still summing k in order. */
void orc_transpose(const float *w, int64_t N, int64_t K, float *out) {
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < K; ++k)
        for (int64_t n = 0; n < N; ++n) out[k * N + n] = w[n * K + k];
}

/* RMSNorm, eps inside the square root. */
void orc_rmsnorm(const float *x, const float *g, int64_t M, int64_t d, float eps, float *h) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *xr = x + m * d;
        float ss = 0.0f;
        for (int64_t j = 0; j < d; ++j) ss += xr[j] * xr[j];
        float inv = 1.0f / sqrtf(ss / (float)d + eps);
        for (int64_t j = 0; j < d; ++j) h[m * d + j] = xr[j] * inv * g[j];
    }
}

/* out[m][n] = sum_k a[m][k] * w[n][k], given wt = transpose of w ([K][N]). */
void orc_linear_t(const float *a, const float *wt, int64_t M, int64_t N, int64_t K, float *out) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t m = 0; m < M; ++m) {
        float *o = out + m * N;
        for (int64_t n = 0; n < N; ++n) o[n] = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float av = a[m * K + k];
            const float *wr = wt + k * N;
            for (int64_t n = 0; n < N; ++n) o[n] += av * wr[n];
        }
    }
}

/* Same product straight from w[N][K] (dot product per output). */
void orc_linear(const float *a, const float *w, int64_t M, int64_t N, int64_t K, float *out) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float s = 0.0f;
            for (int64_t k = 0; k < K; ++k) s += a[m * K + k] * w[n * K + k];
            out[m * N + n] = s;
        }
}

/* Rotary embedding in place on x[M][H][hd]; row m sits at position pos[m].
 * theta_i = base^(-2i/hd); pair (i, i+hd/2). */
void orc_rope(float *x, const int32_t *pos, int64_t M, int64_t H, int64_t hd, double base,
              int64_t row_stride) {
    int64_t half = hd / 2;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t i = 0; i < half; ++i) {
            double theta = pow(base, -2.0 * (double)i / (double)hd);
            double phi = (double)pos[m] * theta;
            float c = (float)cos(phi), s = (float)sin(phi);
            for (int64_t h = 0; h < H; ++h) {
                float *v = x + m * row_stride + h * hd;
                float a = v[i], b = v[i + half];
                v[i] = a * c - b * s;
                v[i + half] = b * c + a * s;
            }
        }
    }
}

static inline float silu(float z) { return z / (1.0f + expf(-z)); }

void orc_silu_mul(const float *g, const float *u, int64_t n, float *out) {
    for (int64_t i = 0; i < n; ++i) out[i] = silu(g[i]) * u[i];
}

/* Softmax-weighted sum for ONE query vector against n_keys keys fetched through
 * get-by-index pointers.  scores/weights in float32. */
static void attend_one(const float *q, const float *const *kp, const float *const *vp,
                       int64_t n_keys, int64_t hd, float *o, float *scratch) {
    float scale = 1.0f / sqrtf((float)hd);
    float mx = -INFINITY;
    for (int64_t j = 0; j < n_keys; ++j) {
        float s = 0.0f;
        for (int64_t t = 0; t < hd; ++t) s += q[t] * kp[j][t];
        s *= scale;
        scratch[j] = s;
        if (s > mx) mx = s;
    }
    float den = 0.0f;
    for (int64_t j = 0; j < n_keys; ++j) {
        scratch[j] = expf(scratch[j] - mx);
        den += scratch[j];
    }
    for (int64_t t = 0; t < hd; ++t) o[t] = 0.0f;
    for (int64_t j = 0; j < n_keys; ++j) {
        float w = scratch[j] / den;
        for (int64_t t = 0; t < hd; ++t) o[t] += w * vp[j][t];
    }
}

/* Causal self-attention over contiguous q,k,v of several independent requests.
 * q: [T][Hq][hd] (row stride q_stride), k, v: [T][Hkv][hd] (row stride kv_stride).
 * cu_seqlens[n_req+1] delimits requests.  rows/n_rows: optional subset of global
 * token rows to evaluate (NULL = all); o is [T][Hq*hd] and only evaluated rows
 * are written. */
int orc_attn_causal(const float *q, int64_t q_stride, const float *k, const float *v,
                    int64_t kv_stride, const int32_t *cu_seqlens, int32_t n_req, int64_t Hq,
                    int64_t Hkv, int64_t hd, const int32_t *rows, int64_t n_rows, float *o) {
    if (Hq % Hkv) return ORC_ERR_ARG;
    int64_t G = Hq / Hkv;
    int64_t T = cu_seqlens[n_req];
    int64_t n_eval = rows ? n_rows : T;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t e = 0; e < n_eval; ++e) {
        int64_t r = rows ? rows[e] : e;
        if (r < 0 || r >= T) { err = 1; continue; }
        int32_t req = 0;
        while (req < n_req && !(r >= cu_seqlens[req] && r < cu_seqlens[req + 1])) ++req;
        if (req >= n_req) { err = 1; continue; }
        int64_t start = cu_seqlens[req];
        int64_t n_keys = r - start + 1; /* keys j <= own position */
        const float **kp = (const float **)malloc(sizeof(float *) * n_keys * 2);
        const float **vp = kp + n_keys;
        float *scratch = (float *)malloc(sizeof(float) * n_keys);
        for (int64_t hq = 0; hq < Hq; ++hq) {
            int64_t hk = hq / G;
            for (int64_t j = 0; j < n_keys; ++j) {
                kp[j] = k + (start + j) * kv_stride + hk * hd;
                vp[j] = v + (start + j) * kv_stride + hk * hd;
            }
            attend_one(q + r * q_stride + hq * hd, kp, vp, n_keys, hd, o + r * Hq * hd + hq * hd,
                       scratch);
        }
        free(scratch);
        free((void *)kp);
    }
    return err ? ORC_ERR_ARG : ORC_OK;
}

/* Write one token's K and V (each [Hkv][hd]) into the paged pools
 * [n_blocks][block][Hkv][hd] at logical position pos of the request whose block
 * table row is tab. */
static int kv_store(float *Kc, float *Vc, int64_t n_blocks, int64_t block, int64_t Hkv, int64_t hd,
                    const int32_t *tab, int64_t max_blk, int64_t pos, const float *k,
                    const float *v) {
    int64_t bi = pos / block, slot = pos % block;
    if (bi >= max_blk) return ORC_ERR_BLOCK;
    int64_t blk = tab[bi];
    if (blk < 0 || blk >= n_blocks) return ORC_ERR_BLOCK;
    int64_t off = ((blk * block + slot) * Hkv) * hd;
    memcpy(Kc + off, k, sizeof(float) * Hkv * hd);
    memcpy(Vc + off, v, sizeof(float) * Hkv * hd);
    return ORC_OK;
}

int orc_kv_write(float *Kc, float *Vc, int64_t n_blocks, int64_t block, int64_t Hkv, int64_t hd,
                 const int32_t *tables, int64_t max_blk, const int32_t *req_of_row,
                 const int32_t *pos_of_row, int64_t M, const float *k, const float *v,
                 int64_t kv_stride) {
    for (int64_t m = 0; m < M; ++m) {
        int rc = kv_store(Kc, Vc, n_blocks, block, Hkv, hd, tables + req_of_row[m] * max_blk,
                          max_blk, pos_of_row[m], k + m * kv_stride, v + m * kv_stride);
        if (rc) return rc;
    }
    return ORC_OK;
}

/* Attention of one query token per request over keys gathered through the block
 * table: request i attends to positions 0..n_keys[i]-1 of its own cache. */
int orc_attn_paged(const float *q, const float *Kc, const float *Vc, int64_t n_blocks,
                   int64_t block, int64_t Hq, int64_t Hkv, int64_t hd, const int32_t *tables,
                   int64_t max_blk, const int32_t *n_keys, int64_t B, float *o) {
    if (Hq % Hkv) return ORC_ERR_ARG;
    int64_t G = Hq / Hkv;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < B; ++i) {
        int64_t n = n_keys[i];
        if (n <= 0 || (n + block - 1) / block > max_blk) { err = 1; continue; }
        const float **kp = (const float **)malloc(sizeof(float *) * n * 2);
        const float **vp = kp + n;
        float *scratch = (float *)malloc(sizeof(float) * n);
        for (int64_t hq = 0; hq < Hq; ++hq) {
            int64_t hk = hq / G;
            int bad = 0;
            for (int64_t j = 0; j < n; ++j) {
                int64_t blk = tables[i * max_blk + j / block];
                if (blk < 0 || blk >= n_blocks) { bad = 1; break; }
                int64_t off = ((blk * block + j % block) * Hkv + hk) * hd;
                kp[j] = Kc + off;
                vp[j] = Vc + off;
            }
            if (bad) { err = 2; break; }
            attend_one(q + (i * Hq + hq) * hd, kp, vp, n, hd, o + (i * Hq + hq) * hd, scratch);
        }
        free(scratch);
        free((void *)kp);
    }
    return err == 2 ? ORC_ERR_BLOCK : (err ? ORC_ERR_ARG : ORC_OK);
}

/* Attention of query rows over the paged cache: row r belongs to request req_of_row[r] and sits at position
 * pos_of_row[r]; it attends to the cached positions 0..pos_of_row[r] of that request (its own key included:
 * the caller has written it).  This is the chunked-prefill case (section 3.1: a prompt processed in chunks;
 * a later chunk's queries see the keys of the earlier chunks in the cache).  q: [T][Hq][hd], row stride
 * q_stride; rows/n_rows as in orc_attn_causal; o: [T][Hq*hd]. */
int orc_attn_cached_rows(const float *q, int64_t q_stride, const int32_t *req_of_row, const int32_t *pos_of_row,
                         int64_t T, const float *Kc, const float *Vc, int64_t n_blocks, int64_t block, int64_t Hq,
                         int64_t Hkv, int64_t hd, const int32_t *tables, int64_t max_blk, const int32_t *rows,
                         int64_t n_rows, float *o) {
    if (Hq % Hkv) return ORC_ERR_ARG;
    int64_t G = Hq / Hkv;
    int64_t n_eval = rows ? n_rows : T;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t e = 0; e < n_eval; ++e) {
        int64_t r = rows ? rows[e] : e;
        if (r < 0 || r >= T) { err = 1; continue; }
        int64_t n = (int64_t)pos_of_row[r] + 1;
        const int32_t *tab = tables + (int64_t)req_of_row[r] * max_blk;
        if (n <= 0 || (n + block - 1) / block > max_blk) { err = 1; continue; }
        const float **kp = (const float **)malloc(sizeof(float *) * n * 2);
        const float **vp = kp + n;
        float *scratch = (float *)malloc(sizeof(float) * n);
        for (int64_t hq = 0; hq < Hq; ++hq) {
            int64_t hk = hq / G;
            int bad = 0;
            for (int64_t j = 0; j < n; ++j) {
                int64_t blk = tab[j / block];
                if (blk < 0 || blk >= n_blocks) { bad = 1; break; }
                int64_t off = ((blk * block + j % block) * Hkv + hk) * hd;
                kp[j] = Kc + off;
                vp[j] = Vc + off;
            }
            if (bad) { err = 2; break; }
            attend_one(q + r * q_stride + hq * hd, kp, vp, n, hd, o + r * Hq * hd + hq * hd, scratch);
        }
        free(scratch);
        free((void *)kp);
    }
    return err == 2 ? ORC_ERR_BLOCK : (err ? ORC_ERR_ARG : ORC_OK);
}

/* Weights of one layer, float32, [out][in]; *_t are their [in][out] copies. */
typedef struct {
    int32_t d, hq, hkv, hd, f, block;
    float eps;
    double rope_base;
    const float *g1, *g2;
    const float *wqkv_t; /* [d][(hq+2hkv)*hd] */
    const float *wo_t;   /* [hq*hd][d] */
    const float *wg_t;   /* [d][f] */
    const float *wu_t;   /* [d][f] */
    const float *wd_t;   /* [f][d] */
} orc_layer;

/* Optional taps of intermediate tensors (any may be NULL). */
typedef struct {
    float *h;    /* [M][d]           after first RMSNorm */
    float *qkv;  /* [M][qkv_dim]     after RoPE on q and k */
    float *attn; /* [M][hq*hd]       attention output (evaluated rows only) */
    float *x1;   /* [M][d]           after attention residual (evaluated rows only) */
    float *act;  /* [M][f]           silu(gate)*up (evaluated rows only) */
} orc_taps;

static void ffn_rows(const orc_layer *L, const float *x_rows, const float *attn_rows,
                     int64_t n, float *y_rows, float *x1_tap, float *act_tap) {
    int64_t d = L->d, f = L->f, qd = (int64_t)L->hq * L->hd;
    float *x1 = (float *)malloc(sizeof(float) * n * d);
    float *h2 = (float *)malloc(sizeof(float) * n * d);
    float *gt = (float *)malloc(sizeof(float) * n * f);
    float *up = (float *)malloc(sizeof(float) * n * f);
    orc_linear_t(attn_rows, L->wo_t, n, d, qd, x1);
    for (int64_t i = 0; i < n * d; ++i) x1[i] = x_rows[i] + x1[i];
    orc_rmsnorm(x1, L->g2, n, d, L->eps, h2);
    orc_linear_t(h2, L->wg_t, n, f, d, gt);
    orc_linear_t(h2, L->wu_t, n, f, d, up);
    orc_silu_mul(gt, up, n * f, gt);
    orc_linear_t(gt, L->wd_t, n, d, f, y_rows);
    for (int64_t i = 0; i < n * d; ++i) y_rows[i] = x1[i] + y_rows[i];
    if (x1_tap) memcpy(x1_tap, x1, sizeof(float) * n * d);
    if (act_tap) memcpy(act_tap, gt, sizeof(float) * n * f);
    free(x1); free(h2); free(gt); free(up);
}

/* Prefill of n_req whole prompts (positions start at 0; no chunking, section
 * 4.5.2).  x: [T][d].  K and V of EVERY token are computed and written to the
 * pools; attention and the rest of the layer are evaluated for the rows listed
 * in rows (NULL = all).  y: [n_eval][d] in the order of rows. */
static int prefill_layer_from(const orc_layer *L, const float *x, const int32_t *cu_seqlens, int32_t n_req,
                              const int32_t *start_pos, const int32_t *tables, int64_t max_blk, float *Kc, float *Vc,
                              int64_t n_blocks, const int32_t *rows, int64_t n_rows, float *y, const orc_taps *taps);

int orc_prefill_layer(const orc_layer *L, const float *x, const int32_t *cu_seqlens, int32_t n_req,
                      const int32_t *tables, int64_t max_blk, float *Kc, float *Vc,
                      int64_t n_blocks, const int32_t *rows, int64_t n_rows, float *y,
                      const orc_taps *taps) {
    return prefill_layer_from(L, x, cu_seqlens, n_req, NULL, tables, max_blk, Kc, Vc, n_blocks, rows, n_rows, y, taps);
}

/* One CHUNK of each of n_req prompts (section 3.1, chunked prefill): request r's rows are its tokens at
 * positions start_pos[r] .. start_pos[r] + len_r - 1; the tokens before start_pos[r] are already in the
 * cache (written by earlier chunks).  K/V of the chunk's tokens are appended at their positions, and every
 * evaluated row attends to cached positions 0..its own, read back through the block table. */
int orc_prefill_chunk_layer(const orc_layer *L, const float *x, const int32_t *cu_seqlens, int32_t n_req,
                            const int32_t *start_pos, const int32_t *tables, int64_t max_blk, float *Kc, float *Vc,
                            int64_t n_blocks, const int32_t *rows, int64_t n_rows, float *y, const orc_taps *taps) {
    if (!start_pos) return ORC_ERR_ARG;
    return prefill_layer_from(L, x, cu_seqlens, n_req, start_pos, tables, max_blk, Kc, Vc, n_blocks, rows, n_rows, y, taps);
}

static int prefill_layer_from(const orc_layer *L, const float *x, const int32_t *cu_seqlens, int32_t n_req,
                              const int32_t *start_pos, const int32_t *tables, int64_t max_blk, float *Kc, float *Vc,
                              int64_t n_blocks, const int32_t *rows, int64_t n_rows, float *y, const orc_taps *taps) {
    int64_t d = L->d, hd = L->hd, Hq = L->hq, Hkv = L->hkv;
    int64_t qd = Hq * hd, kvd = Hkv * hd, nqkv = qd + 2 * kvd;
    int64_t T = cu_seqlens[n_req];
    if (hd % 2 || Hq % Hkv || T <= 0) return ORC_ERR_ARG;
    int64_t n_eval = rows ? n_rows : T;
    float *h = (float *)malloc(sizeof(float) * T * d);
    float *qkv = (float *)malloc(sizeof(float) * T * nqkv);
    int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * T);
    int32_t *req = (int32_t *)malloc(sizeof(int32_t) * T);
    for (int32_t r = 0; r < n_req; ++r)
        for (int64_t t = cu_seqlens[r]; t < cu_seqlens[r + 1]; ++t) {
            pos[t] = (int32_t)(t - cu_seqlens[r]) + (start_pos ? start_pos[r] : 0);
            req[t] = r;
        }
    orc_rmsnorm(x, L->g1, T, d, L->eps, h);
    orc_linear_t(h, L->wqkv_t, T, nqkv, d, qkv);
    orc_rope(qkv, pos, T, Hq, hd, L->rope_base, nqkv);
    orc_rope(qkv + qd, pos, T, Hkv, hd, L->rope_base, nqkv);
    int rc = orc_kv_write(Kc, Vc, n_blocks, L->block, Hkv, hd, tables, max_blk, req, pos, T,
                          qkv + qd, qkv + qd + kvd, nqkv);
    float *attn = NULL, *xe = NULL, *ae = NULL;
    if (rc == ORC_OK) {
        attn = (float *)calloc((size_t)T * qd, sizeof(float));
        if (start_pos)   /* keys of earlier chunks live in the cache only: every key is read back from it */
            rc = orc_attn_cached_rows(qkv, nqkv, req, pos, T, Kc, Vc, n_blocks, L->block, Hq, Hkv, hd, tables, max_blk,
                                      rows, n_rows, attn);
        else
            rc = orc_attn_causal(qkv, nqkv, qkv + qd, qkv + qd + kvd, nqkv, cu_seqlens, n_req, Hq, Hkv,
                                 hd, rows, n_rows, attn);
    }
    if (rc == ORC_OK) {
        xe = (float *)malloc(sizeof(float) * n_eval * d);
        ae = (float *)malloc(sizeof(float) * n_eval * qd);
        for (int64_t e = 0; e < n_eval; ++e) {
            int64_t r = rows ? rows[e] : e;
            memcpy(xe + e * d, x + r * d, sizeof(float) * d);
            memcpy(ae + e * qd, attn + r * qd, sizeof(float) * qd);
        }
        float *x1_tap = NULL, *act_tap = NULL;
        if (taps && taps->x1) x1_tap = (float *)malloc(sizeof(float) * n_eval * d);
        if (taps && taps->act) act_tap = (float *)malloc(sizeof(float) * n_eval * L->f);
        ffn_rows(L, xe, ae, n_eval, y, x1_tap, act_tap);
        if (taps) {
            if (taps->h) memcpy(taps->h, h, sizeof(float) * T * d);
            if (taps->qkv) memcpy(taps->qkv, qkv, sizeof(float) * T * nqkv);
            if (taps->attn) memcpy(taps->attn, attn, sizeof(float) * T * qd);
            for (int64_t e = 0; e < n_eval; ++e) {
                int64_t r = rows ? rows[e] : e;
                if (x1_tap) memcpy(taps->x1 + r * d, x1_tap + e * d, sizeof(float) * d);
                if (act_tap) memcpy(taps->act + r * L->f, act_tap + e * L->f, sizeof(float) * L->f);
            }
        }
        free(x1_tap); free(act_tap);
    }
    free(h); free(qkv); free(pos); free(req); free(attn); free(xe); free(ae);
    return rc;
}

/* One decode step: row i is the new token of request i at position ctx_lens[i]
 * (= number of tokens already cached).  Its K/V are appended to the cache and it
 * attends to ctx_lens[i]+1 keys.  x, y: [B][d]. */
int orc_decode_layer(const orc_layer *L, const float *x, const int32_t *ctx_lens,
                     const int32_t *tables, int64_t max_blk, float *Kc, float *Vc,
                     int64_t n_blocks, int64_t B, float *y, const orc_taps *taps) {
    int64_t d = L->d, hd = L->hd, Hq = L->hq, Hkv = L->hkv;
    int64_t qd = Hq * hd, kvd = Hkv * hd, nqkv = qd + 2 * kvd;
    if (hd % 2 || Hq % Hkv || B <= 0) return ORC_ERR_ARG;
    float *h = (float *)malloc(sizeof(float) * B * d);
    float *qkv = (float *)malloc(sizeof(float) * B * nqkv);
    float *q = (float *)malloc(sizeof(float) * B * qd);
    float *attn = (float *)malloc(sizeof(float) * B * qd);
    int32_t *req = (int32_t *)malloc(sizeof(int32_t) * B);
    int32_t *nk = (int32_t *)malloc(sizeof(int32_t) * B);
    for (int64_t i = 0; i < B; ++i) { req[i] = (int32_t)i; nk[i] = ctx_lens[i] + 1; }
    orc_rmsnorm(x, L->g1, B, d, L->eps, h);
    orc_linear_t(h, L->wqkv_t, B, nqkv, d, qkv);
    orc_rope(qkv, ctx_lens, B, Hq, hd, L->rope_base, nqkv);
    orc_rope(qkv + qd, ctx_lens, B, Hkv, hd, L->rope_base, nqkv);
    int rc = orc_kv_write(Kc, Vc, n_blocks, L->block, Hkv, hd, tables, max_blk, req, ctx_lens, B,
                          qkv + qd, qkv + qd + kvd, nqkv);
    if (rc == ORC_OK) {
        for (int64_t i = 0; i < B; ++i) memcpy(q + i * qd, qkv + i * nqkv, sizeof(float) * qd);
        rc = orc_attn_paged(q, Kc, Vc, n_blocks, L->block, Hq, Hkv, hd, tables, max_blk, nk, B,
                            attn);
    }
    if (rc == ORC_OK) {
        ffn_rows(L, x, attn, B, y, taps ? taps->x1 : NULL, taps ? taps->act : NULL);
        if (taps) {
            if (taps->h) memcpy(taps->h, h, sizeof(float) * B * d);
            if (taps->qkv) memcpy(taps->qkv, qkv, sizeof(float) * B * nqkv);
            if (taps->attn) memcpy(taps->attn, attn, sizeof(float) * B * qd);
        }
    }
    free(h); free(qkv); free(q); free(attn); free(req); free(nk);
    return rc;
}

int orc_num_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
