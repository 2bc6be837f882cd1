/*
 * rapid_serve.h -- C ABI of the MI355X (gfx950) prefill/decode co-execution library.
 *
 * One Llama-style decoder layer is evaluated in two ways that share one paged KV
 * cache on one GPU (paper: abstract, sections 2.1, 4.1):
 *   - PREFILL: a whole prompt at once, compute bound, fills the cache;
 *   - DECODE : one new token per running request, bandwidth bound, reads the cache.
 * The two run concurrently, never in one batch, each on its own HIP stream whose
 * hardware queue is confined to a set of compute units by a CU mask (section 4.2).
 * An adaptive resource manager picks the split (section 4.5.3).
 *
 * Conventions
 *   - Every call returns an int32 status: RS_OK (0) or a negative RS_ERR_*.
 *     rs_last_error() gives a thread-local text for the last failure.  Nothing
 *     throws across this boundary.
 *   - "device" pointers are HIP device memory owned by the CALLER (weights, KV pools,
 *     activations, block tables, context lengths).  The library borrows them until
 *     the enqueued work has finished (rs_sync).  "host" pointers are ordinary memory,
 *     read before the call returns.
 *   - The library owns: its CU-masked streams and events, the block free list, the
 *     profile table, the rotary table and two activation workspaces it allocates in
 *     rs_init (one per side, sized from rs_limits).
 *   - Layer calls only ENQUEUE work on the side's current stream and return.
 *   - All matrices are bf16, row major.  Projection weights are [out_features,
 *     in_features].  Accumulation is fp32.  Indices are int32.
 *   - KV pools (bf16), block = 16 tokens:
 *         K pool: [n_layers][n_blocks][n_kv_heads][head_dim/32][4][16][8]
 *         V pool: [n_layers][n_blocks][n_kv_heads][head_dim][16]   (token-minor)
 *     K is stored after the rotary embedding.  Inside one (block, kv head) of the K pool the
 *     element of token slot t and dim d sits at (((d/32)*4 + (d/8)%4)*16 + p(t))*8 + d%8 with
 *     p(t) = t with bits 2 and 3 swapped (slot order 0-3, 8-11, 4-7, 12-15): every MFMA fragment
 *     load of the attention kernels is then one contiguous run of whole 128-byte lines.
 *   - A context created with device = RS_HOST_ONLY touches no GPU: the allocator,
 *     the manager and the request state machine work, layer calls fail with RS_ERR_STATE.
 */
#ifndef RAPID_SERVE_H
#define RAPID_SERVE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RS_OK 0
#define RS_ERR_BAD_ARG (-1)   /* null pointer, size out of range, unsupported shape */
#define RS_ERR_NO_BLOCKS (-2) /* KV pool exhausted; allocator state unchanged */
#define RS_ERR_BAD_SPLIT (-3) /* illegal CU split */
#define RS_ERR_BAD_BLOCK (-4) /* block id outside the pool, or table too short for a context */
#define RS_ERR_HIP (-5)       /* a HIP runtime call failed */
#define RS_ERR_STATE (-6)     /* call not valid in the context's current state */

#define RS_SIDE_PREFILL 0
#define RS_SIDE_DECODE 1

#define RS_TOTAL_CUS 256
#define RS_CU_GRANULE 32        /* splits are multiples of this (4 CUs in each of the 8 XCDs) */
#define RS_KV_BLOCK 16          /* tokens per KV block */
#define RS_MAX_PREFILL_REQS 64  /* prompts per rs_prefill_layer call */
#define RS_HOST_ONLY (-1)

typedef struct rs_ctx rs_ctx;

/* Layer dimensions.  Supported: head_dim 64 or 128; d_model, ffn_dim multiples of 8;
 * n_q_heads a multiple of n_kv_heads with at most 16 query heads per KV head. */
typedef struct {
    int32_t d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, n_layers;
    float rms_eps;    /* inside the square root */
    float rope_base;  /* theta_i = rope_base^(-2i/head_dim), rotate-half pairing (i, i+head_dim/2) */
    int32_t max_pos;  /* rows of the rotary table: positions 0..max_pos-1 are legal */
} rs_model_desc;

/* Caller-allocated KV pools (device).  layer_stride = elements between layers. */
typedef struct {
    void *k_pool, *v_pool;
    int64_t layer_stride;
    int32_t n_blocks;
} rs_pool_desc;

/* Upper bounds that size the two activation workspaces. */
typedef struct {
    int32_t max_prefill_tokens; /* total tokens of one rs_prefill_layer call */
    int32_t max_decode_batch;   /* rows of one rs_decode_layer call */
    int32_t max_context;        /* largest ctx_len + 1 a decode row may attend to */
} rs_limits;

/* Offline profile for the manager (host memory, copied by rs_init; may be NULL = manager
 * always over-allocates).  Section 4.5.3: per decode load, latency of a decode step for each
 * distinct split and under over-allocation, measured while prefill co-runs.
 * lat_distinct_us is [n_batch][n_ctx][n_split], lat_over_us is [n_batch][n_ctx]. */
typedef struct {
    int32_t n_batch, n_ctx, n_split;
    const int32_t *batch_edges; /* ascending decode batch sizes */
    const int32_t *ctx_edges;   /* ascending totals of cached tokens */
    const int32_t *decode_cus;  /* ascending decode CU counts, multiples of RS_CU_GRANULE */
    const int32_t *lat_distinct_us;
    const int32_t *lat_over_us;
    int32_t slo_us;             /* inter-token latency objective (section 5.3: 50 or 100 ms) */
} rs_profile;

/* Device pointers to one layer's bf16 weights. */
typedef struct {
    const void *g1;   /* [d_model]                       first RMSNorm gain */
    const void *wqkv; /* [(Hq+2Hkv)*hd, d_model]         rows: q heads, k heads, v heads */
    const void *wo;   /* [d_model, Hq*hd] */
    const void *g2;   /* [d_model]                       second RMSNorm gain */
    const void *wg;   /* [ffn_dim, d_model]              SwiGLU gate */
    const void *wu;   /* [ffn_dim, d_model]              SwiGLU up */
    const void *wd;   /* [d_model, ffn_dim] */
} rs_layer_weights;

/* ---- life cycle ---------------------------------------------------------------------- */

/* Creates a context on HIP device `device` (or RS_HOST_ONLY).  Allocates workspaces, the
 * rotary table (angles formed in float64 on the host) and the default stream pair for the
 * split (256,256).  pool may have null pointers only for RS_HOST_ONLY.  prof may be NULL. */
int32_t rs_init(const rs_model_desc *model, const rs_pool_desc *pool, const rs_limits *limits,
                const rs_profile *prof, int32_t device, rs_ctx **out);
/* Waits for both sides, frees everything the library owns. */
int32_t rs_destroy(rs_ctx *ctx);
/* Registers (borrows) the weights of one layer, and, on a GPU context, makes the library's own
 * copy of the five matrices in the order its GEMM kernels read them (MFMA fragment order;
 * device memory of about the same size, owned by the context and freed by rs_destroy; allocates
 * and synchronises the device: a set-up call, not a hot-path call).  The caller's matrices must
 * stay valid and unchanged while the context uses the layer; after changing one, call
 * rs_set_weights again.  Errors: RS_ERR_BAD_ARG (null pointer, layer out of range), RS_ERR_HIP. */
int32_t rs_set_weights(rs_ctx *ctx, int32_t layer, const rs_layer_weights *w);
/* Sparse (mixture-of-experts) feed-forward block for `layer`, as in the mixture-of-experts model the
 * paper evaluates next to the dense one (section 5): router logits h W_r^T over n_experts experts,
 * the two largest per row (lower index first on ties), weights = softmax over those two logits,
 * output = x1 + w0 FFN_e0(h) + w1 FFN_e1(h) with each expert a SwiGLU block of the model's ffn_dim.
 * router: device bf16 [n_experts][d_model]; wg, wu: [n_experts][ffn_dim][d_model]; wd:
 * [n_experts][d_model][ffn_dim].  The router stays borrowed; the experts' matrices are packed during
 * the call and may be freed when it returns.  A layer with a sparse block may pass null wg / wu / wd to rs_set_weights; once set,
 * the sparse block replaces the dense one in rs_prefill_layer / rs_decode_layer and everything built
 * on them.  Needs d_model and ffn_dim multiples of 32 and >= 1024, 2 <= n_experts <= 16, top_k = 2
 * (RS_ERR_BAD_ARG otherwise).  Both projections run as grouped GEMMs over 128-row tiles, one expert
 * per tile.  rs_debug_read_moe_routing waits for the side and returns the experts and weights the
 * last layer call on it chose for its first n_rows rows ([n_rows][2] each, host arrays). */
typedef struct {
    const void *router;
    const void *wg;
    const void *wu;
    const void *wd;
    int32_t n_experts;
    int32_t top_k;
} rs_moe_weights;
int32_t rs_set_moe_weights(rs_ctx *ctx, int32_t layer, const rs_moe_weights *w);
int32_t rs_debug_read_moe_routing(rs_ctx *ctx, int32_t side, int32_t n_rows, int32_t *experts_out, float *weights_out);
/* Declares that the five matrices given to rs_set_weights for `layer` will not be read again: the
 * library keeps only its packed copies and the caller may free or reuse that memory (the two gain
 * vectors stay borrowed).  This halves the weight footprint of a large model: a 70B-shaped stack is
 * 137 GB packed.  RS_ERR_STATE if the shape can still reach the generic GEMM kernel, which reads the
 * caller's row-major matrices (some K not a multiple of 32, or some N below 1024); nothing changes
 * then.  Waits for the device to be idle. */
int32_t rs_release_source_weights(rs_ctx *ctx, int32_t layer);
const char *rs_last_error(void);

/* ---- KV cache manager (section 4.5.1; request flow, section 4.4) ------------------------
 * Single owner of the block pool.  rs_kv_alloc makes request req_id own exactly
 * ceil(n_tokens_total/16) blocks, allocating only the missing tail (a request never shrinks),
 * and writes the request's full ordered id list to block_ids_out[0..*n_blocks_out) (host,
 * capacity cap).  The count depends on the length alone, so prompt blocks can be handed to
 * the prefill side before it runs.  On RS_ERR_NO_BLOCKS (or cap too small: RS_ERR_BAD_ARG)
 * nothing changes.  Free list is LIFO: a fresh pool hands out 0,1,2,..; a released
 * request's blocks are reused next, in their original order. */
int32_t rs_kv_alloc(rs_ctx *ctx, int64_t req_id, int32_t n_tokens_total, int32_t *block_ids_out,
                    int32_t cap, int32_t *n_blocks_out);
int32_t rs_kv_free(rs_ctx *ctx, int64_t req_id);
int32_t rs_kv_num_free(rs_ctx *ctx, int32_t *n_free_out);

/* ---- layer passes ---------------------------------------------------------------------- */

/* Un-chunked prefill of n_req whole prompts through layer `layer` (sections 2.1, 4.5.2:
 * a prefill finishes in one step, positions start at 0).  Enqueued on the PREFILL stream.
 *   x_in, x_out  device bf16 [T, d_model], T = cu_seqlens[n_req] (may alias each other)
 *   cu_seqlens   host int32 [n_req+1], ascending from 0; n_req <= RS_MAX_PREFILL_REQS
 *   block_tables device int32 [n_req, max_blk]; row r holds >= ceil(len_r/16) valid ids
 * Writes K/V of every token into the pools through the tables, then causal attention per
 * prompt, output projection + residual, SwiGLU FFN + residual.  A block id outside the pool
 * is never dereferenced: the access is skipped and rs_sync reports RS_ERR_BAD_BLOCK. */
int32_t rs_prefill_layer(rs_ctx *ctx, int32_t layer, const void *x_in, void *x_out,
                         const int32_t *cu_seqlens, int32_t n_req, const int32_t *block_tables,
                         int32_t max_blk);

/* One decode step through layer `layer` for a batch of B running requests (section 2.1).
 * Enqueued on the DECODE stream.
 *   x_in, x_out  device bf16 [B, d_model]
 *   ctx_lens     device int32 [B]: tokens already cached; row i is the token at position
 *                ctx_lens[i], its K/V are appended there and it attends to ctx_lens[i]+1 keys
 *   block_tables device int32 [B, max_blk]; row i holds >= ceil((ctx_lens[i]+1)/16) valid ids
 *   max_ctx      host upper bound of ctx_lens[i]+1 over the batch (sizes the launch)
 * Results do not depend on the CU split nor on what runs on the other side: every reduction
 * shape is a function of the problem shape alone. */
int32_t rs_decode_layer(rs_ctx *ctx, int32_t layer, const void *x_in, void *x_out,
                        const int32_t *ctx_lens, const int32_t *block_tables, int32_t max_blk,
                        int32_t B, int32_t max_ctx);

/* The same decode step, replayed from a captured HIP graph (section 4.5.2: decode steps are
 * captured as graphs per batch size; section 4.5.3: the CU mask a graph was captured under stays
 * with it).  The first call with a given (layer, pointers, max_blk, B, max_ctx_bucket, current
 * decode stream) records rs_decode_layer's kernel sequence on the decode stream and instantiates
 * it (set-up work: allocates); every call launches the instantiated graph on that stream, one
 * runtime call instead of fourteen.  Pointers are part of the graph: the CONTENTS of x_in,
 * ctx_lens and block_tables are read at replay, so a serving loop keeps them in place and updates
 * them between steps.  max_ctx_bucket plays the role of max_ctx but is baked into the launch
 * shape: a multiple of 512 (or the context limit of rs_init) that bounds ctx_lens[i]+1 for as
 * long as the graph is reused, and block_tables rows must be long enough for it
 * (RS_ERR_BAD_BLOCK otherwise).  After rs_set_cu_split the decode stream differs and a new graph
 * is captured under the new mask.  At most 256 graphs are cached per context (RS_ERR_STATE);
 * rs_destroy frees them.  Results are bit-identical to rs_decode_layer's. */
int32_t rs_decode_layer_graph(rs_ctx *ctx, int32_t layer, const void *x_in, void *x_out,
                              const int32_t *ctx_lens, const int32_t *block_tables, int32_t max_blk,
                              int32_t B, int32_t max_ctx_bucket);

/* One layer over a HYBRID BATCH: chunked prefill co-batched with decode, the scheme the paper argues against
 * and measures itself against (section 3.1: a prompt is cut into chunks of 512 or 1024 tokens and each chunk
 * shares a batch, and so a latency, with the running decode tokens; section 5.1: the comparison system).  Built
 * from the same kernels as the two separate passes so that the comparison can be run on this GPU:
 *   rows [0, T) of x_in / x_out (T = cu_seqlens[n_req]) are one chunk of each of n_req prompts: prompt r's rows
 *                sit at positions start_pos[r] .. start_pos[r] + len_r - 1, the positions before start_pos[r] are
 *                already cached (earlier chunks), and each row attends to all cached positions before it and to
 *                the chunk's rows up to itself; start_pos[r] is a multiple of 16 (host array, like cu_seqlens);
 *   rows [T, T+B) are decode rows exactly as in rs_decode_layer (ctx_lens, decode_tables device arrays).
 * All rows go through every projection together (the weights are read once for the whole batch); each kind
 * takes its own attention kernel.  Enqueued on the PREFILL side's stream with that side's workspace: T + B <=
 * max_prefill_tokens, B <= max_decode_batch (B may be 0: a chunk alone).  Errors as for the two passes. */
int32_t rs_hybrid_layer(rs_ctx *ctx, int32_t layer, const void *x_in, void *x_out, const int32_t *cu_seqlens,
                        const int32_t *start_pos, int32_t n_req, const int32_t *prefill_tables,
                        int32_t max_blk_prefill, const int32_t *ctx_lens, const int32_t *decode_tables,
                        int32_t max_blk_decode, int32_t B, int32_t max_ctx);

/* rs_decode_layer for callers that cannot allocate device memory or have it allocated on their behalf:
 * code recorded into a HIP graph, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels and bit-identical results, but every intermediate of the step (normalised rows, q|k|v,
 * attention output and its per-chunk partial results, the GEMMs' K-slice partial sums, the SwiGLU product)
 * lives in a static device array that is part of the library's code object, RS_STATIC_SCRATCH_BYTES =
 * 32 MiB per GPU, held until the process ends; the call allocates nothing and calls nothing that
 * allocates.  A step that needs more (it grows with B, d_model, ffn_dim and max_ctx: the
 * Llama-3-8B-shaped layer at B = 64 and contexts up to 4096 needs 29 MB) is refused with RS_ERR_BAD_ARG and
 * nothing is enqueued; a layer with a sparse feed-forward block is refused with RS_ERR_STATE.  Every
 * context of the process on one GPU shares that GPU's array: calls that overlap on one GPU (two contexts,
 * or a captured graph replayed while another call runs) race on it; calls on one context's decode stream
 * are ordered and safe.  The array keeps the previous call's contents; the call clears what must start
 * at zero with a kernel.  rs_debug_read_workspace does not see these buffers. */
#define RS_STATIC_SCRATCH_BYTES (32u << 20)
int32_t rs_decode_layer_noalloc(rs_ctx *ctx, int32_t layer, const void *x_in, void *x_out,
                                const int32_t *ctx_lens, const int32_t *block_tables, int32_t max_blk,
                                int32_t B, int32_t max_ctx);

/* ---- CU partitioning (sections 4.2, 4.5.3) -------------------------------------------------
 * Selects the masks for SUBSEQUENT enqueues.  Each count is 0 or a multiple of
 * RS_CU_GRANULE up to 256.  prefill+decode <= 256 gives disjoint masks: prefill takes mask
 * bits from 0 upward, decode from 255 downward.  Mask bit b is unit b/8 of XCD b%8, and unit j
 * of an XCD sits in shader engine j%4, so each side keeps the same units in all 8 XCDs and
 * equally many in each of the four shader engines, and a side's masks are nested (a smaller
 * count is a subset of a larger one).  (256,256) is over-allocation: both sides see every
 * CU.  Any other overlapping pair is RS_ERR_BAD_SPLIT.  A side with 0 CUs refuses work
 * (RS_ERR_STATE).  Work already enqueued keeps the mask it was enqueued with; later work of
 * the same side is ordered after it. */
int32_t rs_set_cu_split(rs_ctx *ctx, int32_t prefill_cus, int32_t decode_cus);
int32_t rs_get_cu_split(rs_ctx *ctx, int32_t *prefill_cus, int32_t *decode_cus);
/* The mask words (8 x uint32) a side's stream was created with, for inspection. */
int32_t rs_get_cu_mask(rs_ctx *ctx, int32_t side, uint32_t mask_out[8]);

/* The manager's choice (pure function of its arguments and the profile given to rs_init):
 *   no prefill pending -> (0,256); no decode running -> (256,0); profiled over-allocation
 *   latency meets the objective -> (256,256); else the fewest decode CUs that meet it and the
 *   rest to prefill; if none meets it, the profiled-fastest split.  Loads are rounded up to
 *   the next profiled bucket. */
int32_t rs_choose_split(rs_ctx *ctx, int32_t decode_batch, int64_t sum_ctx, int32_t prefill_pending,
                        int32_t *prefill_cus, int32_t *decode_cus);

/* ---- streams, synchronisation, timing ------------------------------------------------------ */

/* The hipStream_t a side currently enqueues on (valid until the next rs_set_cu_split). */
int32_t rs_get_stream(rs_ctx *ctx, int32_t side, void **hip_stream_out);
/* Blocks until the side's work is done (this side's stream only: it does not wait for the other side).
 * Reports what the side's kernels met since its last rs_sync, then clears it: RS_ERR_BAD_BLOCK for a block
 * id outside the pool, a position outside the rotary table or a context length outside [1, max_ctx];
 * RS_ERR_BAD_ARG for a token outside the vocabulary.  rs_step_tokens and the engine report the same
 * conditions themselves, one step late, when they read a step's tokens. */
int32_t rs_sync(rs_ctx *ctx, int32_t side);
/* Timing with HIP events on the side's own stream: rs_mark records event slot `slot`
 * (0..RS_MAX_MARKS-1) on the side's current stream; rs_elapsed_ms waits for both marks and gives
 * the time from (side_begin, slot_begin) to (side_end, slot_end). */
#define RS_MAX_MARKS 4096
int32_t rs_mark(rs_ctx *ctx, int32_t side, int32_t slot);
/* Non-blocking: *done_out = 1 if the work in front of the mark has completed, else 0.  For a
 * host loop that keeps one side fed while it watches the other.  RS_ERR_STATE if the slot was
 * never recorded. */
int32_t rs_mark_done(rs_ctx *ctx, int32_t side, int32_t slot, int32_t *done_out);
int32_t rs_elapsed_ms(rs_ctx *ctx, int32_t side_begin, int32_t slot_begin, int32_t side_end, int32_t slot_end,
                      float *ms_out);
/* Per-kernel timing of layer calls.  While on, every layer call records an event between its
 * kernels on the side's stream; rs_kernel_times waits for the side's most recent layer call and
 * gives the duration of each step: 0 RMSNorm, 1 QKV GEMM, 2 RoPE + KV write, 3 attention
 * (decode: with the chunk merge), 4 output GEMM + residual, 5 RMSNorm, 6 gate/up GEMM + SwiGLU,
 * 7 down GEMM + residual (decode GEMMs: with their split-K epilogue). */
#define RS_N_KERNEL_SLOTS 8
int32_t rs_set_kernel_timing(rs_ctx *ctx, int32_t on);
int32_t rs_kernel_times(rs_ctx *ctx, int32_t side, float ms_out[RS_N_KERNEL_SLOTS]);

/* Where a side's workgroups really run: launches n_workgroups short workgroups on the side's
 * stream and counts them per physical compute unit.  hist_out (host, RS_CU_HIST_BINS int32) is
 * indexed by (xcc_id << 8) | (se_id << 5) | (sh_id << 4) | cu_id as read from the hardware-id
 * registers.  Blocks until done.  Used to check that a CU mask confines work (section 4.2). */
#define RS_CU_HIST_BINS 4096
int32_t rs_debug_cu_histogram(rs_ctx *ctx, int32_t side, int32_t n_workgroups, int32_t *hist_out);

/* Streaming-read probe: reads n_bytes (multiple of 16, >= 32 KiB) of device memory once with
 * coalesced 16-byte loads on the side's stream, i.e. on the side's CU partition, and gives the
 * GPU time.  n_bytes / time is the read bandwidth that partition can pull (section 3.3's
 * question, asked of this GPU).  Blocks until done. */
int32_t rs_debug_stream_read(rs_ctx *ctx, int32_t side, const void *buf, int64_t n_bytes, float *ms_out);
/* Matrix-core probe: runs about 10 ms of back-to-back 32x32x16 bf16 MFMAs whose operands never leave
 * registers (8 independent accumulator tiles per wave, 8 waves per compute unit) on the side's stream, i.e. on
 * the side's CU partition, and gives the rate in TFLOP/s.  This is what the partition sustains at the clock
 * it reaches under matrix load -- the ceiling a prefill GEMM can be measured against besides the published
 * peak, which assumes the nominal clock.  Blocks until done. */
int32_t rs_debug_mfma_probe(rs_ctx *ctx, int32_t side, float *tflops_out);
/* rs_debug_cu_histogram with the probe kernel replayed from a captured graph on the side's stream:
 * shows whether a graph launch keeps the stream's CU mask. */
int32_t rs_debug_cu_histogram_graph(rs_ctx *ctx, int32_t side, int32_t n_workgroups, int32_t *hist_out);

/* Copies an intermediate activation buffer of a side's last layer call to host memory (after
 * waiting for that side): which = 0 first RMSNorm output [M,d]; 1 q|k|v with rotated q and k
 * [M,(Hq+2Hkv)hd]; 2 attention output [M,Hq*hd]; 3 hidden state after the attention residual
 * [M,d]; 4 silu(gate)*up [M,ffn].  All bf16, row-major whatever the library's internal layout
 * (n_bytes = whole rows, at most the rows of that call).  For stage-by-stage checks. */
int32_t rs_debug_read_workspace(rs_ctx *ctx, int32_t side, int32_t which, void *host_out, int64_t n_bytes);

/* ---- serving step (request flow of section 4.4, FCFS of 4.5.2, manager of 4.5.3) -------------
 * The library keeps the request table: WAITING (no blocks yet) -> PREFILL_READY (prompt
 * blocks allocated, ids available to the prefill side) -> PREFILLING -> PREFILL_DONE (event
 * completed: the "notification") -> RUNNING (in the decode batch) -> FINISHED (blocks freed).
 *
 * rs_submit adds a request in arrival order (req_id >= 0, unique).  prompt_hidden is device bf16
 * [prompt_len, d_model] (hidden states are this path's inputs; rs_submit_tokens / rs_step_tokens
 * below take token ids).  A decode step that cannot get a block for a request's next token fails
 * with RS_ERR_NO_BLOCKS: the library cannot recompute a hidden-state request, so none is preempted.
 *
 * rs_step performs one scheduling step:
 *   1. promotes requests whose prefill event has completed into the decode batch (FCFS,
 *      up to max_decode_batch) and retires requests that produced all their tokens;
 *   2. allocates prompt blocks for waiting requests in arrival order while the pool allows;
 *   3. asks rs_choose_split and applies it;
 *   4. enqueues one decode step over all n_layers for the running batch (growing each
 *      request's blocks as needed), with decode_hidden (device bf16 [>=batch, d_model]) as
 *      the step's input rows;
 *   5. if the prefill side is idle and a request is PREFILL_READY, enqueues its whole prompt
 *      over all n_layers on the prefill side and records its completion event (rs_step_tokens
 *      takes, in arrival order, as many whole prompts as fit max_prefill_tokens, at most
 *      RS_MAX_PREFILL_REQS, into that one pass; a prompt is never split).
 * Never blocks on the GPU except when `wait_decode` is non-zero (then it waits for this
 * step's decode work, which is what a caller measuring inter-token latency wants). */
typedef struct {
    const void *decode_hidden; /* device */
    void *decode_out;          /* device bf16 [>=batch, d_model], last layer's output */
    int32_t wait_decode;
} rs_step_in;

typedef struct {
    int32_t prefill_cus, decode_cus; /* split used for this step */
    int32_t decode_batch;            /* rows in this step's decode batch */
    int64_t decode_sum_ctx;          /* cached tokens over the batch */
    int32_t prefill_started_tokens;  /* tokens of the prompt whose prefill was enqueued, or 0 */
    int64_t prefill_started_req;     /* its id, or -1 */
    int32_t n_promoted;              /* requests that joined the decode batch */
    int32_t n_finished;              /* requests retired in this step */
    int32_t n_waiting;               /* requests still without blocks */
    float decode_ms;                 /* GPU time of this step's decode work if wait_decode, else -1 */
    int32_t n_preempted;             /* rs_step_tokens: running requests sent back to WAITING for want of blocks */
    int32_t prefill_started_count;   /* prompts in the prefill pass that was started (prefill_started_req is the first,
                                        prefill_started_tokens their total) */
    int32_t n_chunks, chunk_tokens;  /* hybrid batching: prompt parts in this step's batch and their tokens in all
                                        (rs_step_chunks names them) */
} rs_step_out;

int32_t rs_submit(rs_ctx *ctx, int64_t req_id, int32_t prompt_len, int32_t output_len,
                  const void *prompt_hidden);
int32_t rs_step(rs_ctx *ctx, const rs_step_in *in, rs_step_out *out);
/* Request ids of the rows of the most recent rs_step's decode batch, in row order (row i of that
 * step's decode_hidden / decode_out belongs to ids_out[i]).  Rows keep their relative order from
 * step to step; finished requests drop out, newly promoted ones are appended in arrival order. */
int32_t rs_decode_batch_ids(rs_ctx *ctx, int64_t *ids_out, int32_t cap, int32_t *n_out);
/* State of a request: 0 WAITING, 1 PREFILL_READY, 2 PREFILLING, 3 PREFILL_DONE, 4 RUNNING,
 * 5 FINISHED; RS_ERR_BAD_ARG if unknown. */
int32_t rs_request_state(rs_ctx *ctx, int64_t req_id);
/* Host-only contexts have no events: this marks a PREFILLING request's event as completed
 * (lets the state machine be exercised without a GPU).  RS_ERR_STATE on a GPU context. */
int32_t rs_debug_complete_prefill(rs_ctx *ctx, int64_t req_id);

/* ---- token boundary: what turns the layer stack into a generator -------------------------------
 * The paper's request starts as a prompt and ends when generation ends (section 4.4); how tokens
 * become hidden states and back is the usual Llama head: x = E[token]; logits = RMSNorm(x_last;
 * g_final) W_lm^T; greedy choice = the lowest index among the maxima of the float32 logits.
 *
 * rs_set_head: embed and lm_head are device bf16 [vocab][d_model], final_norm device bf16
 * [d_model]; all borrowed (must stay valid and unchanged; the library keeps a packed copy of
 * lm_head, so a changed matrix needs another rs_set_head).  eos_token < 0: no end-of-sequence
 * token.  RS_ERR_BAD_ARG for vocab < 1 or a null pointer.
 *
 * rs_embed: x_out[i][:] = E[tokens[i]][:] for n rows, enqueued on `side`'s stream.  tokens is a
 * device pointer.  A token outside [0, vocab) is never dereferenced: its row is zero-filled and the
 * next rs_sync returns RS_ERR_BAD_ARG.
 *
 * rs_lm_head_greedy: for the n rows of x (device bf16 [n][d_model], n <= the side's row limit)
 * computes the logits and the greedy token, enqueued on `side`'s stream.  logits_out (device
 * float32 [n][vocab]) and tokens_out (device int32 [n]) may each be null.  Uses the side's
 * normalised-row workspace: not to be interleaved with a layer call on the same side from another
 * thread. */
typedef struct {
    const void *embed;
    const void *final_norm;
    const void *lm_head;
    int32_t vocab;
    int32_t eos_token;
} rs_head_weights;
int32_t rs_set_head(rs_ctx *ctx, const rs_head_weights *w);
int32_t rs_embed(rs_ctx *ctx, int32_t side, const int32_t *tokens, int32_t n, void *x_out);
int32_t rs_lm_head_greedy(rs_ctx *ctx, int32_t side, const void *x, int32_t n, float *logits_out,
                          int32_t *tokens_out);

/* ---- closed-loop serving: the whole request life cycle (sections 4.4, 4.5.1, 4.5.2) -------------
 * Same state machine, schedulers and manager as rs_submit / rs_step, but requests are token
 * sequences and the loop closes on the device: a prompt's tokens are embedded, run through all
 * layers on the prefill side, and the head's greedy choice on the last prompt row is the request's
 * first output token; every decode step embeds each running request's latest token, runs all
 * layers and chooses the next one.  Needs rs_set_head.  Do not mix with rs_submit / rs_step on one
 * context.
 *
 * rs_submit_tokens: req_id >= 0, unique; prompt_tokens is a HOST array, copied before the call returns.  The request
 * produces at most max_new_tokens tokens and stops early after the end-of-sequence token (which is
 * part of its output).  prompt_len + max_new_tokens must fit max_context and max_pos.
 *
 * rs_step_tokens: one scheduling step, as rs_step, with these additions.
 *   - Sampled tokens reach the host by an asynchronous copy that the NEXT step looks at, so the
 *     end-of-sequence token is noticed one step late unless wait_decode is set: the request then
 *     runs one step too many, whose token is dropped (the scheduling of step n+1 never waits for
 *     the results of step n).  Token counts are known in advance and are never overrun.
 *   - When a running request cannot get the block its next token needs, the most recently
 *     arrived request that holds blocks and is not being prefilled right now (possibly the
 *     starved request itself) is preempted: its blocks are released, it returns to WAITING at
 *     its original place in the arrival order, and its next prefill runs over prompt + tokens
 *     generated so far (recomputation; nothing is swapped out).  n_preempted counts these.
 *     RS_ERR_NO_BLOCKS if the starved request is the only block holder, or if the victim's
 *     sequence no longer fits max_prefill_tokens.
 *   - Blocks released in a step may still be written by a decode step that is in flight; a
 *     prefill started afterwards is ordered behind that step on the device.
 *
 * rs_request_output: the tokens generated so far (host array), *finished_out = 1 once the request
 * has produced its last token and the host has seen it.
 *
 * rs_debug_push_sampled: host-only contexts have no sampler; this queues the token that the
 * request's next sampling event (its prefill, then each decode step) will yield.  Without a queued
 * token the event yields token 0.  RS_ERR_STATE on a GPU context. */
int32_t rs_submit_tokens(rs_ctx *ctx, int64_t req_id, const int32_t *prompt_tokens, int32_t prompt_len,
                         int32_t max_new_tokens);
int32_t rs_step_tokens(rs_ctx *ctx, int32_t wait_decode, rs_step_out *out);

/* The batching scheme of rs_step_tokens.  chunk_tokens = 0 (the default): the paper's own scheme, whole prompts
 * on the prefill side concurrently with decode steps on the decode side (sections 4.1, 4.5.2).  chunk_tokens > 0
 * (a multiple of 16): HYBRID BATCHING, the scheme the paper compares with (section 3.1; its comparison system in
 * section 5.1 runs chunks of 512 and 1024 tokens).  chunk_tokens is a step's budget of prompt tokens: it is filled
 * in arrival order -- the rest of the prompt in progress, then the next prompts that have their blocks, the last
 * of them possibly in part (a part that does not end its prompt is a multiple of 16 tokens; at most
 * RS_MAX_PREFILL_REQS parts per step) -- and these parts form one batch with the decode rows of all running
 * requests (rs_hybrid_layer over all layers, all CUs, one stream).  The step that takes a prompt's last part
 * yields its first token; a step without a part is an ordinary decode step.  Block accounting, promotion,
 * retirement and preemption are unchanged, and so are the tokens every request receives.  Only while no request
 * is in flight and the engine threads are not running; needs chunk_tokens + max_decode_batch <=
 * max_prefill_tokens (RS_ERR_BAD_ARG otherwise). */
int32_t rs_set_hybrid_batching(rs_ctx *ctx, int32_t chunk_tokens);
/* The prompt parts of the latest rs_step_tokens call under hybrid batching, batch order: request, first position,
 * length (host arrays of `cap` entries, any may be null); *n_out = their number (RS_ERR_BAD_ARG if cap is less). */
int32_t rs_step_chunks(rs_ctx *ctx, int64_t *req_ids_out, int32_t *starts_out, int32_t *lens_out, int32_t cap,
                       int32_t *n_out);
int32_t rs_request_output(rs_ctx *ctx, int64_t req_id, int32_t *tokens_out, int32_t cap, int32_t *n_out,
                          int32_t *finished_out);
/* rs_step_tokens and the engine's decode thread launch every decode step as ONE captured HIP graph (section
 * 4.5.2: decode steps are captured as graphs and replayed; section 4.5.3: a graph keeps the CU mask it was
 * captured under): embedding, every layer and the head are recorded once per (decode batch size, context bound
 * rounded up to 512 tokens, masked decode stream) and replayed with one runtime call; tokens, context lengths
 * and block tables are read from library buffers that are refreshed before every launch.  The first step of a
 * new key records and instantiates (set-up work: allocates inside the runtime); at most 512 graphs are kept.
 * Results are bit-identical to the uncaptured step.  rs_set_step_graphs(ctx, 0) turns this off (the step's
 * kernels are then launched one by one), 1 turns it on, a value n > 1 turns it on and keeps at most n graphs
 * (when a new key arrives at the limit the library waits for the streams the cached graphs were recorded on and
 * drops them all); not while the engine runs (RS_ERR_STATE).
 * rs_step_graph_stats: stats_out[0] graphs captured so far, [1] steps launched as a graph, [2] decode steps
 * enqueued by the serving loop outside of a capture, [3] host nanoseconds those steps' launches took in total
 * (one graph launch, or the step's kernel launches one by one). */
int32_t rs_set_step_graphs(rs_ctx *ctx, int32_t on);
int32_t rs_step_graph_stats(rs_ctx *ctx, int64_t stats_out[4]);
/* Host-clock times in seconds since the context was created: [0] submission, [1] the moment the
 * host saw the request's first token, [2] its latest token (0 while there is none). */
int32_t rs_request_times(rs_ctx *ctx, int64_t req_id, double times_out[3]);
/* Forgets a FINISHED request (rs_submit or rs_submit_tokens) whose output has been read: its record
 * (tokens, times, state) is dropped and the id may be used again; a serving loop that runs for long calls
 * this for every request it has collected, or the table grows with every request.  RS_ERR_STATE while
 * the request is not finished (engine: until its end flag is set), RS_ERR_BAD_ARG if unknown. */
int32_t rs_request_release(rs_ctx *ctx, int64_t req_id);
int32_t rs_debug_push_sampled(rs_ctx *ctx, int64_t req_id, int32_t token);

/* ---- engine: the two asynchronous sides of section 4.4 as two threads ---------------------------
 * rs_engine_start spawns a decode thread and a prefill thread inside the library and returns.
 *   decode thread : owns the request table, the only KV allocator (section 4.5.1), the manager and
 *                   the decode partition; runs the rs_step_tokens loop without ever waiting for a
 *                   prefill;
 *   prefill thread: owns the prefill partition; takes requests whose blocks are allocated, first
 *                   come first served, runs each whole prompt and waits for it (only this thread
 *                   blocks on prefill work), then sends the notification.
 * The threads share no lock: three bounded single-producer / single-consumer rings carry
 * submissions (application -> decode), block ids (decode -> prefill) and notifications
 * (prefill -> decode); the CU count of the prefill partition is published by the manager and picked
 * up by the prefill thread at its next prompt (work in flight keeps the mask it started with).
 * Several prompts may be queued on the prefill thread at once.
 *
 * While the engine runs: rs_submit_tokens (any application thread), rs_request_output,
 * rs_request_times, rs_request_state and rs_engine_stats are the calls to use; rs_step,
 * rs_step_tokens and the layer calls are refused or must not be made, and the allocator and
 * split calls (rs_kv_alloc, rs_kv_free, rs_kv_num_free, rs_set_cu_split, rs_sync, ...) read or
 * change state the engine's threads own: call them only while it is stopped.  Results are published by
 * the decode thread with release stores and read here with acquire loads: a reader never sees a
 * token count ahead of the tokens.  Host-only contexts: queue a request's sampled tokens with
 * rs_debug_push_sampled BEFORE submitting it.
 *
 * rs_engine_stop(drain != 0) returns after every submitted request has finished; with drain == 0
 * it stops after the step in progress (unfinished requests stay unfinished and the context can then
 * only be inspected and destroyed).  It reports the first error an engine thread met, as does
 * rs_engine_stats.  stats_out: [0] submitted, [1] finished, [2] decode-thread iterations,
 * [3] preemptions. */
int32_t rs_engine_start(rs_ctx *ctx);
int32_t rs_engine_stop(rs_ctx *ctx, int32_t drain);
int32_t rs_engine_stats(rs_ctx *ctx, int64_t stats_out[4]);

#ifdef __cplusplus
}
#endif
#endif /* RAPID_SERVE_H */
