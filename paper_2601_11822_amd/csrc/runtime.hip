// Host runtime behind the C ABI: context, KV block allocator, CU-masked stream pool, adaptive
// resource manager, layer drivers and the serving step.  Declarations and their contract are
// in include/rapid_serve.h.
#include <algorithm>
#include <atomic>
#include <memory>
#include <mutex>
#include <thread>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <chrono>
#include <deque>
#include <map>
#include <string>
#include <unordered_map>
#include <tuple>
#include <vector>

#include "../../include/rapid_serve.h"
#include "kernels.h"

namespace {

thread_local std::string g_err;

int32_t fail(int32_t code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

#define HIP_TRY(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) return fail(RS_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// Scratch of rs_decode_layer_noalloc: one array per GPU, part of the library's code object, so a
// call needs no allocation at all.  Host code never uses this name as an address: g_static_scratch[]
// holds each device's own address of it (hipGetSymbolAddress in rs_init, with that device current).
#define RS_MAX_DEVICES 64
static __device__ __align__(256) unsigned char scratch[RS_STATIC_SCRATCH_BYTES];
void *g_static_scratch[RS_MAX_DEVICES] = {};
std::mutex g_static_scratch_mu;

struct Workspace {
    bf16_t *h = nullptr, *qkv = nullptr, *attn = nullptr, *x1 = nullptr, *act = nullptr, *xbuf = nullptr;
    float *partials = nullptr, *part_o = nullptr, *part_ml = nullptr;
    float *ssq = nullptr;   // decode side: per-slice sums of squares of the two normalised inputs, 2 x [64 slices][64 rows]
    size_t partial_cap = 0;
    int rows = 0;
    // sparse feed-forward block (allocated by the first rs_set_moe_weights)
    int32_t *m_sel = nullptr, *m_pos = nullptr, *m_src = nullptr, *m_tile = nullptr;
    float *m_wt = nullptr;
    bf16_t *m_a = nullptr, *m_act = nullptr, *m_out = nullptr;
    int m_cap = 0;   // grouped row capacity (a multiple of 128)
};

constexpr int RS_HEAD_GROUP = 256;

enum ReqState { WAITING = 0, PREFILL_READY, PREFILLING, PREFILL_DONE, RUNNING, FINISHED };

// Bounded single-producer / single-consumer ring: the only coupling between the engine's threads
// (section 4.4: the two sides exchange requests and notifications, never locks).
template <class T, size_t N>
struct SpscRing {
    std::atomic<size_t> head{0}, tail{0};   // head: next slot to pop (consumer's), tail: next to fill (producer's)
    T buf[N];
    bool push(const T &v) {
        const size_t t = tail.load(std::memory_order_relaxed);
        if (t - head.load(std::memory_order_acquire) == N) return false;
        buf[t % N] = v;
        tail.store(t + 1, std::memory_order_release);
        return true;
    }
    bool pop(T &v) {
        const size_t h = head.load(std::memory_order_relaxed);
        if (h == tail.load(std::memory_order_acquire)) return false;
        v = buf[h % N];
        head.store(h + 1, std::memory_order_release);
        return true;
    }
    // consumer only: the element pop would return, without taking it
    const T *front() const {
        const size_t h = head.load(std::memory_order_relaxed);
        return h == tail.load(std::memory_order_acquire) ? nullptr : &buf[h % N];
    }
    bool empty() const { return head.load(std::memory_order_acquire) == tail.load(std::memory_order_acquire); }
};

// What the application reads of an engine request: written by the decode thread only, every field
// published with release stores (tokens first, then their count).
struct Result {
    int32_t max_new = 0;
    std::unique_ptr<int32_t[]> toks;
    std::atomic<int32_t> n{0}, finished{0}, state{WAITING};
    std::atomic<double> t_submit{0}, t_first{0}, t_last{0};
};
struct SubmitMsg {          // application -> decode thread ("waiting" queue)
    int64_t id;
    int32_t prompt_len, max_new;
    std::vector<int32_t> *toks, *script;   // owned by the message
    Result *res;
    double t_submit;
};
struct PrefillMsg {         // decode thread -> prefill thread: blocks are allocated, here are their ids
    int64_t id;
    int32_t slot, n_tok, wait_idx;
    std::vector<int32_t> *blocks;          // owned by the message
};
struct DoneMsg {            // prefill thread -> decode thread: the notification (no KV moves)
    int64_t id;
    int32_t token, rc;
};

struct Request {
    int64_t id;
    int32_t prompt_len, output_len;
    const void *prompt_hidden;
    int state = WAITING;
    int32_t ctx_len = 0;    // tokens cached so far
    int32_t generated = 0;  // decode steps taken
    hipEvent_t done = nullptr;
    bool host_done = false;
    // closed-loop (token) requests
    bool token_mode = false;
    int slot = -1;                 // index of the request's current-token cell and prompt region on the device
    std::vector<int32_t> toks;     // prompt, then every generated token the host has seen
    int32_t n_prefill = 0;         // tokens the next prefill covers (prompt, plus generated ones after a preemption)
    int32_t n_sampled = 0;         // sampling events enqueued so far (known without looking at any token)
    bool complete = false;         // last token seen (end-of-sequence or the token limit)
    int32_t chunk_done = 0;        // hybrid batching: tokens of the prefill in progress that earlier steps took
    std::deque<int32_t> injected;  // host-only contexts: tokens the next sampling events will yield
    double t_submit = 0, t_first = 0, t_last = 0;   // host clock: submission, first and latest token seen
    Result *res = nullptr;         // engine requests: where the application looks
};

struct Side {
    int cus = RS_TOTAL_CUS;
    hipStream_t stream = nullptr;
    std::map<int, hipStream_t> pool;  // by CU count
    std::vector<hipEvent_t> marks;
    hipEvent_t order = nullptr;
    hipEvent_t kt[RS_N_KERNEL_SLOTS + 1] = {};  // boundaries of the last layer call's kernels
    bool kt_valid = false;
};

}  // namespace

struct rs_ctx {
    rs_model_desc m{};
    rs_pool_desc pool{};
    rs_limits lim{};
    int device = RS_HOST_ONLY;
    bool gpu = false;
    std::vector<rs_layer_weights> weights;
    std::vector<bool> have_weights;
    // fragment-packed private copies of the five matrices, read by the direct and the skinny GEMMs
    struct PackedLayer { bf16_t *wqkv = nullptr, *wo = nullptr, *wg = nullptr, *wu = nullptr, *wd = nullptr; };
    std::vector<PackedLayer> packed;
    // sparse feed-forward block of a layer: the experts' matrices packed back to back (stride elements apart)
    struct MoeLayer { int E = 0; const bf16_t *router = nullptr; bf16_t *wg = nullptr, *wu = nullptr, *wd = nullptr;
                      size_t stride_gu = 0, stride_d = 0; };
    std::vector<MoeLayer> moe;
    CosSin *rope = nullptr;
    // One error word per side (kernels OR bits into it: 1 position outside the rotary table, 2 block id outside
    // the pool, 4 token outside the vocabulary, 8 context length outside [1, max_ctx]) and its pinned host
    // mirrors: h_err[side] is what rs_sync reads, h_err[2 + i] travels with decode step buffer i, h_err[4]
    // with a prefill pass of the serving loop.  Every copy and clear runs on the side's own stream: a
    // blocking copy on the null stream would make one side wait for the other.
    int32_t *err_flag = nullptr;
    int32_t *h_err = nullptr;
    int32_t step_err = 0;            // bits met by serving steps and not yet reported
    Workspace ws[2];
    int last_rows[2] = {0, 0};   // rows of each side's last layer call: fixes the packed layout of h/attn/act
    bool decode_fused = false;   // the decode side's last layer call folded its RMSNorms into the projections (no h buffer)
    // captured decode steps, keyed by everything a captured launch bakes in (rs_decode_layer_graph)
    struct GraphKey {
        int32_t layer, max_blk, B, max_ctx;
        const void *x_in, *x_out, *ctx_lens, *tables;
        hipStream_t stream;
        bool operator<(const GraphKey &o) const {
            return std::tie(layer, max_blk, B, max_ctx, x_in, x_out, ctx_lens, tables, stream) <
                   std::tie(o.layer, o.max_blk, o.B, o.max_ctx, o.x_in, o.x_out, o.ctx_lens, o.tables, o.stream);
        }
    };
    std::map<GraphKey, hipGraphExec_t> graphs;
    // whole decode steps of the closed-loop server (embedding, every layer, head), captured per (batch, context
    // bucket, masked decode stream); every pointer in them is a library buffer
    std::map<std::tuple<int32_t, int32_t, hipStream_t>, hipGraphExec_t> step_graphs;
    bool step_graphs_on = true;
    int step_graph_cap = 512;   // captured steps kept; when a new key arrives at the cap all are dropped
    int64_t step_graph_captures = 0, step_graph_launches = 0;
    int64_t steps_enqueued = 0, step_enqueue_ns = 0;   // decode steps of the serving loop and the host time their launches took
    bool capturing = false;      // a decode step is being recorded: no event records on the stream
    // Held while a step is being recorded, and by the prefill thread around its wait on an event of the decode
    // stream: the runtime takes a wait on an event whose stream is recording at that moment for a dependency inside the
    // recording and draws the waiting stream into it (seen once in some ten engine runs: the prefill stream's next
    // wait then failed with "dependency created on uncaptured work in another stream").
    std::mutex capture_mu;
    std::vector<int64_t> last_batch;   // request ids of the rows of the most recent rs_step's decode batch
    Side side[2];
    bool over_alloc = true;
    bool new_stream = false;     // a masked stream was created since the pair was last warmed (set_split)
    bool kernel_timing = false;

    // allocator
    std::vector<int32_t> free_list;
    std::unordered_map<int64_t, std::vector<int32_t>> owned;

    // manager profile
    bool have_prof = false;
    std::vector<int32_t> batch_edges, ctx_edges, decode_cus, lat_distinct, lat_over;
    int32_t slo_us = 0;

    // serving state
    std::deque<int64_t> arrival;  // FCFS order of all live requests
    std::unordered_map<int64_t, Request> reqs;
    std::vector<int64_t> running;  // decode batch, in promotion order
    std::vector<int64_t> dead;     // engine: finished requests whose table entry goes once no staged step names them
    std::vector<int64_t> prefill_ids;   // the prompts of the prefill pass in flight (one pass at a time)
    bool prefill_host_done = false;     // host-only contexts: rs_debug_complete_prefill
    // hybrid batching (the comparison scheme of section 3.1): chunk size in tokens, 0 = off; whether the last chunk
    // of the prompt in prefill_ids has been enqueued; the stream the previous step ran on
    int32_t hybrid_chunk = 0;
    int64_t hyb_cur = -1;                 // the prompt of which a part, not yet the last, has been taken
    hipStream_t hyb_prev_stream = nullptr;
    struct HybPart { int64_t id; int32_t start, n; };
    std::vector<HybPart> last_parts;      // the prompt parts of the latest step (rs_step_chunks)
    int inflight_nb[2] = {0, 0};          // of inflight[f], the first so many are decode rows; the rest are prompts
                                          // whose last part rode in that step (their first tokens)
    hipEvent_t prefill_ev = nullptr;    // end of that pass
    int32_t max_blk_per_req = 0;
    int32_t *d_ctx = nullptr, *d_tab = nullptr, *d_ptab = nullptr;   // device staging
    int32_t *h_ctx[2] = {nullptr, nullptr}, *h_tab[2] = {nullptr, nullptr}, *h_ptab = nullptr;
    hipEvent_t staged[2] = {nullptr, nullptr};
    hipEvent_t pstaged = nullptr;
    int stage_flip = 0;
    // a decode step's end, alternating: a prefill that may reuse just-released blocks waits for the step
    // enqueued before the release
    hipEvent_t step_end[2] = {nullptr, nullptr};
    int step_end_idx = 0;
    bool step_end_valid[2] = {false, false};

    std::chrono::steady_clock::time_point t0 = std::chrono::steady_clock::now();
    double now() const { return std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count(); }

    // token boundary
    rs_head_weights head{};
    bool have_head = false;
    bf16_t *packed_lm = nullptr;
    float *head_part[2] = {nullptr, nullptr};
    int head_group[2] = {64, 64};     // rows per pass of the LM head over its weights
    // closed-loop serving
    int serving_mode = 0;            // 0 none yet, 1 hidden-state requests, 2 token requests
    int n_slots = 0;
    std::vector<int> free_slots;
    int32_t *d_tok = nullptr;        // [n_slots] latest token of each live request
    int32_t *d_prompts = nullptr;    // [n_slots][max_context] token sequences to prefill
    int32_t *h_first = nullptr;      // pinned [n_slots]: the token a prefill chose
    hipStream_t copy_stream = nullptr;   // non-blocking: token uploads must not wait for the partitions' work
    int32_t *d_pslots = nullptr, *h_pslots = nullptr;   // request slots of the prompts of a prefill pass
    int32_t *d_pfirst = nullptr, *h_pfirst = nullptr;   // the tokens that pass chose, prompt order
    int32_t *d_rowslot = nullptr, *h_rowslot[2] = {nullptr, nullptr};
    int32_t *d_sampled = nullptr, *h_sampled[2] = {nullptr, nullptr};
    hipEvent_t sampled_ev[2] = {nullptr, nullptr};
    std::vector<int64_t> inflight[2];   // request ids of the rows of a step whose tokens the host has not read yet
    bool pending[2] = {false, false};

    // engine: a decode thread (owns the request table, the allocator and the decode side) and a prefill
    // thread (owns the prefill side), coupled by three rings
    bool engine = false;                 // threads running; set and cleared by the application thread
    bool engine_ever = false;
    std::thread th_decode, th_prefill;
    std::atomic<bool> stop{false}, stop_prefill{false}, drain{false};
    SpscRing<SubmitMsg, 4096> sub_q;     // producer side serialised by sub_mu (several application threads)
    SpscRing<PrefillMsg, 4096> pre_q;
    SpscRing<DoneMsg, 4096> fin_q;
    std::mutex sub_mu, res_mu;
    std::unordered_map<int64_t, std::unique_ptr<Result>> results;            // under res_mu
    std::unordered_map<int64_t, std::vector<int32_t>> pre_scripts;           // under res_mu
    std::string eng_err;                                                     // under res_mu
    std::atomic<int32_t> prefill_cus_pub{RS_TOTAL_CUS}, eng_rc{0};
    std::atomic<int64_t> eng_steps{0}, eng_finished{0}, eng_preempted{0}, eng_submitted{0};
    int n_prefill_inflight = 0;          // decode thread only
};

namespace {

// Mask bit b is compute unit j = b/8 of XCD b%8, and inside an XCD unit j sits in shader engine j%4 (both read
// back from the hardware-id registers by rs_debug_cu_histogram).  Prefill takes the bits [0, p) and decode the bits
// [256 - d, 256).  That gives each side the same units in every XCD and the same number of units in each of the four
// shader engines (workgroups are dealt to the engines in turn whatever the number of enabled units behind each: an
// uneven share measured 2x slower), and it makes the masks of a side NESTED: a smaller count is a subset of a larger
// one.  Nesting is what keeps a change of split harmless while a prefill pass is still running under the previous
// mask: a decode side that shrinks never lands on units the old pass still occupies.
// Measured and dropped: whole shader engines per side where the counts allow (multiples of 64).  At a fixed split it
// is better for decode (128/128: step 2.6 % faster alone, 1.9 % beside prefill; 192/64: 6 %) at 0.8-2.3 % of the
// prefill rate, but no order of the units is both nested and balanced at the other multiples of 32, and with two
// layouts a move from 128/128 to 160/96 put half of decode's units under the prefill pass still in flight: decode
// steps of 40 ms instead of 10 for the length of that pass, every time the manager moved the split under load.
void mask_for(int side, int cus, uint32_t out[8]) {
    for (int i = 0; i < 8; ++i) out[i] = 0;
    const int lo = side == RS_SIDE_PREFILL ? 0 : RS_TOTAL_CUS - cus;
    for (int b = lo; b < lo + cus; ++b) out[b >> 5] |= 1u << (b & 31);
}

int32_t get_stream(rs_ctx *c, int side, int cus, hipStream_t *out) {
    Side &s = c->side[side];
    auto it = s.pool.find(cus);
    if (it != s.pool.end()) {
        *out = it->second;
        return RS_OK;
    }
    uint32_t mask[8];
    mask_for(side, cus, mask);
    hipStream_t st;
    HIP_TRY(hipExtStreamCreateWithCUMask(&st, 8, mask));
    s.pool[cus] = st;
    c->new_stream = true;
    *out = st;
    return RS_OK;
}

// Whether a decode step of at most 64 rows takes the weight-streaming projections with the RMSNorm folded in
// (a function of the model's shape), and the partial-product elements they need.
bool fused_decode_applies(const rs_ctx *c) {
    const rs_model_desc &m = c->m;
    const int d = m.d_model, qd = m.n_q_heads * m.head_dim, nqkv = qd + 2 * m.n_kv_heads * m.head_dim, f = m.ffn_dim;
    return dgemm_applies(nqkv, d) && dgemm_applies(d, qd) && dgemm_applies(f, d);
}
size_t fused_partial_elems(const rs_ctx *c, int M) {
    if (!fused_decode_applies(c)) return 0;
    const rs_model_desc &m = c->m;
    const int d = m.d_model, qd = m.n_q_heads * m.head_dim, nqkv = qd + 2 * m.n_kv_heads * m.head_dim, f = m.ffn_dim;
    size_t pe = std::max(dgemm_partial_elems(M, nqkv, d, false), dgemm_partial_elems(M, d, qd, false));
    pe = std::max(pe, dgemm_partial_elems(M, f, d, true));
    if (dgemm_applies(d, f)) pe = std::max(pe, dgemm_partial_elems(M, d, f, false));
    return pe;
}

int32_t alloc_ws(rs_ctx *c, Workspace &w, int rows, bool decode) {
    const rs_model_desc &m = c->m;
    const size_t d = m.d_model, qd = (size_t)m.n_q_heads * m.head_dim;
    const size_t nqkv = qd + 2 * (size_t)m.n_kv_heads * m.head_dim, f = m.ffn_dim;
    w.rows = rows;
    if (rows <= 0) return RS_OK;
    // GEMM inputs are kept fragment-packed: whole 32-row tiles x (width rounded to a k block of 16);
    // zeroed once, so that the padding never holds a NaN pattern (producers write valid elements only)
    const size_t prow = (size_t)packed_mt(rows) * 32;
    auto r16 = [&](size_t v) { return (v + 15) / 16 * 16; };
    HIP_TRY(hipMalloc(&w.h, prow * r16(d) * 2));
    HIP_TRY(hipMemset(w.h, 0, prow * r16(d) * 2));
    HIP_TRY(hipMalloc(&w.qkv, rows * nqkv * 2));
    HIP_TRY(hipMalloc(&w.attn, prow * r16(qd) * 2));
    HIP_TRY(hipMemset(w.attn, 0, prow * r16(qd) * 2));
    HIP_TRY(hipMalloc(&w.x1, rows * d * 2));
    HIP_TRY(hipMalloc(&w.act, prow * r16(f) * 2));
    HIP_TRY(hipMemset(w.act, 0, prow * r16(f) * 2));
    HIP_TRY(hipMalloc(&w.xbuf, rows * d * 2));
    {
        const int Mmax = std::min(rows, 64);
        size_t pe = rows > 64 ? RS_DIRECT_PARTIAL_ELEMS : 0;   // more than 64 rows: also the K-sliced path of the large-tile GEMM
        pe = std::max(pe, skinny_partial_elems(Mmax, (int)nqkv, (int)d, EPI_STORE));
        pe = std::max(pe, skinny_partial_elems(Mmax, (int)d, (int)qd, EPI_RESIDUAL));
        pe = std::max(pe, skinny_partial_elems(Mmax, (int)f, (int)d, EPI_SWIGLU));
        pe = std::max(pe, skinny_partial_elems(Mmax, (int)d, (int)f, EPI_RESIDUAL));
        if (decode) pe = std::max(pe, fused_partial_elems(c, Mmax));
        HIP_TRY(hipMalloc(&w.partials, pe * sizeof(float)));
        w.partial_cap = pe;
    }
    if (!decode && c->lim.max_decode_batch > 0) {
        // a hybrid batch (rs_hybrid_layer) runs decode rows through the prefill side's workspace
        const size_t nch = (c->lim.max_context + RS_DECODE_CHUNK - 1) / RS_DECODE_CHUNK;
        const size_t br = std::min(rows, c->lim.max_decode_batch);
        HIP_TRY(hipMalloc(&w.part_o, br * m.n_q_heads * nch * m.head_dim * sizeof(float)));
        HIP_TRY(hipMalloc(&w.part_ml, br * m.n_q_heads * nch * 2 * sizeof(float)));
    }
    if (decode) {
        HIP_TRY(hipMalloc(&w.ssq, 2 * 64 * 64 * sizeof(float)));
        const size_t nch = (c->lim.max_context + RS_DECODE_CHUNK - 1) / RS_DECODE_CHUNK;
        HIP_TRY(hipMalloc(&w.part_o, (size_t)rows * m.n_q_heads * nch * m.head_dim * sizeof(float)));
        HIP_TRY(hipMalloc(&w.part_ml, (size_t)rows * m.n_q_heads * nch * 2 * sizeof(float)));
    }
    return RS_OK;
}

// The decode side's buffers for a step of `rows` rows and contexts up to max_ctx, laid out one after the other
// (256-byte aligned) from `base`; returns the bytes used.  base == nullptr only measures.  The three
// fragment-packed GEMM inputs come first, contiguous: *packed_bytes is their extent (what must start at zero).
size_t carve_decode_ws(const rs_ctx *c, Workspace &w, unsigned char *base, int rows, int max_ctx, size_t *packed_bytes) {
    const rs_model_desc &m = c->m;
    const size_t d = m.d_model, qd = (size_t)m.n_q_heads * m.head_dim;
    const size_t nqkv = qd + 2 * (size_t)m.n_kv_heads * m.head_dim, f = m.ffn_dim;
    const size_t prow = (size_t)packed_mt(rows) * 32;
    auto r16 = [](size_t v) { return (v + 15) / 16 * 16; };
    size_t off = 0;
    auto take = [&](size_t bytes) {
        unsigned char *p = base ? base + off : nullptr;
        off += (bytes + 255) / 256 * 256;
        return p;
    };
    w = Workspace{};
    w.rows = rows;
    w.h = (bf16_t *)take(prow * r16(d) * 2);
    w.attn = (bf16_t *)take(prow * r16(qd) * 2);
    w.act = (bf16_t *)take(prow * r16(f) * 2);
    if (packed_bytes) *packed_bytes = off;
    w.qkv = (bf16_t *)take(rows * nqkv * 2);
    w.x1 = (bf16_t *)take(rows * d * 2);
    const int Mmax = std::min(rows, 64);
    size_t pe = rows > 64 ? RS_DIRECT_PARTIAL_ELEMS : 0;
    pe = std::max(pe, skinny_partial_elems(Mmax, (int)nqkv, (int)d, EPI_STORE));
    pe = std::max(pe, skinny_partial_elems(Mmax, (int)d, (int)qd, EPI_RESIDUAL));
    pe = std::max(pe, skinny_partial_elems(Mmax, (int)f, (int)d, EPI_SWIGLU));
    pe = std::max(pe, skinny_partial_elems(Mmax, (int)d, (int)f, EPI_RESIDUAL));
    pe = std::max(pe, fused_partial_elems(c, Mmax));
    w.ssq = (float *)take(2 * 64 * 64 * sizeof(float));
    w.partials = (float *)take(pe * sizeof(float));
    w.partial_cap = pe;
    const size_t nch = (max_ctx + RS_DECODE_CHUNK - 1) / RS_DECODE_CHUNK;
    w.part_o = (float *)take((size_t)rows * m.n_q_heads * nch * m.head_dim * sizeof(float));
    w.part_ml = (float *)take((size_t)rows * m.n_q_heads * nch * 2 * sizeof(float));
    return off;
}

void free_ws(Workspace &w) {
    void *ptrs[] = {w.h, w.qkv, w.attn, w.x1, w.act, w.xbuf, w.partials, w.part_o, w.part_ml, w.ssq,
                    w.m_sel, w.m_pos, w.m_src, w.m_tile, w.m_wt, w.m_a, w.m_act, w.m_out};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    w = Workspace{};
}

int bucket(const std::vector<int32_t> &edges, int64_t v) {
    for (size_t i = 0; i < edges.size(); ++i)
        if (v <= edges[i]) return (int)i;
    return (int)edges.size() - 1;
}

void choose_split(const rs_ctx *c, int32_t batch, int64_t sum_ctx, bool prefill_pending, int32_t *p,
                  int32_t *d) {
    if (!prefill_pending) { *p = 0; *d = RS_TOTAL_CUS; return; }
    if (batch <= 0) { *p = RS_TOTAL_CUS; *d = 0; return; }
    if (!c->have_prof) { *p = RS_TOTAL_CUS; *d = RS_TOTAL_CUS; return; }
    const int b = bucket(c->batch_edges, batch), x = bucket(c->ctx_edges, sum_ctx);
    const int nc = (int)c->ctx_edges.size(), ns = (int)c->decode_cus.size();
    if (c->lat_over[b * nc + x] <= c->slo_us) { *p = RS_TOTAL_CUS; *d = RS_TOTAL_CUS; return; }
    const int32_t *row = &c->lat_distinct[(size_t)(b * nc + x) * ns];
    int pick = -1;
    for (int s = 0; s < ns; ++s)
        if (row[s] <= c->slo_us) { pick = s; break; }
    if (pick < 0) {
        pick = 0;
        for (int s = 1; s < ns; ++s)
            if (row[s] < row[pick]) pick = s;
    }
    *d = c->decode_cus[pick];
    *p = RS_TOTAL_CUS - *d;
}

int32_t kv_alloc(rs_ctx *c, int64_t req_id, int32_t n_tokens, const std::vector<int32_t> **out) {
    if (n_tokens < 0) return fail(RS_ERR_BAD_ARG, "negative token count");
    const int need = (n_tokens + RS_KV_BLOCK - 1) / RS_KV_BLOCK;
    auto it = c->owned.find(req_id);
    const int have = it == c->owned.end() ? 0 : (int)it->second.size();
    const int extra = need - have;
    if (extra > (int)c->free_list.size())
        return fail(RS_ERR_NO_BLOCKS, "request %lld needs %d more blocks, %zu free", (long long)req_id,
                    extra, c->free_list.size());
    std::vector<int32_t> &v = c->owned[req_id];
    for (int i = 0; i < extra; ++i) {
        v.push_back(c->free_list.back());
        c->free_list.pop_back();
    }
    if (out) *out = &v;
    return RS_OK;
}

// One side's CU count and the stream masked to it.
int32_t set_side(rs_ctx *c, int s, int cus) {
    Side &sd = c->side[s];
    if (c->gpu && cus > 0) {
        hipStream_t st;
        int32_t rc = get_stream(c, s, cus, &st);
        if (rc) return rc;
        if (st != sd.stream && sd.stream) {
            // later work of this side is ordered after what the old stream still holds
            HIP_TRY(hipEventRecord(sd.order, sd.stream));
            HIP_TRY(hipStreamWaitEvent(st, sd.order, 0));
        }
        sd.stream = st;
    }
    sd.cus = cus;
    return RS_OK;
}

int32_t set_split(rs_ctx *c, int32_t p, int32_t d) {
    auto legal = [](int v) { return v >= 0 && v <= RS_TOTAL_CUS && v % RS_CU_GRANULE == 0; };
    if (!legal(p) || !legal(d)) return fail(RS_ERR_BAD_SPLIT, "split (%d,%d): counts must be multiples of %d in [0,256]", p, d, RS_CU_GRANULE);
    const bool over = (p == RS_TOTAL_CUS && d == RS_TOTAL_CUS);
    if (!over && p + d > RS_TOTAL_CUS) return fail(RS_ERR_BAD_SPLIT, "split (%d,%d) overlaps; only (256,256) may", p, d);
    if (c->engine) {   // the prefill side belongs to the prefill thread: it picks the published count up at its next prompt
        int32_t rc = set_side(c, RS_SIDE_DECODE, d);
        if (rc) return rc;
        c->prefill_cus_pub.store(p, std::memory_order_release);
        c->over_alloc = over;
        return RS_OK;
    }
    const int want[2] = {p, d};
    for (int s = 0; s < 2; ++s) {
        int32_t rc = set_side(c, s, want[s]);
        if (rc) return rc;
    }
    c->over_alloc = over;
    if (c->gpu && c->new_stream && p > 0 && d > 0) {
        // The first time two queues have work at the same moment the runtime blocks a launch call for tens of
        // milliseconds (observed once per process: the first layer call that overlapped the other side stalled
        // 30-60 ms, with both streams long created and used one at a time).  A new stream has just joined the
        // pool: overlap a few empty kernels on the pair now, in this set-up call, and wait for them.
        c->new_stream = false;
        for (int i = 0; i < 8; ++i) {
            launch_noop(c->side[0].stream);
            launch_noop(c->side[1].stream);
        }
        HIP_TRY(hipStreamSynchronize(c->side[0].stream));
        HIP_TRY(hipStreamSynchronize(c->side[1].stream));
    }
    return RS_OK;
}

int32_t check_layer_call(rs_ctx *c, int side, int32_t layer, const void *x_in, void *x_out,
                         const int32_t *tables) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    if (!c->gpu) return fail(RS_ERR_STATE, "host-only context cannot run layers");
    if (layer < 0 || layer >= c->m.n_layers) return fail(RS_ERR_BAD_ARG, "layer %d out of range", layer);
    if (!c->have_weights[layer]) return fail(RS_ERR_STATE, "weights of layer %d not set", layer);
    if (!x_in || !x_out || !tables) return fail(RS_ERR_BAD_ARG, "null pointer");
    if (c->side[side].cus <= 0) return fail(RS_ERR_STATE, "side %d has no compute units in the current split", side);
    return RS_OK;
}

// With kernel timing on, records boundary `i` of the current layer call on the side's stream.
void tick(rs_ctx *c, int side, int i) {
    if (!c->kernel_timing || c->capturing) return;
    Side &s = c->side[side];
    if (!s.kt[i] && hipEventCreate(&s.kt[i]) != hipSuccess) return;
    (void)hipEventRecord(s.kt[i], s.stream);
    if (i == RS_N_KERNEL_SLOTS) s.kt_valid = true;
}

// The dense part after attention, shared by both passes.
bool run_post_attention(rs_ctx *c, int side, hipStream_t st, Workspace &w, const rs_layer_weights &lw,
                        const rs_ctx::PackedLayer &pl, const rs_ctx::MoeLayer &ml, const bf16_t *x, bf16_t *y, int M, bool skinny) {
    bool released_needed = false;   // a GEMM needed row-major weights the caller has released
    const rs_model_desc &m = c->m;
    const int d = m.d_model, qd = m.n_q_heads * m.head_dim, f = m.ffn_dim;
    auto gemm = [&](GemmArgs g) {
        g.cus = c->side[side].cus;
        g.partials = w.partials;
        g.partial_cap = w.partial_cap;
        if (skinny) launch_gemm_skinny(st, g, w.partials);
        else if (!launch_gemm_tiled(st, g)) released_needed = true;
    };
    // h, attn and act are fragment-packed by their producers; x1 and y are row-major
    const bf16_t *wo = (const bf16_t *)lw.wo, *wg = (const bf16_t *)lw.wg, *wu = (const bf16_t *)lw.wu, *wd = (const bf16_t *)lw.wd;
    gemm(GemmArgs{w.attn, wo, nullptr, pl.wo, nullptr, x, w.x1, M, d, qd, EPI_RESIDUAL});
    tick(c, side, 5);
    launch_rmsnorm(st, w.x1, (const bf16_t *)lw.g2, w.h, M, d, m.rms_eps);
    tick(c, side, 6);
    if (ml.E > 0) {
        // sparse block: route, gather expert by expert, two grouped GEMMs over all tiles, weighted sum
        const int cap = std::min(w.m_cap, moe_row_cap(M, ml.E));
        MoeArgs ma{w.h, ml.router, w.m_sel, w.m_wt, w.m_pos, w.m_src, w.m_tile, w.m_a, w.m_out, w.x1, y, M, d, ml.E, cap};
        launch_moe_route_and_gather(st, ma);
        GemmArgs gu{w.m_a, nullptr, nullptr, ml.wg, ml.wu, nullptr, w.m_act, cap, f, d, EPI_SWIGLU, 1, c->side[side].cus};
        gu.tile_expert = w.m_tile;
        gu.expert_stride = ml.stride_gu;
        bool ok = launch_gemm_grouped(st, gu);
        tick(c, side, 7);
        GemmArgs gd{w.m_act, nullptr, nullptr, ml.wd, nullptr, nullptr, w.m_out, cap, d, f, EPI_STORE, 0, c->side[side].cus};
        gd.tile_expert = w.m_tile;
        gd.expert_stride = ml.stride_d;
        ok = launch_gemm_grouped(st, gd) && ok;
        launch_moe_combine(st, ma);
        tick(c, side, 8);
        return ok && !released_needed;
    }
    gemm(GemmArgs{w.h, wg, wu, pl.wg, pl.wu, nullptr, w.act, M, f, d, EPI_SWIGLU, 1});
    tick(c, side, 7);
    gemm(GemmArgs{w.act, wd, nullptr, pl.wd, nullptr, w.x1, y, M, d, f, EPI_RESIDUAL});
    tick(c, side, 8);
    return !released_needed;
}

int32_t prefill_layer(rs_ctx *c, int32_t layer, const void *x_in, void *x_out, const int32_t *cu,
                      int32_t n_req, const int32_t *tables, int32_t max_blk) {
    const rs_model_desc &m = c->m;
    if (!cu || n_req < 1 || n_req > RS_MAX_PREFILL_REQS) return fail(RS_ERR_BAD_ARG, "n_req %d out of range", n_req);
    if (cu[0] != 0) return fail(RS_ERR_BAD_ARG, "cu_seqlens must start at 0");
    SeqInfo seq{};
    seq.n_req = n_req;
    int longest = 0;
    for (int r = 0; r <= n_req; ++r) {
        if (r && cu[r] < cu[r - 1]) return fail(RS_ERR_BAD_ARG, "cu_seqlens must ascend");
        if (r) longest = std::max(longest, cu[r] - cu[r - 1]);
        seq.cu[r] = cu[r];
    }
    const int T = cu[n_req];
    Workspace &w = c->ws[RS_SIDE_PREFILL];
    if (T < 1 || T > w.rows) return fail(RS_ERR_BAD_ARG, "%d prefill tokens, workspace holds %d", T, w.rows);
    if (longest > m.max_pos) return fail(RS_ERR_BAD_ARG, "prompt of %d tokens exceeds max_pos %d", longest, m.max_pos);
    if ((longest + RS_KV_BLOCK - 1) / RS_KV_BLOCK > max_blk)
        return fail(RS_ERR_BAD_BLOCK, "block table of %d entries too short for %d tokens", max_blk, longest);
    if (!c->packed[layer].wg && c->moe[layer].E == 0)
        return fail(RS_ERR_STATE, "layer %d has no feed-forward weights (dense ones in rs_set_weights, or rs_set_moe_weights)", layer);
    const rs_layer_weights &lw = c->weights[layer];
    hipStream_t st = c->side[RS_SIDE_PREFILL].stream;
    const int d = m.d_model, hd = m.head_dim, qd = m.n_q_heads * hd, nqkv = qd + 2 * m.n_kv_heads * hd;
    bf16_t *kp = (bf16_t *)c->pool.k_pool + (size_t)layer * c->pool.layer_stride;
    bf16_t *vp = (bf16_t *)c->pool.v_pool + (size_t)layer * c->pool.layer_stride;

    tick(c, RS_SIDE_PREFILL, 0);
    c->last_rows[RS_SIDE_PREFILL] = T;
    launch_rmsnorm(st, (const bf16_t *)x_in, (const bf16_t *)lw.g1, w.h, T, d, m.rms_eps);
    tick(c, RS_SIDE_PREFILL, 1);
    // a pass of at most 64 rows is bound by reading the weights once: it takes the weight-streaming kernels
    const bool skinny = T <= 64;
    GemmArgs gq{w.h, (const bf16_t *)lw.wqkv, nullptr, c->packed[layer].wqkv, nullptr, nullptr, w.qkv,
                T, nqkv, d, EPI_STORE, 0, c->side[RS_SIDE_PREFILL].cus, w.partials, w.partial_cap};
    bool ok = true;
    if (skinny) launch_gemm_skinny(st, gq, w.partials);
    else ok = launch_gemm_tiled(st, gq);
    tick(c, RS_SIDE_PREFILL, 2);
    RopeKvArgs ra{w.qkv, c->rope, kp, vp, tables, nullptr, c->err_flag + RS_SIDE_PREFILL, T, m.n_q_heads, m.n_kv_heads, hd,
                  max_blk, c->pool.n_blocks, m.max_pos, seq};
    launch_rope_kvwrite(st, ra);
    tick(c, RS_SIDE_PREFILL, 3);
    PrefillAttnArgs pa{w.qkv, nqkv, w.attn, kp, vp, tables, c->err_flag + RS_SIDE_PREFILL, m.n_q_heads, m.n_kv_heads, hd,
                       max_blk, c->pool.n_blocks, (float)(1.4426950408889634 / std::sqrt((double)hd)), seq};
    launch_prefill_attention(st, pa);
    tick(c, RS_SIDE_PREFILL, 4);
    ok = run_post_attention(c, RS_SIDE_PREFILL, st, w, lw, c->packed[layer], c->moe[layer], (const bf16_t *)x_in, (bf16_t *)x_out, T, skinny) && ok;
    HIP_TRY(hipGetLastError());
    if (!ok) return fail(RS_ERR_STATE, "layer %d: a GEMM of this pass needs the row-major matrices that were released", layer);
    return RS_OK;
}

// One layer over a hybrid batch (section 3.1: chunked prefill co-batched with decode, the baseline the paper
// compares with): rows [0, T) are one chunk of each of n_req prompts (prompt r's chunk starts at position
// start[r]), rows [T, T+B) are decode rows.  Both kinds share every projection (one pass over the weights for
// all rows) and take their own attention kernel.  Runs on the prefill side's stream and workspace.
int32_t hybrid_layer(rs_ctx *c, int32_t layer, const void *x_in, void *x_out, const int32_t *cu, const int32_t *start,
                     int32_t n_req, const int32_t *ptables, int32_t max_blk_p, const int32_t *ctx_lens,
                     const int32_t *dtables, int32_t max_blk_d, int32_t B, int32_t max_ctx) {
    const rs_model_desc &m = c->m;
    if (!cu || !start || n_req < 1 || n_req > RS_MAX_PREFILL_REQS) return fail(RS_ERR_BAD_ARG, "n_req %d out of range", n_req);
    if (cu[0] != 0) return fail(RS_ERR_BAD_ARG, "cu_seqlens must start at 0");
    SeqInfo seq{};
    seq.n_req = n_req;
    for (int r = 0; r <= n_req; ++r) {
        if (r && cu[r] < cu[r - 1]) return fail(RS_ERR_BAD_ARG, "cu_seqlens must ascend");
        seq.cu[r] = cu[r];
    }
    for (int r = 0; r < n_req; ++r) {
        const int len = cu[r + 1] - cu[r];
        if (start[r] < 0 || start[r] % RS_KV_BLOCK) return fail(RS_ERR_BAD_ARG, "chunk start %d: a non-negative multiple of %d", start[r], RS_KV_BLOCK);
        if (start[r] + len > m.max_pos) return fail(RS_ERR_BAD_ARG, "chunk ends at position %d, max_pos is %d", start[r] + len, m.max_pos);
        if ((start[r] + len + RS_KV_BLOCK - 1) / RS_KV_BLOCK > max_blk_p)
            return fail(RS_ERR_BAD_BLOCK, "block table of %d entries too short for %d tokens", max_blk_p, start[r] + len);
        seq.start[r] = start[r];
    }
    const int T = cu[n_req], M = T + B;
    Workspace &w = c->ws[RS_SIDE_PREFILL];
    if (T < 1 || B < 0 || M > w.rows) return fail(RS_ERR_BAD_ARG, "%d chunk rows + %d decode rows, workspace holds %d", T, B, w.rows);
    if (B > 0) {
        if (!ctx_lens || !dtables) return fail(RS_ERR_BAD_ARG, "null decode arguments");
        if (B > c->lim.max_decode_batch) return fail(RS_ERR_BAD_ARG, "decode batch %d exceeds max_decode_batch %d", B, c->lim.max_decode_batch);
        if (max_ctx < 1 || max_ctx > c->lim.max_context || max_ctx > m.max_pos)
            return fail(RS_ERR_BAD_ARG, "max_ctx %d outside [1, min(%d,%d)]", max_ctx, c->lim.max_context, m.max_pos);
        if ((max_ctx + RS_KV_BLOCK - 1) / RS_KV_BLOCK > max_blk_d)
            return fail(RS_ERR_BAD_BLOCK, "block table of %d entries too short for context %d", max_blk_d, max_ctx);
    }
    if (!c->packed[layer].wg && c->moe[layer].E == 0) return fail(RS_ERR_STATE, "layer %d has no feed-forward weights", layer);
    const rs_layer_weights &lw = c->weights[layer];
    hipStream_t st = c->side[RS_SIDE_PREFILL].stream;
    const int d = m.d_model, hd = m.head_dim, qd = m.n_q_heads * hd, nqkv = qd + 2 * m.n_kv_heads * hd;
    bf16_t *kp = (bf16_t *)c->pool.k_pool + (size_t)layer * c->pool.layer_stride;
    bf16_t *vp = (bf16_t *)c->pool.v_pool + (size_t)layer * c->pool.layer_stride;
    int32_t *err = c->err_flag + RS_SIDE_PREFILL;
    const float sl2 = (float)(1.4426950408889634 / std::sqrt((double)hd));

    tick(c, RS_SIDE_PREFILL, 0);
    c->last_rows[RS_SIDE_PREFILL] = M;
    launch_rmsnorm(st, (const bf16_t *)x_in, (const bf16_t *)lw.g1, w.h, M, d, m.rms_eps);
    tick(c, RS_SIDE_PREFILL, 1);
    const bool skinny = M <= 64;
    GemmArgs gq{w.h, (const bf16_t *)lw.wqkv, nullptr, c->packed[layer].wqkv, nullptr, nullptr, w.qkv,
                M, nqkv, d, EPI_STORE, 0, c->side[RS_SIDE_PREFILL].cus, w.partials, w.partial_cap};
    bool ok = true;
    if (skinny) launch_gemm_skinny(st, gq, w.partials);
    else ok = launch_gemm_tiled(st, gq);
    tick(c, RS_SIDE_PREFILL, 2);
    launch_rope_kvwrite(st, RopeKvArgs{w.qkv, c->rope, kp, vp, ptables, nullptr, err, T, m.n_q_heads, m.n_kv_heads, hd,
                                       max_blk_p, c->pool.n_blocks, m.max_pos, seq});
    if (B > 0) {
        SeqInfo none{};
        launch_rope_kvwrite(st, RopeKvArgs{w.qkv + (size_t)T * nqkv, c->rope, kp, vp, dtables, ctx_lens, err, B, m.n_q_heads,
                                           m.n_kv_heads, hd, max_blk_d, c->pool.n_blocks, m.max_pos, none});
    }
    tick(c, RS_SIDE_PREFILL, 3);
    PrefillAttnArgs pa{w.qkv, nqkv, w.attn, kp, vp, ptables, err, m.n_q_heads, m.n_kv_heads, hd,
                       max_blk_p, c->pool.n_blocks, sl2, seq};
    pa.Mt_out = packed_mt(M);
    launch_prefill_attention(st, pa);
    if (B > 0) {
        DecodeAttnArgs da{w.qkv + (size_t)T * nqkv, nqkv, w.attn, kp, vp, dtables, ctx_lens, err, w.part_o, w.part_ml,
                          B, m.n_q_heads, m.n_kv_heads, hd, max_blk_d, c->pool.n_blocks, max_ctx,
                          (max_ctx + RS_DECODE_CHUNK - 1) / RS_DECODE_CHUNK, sl2, c->side[RS_SIDE_PREFILL].cus < RS_TOTAL_CUS};
        da.out_row0 = T;
        da.out_Mt = packed_mt(M);
        launch_decode_attention(st, da);
    }
    tick(c, RS_SIDE_PREFILL, 4);
    ok = run_post_attention(c, RS_SIDE_PREFILL, st, w, lw, c->packed[layer], c->moe[layer], (const bf16_t *)x_in, (bf16_t *)x_out, M, skinny) && ok;
    HIP_TRY(hipGetLastError());
    if (!ok) return fail(RS_ERR_STATE, "layer %d: a GEMM of this pass needs the row-major matrices that were released", layer);
    return RS_OK;
}

int32_t decode_layer(rs_ctx *c, Workspace &w, int32_t layer, const void *x_in, void *x_out, const int32_t *ctx_lens,
                     const int32_t *tables, int32_t max_blk, int32_t B, int32_t max_ctx) {
    const rs_model_desc &m = c->m;
    if (!ctx_lens) return fail(RS_ERR_BAD_ARG, "null ctx_lens");
    if (B < 1 || B > w.rows) return fail(RS_ERR_BAD_ARG, "decode batch %d, workspace holds %d", B, w.rows);
    if (max_ctx < 1 || max_ctx > c->lim.max_context || max_ctx > m.max_pos)
        return fail(RS_ERR_BAD_ARG, "max_ctx %d outside [1, min(%d,%d)]", max_ctx, c->lim.max_context, m.max_pos);
    if ((max_ctx + RS_KV_BLOCK - 1) / RS_KV_BLOCK > max_blk)
        return fail(RS_ERR_BAD_BLOCK, "block table of %d entries too short for context %d", max_blk, max_ctx);
    if (!c->packed[layer].wg && c->moe[layer].E == 0)
        return fail(RS_ERR_STATE, "layer %d has no feed-forward weights (dense ones in rs_set_weights, or rs_set_moe_weights)", layer);
    const rs_layer_weights &lw = c->weights[layer];
    hipStream_t st = c->side[RS_SIDE_DECODE].stream;
    const int d = m.d_model, hd = m.head_dim, qd = m.n_q_heads * hd, nqkv = qd + 2 * m.n_kv_heads * hd;
    bf16_t *kp = (bf16_t *)c->pool.k_pool + (size_t)layer * c->pool.layer_stride;
    bf16_t *vp = (bf16_t *)c->pool.v_pool + (size_t)layer * c->pool.layer_stride;
    const bool skinny = B <= 64;
    c->last_rows[RS_SIDE_DECODE] = B;
    c->decode_fused = skinny && c->moe[layer].E == 0 && fused_decode_applies(c);
    if (c->decode_fused) {
        // At most 64 rows: every projection is a stream of its weights with the RMSNorm of its input folded in
        // (decode_gemm.hip).  10 launches: QKV stream, its epilogue (row scale, rotary, cache append), attention,
        // chunk merge, O stream + residual, gate/up stream + SwiGLU, down stream + residual.
        const rs_ctx::PackedLayer &pl = c->packed[layer];
        const int f = m.ffn_dim;
        float *ssq1 = w.ssq, *ssq2 = w.ssq + 64 * 64;
        const int dcus = c->side[RS_SIDE_DECODE].cus;
        tick(c, RS_SIDE_DECODE, 0);
        tick(c, RS_SIDE_DECODE, 1);
        const DGemmPlan pq = dgemm_plan(nqkv, d, false);
        launch_dgemm_partials(st, DGemmArgs{nullptr, (const bf16_t *)x_in, (const bf16_t *)lw.g1, ssq1, pl.wqkv, nullptr, w.partials, B, nqkv, d}, pq, dgemm_prefers_half_height(pq, dcus));
        launch_qkv_rope_epilogue(st, QkvEpiArgs{w.partials, ssq1, pq.S, pq.Nv, d, m.rms_eps, w.qkv, c->rope, kp, vp, tables, ctx_lens,
                                                c->err_flag + RS_SIDE_DECODE, B, m.n_q_heads, m.n_kv_heads, hd, max_blk,
                                                c->pool.n_blocks, m.max_pos});
        tick(c, RS_SIDE_DECODE, 2);
        tick(c, RS_SIDE_DECODE, 3);
        DecodeAttnArgs da{w.qkv, nqkv, w.attn, kp, vp, tables, ctx_lens, c->err_flag + RS_SIDE_DECODE, w.part_o, w.part_ml,
                          B, m.n_q_heads, m.n_kv_heads, hd, max_blk, c->pool.n_blocks, max_ctx,
                          (max_ctx + RS_DECODE_CHUNK - 1) / RS_DECODE_CHUNK,
                          (float)(1.4426950408889634 / std::sqrt((double)hd)), c->side[RS_SIDE_DECODE].cus < RS_TOTAL_CUS};
        launch_decode_attention(st, da);
        tick(c, RS_SIDE_DECODE, 4);
        const DGemmPlan po = dgemm_plan(d, qd, false);
        launch_dgemm_partials(st, DGemmArgs{w.attn, nullptr, nullptr, nullptr, pl.wo, nullptr, w.partials, B, d, qd}, po, dgemm_prefers_half_height(po, dcus));
        launch_dgemm_epilogue(st, DEpiArgs{w.partials, po.S, po.Nv, nullptr, 0, d, m.rms_eps, (const bf16_t *)x_in, w.x1, B, d}, EPI_RESIDUAL);
        tick(c, RS_SIDE_DECODE, 5);
        tick(c, RS_SIDE_DECODE, 6);
        const DGemmPlan pg = dgemm_plan(f, d, true);
        launch_dgemm_partials(st, DGemmArgs{nullptr, w.x1, (const bf16_t *)lw.g2, ssq2, pl.wg, pl.wu, w.partials, B, f, d}, pg, dgemm_prefers_half_height(pg, dcus));
        launch_dgemm_epilogue(st, DEpiArgs{w.partials, pg.S, pg.Nv, ssq2, pg.S, d, m.rms_eps, nullptr, w.act, B, f}, EPI_SWIGLU);
        tick(c, RS_SIDE_DECODE, 7);
        if (dgemm_applies(d, f)) {
            const DGemmPlan pd = dgemm_plan(d, f, false);
            launch_dgemm_partials(st, DGemmArgs{w.act, nullptr, nullptr, nullptr, pl.wd, nullptr, w.partials, B, d, f}, pd, dgemm_prefers_half_height(pd, dcus));
            launch_dgemm_epilogue(st, DEpiArgs{w.partials, pd.S, pd.Nv, nullptr, 0, d, m.rms_eps, w.x1, (bf16_t *)x_out, B, d}, EPI_RESIDUAL);
        } else {
            GemmArgs gd{w.act, (const bf16_t *)lw.wd, nullptr, pl.wd, nullptr, w.x1, (bf16_t *)x_out, B, d, f, EPI_RESIDUAL,
                        0, c->side[RS_SIDE_DECODE].cus, w.partials, w.partial_cap};
            launch_gemm_skinny(st, gd, w.partials);
        }
        tick(c, RS_SIDE_DECODE, 8);
        HIP_TRY(hipGetLastError());
        return RS_OK;
    }

    tick(c, RS_SIDE_DECODE, 0);
    launch_rmsnorm(st, (const bf16_t *)x_in, (const bf16_t *)lw.g1, w.h, B, d, m.rms_eps);
    tick(c, RS_SIDE_DECODE, 1);
    GemmArgs g{w.h, (const bf16_t *)lw.wqkv, nullptr, c->packed[layer].wqkv, nullptr, nullptr, w.qkv, B, nqkv, d, EPI_STORE,
               0, c->side[RS_SIDE_DECODE].cus, w.partials, w.partial_cap};
    bool ok = true;
    if (skinny) launch_gemm_skinny(st, g, w.partials);
    else ok = launch_gemm_tiled(st, g);
    tick(c, RS_SIDE_DECODE, 2);
    SeqInfo none{};
    RopeKvArgs ra{w.qkv, c->rope, kp, vp, tables, ctx_lens, c->err_flag + RS_SIDE_DECODE, B, m.n_q_heads, m.n_kv_heads, hd,
                  max_blk, c->pool.n_blocks, m.max_pos, none};
    launch_rope_kvwrite(st, ra);
    tick(c, RS_SIDE_DECODE, 3);
    DecodeAttnArgs da{w.qkv, nqkv, w.attn, kp, vp, tables, ctx_lens, c->err_flag + RS_SIDE_DECODE, w.part_o, w.part_ml,
                      B, m.n_q_heads, m.n_kv_heads, hd, max_blk, c->pool.n_blocks, max_ctx,
                      (max_ctx + RS_DECODE_CHUNK - 1) / RS_DECODE_CHUNK,
                      (float)(1.4426950408889634 / std::sqrt((double)hd)), c->side[RS_SIDE_DECODE].cus < RS_TOTAL_CUS};
    launch_decode_attention(st, da);
    tick(c, RS_SIDE_DECODE, 4);
    ok = run_post_attention(c, RS_SIDE_DECODE, st, w, lw, c->packed[layer], c->moe[layer], (const bf16_t *)x_in, (bf16_t *)x_out, B, skinny) && ok;
    HIP_TRY(hipGetLastError());
    if (!ok) return fail(RS_ERR_STATE, "layer %d: a GEMM of this step needs the row-major matrices that were released", layer);
    return RS_OK;
}

// Final RMSNorm + LM head + greedy choice for n rows of x, in groups of at most 64 rows (the
// weight-streaming GEMM's limit).  The chosen tokens go to `tokens` (row order) and/or to
// tok_by_slot[row_slot[row]].
int32_t head_greedy(rs_ctx *c, int side, const bf16_t *x, int n, float *logits, int32_t *tokens,
                    const int32_t *row_slot, int32_t *tok_by_slot) {
    const rs_model_desc &m = c->m;
    Workspace &w = c->ws[side];
    hipStream_t st = c->side[side].stream;
    const int d = m.d_model, V = c->head.vocab;
    // one pass over the weights per group of rows: the large-tile kernel (up to RS_HEAD_GROUP rows; with K only
    // d_model deep and a very wide N it also beats the weight-streaming kernel at a few rows: 243 against 249 us
    // at one row, 259 against 299 us at 64 rows for a 128256 x 4096 head), else the weight-streaming kernel (64 rows)
    const int group = c->head_group[side];
    for (int g0 = 0; g0 < n; g0 += group) {
        const int mg = std::min(group, n - g0);
        c->last_rows[side] = mg;
        launch_rmsnorm(st, x + (size_t)g0 * d, (const bf16_t *)c->head.final_norm, w.h, mg, d, m.rms_eps);
        GemmArgs g{w.h, (const bf16_t *)c->head.lm_head, nullptr, c->packed_lm, nullptr, nullptr, nullptr, mg, V, d, EPI_STORE,
                   0, c->side[side].cus};
        int S = 1, Nv = V;
        if (mg <= 64 && gemm_skinny_partials_shared(V, d)) {   // a function of the shapes alone
            launch_gemm_skinny_partials(st, g, c->head_part[side], &S, &Nv);
        } else if (!launch_gemm_direct_partials(st, g, c->head_part[side])) {
            if (mg > 64) return fail(RS_ERR_STATE, "head group of %d rows without the large-tile kernel", mg);
            launch_gemm_skinny_partials(st, g, c->head_part[side], &S, &Nv);
        }
        HeadArgmaxArgs ha{c->head_part[side], logits ? logits + (size_t)g0 * V : nullptr, tokens ? tokens + g0 : nullptr,
                          row_slot ? row_slot + g0 : nullptr, tok_by_slot, S, mg, V, Nv};
        launch_head_argmax(st, ha);
    }
    HIP_TRY(hipGetLastError());
    return RS_OK;
}

// The status a set of error bits stands for (see rs_ctx::err_flag).
int32_t report_flag(int32_t flag) {
    if (flag & 4) return fail(RS_ERR_BAD_ARG, "a kernel met a token outside the vocabulary (flag %d)", flag);
    return fail(RS_ERR_BAD_BLOCK, "a kernel skipped an illegal block id, rotary position or context length (flag %d)", flag);
}

// Captured decode steps bake in the addresses of the layer's packed matrices: whenever those may
// change (rs_set_weights, rs_set_moe_weights) every cached graph of the layer is destroyed.
void drop_step_graphs(rs_ctx *c) {
    for (auto &kv : c->step_graphs) (void)hipGraphExecDestroy(kv.second);
    c->step_graphs.clear();
}

void drop_layer_graphs(rs_ctx *c, int32_t layer) {
    drop_step_graphs(c);
    for (auto it = c->graphs.begin(); it != c->graphs.end();) {
        if (it->first.layer == layer) {
            (void)hipGraphExecDestroy(it->second);
            it = c->graphs.erase(it);
        } else {
            ++it;
        }
    }
}

int32_t enter_mode(rs_ctx *c, int mode) {
    if (c->serving_mode && c->serving_mode != mode)
        return fail(RS_ERR_STATE, "hidden-state and token requests cannot be mixed on one context");
    c->serving_mode = mode;
    return RS_OK;
}

int32_t check_head_call(rs_ctx *c, int side, int n) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    if (side < 0 || side > 1) return fail(RS_ERR_BAD_ARG, "side %d", side);
    if (!c->gpu) return fail(RS_ERR_STATE, "host-only context: no device work");
    if (!c->have_head) return fail(RS_ERR_STATE, "rs_set_head has not been called");
    if (c->side[side].cus <= 0 || !c->side[side].stream) return fail(RS_ERR_STATE, "side %d has no CUs", side);
    if (n < 1 || n > c->ws[side].rows) return fail(RS_ERR_BAD_ARG, "%d rows, the side's workspace holds %d", n, c->ws[side].rows);
    return RS_OK;
}

}  // namespace

// ================================================================================ C ABI

extern "C" {

const char *rs_last_error(void) { return g_err.c_str(); }

int32_t rs_init(const rs_model_desc *model, const rs_pool_desc *pool, const rs_limits *limits,
                const rs_profile *prof, int32_t device, rs_ctx **out) {
    if (!model || !pool || !limits || !out) return fail(RS_ERR_BAD_ARG, "null argument");
    const rs_model_desc &m = *model;
    if (m.head_dim != 64 && m.head_dim != 128) return fail(RS_ERR_BAD_ARG, "head_dim %d: only 64 and 128", m.head_dim);
    if (m.d_model < 8 || m.d_model % 8 || m.ffn_dim < 8 || m.ffn_dim % 8)
        return fail(RS_ERR_BAD_ARG, "d_model and ffn_dim must be positive multiples of 8");
    if (m.d_model > 65536) return fail(RS_ERR_BAD_ARG, "d_model %d: at most 65536", m.d_model);
    if (m.n_kv_heads < 1 || m.n_q_heads < 1 || m.n_q_heads % m.n_kv_heads || m.n_q_heads / m.n_kv_heads > 16)
        return fail(RS_ERR_BAD_ARG, "need n_q_heads = G * n_kv_heads with 1 <= G <= 16");
    if (m.n_layers < 1 || m.max_pos < 1 || !(m.rope_base > 1.0f) || !(m.rms_eps >= 0.0f))
        return fail(RS_ERR_BAD_ARG, "bad n_layers / max_pos / rope_base / rms_eps");
    if (pool->n_blocks < 1) return fail(RS_ERR_BAD_ARG, "pool needs at least one block");
    const int64_t per_layer = (int64_t)pool->n_blocks * RS_KV_BLOCK * m.n_kv_heads * m.head_dim;
    if (m.n_layers > 1 && pool->layer_stride < per_layer) return fail(RS_ERR_BAD_ARG, "layer_stride smaller than one layer's pool");
    if (limits->max_prefill_tokens < 0 || limits->max_decode_batch < 0 || limits->max_context < 1)
        return fail(RS_ERR_BAD_ARG, "bad limits");
    if (device != RS_HOST_ONLY && (!pool->k_pool || !pool->v_pool)) return fail(RS_ERR_BAD_ARG, "null KV pool");
    if (prof) {
        if (prof->n_batch < 1 || prof->n_ctx < 1 || prof->n_split < 1 || !prof->batch_edges || !prof->ctx_edges ||
            !prof->decode_cus || !prof->lat_distinct_us || !prof->lat_over_us)
            return fail(RS_ERR_BAD_ARG, "incomplete profile");
        for (int s = 0; s < prof->n_split; ++s) {
            const int v = prof->decode_cus[s];
            if (v <= 0 || v >= RS_TOTAL_CUS || v % RS_CU_GRANULE || (s && v <= prof->decode_cus[s - 1]))
                return fail(RS_ERR_BAD_ARG, "profile decode_cus must ascend in (0,256), multiples of %d", RS_CU_GRANULE);
        }
    }
    rs_ctx *c = new rs_ctx();
    c->m = m;
    c->pool = *pool;
    c->lim = *limits;
    c->device = device;
    c->gpu = device != RS_HOST_ONLY;
    c->weights.resize(m.n_layers);
    c->packed.resize(m.n_layers);
    c->moe.resize(m.n_layers);
    c->have_weights.assign(m.n_layers, false);
    c->free_list.resize(pool->n_blocks);
    for (int i = 0; i < pool->n_blocks; ++i) c->free_list[i] = pool->n_blocks - 1 - i;  // pop -> 0,1,2,..
    c->max_blk_per_req = (limits->max_context + RS_KV_BLOCK - 1) / RS_KV_BLOCK;
    c->n_slots = 4 * std::max(1, limits->max_decode_batch) + 64;
    for (int i = c->n_slots - 1; i >= 0; --i) c->free_slots.push_back(i);
    if (prof) {
        c->have_prof = true;
        c->batch_edges.assign(prof->batch_edges, prof->batch_edges + prof->n_batch);
        c->ctx_edges.assign(prof->ctx_edges, prof->ctx_edges + prof->n_ctx);
        c->decode_cus.assign(prof->decode_cus, prof->decode_cus + prof->n_split);
        const size_t cells = (size_t)prof->n_batch * prof->n_ctx;
        c->lat_distinct.assign(prof->lat_distinct_us, prof->lat_distinct_us + cells * prof->n_split);
        c->lat_over.assign(prof->lat_over_us, prof->lat_over_us + cells);
        c->slo_us = prof->slo_us;
    }
    *out = c;
    if (!c->gpu) return RS_OK;

    auto bail = [&](int32_t rc) { rs_destroy(c); *out = nullptr; return rc; };
    int32_t rc;
    auto gpu_setup = [&]() -> int32_t {
        HIP_TRY(hipSetDevice(device));
        if (device < 0 || device >= RS_MAX_DEVICES) return fail(RS_ERR_BAD_ARG, "device %d: at most %d devices", device, RS_MAX_DEVICES);
        {   // this device's copy of the static scratch array (each GPU holds its own, at its own address)
            std::lock_guard<std::mutex> lk(g_static_scratch_mu);
            if (!g_static_scratch[device]) {
                void *ptr = nullptr;
                HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
                g_static_scratch[device] = ptr;
            }
        }
        gemm_kernels_init();
        decode_gemm_kernels_init();
        attention_kernels_init();
        // rotary table, angles in float64
        const int half = m.head_dim / 2;
        std::vector<CosSin> tab((size_t)m.max_pos * half);
        for (int i = 0; i < half; ++i) {
            const double theta = std::pow((double)m.rope_base, -2.0 * i / (double)m.head_dim);
            for (int p = 0; p < m.max_pos; ++p) {
                const double phi = (double)p * theta;
                tab[(size_t)p * half + i] = CosSin{(float)std::cos(phi), (float)std::sin(phi)};
            }
        }
        HIP_TRY(hipMalloc(&c->rope, tab.size() * sizeof(CosSin)));
        HIP_TRY(hipMemcpy(c->rope, tab.data(), tab.size() * sizeof(CosSin), hipMemcpyHostToDevice));
        HIP_TRY(hipMalloc(&c->err_flag, 2 * sizeof(int32_t)));
        HIP_TRY(hipMemset(c->err_flag, 0, 2 * sizeof(int32_t)));
        HIP_TRY(hipHostMalloc((void **)&c->h_err, 8 * sizeof(int32_t)));
        std::memset(c->h_err, 0, 8 * sizeof(int32_t));
        int32_t r = alloc_ws(c, c->ws[RS_SIDE_PREFILL], limits->max_prefill_tokens, false);
        if (r) return r;
        r = alloc_ws(c, c->ws[RS_SIDE_DECODE], limits->max_decode_batch, true);
        if (r) return r;
        for (int s = 0; s < 2; ++s) {
            HIP_TRY(hipEventCreateWithFlags(&c->side[s].order, hipEventDisableTiming));
            c->side[s].marks.assign(RS_MAX_MARKS, nullptr);
        }
        // staging for the serving step
        const size_t nb = std::max(1, limits->max_decode_batch);
        const size_t tab_elems = nb * c->max_blk_per_req;
        HIP_TRY(hipMalloc(&c->d_ctx, nb * sizeof(int32_t)));
        HIP_TRY(hipMalloc(&c->d_tab, tab_elems * sizeof(int32_t)));
        HIP_TRY(hipMalloc(&c->d_ptab, (size_t)RS_MAX_PREFILL_REQS * c->max_blk_per_req * sizeof(int32_t)));
        HIP_TRY(hipEventCreateWithFlags(&c->prefill_ev, hipEventDisableTiming));
        for (int i = 0; i < 2; ++i) {
            HIP_TRY(hipHostMalloc(&c->h_ctx[i], nb * sizeof(int32_t)));
            HIP_TRY(hipHostMalloc(&c->h_tab[i], tab_elems * sizeof(int32_t)));
            HIP_TRY(hipEventCreateWithFlags(&c->staged[i], hipEventDisableTiming));
        }
        HIP_TRY(hipHostMalloc(&c->h_ptab, (size_t)RS_MAX_PREFILL_REQS * c->max_blk_per_req * sizeof(int32_t)));
        HIP_TRY(hipEventCreateWithFlags(&c->pstaged, hipEventDisableTiming));
        for (int i = 0; i < 2; ++i) HIP_TRY(hipEventCreateWithFlags(&c->step_end[i], hipEventDisableTiming));
        return set_split(c, RS_TOTAL_CUS, RS_TOTAL_CUS);
    };
    rc = gpu_setup();
    if (rc) return bail(rc);
    return RS_OK;
}

int32_t rs_destroy(rs_ctx *c) {
    if (!c) return RS_OK;
    if (c->engine) (void)rs_engine_stop(c, 0);
    if (c->gpu) {
        (void)hipSetDevice(c->device);
        (void)hipDeviceSynchronize();
        for (auto &kv : c->reqs)
            if (kv.second.done) (void)hipEventDestroy(kv.second.done);
        for (int s = 0; s < 2; ++s) {
            for (hipEvent_t e : c->side[s].marks)
                if (e) (void)hipEventDestroy(e);
            if (c->side[s].order) (void)hipEventDestroy(c->side[s].order);
            for (hipEvent_t e : c->side[s].kt)
                if (e) (void)hipEventDestroy(e);
            for (auto &kv : c->side[s].pool) (void)hipStreamDestroy(kv.second);
            free_ws(c->ws[s]);
        }
        for (auto &kv : c->graphs) (void)hipGraphExecDestroy(kv.second);
        drop_step_graphs(c);
        for (auto &pl : c->packed)
            for (bf16_t *q : {pl.wqkv, pl.wo, pl.wg, pl.wu, pl.wd})
                if (q) (void)hipFree(q);
        for (auto &ml : c->moe)
            for (bf16_t *q : {ml.wg, ml.wu, ml.wd})
                if (q) (void)hipFree(q);
        if (c->rope) (void)hipFree(c->rope);
        if (c->err_flag) (void)hipFree(c->err_flag);
        if (c->h_err) (void)hipHostFree(c->h_err);
        if (c->d_ctx) (void)hipFree(c->d_ctx);
        if (c->d_tab) (void)hipFree(c->d_tab);
        if (c->d_ptab) (void)hipFree(c->d_ptab);
        for (int i = 0; i < 2; ++i) {
            if (c->h_ctx[i]) (void)hipHostFree(c->h_ctx[i]);
            if (c->h_tab[i]) (void)hipHostFree(c->h_tab[i]);
            if (c->staged[i]) (void)hipEventDestroy(c->staged[i]);
        }
        if (c->h_ptab) (void)hipHostFree(c->h_ptab);
        if (c->pstaged) (void)hipEventDestroy(c->pstaged);
        for (int i = 0; i < 2; ++i) {
            if (c->step_end[i]) (void)hipEventDestroy(c->step_end[i]);
            if (c->head_part[i]) (void)hipFree(c->head_part[i]);
            if (c->h_rowslot[i]) (void)hipHostFree(c->h_rowslot[i]);
            if (c->h_sampled[i]) (void)hipHostFree(c->h_sampled[i]);
            if (c->sampled_ev[i]) (void)hipEventDestroy(c->sampled_ev[i]);
        }
        for (void *q : {(void *)c->packed_lm, (void *)c->d_tok, (void *)c->d_prompts, (void *)c->d_rowslot, (void *)c->d_sampled,
                        (void *)c->d_pslots, (void *)c->d_pfirst})
            if (q) (void)hipFree(q);
        if (c->h_first) (void)hipHostFree(c->h_first);
        if (c->h_pslots) (void)hipHostFree(c->h_pslots);
        if (c->h_pfirst) (void)hipHostFree(c->h_pfirst);
        if (c->prefill_ev) (void)hipEventDestroy(c->prefill_ev);
        if (c->copy_stream) (void)hipStreamDestroy(c->copy_stream);
    }
    delete c;
    return RS_OK;
}

int32_t rs_set_weights(rs_ctx *c, int32_t layer, const rs_layer_weights *w) {
    if (!c || !w) return fail(RS_ERR_BAD_ARG, "null argument");
    if (layer < 0 || layer >= c->m.n_layers) return fail(RS_ERR_BAD_ARG, "layer %d out of range", layer);
    if (!w->g1 || !w->wqkv || !w->wo || !w->g2) return fail(RS_ERR_BAD_ARG, "null weight pointer");
    const bool dense_ffn = w->wg || w->wu || w->wd;   // all three null: the layer's feed-forward block is a sparse one (rs_set_moe_weights)
    if (dense_ffn && (!w->wg || !w->wu || !w->wd)) return fail(RS_ERR_BAD_ARG, "null weight pointer");
    if (c->gpu) {
        // the GEMM kernels stream the matrices in MFMA fragment order: repack them once, here
        HIP_TRY(hipSetDevice(c->device));
        HIP_TRY(hipDeviceSynchronize());   // a captured step of this layer may still be running
        drop_layer_graphs(c, layer);
        const rs_model_desc &m = c->m;
        const int d = m.d_model, qd = m.n_q_heads * m.head_dim, nqkv = qd + 2 * m.n_kv_heads * m.head_dim, f = m.ffn_dim;
        rs_ctx::PackedLayer &pl = c->packed[layer];
        struct Item { bf16_t **dst; const void *src; int N, K; };
        const Item items[5] = {{&pl.wqkv, w->wqkv, nqkv, d}, {&pl.wo, w->wo, d, qd}, {&pl.wg, w->wg, f, d},
                               {&pl.wu, w->wu, f, d}, {&pl.wd, w->wd, d, f}};
        for (const Item &it : items) {
            if (!it.src) continue;
            if (!*it.dst) HIP_TRY(hipMalloc((void **)it.dst, packed_weight_elems(it.N, it.K) * sizeof(bf16_t)));
            launch_pack_weights(nullptr, (const bf16_t *)it.src, *it.dst, it.N, it.K);
        }
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipDeviceSynchronize());
    }
    c->weights[layer] = *w;
    c->have_weights[layer] = true;
    return RS_OK;
}

int32_t rs_set_moe_weights(rs_ctx *c, int32_t layer, const rs_moe_weights *w) {
    if (!c || !w) return fail(RS_ERR_BAD_ARG, "null argument");
    if (layer < 0 || layer >= c->m.n_layers) return fail(RS_ERR_BAD_ARG, "layer %d out of range", layer);
    if (w->n_experts < 2 || w->n_experts > RS_MOE_MAX_EXPERTS) return fail(RS_ERR_BAD_ARG, "n_experts %d: 2 to %d", w->n_experts, RS_MOE_MAX_EXPERTS);
    if (w->top_k != 2) return fail(RS_ERR_BAD_ARG, "top_k %d: only 2", w->top_k);
    const rs_model_desc &m = c->m;
    const int d = m.d_model, f = m.ffn_dim, E = w->n_experts;
    // both products run as grouped large-tile GEMMs
    if (d % 32 || f % 32 || d < 1024 || f < 1024)
        return fail(RS_ERR_BAD_ARG, "the sparse block needs d_model and ffn_dim to be multiples of 32 and at least 1024");
    rs_ctx::MoeLayer &ml = c->moe[layer];
    if (c->gpu) {
        if (!w->router || !w->wg || !w->wu || !w->wd) return fail(RS_ERR_BAD_ARG, "null weight pointer");
        HIP_TRY(hipSetDevice(c->device));
        HIP_TRY(hipDeviceSynchronize());
        drop_layer_graphs(c, layer);
        ml.stride_gu = packed_weight_elems(f, d);
        ml.stride_d = packed_weight_elems(d, f);
        if (ml.E != E) {
            for (bf16_t **q : {&ml.wg, &ml.wu, &ml.wd})
                if (*q) { (void)hipFree(*q); *q = nullptr; }
        }
        if (!ml.wg) {
            HIP_TRY(hipMalloc((void **)&ml.wg, ml.stride_gu * E * sizeof(bf16_t)));
            HIP_TRY(hipMalloc((void **)&ml.wu, ml.stride_gu * E * sizeof(bf16_t)));
            HIP_TRY(hipMalloc((void **)&ml.wd, ml.stride_d * E * sizeof(bf16_t)));
        }
        for (int e = 0; e < E; ++e) {
            launch_pack_weights(nullptr, (const bf16_t *)w->wg + (size_t)e * f * d, ml.wg + e * ml.stride_gu, f, d);
            launch_pack_weights(nullptr, (const bf16_t *)w->wu + (size_t)e * f * d, ml.wu + e * ml.stride_gu, f, d);
            launch_pack_weights(nullptr, (const bf16_t *)w->wd + (size_t)e * d * f, ml.wd + e * ml.stride_d, d, f);
        }
        // per-side buffers of the grouped layout, sized for the side's row limit
        for (int s = 0; s < 2; ++s) {
            Workspace &ws = c->ws[s];
            const int cap = moe_row_cap(ws.rows, RS_MOE_MAX_EXPERTS);
            if (ws.rows <= 0 || ws.m_cap >= cap) continue;
            ws.m_cap = cap;
            HIP_TRY(hipMalloc((void **)&ws.m_sel, (size_t)ws.rows * 2 * sizeof(int32_t)));
            HIP_TRY(hipMalloc((void **)&ws.m_pos, (size_t)ws.rows * 2 * sizeof(int32_t)));
            HIP_TRY(hipMalloc((void **)&ws.m_wt, (size_t)ws.rows * 2 * sizeof(float)));
            HIP_TRY(hipMalloc((void **)&ws.m_src, (size_t)cap * sizeof(int32_t)));
            HIP_TRY(hipMalloc((void **)&ws.m_tile, (size_t)(2 * (cap / 128) + 1) * sizeof(int32_t)));   // tile table + work list
            HIP_TRY(hipMalloc((void **)&ws.m_a, (size_t)cap * d * sizeof(bf16_t)));
            HIP_TRY(hipMalloc((void **)&ws.m_act, (size_t)cap * f * sizeof(bf16_t)));
            HIP_TRY(hipMalloc((void **)&ws.m_out, (size_t)cap * d * sizeof(bf16_t)));
            HIP_TRY(hipMemset(ws.m_a, 0, (size_t)cap * d * sizeof(bf16_t)));
            HIP_TRY(hipMemset(ws.m_act, 0, (size_t)cap * f * sizeof(bf16_t)));
        }
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipDeviceSynchronize());
    }
    ml.router = (const bf16_t *)w->router;
    ml.E = E;
    return RS_OK;
}

int32_t rs_debug_read_moe_routing(rs_ctx *c, int32_t side, int32_t n_rows, int32_t *experts_out, float *weights_out) {
    if (!c || side < 0 || side > 1 || !experts_out || !weights_out) return fail(RS_ERR_BAD_ARG, "bad argument");
    if (!c->gpu) return fail(RS_ERR_STATE, "host-only context");
    Workspace &w = c->ws[side];
    if (!w.m_sel || n_rows < 1 || n_rows > w.rows) return fail(RS_ERR_BAD_ARG, "no routing of %d rows to read", n_rows);
    HIP_TRY(hipSetDevice(c->device));
    if (c->side[side].stream) HIP_TRY(hipStreamSynchronize(c->side[side].stream));
    HIP_TRY(hipMemcpy(experts_out, w.m_sel, (size_t)n_rows * 2 * sizeof(int32_t), hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(weights_out, w.m_wt, (size_t)n_rows * 2 * sizeof(float), hipMemcpyDeviceToHost));
    return RS_OK;
}

int32_t rs_release_source_weights(rs_ctx *c, int32_t layer) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    if (layer < 0 || layer >= c->m.n_layers) return fail(RS_ERR_BAD_ARG, "layer %d out of range", layer);
    if (!c->have_weights[layer]) return fail(RS_ERR_STATE, "weights of layer %d not set", layer);
    const rs_model_desc &m = c->m;
    const int d = m.d_model, qd = m.n_q_heads * m.head_dim, nqkv = qd + 2 * m.n_kv_heads * m.head_dim, f = m.ffn_dim;
    // every pass of more than 64 rows must qualify for the large-tile kernel (K a multiple of 32, N >= 1024);
    // passes of up to 64 rows always take the weight-streaming kernel: both read the packed copies only
    const bool packed_only = d % 32 == 0 && qd % 32 == 0 && f % 32 == 0 && nqkv >= 1024 && d >= 1024 && f >= 1024;
    if (!packed_only)
        return fail(RS_ERR_STATE, "this shape still reads the caller's matrices (generic GEMM kernel for K %% 32 != 0 or N < 1024)");
    if (c->gpu) {
        HIP_TRY(hipSetDevice(c->device));
        HIP_TRY(hipDeviceSynchronize());
    }
    rs_layer_weights &w = c->weights[layer];
    w.wqkv = w.wo = w.wg = w.wu = w.wd = nullptr;
    return RS_OK;
}

int32_t rs_set_head(rs_ctx *c, const rs_head_weights *w) {
    if (!c || !w) return fail(RS_ERR_BAD_ARG, "null argument");
    if (w->vocab < 1) return fail(RS_ERR_BAD_ARG, "vocab %d", w->vocab);
    if (c->gpu) {
        if (!w->embed || !w->final_norm || !w->lm_head) return fail(RS_ERR_BAD_ARG, "null head pointer");
        HIP_TRY(hipSetDevice(c->device));
        HIP_TRY(hipDeviceSynchronize());   // the packed copy and the partial-sum buffers may be in use
        drop_step_graphs(c);
        const int d = c->m.d_model;
        if (c->packed_lm) { (void)hipFree(c->packed_lm); c->packed_lm = nullptr; }
        HIP_TRY(hipMalloc((void **)&c->packed_lm, packed_weight_elems(w->vocab, d) * sizeof(bf16_t)));
        launch_pack_weights(nullptr, (const bf16_t *)w->lm_head, c->packed_lm, w->vocab, d);
        for (int s = 0; s < 2; ++s) {
            if (c->head_part[s]) { (void)hipFree(c->head_part[s]); c->head_part[s] = nullptr; }
            if (c->ws[s].rows > 0) {
                // more than 64 rows per call and a shape the large-tile kernel takes: groups of up to 256 rows
                const bool big = c->ws[s].rows > 64 && d % 32 == 0 && w->vocab >= 1024 && w->vocab % 4 == 0;
                c->head_group[s] = big ? std::min(c->ws[s].rows, RS_HEAD_GROUP) : 64;
                const size_t elems = std::max(skinny_partial_elems(64, w->vocab, d, EPI_STORE), (size_t)c->head_group[s] * w->vocab);
                HIP_TRY(hipMalloc((void **)&c->head_part[s], elems * sizeof(float)));
            }
        }
        if (!c->d_tok) {
            const size_t ns = (size_t)c->n_slots, mc = (size_t)c->lim.max_context, nb = std::max(1, c->lim.max_decode_batch);
            HIP_TRY(hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking));
            HIP_TRY(hipMalloc((void **)&c->d_tok, ns * sizeof(int32_t)));
            HIP_TRY(hipMemset(c->d_tok, 0, ns * sizeof(int32_t)));
            HIP_TRY(hipMalloc((void **)&c->d_prompts, ns * mc * sizeof(int32_t)));
            HIP_TRY(hipHostMalloc((void **)&c->h_first, ns * sizeof(int32_t)));
            HIP_TRY(hipMalloc((void **)&c->d_pslots, RS_MAX_PREFILL_REQS * sizeof(int32_t)));
            HIP_TRY(hipMalloc((void **)&c->d_pfirst, RS_MAX_PREFILL_REQS * sizeof(int32_t)));
            HIP_TRY(hipHostMalloc((void **)&c->h_pslots, RS_MAX_PREFILL_REQS * sizeof(int32_t)));
            HIP_TRY(hipHostMalloc((void **)&c->h_pfirst, RS_MAX_PREFILL_REQS * sizeof(int32_t)));
            // decode rows, and behind them (hybrid batching) the prompts that end in the same step
            const size_t nr = nb + RS_MAX_PREFILL_REQS;
            HIP_TRY(hipMalloc((void **)&c->d_rowslot, nr * sizeof(int32_t)));
            HIP_TRY(hipMalloc((void **)&c->d_sampled, nr * sizeof(int32_t)));
            for (int i = 0; i < 2; ++i) {
                HIP_TRY(hipHostMalloc((void **)&c->h_rowslot[i], nr * sizeof(int32_t)));
                HIP_TRY(hipHostMalloc((void **)&c->h_sampled[i], nr * sizeof(int32_t)));
                HIP_TRY(hipEventCreateWithFlags(&c->sampled_ev[i], hipEventDisableTiming));
            }
        }
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipDeviceSynchronize());
    }
    c->head = *w;
    c->have_head = true;
    return RS_OK;
}

int32_t rs_embed(rs_ctx *c, int32_t side, const int32_t *tokens, int32_t n, void *x_out) {
    int32_t rc = check_head_call(c, side, n);
    if (rc) return rc;
    if (!tokens || !x_out) return fail(RS_ERR_BAD_ARG, "null argument");
    HIP_TRY(hipSetDevice(c->device));
    launch_embed(c->side[side].stream, EmbedArgs{tokens, nullptr, (const bf16_t *)c->head.embed, (bf16_t *)x_out, c->err_flag + side, n,
                                                 c->m.d_model, c->head.vocab});
    HIP_TRY(hipGetLastError());
    return RS_OK;
}

int32_t rs_lm_head_greedy(rs_ctx *c, int32_t side, const void *x, int32_t n, float *logits_out, int32_t *tokens_out) {
    int32_t rc = check_head_call(c, side, n);
    if (rc) return rc;
    if (!x) return fail(RS_ERR_BAD_ARG, "null x");
    HIP_TRY(hipSetDevice(c->device));
    return head_greedy(c, side, (const bf16_t *)x, n, logits_out, tokens_out, nullptr, nullptr);
}

int32_t rs_kv_alloc(rs_ctx *c, int64_t req_id, int32_t n_tokens_total, int32_t *block_ids_out, int32_t cap,
                    int32_t *n_blocks_out) {
    if (!c || !n_blocks_out || (cap > 0 && !block_ids_out) || cap < 0) return fail(RS_ERR_BAD_ARG, "null argument");
    if (n_tokens_total < 0) return fail(RS_ERR_BAD_ARG, "negative token count");
    const int need = (n_tokens_total + RS_KV_BLOCK - 1) / RS_KV_BLOCK;
    auto it = c->owned.find(req_id);
    const int have = it == c->owned.end() ? 0 : (int)it->second.size();
    if (std::max(need, have) > cap) return fail(RS_ERR_BAD_ARG, "id buffer of %d too small for %d blocks", cap, std::max(need, have));
    const std::vector<int32_t> *v = nullptr;
    int32_t rc = kv_alloc(c, req_id, n_tokens_total, &v);
    if (rc) return rc;
    std::copy(v->begin(), v->end(), block_ids_out);
    *n_blocks_out = (int32_t)v->size();
    return RS_OK;
}

int32_t rs_kv_free(rs_ctx *c, int64_t req_id) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    auto it = c->owned.find(req_id);
    if (it == c->owned.end()) return fail(RS_ERR_BAD_ARG, "request %lld owns no blocks", (long long)req_id);
    for (auto b = it->second.rbegin(); b != it->second.rend(); ++b) c->free_list.push_back(*b);
    c->owned.erase(it);
    return RS_OK;
}

int32_t rs_kv_num_free(rs_ctx *c, int32_t *n) {
    if (!c || !n) return fail(RS_ERR_BAD_ARG, "null argument");
    *n = (int32_t)c->free_list.size();
    return RS_OK;
}

int32_t rs_prefill_layer(rs_ctx *c, int32_t layer, const void *x_in, void *x_out, const int32_t *cu_seqlens,
                         int32_t n_req, const int32_t *block_tables, int32_t max_blk) {
    int32_t rc = check_layer_call(c, RS_SIDE_PREFILL, layer, x_in, x_out, block_tables);
    if (rc) return rc;
    return prefill_layer(c, layer, x_in, x_out, cu_seqlens, n_req, block_tables, max_blk);
}

int32_t rs_decode_layer(rs_ctx *c, int32_t layer, const void *x_in, void *x_out, const int32_t *ctx_lens,
                        const int32_t *block_tables, int32_t max_blk, int32_t B, int32_t max_ctx) {
    int32_t rc = check_layer_call(c, RS_SIDE_DECODE, layer, x_in, x_out, block_tables);
    if (rc) return rc;
    return decode_layer(c, c->ws[RS_SIDE_DECODE], layer, x_in, x_out, ctx_lens, block_tables, max_blk, B, max_ctx);
}

int32_t rs_hybrid_layer(rs_ctx *c, int32_t layer, const void *x_in, void *x_out, const int32_t *cu_seqlens,
                        const int32_t *start_pos, int32_t n_req, const int32_t *prefill_tables, int32_t max_blk_prefill,
                        const int32_t *ctx_lens, const int32_t *decode_tables, int32_t max_blk_decode, int32_t B,
                        int32_t max_ctx) {
    int32_t rc = check_layer_call(c, RS_SIDE_PREFILL, layer, x_in, x_out, prefill_tables);
    if (rc) return rc;
    return hybrid_layer(c, layer, x_in, x_out, cu_seqlens, start_pos, n_req, prefill_tables, max_blk_prefill, ctx_lens,
                        decode_tables, max_blk_decode, B, max_ctx);
}

int32_t rs_decode_layer_noalloc(rs_ctx *c, int32_t layer, const void *x_in, void *x_out, const int32_t *ctx_lens,
                                const int32_t *block_tables, int32_t max_blk, int32_t B, int32_t max_ctx) {
    int32_t rc = check_layer_call(c, RS_SIDE_DECODE, layer, x_in, x_out, block_tables);
    if (rc) return rc;
    if (c->moe[layer].E > 0) return fail(RS_ERR_STATE, "layer %d has a sparse feed-forward block: not served from the static scratch", layer);
    if (B < 1 || max_ctx < 1) return fail(RS_ERR_BAD_ARG, "decode batch %d, max_ctx %d", B, max_ctx);
    unsigned char *base = (unsigned char *)g_static_scratch[c->device];
    if (!base) return fail(RS_ERR_STATE, "the static scratch array of device %d was not resolved", c->device);
    Workspace w;
    size_t packed = 0;
    const size_t need = carve_decode_ws(c, w, base, B, max_ctx, &packed);
    if (need > RS_STATIC_SCRATCH_BYTES)
        return fail(RS_ERR_BAD_ARG, "a step of %d rows over contexts up to %d needs %zu bytes of scratch; the static array holds %zu",
                    B, max_ctx, need, (size_t)RS_STATIC_SCRATCH_BYTES);
    // the array keeps the last call's contents, in that call's layout: the padding of the packed GEMM inputs
    // must read as zero (a fill kernel, not a memset: the call may be recorded into a graph)
    launch_fill_zero(c->side[RS_SIDE_DECODE].stream, base, packed);
    return decode_layer(c, w, layer, x_in, x_out, ctx_lens, block_tables, max_blk, B, max_ctx);
}

int32_t rs_decode_layer_graph(rs_ctx *c, int32_t layer, const void *x_in, void *x_out, const int32_t *ctx_lens,
                              const int32_t *block_tables, int32_t max_blk, int32_t B, int32_t max_ctx_bucket) {
    int32_t rc = check_layer_call(c, RS_SIDE_DECODE, layer, x_in, x_out, block_tables);
    if (rc) return rc;
    if (max_ctx_bucket < 1 || (max_ctx_bucket % RS_DECODE_CHUNK && max_ctx_bucket != c->lim.max_context))
        return fail(RS_ERR_BAD_ARG, "max_ctx_bucket %d: a multiple of %d, or the context limit %d", max_ctx_bucket,
                    RS_DECODE_CHUNK, c->lim.max_context);
    hipStream_t st = c->side[RS_SIDE_DECODE].stream;
    const rs_ctx::GraphKey key{layer, max_blk, B, max_ctx_bucket, x_in, x_out, ctx_lens, block_tables, st};
    auto it = c->graphs.find(key);
    if (it == c->graphs.end()) {
        if (c->graphs.size() >= 256) return fail(RS_ERR_STATE, "256 captured decode steps are cached already");
        hipGraph_t graph = nullptr;
        hipGraphExec_t exec = nullptr;
        HIP_TRY(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
        c->capturing = true;
        rc = decode_layer(c, c->ws[RS_SIDE_DECODE], layer, x_in, x_out, ctx_lens, block_tables, max_blk, B, max_ctx_bucket);
        c->capturing = false;
        const hipError_t e = hipStreamEndCapture(st, &graph);
        if (rc) {
            if (graph) (void)hipGraphDestroy(graph);
            return rc;
        }
        HIP_TRY(e);
        const hipError_t ei = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        HIP_TRY(ei);
        it = c->graphs.emplace(key, exec).first;
    }
    c->last_rows[RS_SIDE_DECODE] = B;
    HIP_TRY(hipGraphLaunch(it->second, st));
    return RS_OK;
}

int32_t rs_set_step_graphs(rs_ctx *c, int32_t on) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    if (c->engine) return fail(RS_ERR_STATE, "the engine's threads drive this context");
    c->step_graphs_on = on != 0;
    c->step_graph_cap = on > 1 ? on : 512;
    return RS_OK;
}

int32_t rs_step_graph_stats(rs_ctx *c, int64_t stats_out[4]) {
    if (!c || !stats_out) return fail(RS_ERR_BAD_ARG, "null argument");
    stats_out[0] = c->step_graph_captures;
    stats_out[1] = c->step_graph_launches;
    stats_out[2] = c->steps_enqueued;
    stats_out[3] = c->step_enqueue_ns;
    return RS_OK;
}

int32_t rs_debug_cu_histogram_graph(rs_ctx *c, int32_t side, int32_t n_workgroups, int32_t *hist_out) {
    if (!c || !hist_out || side < 0 || side > 1 || n_workgroups < 1 || n_workgroups > (1 << 20))
        return fail(RS_ERR_BAD_ARG, "bad argument");
    if (!c->gpu) return fail(RS_ERR_STATE, "host-only context");
    if (c->side[side].cus <= 0) return fail(RS_ERR_STATE, "side has no compute units");
    hipStream_t st = c->side[side].stream;
    int32_t *d = nullptr;
    HIP_TRY(hipMalloc(&d, RS_CU_HIST_BINS * sizeof(int32_t)));
    auto run = [&]() -> int32_t {
        HIP_TRY(hipMemset(d, 0, RS_CU_HIST_BINS * sizeof(int32_t)));   // outside the capture
        HIP_TRY(hipStreamSynchronize(st));
        hipGraph_t graph = nullptr;
        hipGraphExec_t exec = nullptr;
        HIP_TRY(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
        launch_cu_probe(st, d, n_workgroups);
        HIP_TRY(hipStreamEndCapture(st, &graph));
        const hipError_t ei = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        HIP_TRY(ei);
        const hipError_t el = hipGraphLaunch(exec, st);
        const hipError_t es = hipStreamSynchronize(st);
        (void)hipGraphExecDestroy(exec);
        HIP_TRY(el);
        HIP_TRY(es);
        HIP_TRY(hipMemcpy(hist_out, d, RS_CU_HIST_BINS * sizeof(int32_t), hipMemcpyDeviceToHost));
        return RS_OK;
    };
    const int32_t rc = run();
    (void)hipFree(d);
    return rc;
}

int32_t rs_set_cu_split(rs_ctx *c, int32_t p, int32_t d) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    return set_split(c, p, d);
}

int32_t rs_get_cu_split(rs_ctx *c, int32_t *p, int32_t *d) {
    if (!c || !p || !d) return fail(RS_ERR_BAD_ARG, "null argument");
    *p = c->side[0].cus;
    *d = c->side[1].cus;
    return RS_OK;
}

int32_t rs_get_cu_mask(rs_ctx *c, int32_t side, uint32_t mask_out[8]) {
    if (!c || !mask_out || side < 0 || side > 1) return fail(RS_ERR_BAD_ARG, "bad argument");
    mask_for(side, c->side[side].cus, mask_out);
    return RS_OK;
}

int32_t rs_choose_split(rs_ctx *c, int32_t batch, int64_t sum_ctx, int32_t prefill_pending, int32_t *p, int32_t *d) {
    if (!c || !p || !d) return fail(RS_ERR_BAD_ARG, "null argument");
    choose_split(c, batch, sum_ctx, prefill_pending != 0, p, d);
    return RS_OK;
}

int32_t rs_get_stream(rs_ctx *c, int32_t side, void **out) {
    if (!c || !out || side < 0 || side > 1) return fail(RS_ERR_BAD_ARG, "bad argument");
    if (!c->gpu) return fail(RS_ERR_STATE, "host-only context has no streams");
    *out = (void *)c->side[side].stream;
    return RS_OK;
}

int32_t rs_sync(rs_ctx *c, int32_t side) {
    if (!c || side < 0 || side > 1) return fail(RS_ERR_BAD_ARG, "bad argument");
    if (!c->gpu) return RS_OK;
    hipStream_t st = c->side[side].stream;
    if (!st) return RS_OK;
    // the side's own error word, copied and cleared on the side's own stream: nothing here waits for the other side
    HIP_TRY(hipMemcpyAsync(&c->h_err[side], c->err_flag + side, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    int32_t flag = c->h_err[side] | (side == RS_SIDE_DECODE ? c->step_err : 0);
    if (side == RS_SIDE_DECODE) c->step_err = 0;
    if (c->h_err[side]) {
        HIP_TRY(hipMemsetAsync(c->err_flag + side, 0, sizeof(int32_t), st));
        HIP_TRY(hipStreamSynchronize(st));
    }
    return flag ? report_flag(flag) : RS_OK;
}

int32_t rs_mark(rs_ctx *c, int32_t side, int32_t slot) {
    if (!c || side < 0 || side > 1 || slot < 0 || slot >= RS_MAX_MARKS) return fail(RS_ERR_BAD_ARG, "bad argument");
    if (!c->gpu) return fail(RS_ERR_STATE, "host-only context");
    hipEvent_t &e = c->side[side].marks[slot];
    if (!e) HIP_TRY(hipEventCreate(&e));
    HIP_TRY(hipEventRecord(e, c->side[side].stream));
    return RS_OK;
}

int32_t rs_mark_done(rs_ctx *c, int32_t side, int32_t slot, int32_t *done_out) {
    if (!c || !done_out || side < 0 || side > 1 || slot < 0 || slot >= RS_MAX_MARKS) return fail(RS_ERR_BAD_ARG, "bad argument");
    if (!c->gpu) return fail(RS_ERR_STATE, "host-only context");
    hipEvent_t e = c->side[side].marks[slot];
    if (!e) return fail(RS_ERR_STATE, "mark not recorded");
    const hipError_t q = hipEventQuery(e);
    if (q != hipSuccess && q != hipErrorNotReady) HIP_TRY(q);
    *done_out = q == hipSuccess ? 1 : 0;
    return RS_OK;
}

int32_t rs_elapsed_ms(rs_ctx *c, int32_t side_a, int32_t a, int32_t side_b, int32_t b, float *ms) {
    if (!c || !ms || side_a < 0 || side_a > 1 || side_b < 0 || side_b > 1 || a < 0 || b < 0 || a >= RS_MAX_MARKS ||
        b >= RS_MAX_MARKS)
        return fail(RS_ERR_BAD_ARG, "bad argument");
    if (!c->gpu) return fail(RS_ERR_STATE, "host-only context");
    hipEvent_t ea = c->side[side_a].marks[a], eb = c->side[side_b].marks[b];
    if (!ea || !eb) return fail(RS_ERR_STATE, "mark not recorded");
    HIP_TRY(hipEventSynchronize(ea));
    HIP_TRY(hipEventSynchronize(eb));
    HIP_TRY(hipEventElapsedTime(ms, ea, eb));
    return RS_OK;
}

int32_t rs_set_kernel_timing(rs_ctx *c, int32_t on) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    if (!c->gpu) return fail(RS_ERR_STATE, "host-only context");
    c->kernel_timing = on != 0;
    c->side[0].kt_valid = c->side[1].kt_valid = false;
    return RS_OK;
}

int32_t rs_kernel_times(rs_ctx *c, int32_t side, float ms_out[RS_N_KERNEL_SLOTS]) {
    if (!c || !ms_out || side < 0 || side > 1) return fail(RS_ERR_BAD_ARG, "bad argument");
    if (!c->gpu) return fail(RS_ERR_STATE, "host-only context");
    Side &s = c->side[side];
    if (!s.kt_valid) return fail(RS_ERR_STATE, "no timed layer call on this side yet");
    HIP_TRY(hipEventSynchronize(s.kt[RS_N_KERNEL_SLOTS]));
    for (int i = 0; i < RS_N_KERNEL_SLOTS; ++i) HIP_TRY(hipEventElapsedTime(&ms_out[i], s.kt[i], s.kt[i + 1]));
    return RS_OK;
}

int32_t rs_debug_read_workspace(rs_ctx *c, int32_t side, int32_t which, void *host_out, int64_t n_bytes) {
    if (!c || !host_out || side < 0 || side > 1 || n_bytes < 0) return fail(RS_ERR_BAD_ARG, "bad argument");
    if (!c->gpu) return fail(RS_ERR_STATE, "host-only context");
    const Workspace &w = c->ws[side];
    const rs_model_desc &m = c->m;
    const size_t qd = (size_t)m.n_q_heads * m.head_dim, nqkv = qd + 2 * (size_t)m.n_kv_heads * m.head_dim;
    const void *src = nullptr;
    size_t cap = 0;
    switch (which) {
        case 0:
            if (side == RS_SIDE_DECODE && c->decode_fused)
                return fail(RS_ERR_STATE, "this decode step folded its RMSNorms into the projections: no normalised rows were written");
            src = w.h; cap = (size_t)w.rows * m.d_model * 2; break;  // (decode buffers are at least 64 rows)
        case 1: src = w.qkv; cap = (size_t)w.rows * nqkv * 2; break;
        case 2: src = w.attn; cap = (size_t)w.rows * qd * 2; break;
        case 3: src = w.x1; cap = (size_t)w.rows * m.d_model * 2; break;
        case 4: src = w.act; cap = (size_t)w.rows * m.ffn_dim * 2; break;
        default: return fail(RS_ERR_BAD_ARG, "unknown workspace buffer %d", which);
    }
    if (!src || (size_t)n_bytes > cap) return fail(RS_ERR_BAD_ARG, "workspace buffer %d holds %zu bytes", which, cap);
    if (c->side[side].stream) HIP_TRY(hipStreamSynchronize(c->side[side].stream));
    if (which == 0 || which == 2 || which == 4) {
        // undo the fragment-packed layout of the GEMM inputs: row-major out
        const int width = which == 0 ? m.d_model : which == 2 ? (int)qd : m.ffn_dim;
        const int rows = (int)((size_t)n_bytes / 2 / width);
        const int Mt = packed_mt(c->last_rows[side]);
        if (c->last_rows[side] < 1 || rows > c->last_rows[side])
            return fail(RS_ERR_BAD_ARG, "the side's last layer call had %d rows", c->last_rows[side]);
        std::vector<uint16_t> raw((size_t)Mt * 32 * ((width + 15) / 16 * 16));
        HIP_TRY(hipMemcpy(raw.data(), src, raw.size() * 2, hipMemcpyDeviceToHost));
        uint16_t *dst = (uint16_t *)host_out;
        for (int r = 0; r < rows; ++r)
            for (int k = 0; k < width; ++k) dst[(size_t)r * width + k] = raw[packed_offset(r, k, Mt) + (k & 7)];
        return RS_OK;
    }
    HIP_TRY(hipMemcpy(host_out, src, (size_t)n_bytes, hipMemcpyDeviceToHost));
    return RS_OK;
}

int32_t rs_debug_stream_read(rs_ctx *c, int32_t side, const void *buf, int64_t n_bytes, float *ms_out) {
    if (!c || !buf || !ms_out || side < 0 || side > 1 || n_bytes < 32768 || n_bytes % 16) return fail(RS_ERR_BAD_ARG, "bad argument");
    if (!c->gpu) return fail(RS_ERR_STATE, "host-only context");
    if (c->side[side].cus <= 0) return fail(RS_ERR_STATE, "side has no compute units");
    hipStream_t st = c->side[side].stream;
    int32_t rc = rs_mark(c, side, RS_MAX_MARKS - 4);
    if (rc) return rc;
    launch_stream_read(st, buf, (size_t)n_bytes, c->side[side].cus * 16);
    rc = rs_mark(c, side, RS_MAX_MARKS - 3);
    if (rc) return rc;
    return rs_elapsed_ms(c, side, RS_MAX_MARKS - 4, side, RS_MAX_MARKS - 3, ms_out);
}

int32_t rs_debug_mfma_probe(rs_ctx *c, int32_t side, float *tflops_out) {
    if (!c || !tflops_out || side < 0 || side > 1) return fail(RS_ERR_BAD_ARG, "bad argument");
    if (!c->gpu) return fail(RS_ERR_STATE, "host-only context");
    if (c->side[side].cus <= 0) return fail(RS_ERR_STATE, "side has no compute units");
    hipStream_t st = c->side[side].stream;
    float *sink = (float *)c->ws[side].partials;   // never written (the kernel's store is dead by construction)
    if (!sink) sink = (float *)c->err_flag;
    const int wgs = c->side[side].cus * 2;
    (void)launch_mfma_probe(st, sink, wgs, 2000);                     // warm-up: clocks settle under the load
    int32_t rc = rs_mark(c, side, RS_MAX_MARKS - 4);
    if (rc) return rc;
    const double flops = launch_mfma_probe(st, sink, wgs, 40000);   // about 10 ms
    rc = rs_mark(c, side, RS_MAX_MARKS - 3);
    if (rc) return rc;
    float ms = 0.f;
    rc = rs_elapsed_ms(c, side, RS_MAX_MARKS - 4, side, RS_MAX_MARKS - 3, &ms);
    if (rc) return rc;
    *tflops_out = (float)(flops / (ms * 1e-3) / 1e12);
    return RS_OK;
}

int32_t rs_debug_cu_histogram(rs_ctx *c, int32_t side, int32_t n_workgroups, int32_t *hist_out) {
    if (!c || !hist_out || side < 0 || side > 1 || n_workgroups < 1 || n_workgroups > (1 << 20))
        return fail(RS_ERR_BAD_ARG, "bad argument");
    if (!c->gpu) return fail(RS_ERR_STATE, "host-only context");
    if (c->side[side].cus <= 0) return fail(RS_ERR_STATE, "side has no compute units");
    int32_t *d = nullptr;
    HIP_TRY(hipMalloc(&d, RS_CU_HIST_BINS * sizeof(int32_t)));
    hipStream_t st = c->side[side].stream;
    hipError_t e = hipMemsetAsync(d, 0, RS_CU_HIST_BINS * sizeof(int32_t), st);
    if (e == hipSuccess) {
        launch_cu_probe(st, d, n_workgroups);
        e = hipMemcpyAsync(hist_out, d, RS_CU_HIST_BINS * sizeof(int32_t), hipMemcpyDeviceToHost, st);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(d);
    if (e != hipSuccess) return fail(RS_ERR_HIP, "cu probe: %s", hipGetErrorString(e));
    return RS_OK;
}

// ---------------------------------------------------------------------------- serving step

int32_t rs_submit(rs_ctx *c, int64_t req_id, int32_t prompt_len, int32_t output_len, const void *prompt_hidden) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    if (req_id < 0) return fail(RS_ERR_BAD_ARG, "request ids are non-negative");
    if (prompt_len < 1 || output_len < 1) return fail(RS_ERR_BAD_ARG, "prompt_len and output_len must be >= 1");
    if (c->gpu && !prompt_hidden) return fail(RS_ERR_BAD_ARG, "null prompt_hidden");
    if (c->reqs.count(req_id)) return fail(RS_ERR_BAD_ARG, "request %lld already known", (long long)req_id);
    if (prompt_len + output_len > c->lim.max_context || prompt_len + output_len > c->m.max_pos)
        return fail(RS_ERR_BAD_ARG, "prompt+output %d exceeds max_context/max_pos", prompt_len + output_len);
    if (c->gpu && prompt_len > c->ws[RS_SIDE_PREFILL].rows) return fail(RS_ERR_BAD_ARG, "prompt longer than max_prefill_tokens");
    int32_t mrc = enter_mode(c, 1);
    if (mrc) return mrc;
    Request r{};
    r.id = req_id;
    r.prompt_len = prompt_len;
    r.output_len = output_len;
    r.prompt_hidden = prompt_hidden;
    c->reqs[req_id] = r;
    c->arrival.push_back(req_id);
    return RS_OK;
}

int32_t rs_decode_batch_ids(rs_ctx *c, int64_t *ids_out, int32_t cap, int32_t *n_out) {
    if (!c || !n_out || cap < 0 || (cap > 0 && !ids_out)) return fail(RS_ERR_BAD_ARG, "null argument");
    if ((int)c->last_batch.size() > cap) return fail(RS_ERR_BAD_ARG, "id buffer of %d too small for %d rows", cap, (int)c->last_batch.size());
    std::copy(c->last_batch.begin(), c->last_batch.end(), ids_out);
    *n_out = (int32_t)c->last_batch.size();
    return RS_OK;
}

int32_t rs_request_state(rs_ctx *c, int64_t req_id) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    if (c->engine_ever) {
        std::lock_guard<std::mutex> lr(c->res_mu);
        auto ir = c->results.find(req_id);
        if (ir == c->results.end()) return fail(RS_ERR_BAD_ARG, "unknown request");
        return ir->second->state.load(std::memory_order_acquire);
    }
    auto it = c->reqs.find(req_id);
    if (it == c->reqs.end()) return fail(RS_ERR_BAD_ARG, "unknown request");
    return it->second.state;
}

int32_t rs_debug_complete_prefill(rs_ctx *c, int64_t req_id) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    if (c->gpu) return fail(RS_ERR_STATE, "only for host-only contexts");
    auto it = c->reqs.find(req_id);
    if (it == c->reqs.end() || it->second.state != PREFILLING) return fail(RS_ERR_STATE, "request is not prefilling");
    c->prefill_host_done = true;   // the whole pass the request is part of
    return RS_OK;
}

// ---- the serving step, for hidden-state requests (rs_step) and token requests (rs_step_tokens) ----
namespace {

int32_t out_count(const Request &r) { return (int32_t)r.toks.size() - r.prompt_len; }

void set_state(Request &r, int st) {
    r.state = st;
    if (r.res) r.res->state.store(st, std::memory_order_release);
}

// A sampled token reaches the host: kept unless the request already has its last token.
void accept_token(rs_ctx *c, Request &r, int32_t tok) {
    if (r.complete) return;
    r.toks.push_back(tok);
    r.t_last = c->now();
    if (out_count(r) == 1) r.t_first = r.t_last;
    if ((c->head.eos_token >= 0 && tok == c->head.eos_token) || out_count(r) >= r.output_len) r.complete = true;
    if (r.res) {   // token, then times, then the count that makes them visible, then the end flag
        const int32_t n = out_count(r);
        r.res->toks[n - 1] = tok;
        r.res->t_last.store(r.t_last, std::memory_order_relaxed);
        if (n == 1) r.res->t_first.store(r.t_first, std::memory_order_relaxed);
        r.res->n.store(n, std::memory_order_release);
        if (r.complete) r.res->finished.store(1, std::memory_order_release);
    }
}

int32_t next_injected(Request &r) {
    if (r.injected.empty()) return 0;
    const int32_t t = r.injected.front();
    r.injected.pop_front();
    return t;
}

// Reads the tokens of the decode step staged in buffer f (its copy must have completed).
void harvest(rs_ctx *c, int f) {
    if (!c->pending[f]) return;
    for (size_t i = 0; i < c->inflight[f].size(); ++i) {
        Request &r = c->reqs[c->inflight[f][i]];
        if ((int)i >= c->inflight_nb[f]) {   // hybrid batching: a prompt whose last part rode in that step
            set_state(r, PREFILL_DONE);
            r.ctx_len = r.n_prefill;
        }
        accept_token(c, r, c->gpu ? c->h_sampled[f][i] : next_injected(r));
    }
    if (c->gpu) c->step_err |= c->h_err[2 + f];   // reported by the serving step that harvested it
    c->pending[f] = false;
    c->inflight[f].clear();
}

// Oldest first; with must = false only what has already arrived.
int32_t harvest_ready(rs_ctx *c, bool must) {
    const int order[2] = {c->stage_flip ^ 1, c->stage_flip};
    for (int f : order) {
        if (!c->pending[f]) continue;
        if (c->gpu) {
            if (must) HIP_TRY(hipEventSynchronize(c->sampled_ev[f]));
            else {
                hipError_t q = hipEventQuery(c->sampled_ev[f]);
                if (q == hipErrorNotReady) return RS_OK;   // the newer one cannot be ready either
                if (q != hipSuccess) return fail(RS_ERR_HIP, "hipEventQuery: %s", hipGetErrorString(q));
            }
        }
        harvest(c, f);
    }
    return RS_OK;
}

bool in_flight(const rs_ctx *c, int64_t id) {
    for (int f = 0; f < 2; ++f)
        if (c->pending[f] && std::find(c->inflight[f].begin(), c->inflight[f].end(), id) != c->inflight[f].end()) return true;
    return false;
}

void release_request(rs_ctx *c, Request &r) {
    if (c->engine) c->dead.push_back(r.id);
    set_state(r, FINISHED);
    rs_kv_free(c, r.id);
    if (r.done) { (void)hipEventDestroy(r.done); r.done = nullptr; }
    if (r.slot >= 0) { c->free_slots.push_back(r.slot); r.slot = -1; }
}

bool wants_retire(const Request &r) {
    return r.token_mode ? (r.complete || r.n_sampled >= r.output_len) : r.generated >= r.output_len;
}

int retire_finished(rs_ctx *c) {
    int n = 0;
    for (size_t i = 0; i < c->running.size();) {
        Request &r = c->reqs[c->running[i]];
        if (wants_retire(r)) {
            release_request(c, r);
            c->running.erase(c->running.begin() + i);
            ++n;
        } else {
            ++i;
        }
    }
    return n;
}

// One prefill pass over several whole token prompts on the prefill side's current stream: block tables and
// slots staged, embedding, every layer, then the head on each prompt's last row.  The chosen tokens are in
// c->h_pfirst[0..n) (prompt order) once the stream has reached the end of what is enqueued here; each
// request's token cell is written too.
struct PromptItem {
    int32_t slot, n_tok;
    const std::vector<int32_t> *blocks;
};
int32_t enqueue_prompts(rs_ctx *c, const PromptItem *items, int n, hipEvent_t wait_for) {
    const int mb = c->max_blk_per_req;
    hipStream_t st = c->side[RS_SIDE_PREFILL].stream;
    Workspace &w = c->ws[RS_SIDE_PREFILL];
    HIP_TRY(hipEventSynchronize(c->pstaged));   // the staging buffers' previous contents have been copied
    int32_t cu[RS_MAX_PREFILL_REQS + 1];
    cu[0] = 0;
    SeqInfo seq{};
    seq.n_req = n;
    for (int q = 0; q < n; ++q) {
        cu[q + 1] = cu[q] + items[q].n_tok;
        c->h_pslots[q] = items[q].slot;
        const std::vector<int32_t> &ids = *items[q].blocks;
        for (int j = 0; j < mb; ++j) c->h_ptab[(size_t)q * mb + j] = j < (int)ids.size() ? ids[j] : -1;
    }
    for (int q = 0; q <= n; ++q) seq.cu[q] = cu[q];
    const int T = cu[n];
    if (wait_for) {
        std::lock_guard<std::mutex> hold(c->capture_mu);   // not while the decode stream is recording a step
        HIP_TRY(hipStreamWaitEvent(st, wait_for, 0));
    }
    HIP_TRY(hipMemcpyAsync(c->d_ptab, c->h_ptab, (size_t)n * mb * sizeof(int32_t), hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(c->d_pslots, c->h_pslots, n * sizeof(int32_t), hipMemcpyHostToDevice, st));
    HIP_TRY(hipEventRecord(c->pstaged, st));
    EmbedArgs ea{c->d_prompts, nullptr, (const bf16_t *)c->head.embed, w.xbuf, c->err_flag + RS_SIDE_PREFILL, T, c->m.d_model, c->head.vocab};
    ea.slots = c->d_pslots;
    ea.slot_stride = c->lim.max_context;
    ea.seq = seq;
    launch_embed(st, ea);
    for (int l = 0; l < c->m.n_layers; ++l) {
        if (!c->have_weights[l]) return fail(RS_ERR_STATE, "weights of layer %d not set", l);
        int32_t rc = prefill_layer(c, l, w.xbuf, w.xbuf, cu, n, c->d_ptab, mb);
        if (rc) return rc;
    }
    launch_gather_last_rows(st, w.xbuf, w.x1, c->m.d_model, seq);   // x1 is free once the layers are enqueued
    int32_t rc = head_greedy(c, RS_SIDE_PREFILL, w.x1, n, nullptr, c->d_pfirst, c->d_pslots, c->d_tok);
    if (rc) return rc;
    HIP_TRY(hipMemcpyAsync(c->h_pfirst, c->d_pfirst, n * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(&c->h_err[4], c->err_flag + RS_SIDE_PREFILL, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    return RS_OK;
}

int32_t serve_step(rs_ctx *c, const rs_step_in *in, rs_step_out *out, bool token_mode) {
    *out = rs_step_out{};
    out->prefill_started_req = -1;
    out->decode_ms = -1.f;
    if (c->hybrid_chunk && !token_mode) return fail(RS_ERR_STATE, "hybrid batching serves token requests only (rs_step_tokens)");
    const int maxB = c->lim.max_decode_batch;
    if (c->gpu) HIP_TRY(hipSetDevice(c->device));

    // 0. tokens of earlier steps that have reached the host, and the error bits their kernels raised
    if (token_mode) {
        int32_t rc = harvest_ready(c, false);
        if (rc) return rc;
    }
    if (c->step_err) {
        const int32_t flag = c->step_err;
        c->step_err = 0;
        return report_flag(flag);
    }
    // 1a. the prefill "notification": event completed -> PREFILL_DONE
    if (c->engine) {
        DoneMsg dm;
        while (c->fin_q.pop(dm)) {
            c->n_prefill_inflight--;
            if (dm.rc) return fail(dm.rc, "the prefill thread failed on request %lld", (long long)dm.id);
            Request &r = c->reqs[dm.id];
            set_state(r, PREFILL_DONE);
            r.ctx_len = r.n_prefill;
            accept_token(c, r, c->gpu ? dm.token : next_injected(r));
            if (wants_retire(r)) { release_request(c, r); out->n_finished++; }
        }
    } else if (!c->prefill_ids.empty()) {
        bool done = c->prefill_host_done;
        if (c->gpu) {
            hipError_t q = hipEventQuery(c->prefill_ev);
            if (q == hipSuccess) done = true;
            else if (q != hipErrorNotReady) return fail(RS_ERR_HIP, "hipEventQuery: %s", hipGetErrorString(q));
        }
        if (done) {
            c->prefill_host_done = false;
            if (c->gpu && token_mode) c->step_err |= c->h_err[4];
            for (size_t i = 0; i < c->prefill_ids.size(); ++i) {
                Request &r = c->reqs[c->prefill_ids[i]];
                set_state(r, PREFILL_DONE);
                r.ctx_len = token_mode ? r.n_prefill : r.prompt_len;
                if (token_mode) {   // the prefill's own token
                    accept_token(c, r, c->gpu ? c->h_pfirst[i] : next_injected(r));
                    if (wants_retire(r)) { release_request(c, r); out->n_finished++; }
                }
            }
            c->prefill_ids.clear();
        }
    }
    if (c->hybrid_chunk)   // hybrid batching: first tokens arrive with the harvest; a request they end goes here
        for (int64_t id : c->arrival) {
            Request &r = c->reqs[id];
            if (r.state == PREFILL_DONE && wants_retire(r)) { release_request(c, r); out->n_finished++; }
        }
    // 1b. retire requests that produced all their tokens
    out->n_finished += retire_finished(c);
    while (!c->arrival.empty() && c->reqs[c->arrival.front()].state == FINISHED) c->arrival.pop_front();
    // engine: the application reads results from the Result records, so the decode thread's own table entry of a
    // finished request goes as soon as no staged step still names it (the table would otherwise grow for ever)
    for (size_t i = 0; i < c->dead.size();) {
        const int64_t id = c->dead[i];
        if (in_flight(c, id) || std::find(c->arrival.begin(), c->arrival.end(), id) != c->arrival.end()) { ++i; continue; }
        c->reqs.erase(id);
        c->dead[i] = c->dead.back();
        c->dead.pop_back();
    }
    // 1c. promote finished prefills into the decode batch, FCFS
    for (int64_t id : c->arrival) {
        Request &r = c->reqs[id];
        if (r.state == PREFILL_DONE && (int)c->running.size() < maxB) {
            set_state(r, RUNNING);
            c->running.push_back(id);
            out->n_promoted++;
        }
    }
    // 2. blocks for waiting requests in arrival order (stop at the first that does not fit)
    for (int64_t id : c->arrival) {
        Request &r = c->reqs[id];
        if (r.state != WAITING) continue;
        if (kv_alloc(c, id, token_mode ? r.n_prefill : r.prompt_len, nullptr) != RS_OK) break;
        set_state(r, PREFILL_READY);
    }

    // 3. room for every running request's next token; in token mode a request that cannot grow
    //    sends the most recently arrived running request back to WAITING (recomputation)
    bool synced = false;
    for (size_t i = 0; i < c->running.size();) {
        Request &r = c->reqs[c->running[i]];
        if (kv_alloc(c, r.id, r.ctx_len + 1, nullptr) == RS_OK) { ++i; continue; }
        if (!token_mode)
            return fail(RS_ERR_NO_BLOCKS, "no block to grow request %lld (hidden-state requests are not preempted)", (long long)r.id);
        if (!synced) {   // the victim's sequence must be complete on the host; late tokens may also end requests
            int32_t rc = harvest_ready(c, true);
            if (rc) return rc;
            out->n_finished += retire_finished(c);
            synced = true;
            i = 0;
            continue;
        }
        Request *vp = nullptr;
        for (auto it = c->arrival.rbegin(); it != c->arrival.rend() && !vp; ++it) {
            Request &q = c->reqs[*it];
            if (q.state == RUNNING || q.state == PREFILL_DONE || q.state == PREFILL_READY) vp = &q;
        }
        Request &v = *vp;   // exists: r itself is RUNNING
        if (v.id == r.id) {
            bool other = false;
            for (auto &kv : c->owned) other = other || (kv.first != r.id && !kv.second.empty());
            if (!other) return fail(RS_ERR_NO_BLOCKS, "request %lld alone does not fit the pool", (long long)r.id);
        }
        const int32_t n_all = (int32_t)v.toks.size();
        if (c->gpu && n_all > c->ws[RS_SIDE_PREFILL].rows)
            return fail(RS_ERR_NO_BLOCKS, "request %lld cannot be preempted: %d tokens exceed max_prefill_tokens", (long long)v.id, n_all);
        if (c->gpu && n_all > v.prompt_len) {   // generated tokens join the sequence to prefill
            HIP_TRY(hipMemcpyAsync(c->d_prompts + (size_t)v.slot * c->lim.max_context + v.prompt_len, v.toks.data() + v.prompt_len,
                                   (size_t)(n_all - v.prompt_len) * sizeof(int32_t), hipMemcpyHostToDevice, c->copy_stream));
            HIP_TRY(hipStreamSynchronize(c->copy_stream));
        }
        if (v.state == RUNNING) c->running.erase(std::find(c->running.begin(), c->running.end(), v.id));
        rs_kv_free(c, v.id);
        set_state(v, WAITING);
        v.n_prefill = n_all;
        v.ctx_len = 0;
        out->n_preempted++;
        i = 0;
    }
    for (int64_t id : c->arrival)
        if (c->reqs[id].state == WAITING) out->n_waiting++;

    // 4. the split for this step
    int64_t next_prefill = -1;
    if (c->prefill_ids.empty())
        for (int64_t id : c->arrival)
            if (c->reqs[id].state == PREFILL_READY) { next_prefill = id; break; }
    const bool prefill_pending = !c->prefill_ids.empty() || next_prefill >= 0 || c->n_prefill_inflight > 0;
    const int B = (int)c->running.size();
    int64_t sum_ctx = 0;
    for (int64_t id : c->running) sum_ctx += c->reqs[id].ctx_len;
    int32_t p, d;
    choose_split(c, B, sum_ctx, prefill_pending, &p, &d);
    const bool hyb = c->hybrid_chunk > 0;
    if (hyb) p = d = RS_TOTAL_CUS;   // one batch, the whole chip
    if (B == 0 && !prefill_pending) { p = c->engine ? c->prefill_cus_pub.load() : c->side[0].cus; d = c->side[1].cus; }
    else {
        int32_t rc = set_split(c, p, d);
        if (rc) return rc;
    }
    out->prefill_cus = p;
    out->decode_cus = d;
    out->decode_batch = B;
    out->decode_sum_ctx = sum_ctx;

    // a prefill started below may have been given blocks released above, which the decode step enqueued by
    // the previous call may still write: it is ordered behind that step
    const int prev_end = c->step_end_idx;

    // 5h. hybrid batching: this step's budget of prompt tokens is filled in arrival order -- the rest of the prompt
    //     in progress, then the next prompts that have their blocks, the last possibly in part (a part that does not
    //     end its prompt is whole blocks, so that the next one starts on a block boundary)
    struct Part { Request *r; int32_t start, n; bool last; };
    std::vector<Part> parts;
    if (hyb) {
        int budget = c->hybrid_chunk;
        while (budget > 0 && (int)parts.size() < RS_MAX_PREFILL_REQS) {
            Request *r = nullptr;
            const bool fresh = c->hyb_cur < 0;
            if (!fresh) r = &c->reqs[c->hyb_cur];
            else
                for (int64_t id : c->arrival)
                    if (c->reqs[id].state == PREFILL_READY) { r = &c->reqs[id]; break; }
            if (!r) break;
            const int32_t done = fresh ? 0 : r->chunk_done, rest = r->n_prefill - done;
            int32_t n = std::min(budget, rest);
            if (n < rest) n -= n % RS_KV_BLOCK;
            if (n == 0) break;
            if (fresh) {   // taken up with its first part
                r->n_sampled++;
                set_state(*r, PREFILLING);
                c->hyb_cur = r->id;
                if (out->prefill_started_req < 0) out->prefill_started_req = r->id;
                out->prefill_started_tokens += r->n_prefill;
                out->prefill_started_count++;
            }
            parts.push_back(Part{r, done, n, done + n == r->n_prefill});
            r->chunk_done = done + n;
            budget -= n;
            if (parts.back().last) c->hyb_cur = -1;
        }
    }
    c->last_parts.clear();
    int n_chunk = 0, F = 0;   // prompt rows of this step's batch; prompts that end in it
    for (const Part &pt : parts) {
        c->last_parts.push_back(rs_ctx::HybPart{pt.r->id, pt.start, pt.n});
        n_chunk += pt.n;
        F += pt.last;
    }
    out->n_chunks = (int32_t)parts.size();
    out->chunk_tokens = n_chunk;

    // 5. one decode step over the running batch (hybrid batching: and the chunk, in one batch)
    c->last_batch.assign(c->running.begin(), c->running.end());
    if (B > 0 || n_chunk > 0) {
        int max_ctx = 1;
        for (int64_t id : c->running) max_ctx = std::max(max_ctx, c->reqs[id].ctx_len + 1);
        const int nS = B + F;   // rows whose next token this step chooses
        const int flip = nS > 0 ? (c->stage_flip ^= 1) : c->stage_flip;
        if (nS > 0 && token_mode && c->pending[flip]) {   // the staging buffers are about to be rewritten
            if (c->gpu) HIP_TRY(hipEventSynchronize(c->sampled_ev[flip]));
            harvest(c, flip);
        }
        if (c->gpu) {
            if (nS > 0) HIP_TRY(hipEventSynchronize(c->staged[flip]));
            const int mb = c->max_blk_per_req;
            for (int i = 0; i < B; ++i) {
                Request &r = c->reqs[c->running[i]];
                c->h_ctx[flip][i] = r.ctx_len;
                if (token_mode) c->h_rowslot[flip][i] = r.slot;
                const std::vector<int32_t> &ids = c->owned[r.id];
                for (int j = 0; j < mb; ++j) c->h_tab[flip][(size_t)i * mb + j] = j < (int)ids.size() ? ids[j] : -1;
            }
            // a step with a chunk runs on the prefill side's stream and workspace (which holds chunk + batch rows),
            // a step without one is an ordinary decode step; consecutive steps on different streams are ordered
            const int sd = n_chunk > 0 ? RS_SIDE_PREFILL : RS_SIDE_DECODE;
            hipStream_t st = c->side[sd].stream;
            if (hyb) {
                if (c->hyb_prev_stream && c->hyb_prev_stream != st && c->step_end_valid[c->step_end_idx])
                    HIP_TRY(hipStreamWaitEvent(st, c->step_end[c->step_end_idx], 0));
                c->hyb_prev_stream = st;
            }
            {   // the slots of the prompts that end in this step follow the decode rows' (their first tokens are
                // chosen, copied back and harvested with the decode rows' tokens)
                int j = B;
                for (const Part &pt : parts)
                    if (pt.last) c->h_rowslot[flip][j++] = pt.r->slot;
            }
            if (nS > 0) {
                if (B > 0) {
                    HIP_TRY(hipMemcpyAsync(c->d_ctx, c->h_ctx[flip], B * sizeof(int32_t), hipMemcpyHostToDevice, st));
                    HIP_TRY(hipMemcpyAsync(c->d_tab, c->h_tab[flip], (size_t)B * mb * sizeof(int32_t), hipMemcpyHostToDevice, st));
                }
                if (token_mode)
                    HIP_TRY(hipMemcpyAsync(c->d_rowslot, c->h_rowslot[flip], nS * sizeof(int32_t), hipMemcpyHostToDevice, st));
                HIP_TRY(hipEventRecord(c->staged[flip], st));
            }
            int32_t pcu[RS_MAX_PREFILL_REQS + 1] = {0}, pstart[RS_MAX_PREFILL_REQS] = {0};
            if (n_chunk > 0) {   // block tables and slots of the prompts with a part in this step
                HIP_TRY(hipEventSynchronize(c->pstaged));
                for (size_t q = 0; q < parts.size(); ++q) {
                    const std::vector<int32_t> &ids = c->owned[parts[q].r->id];
                    for (int j = 0; j < mb; ++j) c->h_ptab[q * mb + j] = j < (int)ids.size() ? ids[j] : -1;
                    c->h_pslots[q] = parts[q].r->slot;
                    pcu[q + 1] = pcu[q] + parts[q].n;
                    pstart[q] = parts[q].start;
                }
                HIP_TRY(hipMemcpyAsync(c->d_ptab, c->h_ptab, parts.size() * mb * sizeof(int32_t), hipMemcpyHostToDevice, st));
                HIP_TRY(hipMemcpyAsync(c->d_pslots, c->h_pslots, parts.size() * sizeof(int32_t), hipMemcpyHostToDevice, st));
                HIP_TRY(hipEventRecord(c->pstaged, st));
            }
            if (in->wait_decode) { int32_t rc = rs_mark(c, sd, RS_MAX_MARKS - 2); if (rc) return rc; }
            Workspace &w = c->ws[sd];
            // the step's kernels: embedding (token mode), every layer, head (token mode)
            auto enqueue_kernels = [&](int ctx_bound) -> int32_t {
                if (n_chunk > 0) {   // hybrid batch: rows [0, n_chunk) the prompt parts, rows [n_chunk, n_chunk + B) the decode rows
                    const int dm = c->m.d_model, np = (int)parts.size();
                    SeqInfo seq{}, fin{};
                    seq.n_req = np;
                    for (int q = 0; q < np; ++q) {
                        seq.cu[q + 1] = pcu[q + 1];
                        seq.start[q] = pstart[q];
                        if (parts[q].last) fin.cu[++fin.n_req] = pcu[q + 1];   // the last row of a prompt that ends here
                    }
                    EmbedArgs ea{c->d_prompts, nullptr, (const bf16_t *)c->head.embed, w.xbuf, c->err_flag + sd, n_chunk, dm, c->head.vocab};
                    ea.slots = c->d_pslots;
                    ea.slot_stride = c->lim.max_context;
                    ea.seq = seq;
                    launch_embed(st, ea);
                    launch_embed(st, EmbedArgs{c->d_tok, c->d_rowslot, (const bf16_t *)c->head.embed, w.xbuf + (size_t)n_chunk * dm,
                                               c->err_flag + sd, B, dm, c->head.vocab});
                    for (int l = 0; l < c->m.n_layers; ++l) {
                        if (!c->have_weights[l]) return fail(RS_ERR_STATE, "weights of layer %d not set", l);
                        int32_t rc = hybrid_layer(c, l, w.xbuf, w.xbuf, pcu, pstart, np, c->d_ptab, mb, c->d_ctx, c->d_tab, mb, B, ctx_bound);
                        if (rc) return rc;
                    }
                    if (B > 0) {
                        int32_t rc = head_greedy(c, sd, w.xbuf + (size_t)n_chunk * dm, B, nullptr, c->d_sampled, c->d_rowslot, c->d_tok);
                        if (rc) return rc;
                    }
                    if (F > 0) {   // first tokens of the prompts that end here (x1 is free after the layers)
                        launch_gather_last_rows(st, w.xbuf, w.x1, dm, fin);
                        return head_greedy(c, sd, w.x1, F, nullptr, c->d_sampled + B, c->d_rowslot + B, c->d_tok);
                    }
                    return RS_OK;
                }
                const void *x_first = in->decode_hidden;
                void *x_out = in->decode_out;
                if (token_mode) {
                    launch_embed(st, EmbedArgs{c->d_tok, c->d_rowslot, (const bf16_t *)c->head.embed, w.xbuf, c->err_flag + RS_SIDE_DECODE, B,
                                               c->m.d_model, c->head.vocab});
                    x_first = w.xbuf;
                    x_out = w.xbuf;
                }
                for (int l = 0; l < c->m.n_layers; ++l) {
                    if (!c->have_weights[l]) return fail(RS_ERR_STATE, "weights of layer %d not set", l);
                    int32_t rc = decode_layer(c, w, l, l == 0 ? x_first : (const void *)x_out, x_out, c->d_ctx, c->d_tab, mb, B, ctx_bound);
                    if (rc) return rc;
                }
                if (token_mode) return head_greedy(c, RS_SIDE_DECODE, w.xbuf, B, nullptr, c->d_sampled, c->d_rowslot, c->d_tok);
                return RS_OK;
            };
            const auto t_enq = std::chrono::steady_clock::now();
            bool captured_now = false;
            if (token_mode && c->step_graphs_on && n_chunk == 0) {
                // Section 4.5.2: decode steps are captured as graphs per batch size and replayed.  The key is
                // (batch, context bucket, masked stream): the captured launches bake in the batch, a bound on the
                // contexts (a multiple of 512 tokens) and the stream's CU mask; everything else they read --
                // tokens, context lengths, block tables -- sits in library buffers refreshed before every launch.
                const int cap = std::min(c->lim.max_context, c->m.max_pos);
                const int bucket = std::min(((max_ctx + RS_DECODE_CHUNK - 1) / RS_DECODE_CHUNK) * RS_DECODE_CHUNK, cap);
                const auto key = std::make_tuple((int32_t)B, (int32_t)bucket, st);
                auto it = c->step_graphs.find(key);
                if (it == c->step_graphs.end()) {
                    if ((int)c->step_graphs.size() >= c->step_graph_cap) {   // set-up work either way; start over
                        // a replay of a cached graph may still be running: wait for the streams they were recorded on
                        std::vector<hipStream_t> seen;
                        for (auto &kv : c->step_graphs) {
                            hipStream_t gs = std::get<2>(kv.first);
                            if (std::find(seen.begin(), seen.end(), gs) == seen.end()) {
                                seen.push_back(gs);
                                HIP_TRY(hipStreamSynchronize(gs));
                            }
                        }
                        drop_step_graphs(c);
                    }
                    hipGraph_t graph = nullptr;
                    hipGraphExec_t exec = nullptr;
                    int32_t rc;
                    hipError_t e;
                    {
                        std::lock_guard<std::mutex> hold(c->capture_mu);
                        HIP_TRY(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
                        c->capturing = true;
                        rc = enqueue_kernels(bucket);
                        c->capturing = false;
                        e = hipStreamEndCapture(st, &graph);
                    }
                    if (rc) {
                        if (graph) (void)hipGraphDestroy(graph);
                        return rc;
                    }
                    HIP_TRY(e);
                    const hipError_t ei = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
                    (void)hipGraphDestroy(graph);
                    HIP_TRY(ei);
                    it = c->step_graphs.emplace(key, exec).first;
                    c->step_graph_captures++;
                    captured_now = true;
                }
                HIP_TRY(hipGraphLaunch(it->second, st));
                c->step_graph_launches++;
            } else {
                const int32_t rc = enqueue_kernels(max_ctx);
                if (rc) return rc;
            }
            if (!captured_now) {   // steady state only: a step that recorded its graph is set-up work
                c->steps_enqueued++;
                c->step_enqueue_ns += std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - t_enq).count();
            }
            if (token_mode && nS > 0) {
                HIP_TRY(hipMemcpyAsync(c->h_sampled[flip], c->d_sampled, nS * sizeof(int32_t), hipMemcpyDeviceToHost, st));
                HIP_TRY(hipMemcpyAsync(&c->h_err[2 + flip], c->err_flag + sd, sizeof(int32_t), hipMemcpyDeviceToHost, st));
                HIP_TRY(hipEventRecord(c->sampled_ev[flip], st));
            }
            c->step_end_idx ^= 1;
            HIP_TRY(hipEventRecord(c->step_end[c->step_end_idx], st));
            c->step_end_valid[c->step_end_idx] = true;
            if (in->wait_decode) {
                int32_t rc = rs_mark(c, sd, RS_MAX_MARKS - 1);
                if (rc) return rc;
                rc = rs_elapsed_ms(c, sd, RS_MAX_MARKS - 2, sd, RS_MAX_MARKS - 1, &out->decode_ms);
                if (rc) return rc;
            }
        }
        if (token_mode && nS > 0) {
            c->inflight[flip].assign(c->running.begin(), c->running.end());
            c->inflight_nb[flip] = B;
            for (const Part &pt : parts)
                if (pt.last) c->inflight[flip].push_back(pt.r->id);
            c->pending[flip] = true;
        }
        for (int64_t id : c->running) {
            Request &r = c->reqs[id];
            r.ctx_len++;
            r.generated++;
            r.n_sampled++;
        }
        if (token_mode && in->wait_decode && nS > 0) {
            int32_t rc = harvest_ready(c, true);
            if (rc) return rc;
        }
    }
    if (hyb) return RS_OK;   // no separate prefill pass under hybrid batching

    // 6. engine: every request whose blocks are allocated goes to the prefill thread, in arrival order
    if (c->engine) {
        if (p > 0)
            for (int64_t id : c->arrival) {
                Request &r = c->reqs[id];
                if (r.state != PREFILL_READY) continue;
                PrefillMsg pm{id, r.slot, r.n_prefill, c->step_end_valid[prev_end] ? prev_end : -1,
                              new std::vector<int32_t>(c->owned[id])};
                if (!c->pre_q.push(pm)) { delete pm.blocks; break; }   // ring full: next step
                r.n_sampled++;
                set_state(r, PREFILLING);
                c->n_prefill_inflight++;
                if (out->prefill_started_req < 0) out->prefill_started_req = id;
                out->prefill_started_tokens += r.n_prefill;
                out->prefill_started_count++;
            }
        return RS_OK;
    }
    // 6. start the next prefill pass if the prefill side is idle: whole prompts in arrival order, as many as
    //    fit the prefill workspace (token requests; a hidden-state request runs alone)
    if (next_prefill >= 0 && c->side[RS_SIDE_PREFILL].cus > 0) {
        std::vector<int64_t> ids;
        int32_t total = 0;
        for (int64_t id : c->arrival) {
            Request &r = c->reqs[id];
            if (r.state != PREFILL_READY) continue;
            const int32_t n_tok = token_mode ? r.n_prefill : r.prompt_len;
            if (!ids.empty() && (!token_mode || total + n_tok > c->lim.max_prefill_tokens || (int)ids.size() >= RS_MAX_PREFILL_REQS)) break;
            ids.push_back(id);
            total += n_tok;
        }
        if (c->gpu) {
            hipStream_t st = c->side[RS_SIDE_PREFILL].stream;
            hipEvent_t wait_for = c->step_end_valid[prev_end] ? c->step_end[prev_end] : nullptr;
            if (token_mode) {
                std::vector<PromptItem> items;
                for (int64_t id : ids) items.push_back(PromptItem{c->reqs[id].slot, c->reqs[id].n_prefill, &c->owned[id]});
                int32_t rc = enqueue_prompts(c, items.data(), (int)items.size(), wait_for);
                if (rc) return rc;
            } else {
                Request &r = c->reqs[ids[0]];
                const int mb = c->max_blk_per_req;
                HIP_TRY(hipEventSynchronize(c->pstaged));
                const std::vector<int32_t> &bl = c->owned[r.id];
                for (int j = 0; j < mb; ++j) c->h_ptab[j] = j < (int)bl.size() ? bl[j] : -1;
                if (wait_for) HIP_TRY(hipStreamWaitEvent(st, wait_for, 0));
                HIP_TRY(hipMemcpyAsync(c->d_ptab, c->h_ptab, mb * sizeof(int32_t), hipMemcpyHostToDevice, st));
                HIP_TRY(hipEventRecord(c->pstaged, st));
                const int32_t cu[2] = {0, r.prompt_len};
                Workspace &w = c->ws[RS_SIDE_PREFILL];
                for (int l = 0; l < c->m.n_layers; ++l) {
                    if (!c->have_weights[l]) return fail(RS_ERR_STATE, "weights of layer %d not set", l);
                    int32_t rc = prefill_layer(c, l, l == 0 ? r.prompt_hidden : (const void *)w.xbuf, w.xbuf, cu, 1, c->d_ptab, mb);
                    if (rc) return rc;
                }
            }
            HIP_TRY(hipEventRecord(c->prefill_ev, st));
        }
        for (int64_t id : ids) {
            Request &r = c->reqs[id];
            if (token_mode) r.n_sampled++;
            set_state(r, PREFILLING);
        }
        c->prefill_ids = ids;
        out->prefill_started_req = ids[0];
        out->prefill_started_tokens = total;
        out->prefill_started_count = (int32_t)ids.size();
    }
    return RS_OK;
}

}  // namespace

// ---- the two-thread engine (section 4.4) -------------------------------------------------------
namespace {

// Prefill thread: one pass over the prompts it has taken, then wait for it (this thread only).
int32_t engine_run_prompts(rs_ctx *c, const std::vector<PrefillMsg> &ms) {
    int32_t rc = set_side(c, RS_SIDE_PREFILL, c->prefill_cus_pub.load(std::memory_order_acquire));
    if (rc) return rc;
    if (c->side[RS_SIDE_PREFILL].cus <= 0) return fail(RS_ERR_STATE, "a prompt was handed over while the prefill side has no CUs");
    std::vector<PromptItem> items;
    int wait_idx = -1;
    for (const PrefillMsg &m : ms) {
        items.push_back(PromptItem{m.slot, m.n_tok, m.blocks});
        if (m.wait_idx >= 0) wait_idx = m.wait_idx;   // the newest message names the newest decode step to stay behind
    }
    // blocks released by the decode thread may still be written by the decode step it had in flight
    rc = enqueue_prompts(c, items.data(), (int)items.size(), wait_idx >= 0 ? c->step_end[wait_idx] : nullptr);
    if (rc) return rc;
    HIP_TRY(hipStreamSynchronize(c->side[RS_SIDE_PREFILL].stream));
    if (c->h_err[4]) return report_flag(c->h_err[4]);
    return RS_OK;
}

void engine_fail(rs_ctx *c, int32_t rc) {
    std::lock_guard<std::mutex> lk(c->res_mu);
    if (!c->eng_rc.load()) {
        c->eng_err = g_err;
        c->eng_rc.store(rc);
    }
}

void prefill_main(rs_ctx *c) {
    if (c->gpu) (void)hipSetDevice(c->device);
    std::vector<PrefillMsg> ms;
    for (;;) {
        PrefillMsg m;
        if (!c->pre_q.pop(m)) {
            if (c->stop_prefill.load(std::memory_order_acquire)) break;
            std::this_thread::sleep_for(std::chrono::microseconds(50));
            continue;
        }
        // first come first served, never chunked: as many whole prompts, in order, as fit the workspace
        ms.assign(1, m);
        int32_t total = m.n_tok;
        for (const PrefillMsg *nx; (nx = c->pre_q.front()) != nullptr;) {
            if (total + nx->n_tok > c->lim.max_prefill_tokens || (int)ms.size() >= RS_MAX_PREFILL_REQS) break;
            total += nx->n_tok;
            (void)c->pre_q.pop(m);
            ms.push_back(m);
        }
        int32_t rc = RS_OK;
        if (c->gpu) rc = engine_run_prompts(c, ms);
        if (rc) engine_fail(c, rc);
        for (size_t i = 0; i < ms.size(); ++i) {
            delete ms[i].blocks;
            const DoneMsg dm{ms[i].id, (c->gpu && !rc) ? c->h_pfirst[i] : 0, rc};
            while (!c->fin_q.push(dm)) std::this_thread::yield();
        }
    }
}

// Decode thread: a new request enters the table ("waiting" queue of the decode side).
int32_t engine_admit(rs_ctx *c, const SubmitMsg &m) {
    std::unique_ptr<std::vector<int32_t>> toks(m.toks), script(m.script);
    Request r{};
    r.id = m.id;
    r.prompt_len = m.prompt_len;
    r.output_len = m.max_new;
    r.token_mode = true;
    r.n_prefill = m.prompt_len;
    r.toks = std::move(*toks);
    r.t_submit = m.t_submit;
    r.res = m.res;
    if (script) r.injected.assign(script->begin(), script->end());
    if (c->free_slots.empty()) return fail(RS_ERR_STATE, "no request slot for %lld", (long long)m.id);   // submit keeps within n_slots
    r.slot = c->free_slots.back();
    c->free_slots.pop_back();
    if (c->gpu) {
        HIP_TRY(hipMemcpyAsync(c->d_prompts + (size_t)r.slot * c->lim.max_context, r.toks.data(), (size_t)r.prompt_len * sizeof(int32_t),
                               hipMemcpyHostToDevice, c->copy_stream));
        HIP_TRY(hipStreamSynchronize(c->copy_stream));
    }
    c->reqs[m.id] = std::move(r);
    c->arrival.push_back(m.id);
    return RS_OK;
}

void decode_main(rs_ctx *c) {
    if (c->gpu) (void)hipSetDevice(c->device);
    rs_step_in in{nullptr, nullptr, 0};
    rs_step_out out;
    for (;;) {
        int32_t rc = RS_OK;
        SubmitMsg sm;
        while (!rc && c->sub_q.pop(sm)) rc = engine_admit(c, sm);
        if (!rc) rc = serve_step(c, &in, &out, true);
        if (rc) { engine_fail(c, rc); break; }
        c->eng_steps.fetch_add(1, std::memory_order_relaxed);
        c->eng_finished.fetch_add(out.n_finished, std::memory_order_release);
        c->eng_preempted.fetch_add(out.n_preempted, std::memory_order_relaxed);
        if (c->stop.load(std::memory_order_acquire)) {
            const bool idle = c->arrival.empty() && c->n_prefill_inflight == 0 && c->sub_q.empty() && !c->pending[0] && !c->pending[1];
            if (!c->drain.load() || idle) break;
        }
        if (out.decode_batch == 0) std::this_thread::sleep_for(std::chrono::microseconds(50));
    }
    (void)harvest_ready(c, true);   // tokens of the last steps
}

}  // namespace

int32_t rs_engine_start(rs_ctx *c) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    if (c->engine) return fail(RS_ERR_STATE, "the engine is already running");
    if (!c->have_head) return fail(RS_ERR_STATE, "rs_set_head has not been called");
    if (!c->arrival.empty()) return fail(RS_ERR_STATE, "requests are live on this context");
    if (c->hybrid_chunk) return fail(RS_ERR_STATE, "hybrid batching is on: the engine threads serve with two sides");
    int32_t rc = enter_mode(c, 2);
    if (rc) return rc;
    if (c->gpu) {
        HIP_TRY(hipSetDevice(c->device));
        HIP_TRY(hipDeviceSynchronize());
    }
    c->stop.store(false);
    c->stop_prefill.store(false);
    c->drain.store(false);
    c->eng_rc.store(0);
    c->prefill_cus_pub.store(c->side[RS_SIDE_PREFILL].cus);
    c->engine = true;
    c->engine_ever = true;
    c->th_prefill = std::thread(prefill_main, c);
    c->th_decode = std::thread(decode_main, c);
    return RS_OK;
}

int32_t rs_engine_stop(rs_ctx *c, int32_t drain) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    if (!c->engine) return fail(RS_ERR_STATE, "the engine is not running");
    c->drain.store(drain != 0);
    c->stop.store(true, std::memory_order_release);
    c->th_decode.join();
    c->stop_prefill.store(true, std::memory_order_release);
    c->th_prefill.join();
    PrefillMsg pm;
    while (c->pre_q.pop(pm)) delete pm.blocks;
    SubmitMsg sm;
    while (c->sub_q.pop(sm)) { delete sm.toks; delete sm.script; }
    DoneMsg dm;
    while (c->fin_q.pop(dm)) {}
    c->engine = false;
    if (c->gpu) HIP_TRY(hipDeviceSynchronize());
    const int32_t rc = c->eng_rc.load();
    if (rc) {
        std::lock_guard<std::mutex> lk(c->res_mu);
        return fail(rc, "engine thread: %s", c->eng_err.c_str());
    }
    return RS_OK;
}

int32_t rs_engine_stats(rs_ctx *c, int64_t stats_out[4]) {
    if (!c || !stats_out) return fail(RS_ERR_BAD_ARG, "null argument");
    stats_out[0] = c->eng_submitted.load();
    stats_out[1] = c->eng_finished.load(std::memory_order_acquire);
    stats_out[2] = c->eng_steps.load();
    stats_out[3] = c->eng_preempted.load();
    const int32_t rc = c->eng_rc.load();
    if (rc) {
        std::lock_guard<std::mutex> lk(c->res_mu);
        return fail(rc, "engine thread: %s", c->eng_err.c_str());
    }
    return RS_OK;
}

int32_t rs_set_hybrid_batching(rs_ctx *c, int32_t chunk_tokens) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    if (c->engine) return fail(RS_ERR_STATE, "the engine threads serve with two sides; stop the engine first");
    if (!c->arrival.empty() || !c->running.empty() || !c->prefill_ids.empty())
        return fail(RS_ERR_STATE, "the batching scheme changes only while no request is in flight");
    if (chunk_tokens < 0 || chunk_tokens % RS_KV_BLOCK)
        return fail(RS_ERR_BAD_ARG, "chunk of %d tokens: 0 (off) or a multiple of %d", chunk_tokens, RS_KV_BLOCK);
    if (chunk_tokens > 0 && chunk_tokens + c->lim.max_decode_batch > c->lim.max_prefill_tokens)
        return fail(RS_ERR_BAD_ARG, "a chunk of %d tokens and %d decode rows exceed max_prefill_tokens %d", chunk_tokens,
                    c->lim.max_decode_batch, c->lim.max_prefill_tokens);
    c->hybrid_chunk = chunk_tokens;
    c->hyb_cur = -1;
    c->hyb_prev_stream = nullptr;
    c->last_parts.clear();
    return RS_OK;
}

int32_t rs_step_chunks(rs_ctx *c, int64_t *req_ids_out, int32_t *starts_out, int32_t *lens_out, int32_t cap, int32_t *n_out) {
    if (!c || !n_out) return fail(RS_ERR_BAD_ARG, "null argument");
    const int n = (int)c->last_parts.size();
    *n_out = n;
    if (n > cap) return fail(RS_ERR_BAD_ARG, "%d parts, room for %d", n, cap);
    for (int i = 0; i < n; ++i) {
        if (req_ids_out) req_ids_out[i] = c->last_parts[i].id;
        if (starts_out) starts_out[i] = c->last_parts[i].start;
        if (lens_out) lens_out[i] = c->last_parts[i].n;
    }
    return RS_OK;
}

int32_t rs_step(rs_ctx *c, const rs_step_in *in, rs_step_out *out) {
    if (!c || !in || !out) return fail(RS_ERR_BAD_ARG, "null argument");
    if (c->gpu && (!in->decode_hidden || !in->decode_out)) return fail(RS_ERR_BAD_ARG, "null decode buffers");
    if (c->engine) return fail(RS_ERR_STATE, "the engine's threads drive this context");
    int32_t rc = enter_mode(c, 1);
    if (rc) return rc;
    return serve_step(c, in, out, false);
}

int32_t rs_submit_tokens(rs_ctx *c, int64_t req_id, const int32_t *prompt_tokens, int32_t prompt_len, int32_t max_new_tokens) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    if (!c->have_head) return fail(RS_ERR_STATE, "rs_set_head has not been called");
    if (req_id < 0) return fail(RS_ERR_BAD_ARG, "request ids are non-negative");
    if (!prompt_tokens || prompt_len < 1 || max_new_tokens < 1) return fail(RS_ERR_BAD_ARG, "need a prompt and max_new_tokens >= 1");
    if (c->reqs.count(req_id)) return fail(RS_ERR_BAD_ARG, "request %lld already known", (long long)req_id);
    if (prompt_len + max_new_tokens > c->lim.max_context || prompt_len + max_new_tokens > c->m.max_pos)
        return fail(RS_ERR_BAD_ARG, "prompt+output %d exceeds max_context/max_pos", prompt_len + max_new_tokens);
    if (c->gpu && prompt_len > c->ws[RS_SIDE_PREFILL].rows) return fail(RS_ERR_BAD_ARG, "prompt longer than max_prefill_tokens");
    for (int i = 0; i < prompt_len; ++i)
        if (prompt_tokens[i] < 0 || prompt_tokens[i] >= c->head.vocab)
            return fail(RS_ERR_BAD_ARG, "prompt token %d at %d outside the vocabulary of %d", prompt_tokens[i], i, c->head.vocab);
    if (c->engine) {
        std::lock_guard<std::mutex> lk(c->sub_mu);   // among application threads only
        if (c->eng_submitted.load() - c->eng_finished.load(std::memory_order_acquire) >= c->n_slots)
            return fail(RS_ERR_STATE, "too many live requests (%d)", c->n_slots);
        Result *res;
        std::vector<int32_t> *script = nullptr;
        {
            std::lock_guard<std::mutex> lr(c->res_mu);
            if (c->results.count(req_id)) return fail(RS_ERR_BAD_ARG, "request %lld already known", (long long)req_id);
            auto up = std::make_unique<Result>();
            up->max_new = max_new_tokens;
            up->toks.reset(new int32_t[max_new_tokens]);
            up->t_submit.store(c->now());
            res = up.get();
            c->results[req_id] = std::move(up);
            auto ps = c->pre_scripts.find(req_id);
            if (ps != c->pre_scripts.end()) {
                script = new std::vector<int32_t>(std::move(ps->second));
                c->pre_scripts.erase(ps);
            }
        }
        SubmitMsg m{req_id, prompt_len, max_new_tokens, new std::vector<int32_t>(prompt_tokens, prompt_tokens + prompt_len), script, res,
                    res->t_submit.load()};
        if (!c->sub_q.push(m)) {
            delete m.toks;
            delete m.script;
            std::lock_guard<std::mutex> lr(c->res_mu);
            c->results.erase(req_id);
            return fail(RS_ERR_STATE, "submission queue full");
        }
        c->eng_submitted.fetch_add(1);
        return RS_OK;
    }
    if (c->engine_ever) return fail(RS_ERR_STATE, "this context was driven by the engine: start it again to submit");
    if (c->free_slots.empty()) return fail(RS_ERR_STATE, "too many live requests (%d)", c->n_slots);
    int32_t rc = enter_mode(c, 2);
    if (rc) return rc;
    Request r{};
    r.id = req_id;
    r.prompt_len = prompt_len;
    r.output_len = max_new_tokens;
    r.token_mode = true;
    r.n_prefill = prompt_len;
    r.toks.assign(prompt_tokens, prompt_tokens + prompt_len);
    r.t_submit = c->now();
    r.slot = c->free_slots.back();
    if (c->gpu) {
        HIP_TRY(hipSetDevice(c->device));
        // on a stream of its own that does not synchronise with others: a plain blocking copy would wait
        // for whatever prefill is in flight and hold up the caller's step loop for that long
        HIP_TRY(hipMemcpyAsync(c->d_prompts + (size_t)r.slot * c->lim.max_context, prompt_tokens,
                               (size_t)prompt_len * sizeof(int32_t), hipMemcpyHostToDevice, c->copy_stream));
        HIP_TRY(hipStreamSynchronize(c->copy_stream));
    }
    c->free_slots.pop_back();
    c->reqs[req_id] = std::move(r);
    c->arrival.push_back(req_id);
    return RS_OK;
}

int32_t rs_step_tokens(rs_ctx *c, int32_t wait_decode, rs_step_out *out) {
    if (!c || !out) return fail(RS_ERR_BAD_ARG, "null argument");
    if (!c->have_head) return fail(RS_ERR_STATE, "rs_set_head has not been called");
    if (c->engine) return fail(RS_ERR_STATE, "the engine's threads drive this context");
    int32_t rc = enter_mode(c, 2);
    if (rc) return rc;
    rs_step_in in{nullptr, nullptr, wait_decode};
    return serve_step(c, &in, out, true);
}

int32_t rs_request_output(rs_ctx *c, int64_t req_id, int32_t *tokens_out, int32_t cap, int32_t *n_out, int32_t *finished_out) {
    if (!c || !n_out || cap < 0 || (cap > 0 && !tokens_out)) return fail(RS_ERR_BAD_ARG, "null argument");
    if (c->engine_ever) {
        Result *res = nullptr;
        {
            std::lock_guard<std::mutex> lr(c->res_mu);
            auto ir = c->results.find(req_id);
            if (ir != c->results.end()) res = ir->second.get();
        }
        if (!res) return fail(RS_ERR_BAD_ARG, "unknown token request");
        const int32_t fin = res->finished.load(std::memory_order_acquire);   // before the count: a set flag means the count is final
        const int32_t n = res->n.load(std::memory_order_acquire);
        if (n > cap) return fail(RS_ERR_BAD_ARG, "buffer of %d too small for %d tokens", cap, n);
        std::copy(res->toks.get(), res->toks.get() + n, tokens_out);
        *n_out = n;
        if (finished_out) *finished_out = fin;
        return RS_OK;
    }
    auto it = c->reqs.find(req_id);
    if (it == c->reqs.end() || !it->second.token_mode) return fail(RS_ERR_BAD_ARG, "unknown token request");
    const Request &r = it->second;
    const int32_t n = out_count(r);
    if (n > cap) return fail(RS_ERR_BAD_ARG, "buffer of %d too small for %d tokens", cap, n);
    std::copy(r.toks.begin() + r.prompt_len, r.toks.end(), tokens_out);
    *n_out = n;
    if (finished_out) *finished_out = r.complete ? 1 : 0;
    return RS_OK;
}

int32_t rs_request_release(rs_ctx *c, int64_t req_id) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    if (c->engine_ever) {
        std::lock_guard<std::mutex> lr(c->res_mu);
        auto ir = c->results.find(req_id);
        if (ir == c->results.end()) return fail(RS_ERR_BAD_ARG, "unknown request");
        if (!ir->second->finished.load(std::memory_order_acquire) || ir->second->state.load(std::memory_order_acquire) != FINISHED)
            return fail(RS_ERR_STATE, "request %lld has not finished", (long long)req_id);
        c->results.erase(ir);
        return RS_OK;
    }
    auto it = c->reqs.find(req_id);
    if (it == c->reqs.end()) return fail(RS_ERR_BAD_ARG, "unknown request");
    if (it->second.state != FINISHED || in_flight(c, req_id))
        return fail(RS_ERR_STATE, "request %lld has not finished", (long long)req_id);
    c->arrival.erase(std::remove(c->arrival.begin(), c->arrival.end(), req_id), c->arrival.end());
    c->reqs.erase(it);
    return RS_OK;
}

int32_t rs_request_times(rs_ctx *c, int64_t req_id, double times_out[3]) {
    if (!c || !times_out) return fail(RS_ERR_BAD_ARG, "null argument");
    if (c->engine_ever) {
        std::lock_guard<std::mutex> lr(c->res_mu);
        auto ir = c->results.find(req_id);
        if (ir == c->results.end()) return fail(RS_ERR_BAD_ARG, "unknown token request");
        (void)ir->second->n.load(std::memory_order_acquire);
        times_out[0] = ir->second->t_submit.load();
        times_out[1] = ir->second->t_first.load();
        times_out[2] = ir->second->t_last.load();
        return RS_OK;
    }
    auto it = c->reqs.find(req_id);
    if (it == c->reqs.end() || !it->second.token_mode) return fail(RS_ERR_BAD_ARG, "unknown token request");
    times_out[0] = it->second.t_submit;
    times_out[1] = it->second.t_first;
    times_out[2] = it->second.t_last;
    return RS_OK;
}

int32_t rs_debug_push_sampled(rs_ctx *c, int64_t req_id, int32_t token) {
    if (!c) return fail(RS_ERR_BAD_ARG, "null context");
    if (c->gpu) return fail(RS_ERR_STATE, "only for host-only contexts");
    if (c->engine) {   // the table belongs to the decode thread: the script travels with the submission
        std::lock_guard<std::mutex> lr(c->res_mu);
        if (c->results.count(req_id)) return fail(RS_ERR_STATE, "with the engine running, queue a request's tokens before submitting it");
        c->pre_scripts[req_id].push_back(token);
        return RS_OK;
    }
    auto it = c->reqs.find(req_id);
    if (it == c->reqs.end() || !it->second.token_mode) return fail(RS_ERR_BAD_ARG, "unknown token request");
    it->second.injected.push_back(token);
    return RS_OK;
}

}  // extern "C"
