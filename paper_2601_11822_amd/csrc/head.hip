// Token boundary of the model: embedding lookup in front of the first layer, greedy choice behind
// the LM-head product (which runs in the weight-streaming GEMM and leaves float32 partial sums).
#include "kernels.h"

// ---------------------------------------------------------------------------------------------
// x[row][:] = E[token(row)][:].  One workgroup per row, 16-byte copies.  The token of a row is
// tokens[row], or tokens[row_slot[row]] when an indirection is given (the serving loop keeps one
// current token per request slot and a per-step row -> slot map).  A token outside the vocabulary
// is never used as an index: the row is zero-filled and the error flag raised.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void embed_kernel(EmbedArgs a) {
    const int row = blockIdx.x;
    int tok;
    if (a.slots) {
        int q = 0;
        while (q + 1 < a.seq.n_req && row >= a.seq.cu[q + 1]) ++q;
        tok = a.tokens[(size_t)a.slots[q] * a.slot_stride + a.seq.start[q] + (row - a.seq.cu[q])];
    } else {
        tok = a.tokens[a.row_slot ? a.row_slot[row] : row];
    }
    const bool ok = (unsigned)tok < (unsigned)a.vocab;
    if (!ok && threadIdx.x == 0) atomicOr(a.err_flag, 4);
    const bf16_t *src = a.table + (size_t)(ok ? tok : 0) * a.d;
    bf16_t *dst = a.x + (size_t)row * a.d;
    for (int c = threadIdx.x; c < (a.d >> 3); c += 256) st_bf16x8(dst + c * 8, ok ? ld_bf16x8(src + c * 8) : zero_bf16x8());
}

void launch_embed(hipStream_t st, const EmbedArgs &a) {
    if (a.n <= 0) return;
    hipLaunchKernelGGL(embed_kernel, dim3(a.n), dim3(256), 0, st, a);
}

__global__ __launch_bounds__(256) void gather_last_rows_kernel(const bf16_t *__restrict__ x, bf16_t *__restrict__ out, int d, SeqInfo seq) {
    const int q = blockIdx.x;
    const bf16_t *src = x + (size_t)(seq.cu[q + 1] - 1) * d;
    for (int c = threadIdx.x; c < (d >> 3); c += 256) st_bf16x8(out + (size_t)q * d + c * 8, ld_bf16x8(src + c * 8));
}

void launch_gather_last_rows(hipStream_t st, const bf16_t *x, bf16_t *out, int d, const SeqInfo &seq) {
    if (seq.n_req <= 0) return;
    hipLaunchKernelGGL(gather_last_rows_kernel, dim3(seq.n_req), dim3(256), 0, st, x, out, d, seq);
}

// ---------------------------------------------------------------------------------------------
// Greedy choice over one row of logits per workgroup.  logit(m, n) = sum over the S K-slices, in
// slice order, of part[s][m][n]; the chosen token is the lowest n among the row's maxima (the
// comparison is taken on the float32 sums; NaN never wins).  Optionally writes the float32 logits
// and scatters the token to tok_by_slot[row_slot[m]].
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void head_argmax_kernel(HeadArgmaxArgs a) {
    __shared__ float s_val[256];
    __shared__ int s_arg[256];
    const int m = blockIdx.x, tid = threadIdx.x;
    float best = -INFINITY;
    int arg = 0x7fffffff;
    auto take = [&](float v, int n) {
        if (v > best || (v == best && n < arg)) { best = v; arg = n; }
    };
    const int n4 = ((a.N & 3) == 0 && (a.Nv & 3) == 0) ? a.N : 0;   // vector path needs aligned rows
    for (int n = tid * 4; n < n4; n += 1024) {
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < a.S; ++s) v += *(const f32x4 *)(a.part + ((size_t)s * a.M + m) * a.Nv + n);
        if (a.logits) *(f32x4 *)(a.logits + (size_t)m * a.N + n) = v;
#pragma unroll
        for (int i = 0; i < 4; ++i) take(v[i], n + i);
    }
    for (int n = n4 + tid; n < a.N; n += 256) {
        float v = 0.f;
        for (int s = 0; s < a.S; ++s) v += a.part[((size_t)s * a.M + m) * a.Nv + n];
        if (a.logits) a.logits[(size_t)m * a.N + n] = v;
        take(v, n);
    }
    s_val[tid] = best;
    s_arg[tid] = arg;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (tid < o) {
            const float v = s_val[tid + o];
            const int g = s_arg[tid + o];
            if (v > s_val[tid] || (v == s_val[tid] && g < s_arg[tid])) { s_val[tid] = v; s_arg[tid] = g; }
        }
        __syncthreads();
    }
    if (tid == 0) {
        const int tok = s_arg[0] == 0x7fffffff ? 0 : s_arg[0];   // a row of NaNs: token 0
        if (a.tokens) a.tokens[m] = tok;
        if (a.tok_by_slot) a.tok_by_slot[a.row_slot ? a.row_slot[m] : m] = tok;
    }
}

void launch_head_argmax(hipStream_t st, const HeadArgmaxArgs &a) {
    if (a.M <= 0) return;
    hipLaunchKernelGGL(head_argmax_kernel, dim3(a.M), dim3(256), 0, st, a);
}
