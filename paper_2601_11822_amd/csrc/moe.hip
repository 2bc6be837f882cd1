// Sparse (mixture-of-experts) feed-forward block around the grouped form of the large-tile GEMM:
// route each row to its two experts, lay the (row, expert) assignments out expert by expert in
// whole 128-row tiles, gather the normalised rows into that order, run gate/up and down once over
// all tiles (each tile reads its own expert's weights), and add the two weighted results back.
#include "kernels.h"

// ---------------------------------------------------------------------------------------------
// Router: logits of row m = h[m] . Wr[e] for the E experts (h fragment-packed, Wr row-major), then
// the two largest (lower index first on ties) and the softmax over those two.  One workgroup per R
// consecutive rows, 256 / R threads per row.  R = 8 for long passes: in the packed layout the same
// 16-byte chunk of 8 consecutive rows is one 128-byte line, so the 8 threads that share a chunk index
// read whole lines (a row on its own touches 8 times the bytes it uses); R = 1 for short ones, where
// the number of workgroups and the short loop matter more.
// ---------------------------------------------------------------------------------------------
template <int R>
__global__ __launch_bounds__(256) void moe_router_kernel(MoeArgs a) {
    __shared__ float red[4][R][RS_MOE_MAX_EXPERTS];
    const int tid = threadIdx.x;
    const int r = tid % R, t = tid / R;   // row within the group, thread within the row
    const int m = blockIdx.x * R + r;
    const int Mt = packed_mt(a.M);
    const int mc = min(m, a.M - 1);
    float acc[RS_MOE_MAX_EXPERTS];
#pragma unroll
    for (int e = 0; e < RS_MOE_MAX_EXPERTS; ++e) acc[e] = 0.f;
    for (int c = t; c < (a.d >> 3); c += 256 / R) {
        const bf16x8 hv = ld_bf16x8(a.h + packed_offset(mc, c * 8, Mt));
#pragma unroll
        for (int e = 0; e < RS_MOE_MAX_EXPERTS; ++e) {
            if (e >= a.E) break;
            const bf16x8 wv = ld_bf16x8(a.router + (size_t)e * a.d + c * 8);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[e] += (float)hv[i] * (float)wv[i];
        }
    }
    // lanes with equal (lane % R) hold the same row: butterfly over the other lane bits, then the 4 waves
#pragma unroll
    for (int e = 0; e < RS_MOE_MAX_EXPERTS; ++e) {
        float v = acc[e];
#pragma unroll
        for (int o = 32; o >= R; o >>= 1) v += __shfl_xor(v, o, 64);
        if ((tid & 63) < R) red[tid >> 6][r][e] = v;
    }
    __syncthreads();
    if (tid < R && m < a.M) {
        float lg[RS_MOE_MAX_EXPERTS];
        for (int e = 0; e < a.E; ++e) lg[e] = (red[0][r][e] + red[1][r][e]) + (red[2][r][e] + red[3][r][e]);
        int e0 = 0;
        for (int e = 1; e < a.E; ++e)
            if (lg[e] > lg[e0]) e0 = e;
        int e1 = -1;
        for (int e = 0; e < a.E; ++e)
            if (e != e0 && (e1 < 0 || lg[e] > lg[e1])) e1 = e;
        const float eb = expf(lg[e1] - lg[e0]);
        a.sel[2 * m] = e0;
        a.sel[2 * m + 1] = e1;
        a.wt[2 * m] = 1.0f / (1.0f + eb);
        a.wt[2 * m + 1] = eb / (1.0f + eb);
    }
}

// ---------------------------------------------------------------------------------------------
// Plan (one workgroup): per-expert counts, each expert's segment padded to whole 128-row tiles (a
// segment of two or more tiles starts on a 256-row boundary, after an idle tile if need be, so that
// the grouped GEMM can take its tiles in pairs), the expert of every tile (-1 for a tile not in use), the source row of every grouped row
// (-1 for padding) and the grouped position of every assignment.  The order of rows inside a
// segment is arbitrary (an atomic cursor): a row's result does not depend on where it sits.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void moe_plan_kernel(MoeArgs a) {
    __shared__ int cnt[RS_MOE_MAX_EXPERTS], off[RS_MOE_MAX_EXPERTS], cur[RS_MOE_MAX_EXPERTS];
    const int tid = threadIdx.x;
    if (tid < RS_MOE_MAX_EXPERTS) cnt[tid] = cur[tid] = 0;
    __syncthreads();
    for (int i = tid; i < 2 * a.M; i += 1024) atomicAdd(&cnt[a.sel[i]], 1);
    for (int i = tid; i < a.Mg_cap; i += 1024) a.src[i] = -1;
    __syncthreads();
    if (tid == 0) {
        int t = 0;
        for (int e = 0; e < a.E; ++e) {
            const int nt = (cnt[e] + 127) >> 7;
            if (nt >= 2 && (t & 1)) a.tile_expert[t++] = -1;   // longer segments start on a 256-row boundary
            off[e] = t * 128;
            for (int j = 0; j < nt; ++j) a.tile_expert[t + j] = e;
            t += nt;
        }
        const int n128 = a.Mg_cap / 128;
        for (int j = t; j < n128; ++j) a.tile_expert[j] = -1;
        // the grouped GEMM's work list, behind the tile table: aligned pairs of one expert, else single tiles
        int32_t *units = a.tile_expert + n128;
        int nu = 0;
        for (int e = 0, j = 0; e < a.E; ++e) {
            const int nt = (cnt[e] + 127) >> 7;
            if (nt >= 2 && (j & 1)) ++j;
            int k = 0;
            for (; k + 2 <= nt && !((j + k) & 1); k += 2) units[1 + nu++] = 2 * (j + k) + 1;
            for (; k < nt; ++k) units[1 + nu++] = 2 * (j + k);
            j += nt;
        }
        units[0] = nu;
    }
    __syncthreads();
    for (int i = tid; i < 2 * a.M; i += 1024) {
        const int e = a.sel[i];
        const int p = off[e] + atomicAdd(&cur[e], 1);
        a.pos[i] = p;
        a.src[p] = i >> 1;
    }
}

// Gathered, fragment-packed GEMM input: grouped row g takes the chunks of its source row (zeros for padding).
__global__ __launch_bounds__(256) void moe_gather_kernel(MoeArgs a) {
    const int chunks = a.d >> 3;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)a.Mg_cap * chunks) return;
    // consecutive threads take consecutive rows of one k chunk: whole 128-byte lines on the writing side
    const int g = (int)(idx % a.Mg_cap), c = (int)(idx / a.Mg_cap);
    if (a.tile_expert[g >> 7] < 0) return;   // tile not in use: the GEMMs skip it too
    const int s = a.src[g];
    const bf16x8 v = s >= 0 ? ld_bf16x8(a.h + packed_offset(s, c * 8, packed_mt(a.M))) : zero_bf16x8();
    st_bf16x8(a.a_g + packed_offset(g, c * 8, a.Mg_cap >> 5), v);
}

// y[m] = x1[m] + w0 * out[pos0] + w1 * out[pos1], float32 arithmetic.  One workgroup per row.
__global__ __launch_bounds__(256) void moe_combine_kernel(MoeArgs a) {
    const int m = blockIdx.x;
    const float w0 = a.wt[2 * m], w1 = a.wt[2 * m + 1];
    const bf16_t *o0 = a.out_g + (size_t)a.pos[2 * m] * a.d, *o1 = a.out_g + (size_t)a.pos[2 * m + 1] * a.d;
    const bf16_t *xr = a.x1 + (size_t)m * a.d;
    bf16_t *yr = a.y + (size_t)m * a.d;
    for (int c = threadIdx.x; c < (a.d >> 3); c += 256) {
        const bf16x8 x = ld_bf16x8(xr + c * 8), p = ld_bf16x8(o0 + c * 8), q = ld_bf16x8(o1 + c * 8);
        bf16x8 r;
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] = (bf16_t)((float)x[i] + (w0 * (float)p[i] + w1 * (float)q[i]));
        st_bf16x8(yr + c * 8, r);
    }
}

void launch_moe_route_and_gather(hipStream_t st, const MoeArgs &a) {
    if (a.M <= 0) return;
    if (a.M >= 512)   // a function of the row count alone
        hipLaunchKernelGGL(moe_router_kernel<8>, dim3((a.M + 7) / 8), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(moe_router_kernel<1>, dim3(a.M), dim3(256), 0, st, a);
    hipLaunchKernelGGL(moe_plan_kernel, dim3(1), dim3(1024), 0, st, a);
    const long n = (long)a.Mg_cap * (a.d >> 3);
    hipLaunchKernelGGL(moe_gather_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a);
}

void launch_moe_combine(hipStream_t st, const MoeArgs &a) {
    if (a.M <= 0) return;
    hipLaunchKernelGGL(moe_combine_kernel, dim3(a.M), dim3(256), 0, st, a);
}
