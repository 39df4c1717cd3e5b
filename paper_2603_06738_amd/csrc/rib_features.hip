// RIB feature generator (paper Sec. 3.1 Eq. 1-3) and its backward.
//
// The work is tiny next to the attention it feeds (N <= 65536 tokens, 42 -> 32 -> heads*r
// features) and runs once per weight update, so these are plain vector-ALU kernels laid out
// for coalesced access and a fixed summation order, not for the matrix cores.
//
//   forward:  one workgroup per 64 tokens: Fourier features (fp64 sines / cosines of the
//             token's row and column coordinate, rounded to fp32) into LDS, the shared hidden
//             layer into LDS, then every (head, token, column) output as a d_h-long dot product.
//   backward: (1) the same two stages, kept in the workspace (r_in, h) together with
//             dpre = ReLU'(pre) * sum over heads of dF W_p^T;
//             (2) per 256-token chunk, one thread per weight-gradient element sums its chunk;
//             (3) chunks are added in ascending order.
#include <hip/hip_runtime.h>

#include "rib_common.h"

namespace rib {
namespace {

constexpr int kTok = 64;        // tokens per workgroup in the token-parallel kernels
constexpr int kChunk = 256;     // tokens per partial sum in the weight-gradient kernel
constexpr int kGenNT = 256;

struct Gen {
    int M, N, heads, r, L, d_h, n_in;
};

// Fourier features of the workgroup's tokens -> rin[kTok][n_in] (LDS).  One thread per
// (token, axis): coordinate in fp64, then 2L sines / cosines in fp64.
__device__ __forceinline__ void stage_fourier(const Gen &g, int n0, float *rin)
{
    for (int e = threadIdx.x; e < kTok * 2; e += kGenNT) {
        const int t = e >> 1, axis = e & 1, n = n0 + t;
        if (n >= g.N) continue;
        const int iy = n / g.M, ix = n - iy * g.M;
        const int i = axis == 0 ? iy : ix;
        const double x = g.M > 1 ? -1.0 + 2.0 * (double)i / (double)(g.M - 1) : 0.0;
        float *row = rin + t * g.n_in;
        row[axis] = (float)x;
        double f = 1.0;
        for (int l = 0; l < g.L; ++l) {
            double s, c;
            sincos(f * x, &s, &c);
            row[2 + 4 * l + axis] = (float)s;
            row[4 + 4 * l + axis] = (float)c;
            f *= 2.0;
        }
    }
}

// pre-activation of the shared hidden layer for (token t, unit c): r_in[t] . W_h[:, c] + b_h[c]
__device__ __forceinline__ float hidden_pre(const Gen &g, const float *rin_row, const float *__restrict__ W_h,
                                            const float *__restrict__ b_h, int c)
{
    float acc = b_h[c];
    for (int a = 0; a < g.n_in; ++a) acc = fmaf(rin_row[a], W_h[a * g.d_h + c], acc);
    return acc;
}

template <typename T>
__global__ __launch_bounds__(kGenNT) void features_fwd_kernel(Gen g, const float *__restrict__ W_h,
                                                              const float *__restrict__ b_h,
                                                              const float *__restrict__ W_pq,
                                                              const float *__restrict__ W_pk, T *__restrict__ f_q,
                                                              T *__restrict__ f_k)
{
    extern __shared__ float lds[];
    float *rin = lds, *hs = lds + kTok * g.n_in;
    const int n0 = blockIdx.x * kTok;
    const int live = min(kTok, g.N - n0);
    stage_fourier(g, n0, rin);
    __syncthreads();
    for (int e = threadIdx.x; e < live * g.d_h; e += kGenNT) {
        const int t = e / g.d_h, c = e - t * g.d_h;
        hs[t * g.d_h + c] = fmaxf(hidden_pre(g, rin + t * g.n_in, W_h, b_h, c), 0.f);
    }
    __syncthreads();
    // outputs: (which, head, token, column) with the column fastest
    const int per_head = live * g.r;
    for (int e = threadIdx.x; e < 2 * g.heads * per_head; e += kGenNT) {
        const int wh = e / per_head, rem = e - wh * per_head;
        const int which = wh / g.heads, hd = wh - which * g.heads;
        const int t = rem / g.r, j = rem - t * g.r;
        const float *W = (which ? W_pk : W_pq) + (size_t)hd * g.d_h * g.r + j;
        const float *h = hs + t * g.d_h;
        float acc = 0.f;
        for (int c = 0; c < g.d_h; ++c) acc = fmaf(h[c], W[c * g.r], acc);
        T *dst = (which ? f_k : f_q) + ((size_t)hd * g.N + n0 + t) * g.r + j;
        store_as(dst, acc);
    }
}

// Backward stage 1: r_in, h and dpre of every token into the workspace.
__global__ __launch_bounds__(kGenNT) void features_hidden_kernel(Gen g, const float *__restrict__ W_h,
                                                                 const float *__restrict__ b_h,
                                                                 const float *__restrict__ W_pq,
                                                                 const float *__restrict__ W_pk,
                                                                 const float *__restrict__ df_q,
                                                                 const float *__restrict__ df_k, float *__restrict__ ws_rin,
                                                                 float *__restrict__ ws_h, float *__restrict__ ws_dpre)
{
    extern __shared__ float lds[];
    float *rin = lds;
    const int n0 = blockIdx.x * kTok;
    const int live = min(kTok, g.N - n0);
    stage_fourier(g, n0, rin);
    __syncthreads();
    for (int e = threadIdx.x; e < live * g.n_in; e += kGenNT) ws_rin[(size_t)n0 * g.n_in + e] = rin[e];
    for (int e = threadIdx.x; e < live * g.d_h; e += kGenNT) {
        const int t = e / g.d_h, c = e - t * g.d_h;
        const float pre = hidden_pre(g, rin + t * g.n_in, W_h, b_h, c);
        // dh[t][c] = sum over heads and columns of dF_q W_pq + dF_k W_pk, heads ascending
        float dh = 0.f;
        for (int hd = 0; hd < g.heads; ++hd) {
            const float *gq = df_q + ((size_t)hd * g.N + n0 + t) * g.r;
            const float *gk = df_k + ((size_t)hd * g.N + n0 + t) * g.r;
            const float *wq = W_pq + ((size_t)hd * g.d_h + c) * g.r;
            const float *wk = W_pk + ((size_t)hd * g.d_h + c) * g.r;
            for (int j = 0; j < g.r; ++j) dh = fmaf(gq[j], wq[j], dh);
            for (int j = 0; j < g.r; ++j) dh = fmaf(gk[j], wk[j], dh);
        }
        ws_h[(size_t)n0 * g.d_h + e] = fmaxf(pre, 0.f);
        ws_dpre[(size_t)n0 * g.d_h + e] = pre > 0.f ? dh : 0.f;
    }
}

// Gradient elements in one flat index space:
//   [0, P)            dW_pq[hd][c][j]   = sum_n h[n][c]    dF_q[hd][n][j]       P = heads*d_h*r
//   [P, 2P)           dW_pk
//   [2P, 2P + I)      dW_h[a][c]        = sum_n r_in[n][a] dpre[n][c]           I = n_in*d_h
//   [2P + I, .. + d_h) db_h[c]          = sum_n dpre[n][c]
__device__ __forceinline__ int n_grad_elems(const Gen &g) { return 2 * g.heads * g.d_h * g.r + g.n_in * g.d_h + g.d_h; }

// Backward stage 2: partial[chunk][e] = the sum over the chunk's tokens, ascending.
__global__ __launch_bounds__(kGenNT) void features_wgrad_kernel(Gen g, const float *__restrict__ df_q,
                                                                const float *__restrict__ df_k,
                                                                const float *__restrict__ ws_rin,
                                                                const float *__restrict__ ws_h,
                                                                const float *__restrict__ ws_dpre, float *__restrict__ partial)
{
    const int e = blockIdx.x * kGenNT + threadIdx.x, total = n_grad_elems(g);
    if (e >= total) return;
    const int n0 = blockIdx.y * kChunk, n1 = min(g.N, n0 + kChunk);
    const int P = g.heads * g.d_h * g.r, I = g.n_in * g.d_h;
    const float *a, *b;          // the two factors, with their strides per token
    int sa, sb;
    if (e < 2 * P) {
        const int which = e >= P, ee = e - which * P;
        const int hd = ee / (g.d_h * g.r), rem = ee - hd * g.d_h * g.r, c = rem / g.r, j = rem - c * g.r;
        a = ws_h + c, sa = g.d_h;
        b = (which ? df_k : df_q) + (size_t)hd * g.N * g.r + j, sb = g.r;
    } else if (e < 2 * P + I) {
        const int ee = e - 2 * P, ai = ee / g.d_h, c = ee - ai * g.d_h;
        a = ws_rin + ai, sa = g.n_in;
        b = ws_dpre + c, sb = g.d_h;
    } else {
        a = nullptr, sa = 0;
        b = ws_dpre + (e - 2 * P - I), sb = g.d_h;
    }
    float acc = 0.f;
    if (a) {
#pragma unroll 8
        for (int n = n0; n < n1; ++n) acc = fmaf(a[(size_t)n * sa], b[(size_t)n * sb], acc);
    } else {
#pragma unroll 8
        for (int n = n0; n < n1; ++n) acc += b[(size_t)n * sb];
    }
    partial[(size_t)blockIdx.y * total + e] = acc;
}

// Backward stage 3: chunks ascending, scattered to the four gradient tensors.
__global__ __launch_bounds__(kGenNT) void features_reduce_kernel(Gen g, int nchunks, const float *__restrict__ partial,
                                                                 float *__restrict__ dW_h, float *__restrict__ db_h,
                                                                 float *__restrict__ dW_pq, float *__restrict__ dW_pk)
{
    const int e = blockIdx.x * kGenNT + threadIdx.x, total = n_grad_elems(g);
    if (e >= total) return;
    float acc = 0.f;
    for (int ch = 0; ch < nchunks; ++ch) acc += partial[(size_t)ch * total + e];
    const int P = g.heads * g.d_h * g.r, I = g.n_in * g.d_h;
    if (e < P) dW_pq[e] = acc;
    else if (e < 2 * P) dW_pk[e - P] = acc;
    else if (e < 2 * P + I) dW_h[e - 2 * P] = acc;
    else db_h[e - 2 * P - I] = acc;
}

bool make_gen(const rib_gen_params *p, Gen *g, rib_status *st)
{
    if (p == nullptr) return *st = RIB_ERR_NULL, false;
    if (p->window < 1 || p->window > 256 || p->heads < 1 || p->heads > 64 || p->r < 1 || p->r > 64 || p->L < 0 ||
        p->L > 16 || p->d_h < 1 || p->d_h > 64)
        return *st = RIB_ERR_SHAPE, false;
    if (p->dtype != RIB_F32 && p->dtype != RIB_BF16) return *st = RIB_ERR_DTYPE, false;
    g->M = p->window, g->N = p->window * p->window, g->heads = p->heads, g->r = p->r, g->L = p->L, g->d_h = p->d_h;
    g->n_in = 2 + 4 * p->L;
    return *st = RIB_OK, true;
}

struct GenWs {
    size_t rin_off, h_off, dpre_off, partial_off, total;
    int nchunks;
};

GenWs gen_ws_layout(const Gen &g)
{
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    GenWs l;
    l.nchunks = (g.N + kChunk - 1) / kChunk;
    const size_t elems = (size_t)2 * g.heads * g.d_h * g.r + (size_t)g.n_in * g.d_h + g.d_h;
    l.rin_off = 0;
    l.h_off = up((size_t)g.N * g.n_in * 4);
    l.dpre_off = l.h_off + up((size_t)g.N * g.d_h * 4);
    l.partial_off = l.dpre_off + up((size_t)g.N * g.d_h * 4);
    l.total = l.partial_off + up((size_t)l.nchunks * elems * 4);
    return l;
}

}  // namespace
}  // namespace rib

using namespace rib;

extern "C" {

rib_status rib_features_fwd(const rib_gen_params *p, const float *W_h, const float *b_h, const float *W_pq,
                            const float *W_pk, void *f_q, void *f_k, void *stream)
{
    Gen g;
    rib_status st;
    if (!make_gen(p, &g, &st)) return st;
    if (!W_h || !b_h || !W_pq || !W_pk || !f_q || !f_k) return RIB_ERR_NULL;
    const dim3 grid((unsigned)((g.N + kTok - 1) / kTok)), block(kGenNT);
    const size_t lds = (size_t)kTok * (g.n_in + g.d_h) * sizeof(float);
    hipStream_t s = (hipStream_t)stream;
    if (p->dtype == RIB_BF16)
        hipLaunchKernelGGL(features_fwd_kernel<bf16_t>, grid, block, lds, s, g, W_h, b_h, W_pq, W_pk, (bf16_t *)f_q,
                           (bf16_t *)f_k);
    else
        hipLaunchKernelGGL(features_fwd_kernel<float>, grid, block, lds, s, g, W_h, b_h, W_pq, W_pk, (float *)f_q,
                           (float *)f_k);
    return hipGetLastError() == hipSuccess ? RIB_OK : RIB_ERR_LAUNCH;
}

size_t rib_features_bwd_workspace_bytes(const rib_gen_params *p)
{
    Gen g;
    rib_status st;
    if (!make_gen(p, &g, &st)) return 0;
    return gen_ws_layout(g).total;
}

rib_status rib_features_bwd(const rib_gen_params *p, const float *W_h, const float *b_h, const float *W_pq,
                            const float *W_pk, const float *df_q, const float *df_k, float *dW_h, float *db_h,
                            float *dW_pq, float *dW_pk, void *workspace, size_t workspace_bytes, void *stream)
{
    Gen g;
    rib_status st;
    if (!make_gen(p, &g, &st)) return st;
    if (!W_h || !b_h || !W_pq || !W_pk || !df_q || !df_k || !dW_h || !db_h || !dW_pq || !dW_pk) return RIB_ERR_NULL;
    const GenWs l = gen_ws_layout(g);
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < l.total) return RIB_ERR_WORKSPACE;
    char *ws = (char *)workspace;
    float *ws_rin = (float *)(ws + l.rin_off), *ws_h = (float *)(ws + l.h_off), *ws_dpre = (float *)(ws + l.dpre_off),
          *partial = (float *)(ws + l.partial_off);
    hipStream_t s = (hipStream_t)stream;
    const int total = 2 * g.heads * g.d_h * g.r + g.n_in * g.d_h + g.d_h;
    hipLaunchKernelGGL(features_hidden_kernel, dim3((unsigned)((g.N + kTok - 1) / kTok)), dim3(kGenNT),
                       (size_t)kTok * g.n_in * sizeof(float), s, g, W_h, b_h, W_pq, W_pk, df_q, df_k, ws_rin, ws_h, ws_dpre);
    if (hipGetLastError() != hipSuccess) return RIB_ERR_LAUNCH;
    const unsigned eb = (unsigned)((total + kGenNT - 1) / kGenNT);
    hipLaunchKernelGGL(features_wgrad_kernel, dim3(eb, (unsigned)l.nchunks), dim3(kGenNT), 0, s, g, df_q, df_k, ws_rin, ws_h,
                       ws_dpre, partial);
    if (hipGetLastError() != hipSuccess) return RIB_ERR_LAUNCH;
    hipLaunchKernelGGL(features_reduce_kernel, dim3(eb), dim3(kGenNT), 0, s, g, l.nchunks, partial, dW_h, db_h, dW_pq, dW_pk);
    return hipGetLastError() == hipSuccess ? RIB_OK : RIB_ERR_LAUNCH;
}

}  // extern "C"
