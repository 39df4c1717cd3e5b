// Shared device/host declarations of the RIB window-attention library (gfx950).
// Internal header: the public interface is include/rib_attn.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rib_attn.h"

namespace rib {

// Problem geometry handed to every kernel by value.
struct Geo {
    int B, H, W, heads, d, r, M, s;
    int N;            // M*M tokens per window
    int nwx, nwy;     // windows per row / column of one image
    int C;            // heads*d
    int64_t tstride;  // elements between consecutive tokens of q, k, v
    float scale_c, scale_p;
    int64_t units;    // B*nwy*nwx*heads (window, head) pairs
    uint32_t inv_m;   // ceil(2^32 / M): n / M == mulhi(n, inv_m) for every n < 2^24 (M >= 2)
    // Gated epilogue (CLA, paper Eq. 9), forward only: when `gate` is set the kernels store
    // O * gate to their output and, if `out_raw` is set too, the ungated O there (both dense
    // [B][H][W][C] in the problem's storage type).  Null for the plain operator.
    const void *gate;
    void *out_raw;
    int flags;        // rib_params.flags
};

using bf16_t = uint16_t;  // raw bf16 storage

// Dynamic LDS the matrix-core kernels may ask for: the 160 KB of a gfx950 CU minus room
// for the few hundred bytes of static LDS the compiler adds (workgroup reductions).
constexpr int kMaxDynLds = 160 * 1024 - 2048;

__device__ __forceinline__ float widen(float x) { return x; }
__device__ __forceinline__ float widen(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

// Round-to-nearest-even fp32 -> bf16 (NaN kept quiet).
__device__ __forceinline__ bf16_t narrow_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ void store_as(float *p, float x) { *p = x; }
__device__ __forceinline__ void store_as(bf16_t *p, float x) { *p = narrow_bf16(x); }

// Sec. 2.2 window partition after a cyclic shift: window-local token n of window
// w (numbered (b*nwy + wy)*nwx + wx) -> token index (b*H + y)*W + x in the grid.
__device__ __forceinline__ int64_t grid_token(const Geo &g, int w, int n)
{
    int wx = w % g.nwx;
    int t = w / g.nwx;
    int wy = t % g.nwy;
    int b = t / g.nwy;
    int iy = n / g.M, ix = n - iy * g.M;
    int y = wy * g.M + iy + g.s;
    if (y >= g.H) y -= g.H;
    int x = wx * g.M + ix + g.s;
    if (x >= g.W) x -= g.W;
    return ((int64_t)b * g.H + y) * g.W + x;
}

// Token table of window w: entry n = grid token of window-local token n (Sec. 2.2
// partition after the cyclic shift), -1 for n >= N.  One integer division per thread;
// the walk from n to n + NT is done with adds and a carry.
template <int NT>
__device__ __forceinline__ void fill_tok_table(const Geo &g, int w, int *tok, int count)
{
    const int wx = w % g.nwx, t = w / g.nwx, wy = t % g.nwy, b = t / g.nwy;
    const int sy = NT / g.M, sx = NT - sy * g.M;
    const int y0 = wy * g.M + g.s, x0 = wx * g.M + g.s;
    int n = threadIdx.x;
    int iy = n / g.M, ix = n - iy * g.M;
    for (; n < count; n += NT) {
        int y = y0 + iy, x = x0 + ix;
        if (y >= g.H) y -= g.H;
        if (x >= g.W) x -= g.W;
        tok[n] = n < g.N ? (b * g.H + y) * g.W + x : -1;
        ix += sx;
        iy += sy;
        if (ix >= g.M) {
            ix -= g.M;
            ++iy;
        }
    }
}

// The same map in separable form, 2*M integers instead of N: grid token of window-local
// token n = iy*M + ix is rowb[iy] + colo[ix] (row base of the wrapped pixel row, wrapped
// pixel column).  Large windows (N = 9216) would otherwise spend 36 KB of LDS on the table.
// Indexing syntax matches the plain table so that code can be written for either.
struct TokMap {
    const int *rowb, *colo;
    uint32_t inv_m;
    int M;
    __device__ __forceinline__ int operator[](int n) const
    {
        const int iy = (int)__umulhi((uint32_t)n, inv_m);
        return rowb[iy] + colo[n - iy * M];
    }
    // tokens n0 .. n0+3 of one window row (n0 a multiple of 4, M a multiple of 4)
    __device__ __forceinline__ void quad(int n0, int (&t)[4]) const
    {
        const int iy = (int)__umulhi((uint32_t)n0, inv_m);
        const int rb = rowb[iy];
        const int4 c = *(const int4 *)(colo + (n0 - iy * M));
        t[0] = rb + c.x, t[1] = rb + c.y, t[2] = rb + c.z, t[3] = rb + c.w;
    }
};

// Fills lds[0, 2M) and returns the map; the caller synchronises the workgroup.  `lds` must be
// 16-byte aligned and M a multiple of 4 for quad().
template <int NT>
__device__ __forceinline__ TokMap fill_tok_map(const Geo &g, int w, int *lds)
{
    const int wx = w % g.nwx, t = w / g.nwx, wy = t % g.nwy, b = t / g.nwy;
    for (int i = threadIdx.x; i < 2 * g.M; i += NT) {
        if (i < g.M) {
            int y = wy * g.M + g.s + i;
            if (y >= g.H) y -= g.H;
            lds[i] = (b * g.H + y) * g.W;
        } else {
            int x = wx * g.M + g.s + (i - g.M);
            if (x >= g.W) x -= g.W;
            lds[i] = x;
        }
    }
    TokMap m;
    m.rowb = lds;
    m.colo = lds + g.M;
    m.inv_m = g.inv_m;
    m.M = g.M;
    return m;
}

// Before a launch of a kernel that uses dynamic LDS: raises the kernel's dynamic-LDS limit to
// kMaxDynLds on the CURRENT device, once per (kernel, device); a failure is returned and not
// remembered, so a later call tries again.  If `cus` is given it receives the number of compute
// units of the current device (looked up once per device).  Thread-safe.
hipError_t prepare_kernel(const void *kern, int *cus);

// Launchers (each returns the hipError_t of its launches).
hipError_t launch_valu_fwd(const Geo &g, int dtype, const void *q, const void *k, const void *v,
                           const void *fq, const void *fk, void *out, float *lse, hipStream_t st);
hipError_t launch_valu_bwd(const Geo &g, int dtype, const void *q, const void *k, const void *v,
                           const void *fq, const void *fk, const void *out, const void *dout,
                           const float *lse, void *dq, void *dk, void *dv, float *dfq, float *dfk,
                           void *ws, hipStream_t st, void *gated_dout = nullptr, void *dgate = nullptr);
size_t valu_bwd_workspace(const Geo &g);

// Backward scratch layout (both kernel families): delta [units][N] fp32, then the
// per-unit RIB gradient partials dF_q, dF_k [units][N][r] fp32, each 256-byte aligned.
struct BwdWs {
    size_t delta_off, dfq_off, dfk_off, total;
};
BwdWs bwd_ws_layout(const Geo &g);
// Gated backward: the same scratch followed by one grid tensor for dO = dO' * gate.
size_t gated_dout_bytes(const Geo &g, int dtype);
// delta, dO = dO' * gate (into `dout`, storage type) and dgate = dO' * O in one pass.
hipError_t launch_delta_gated(const Geo &g, int dtype, const void *out_raw, const void *dout_gated, const void *gate,
                              float *delta, void *dout, void *dgate, hipStream_t st);
// delta[u][i] = dO[i].O[i] per head (dtype = RIB_F32 / RIB_BF16 storage of out, dout).
hipError_t launch_delta(const Geo &g, int dtype, const void *out, const void *dout, float *delta, hipStream_t st);
// dF[hd][e] = sum over windows (ascending) of part[(w*heads + hd)][e].
hipError_t launch_reduce_df(const Geo &g, const float *part_q, const float *part_k, float *dfq, float *dfk,
                            hipStream_t st);

// Matrix-core forward (bf16): whether it serves this problem, and its launcher.
bool mfma_fwd_supported(const Geo &g, int dtype);
hipError_t launch_mfma_fwd(const Geo &g, int force_max, const void *q, const void *k, const void *v,
                           const void *fq, const void *fk, void *out, float *lse, hipStream_t st);
// Matrix-core backward (bf16).
bool mfma_bwd_supported(const Geo &g, int dtype);
hipError_t launch_mfma_bwd(const Geo &g, const void *q, const void *k, const void *v, const void *fq,
                           const void *fk, const void *out, const void *dout, const float *lse, void *dq,
                           void *dk, void *dv, float *dfq, float *dfk, void *ws, hipStream_t st,
                           void *gated_dout = nullptr, void *dgate = nullptr);
// Matrix-core kernels for fp32 storage (fp32 MFMA, fp32 throughout), forward and backward.
bool mfma_f32_supported(const Geo &g, int dtype);
hipError_t launch_mfma_f32_fwd(const Geo &g, const void *q, const void *k, const void *v, const void *fq,
                               const void *fk, void *out, float *lse, hipStream_t st);
hipError_t launch_mfma_f32_bwd(const Geo &g, const void *q, const void *k, const void *v, const void *fq,
                               const void *fk, const void *out, const void *dout, const float *lse, void *dq, void *dk,
                               void *dv, float *dfq, float *dfk, void *ws, hipStream_t st, void *gated_dout = nullptr,
                               void *dgate = nullptr);
// With g.gate set, `dout` is the gradient of the GATED output: the launchers above first run
// launch_delta_gated (delta, dO into gated_dout, dgate) and feed gated_dout to the main kernels.

}  // namespace rib
