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

// Launchers (each returns the hipError_t of its launches).
hipError_t launch_valu_fwd(const Geo &g, int dtype, const void *q, const void *k, const void *v,
                           const void *fq, const void *fk, void *out, float *lse, hipStream_t st);
hipError_t launch_valu_bwd(const Geo &g, int dtype, const void *q, const void *k, const void *v,
                           const void *fq, const void *fk, const void *out, const void *dout,
                           const float *lse, void *dq, void *dk, void *dv, float *dfq, float *dfk,
                           void *ws, hipStream_t st);
size_t valu_bwd_workspace(const Geo &g);

// Backward scratch layout (both kernel families): delta [units][N] fp32, then the
// per-unit RIB gradient partials dF_q, dF_k [units][N][r] fp32, each 256-byte aligned.
struct BwdWs {
    size_t delta_off, dfq_off, dfk_off, total;
};
BwdWs bwd_ws_layout(const Geo &g);
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
                           void *dk, void *dv, float *dfq, float *dfk, void *ws, hipStream_t st);

}  // namespace rib
