// Host side of the C ABI declared in include/rib_attn.h: argument validation,
// kernel-family selection and launches.  Nothing here allocates device memory or
// synchronises.
#include <atomic>
#include <cmath>
#include <initializer_list>
#include <mutex>
#include <set>
#include <utility>

#include "rib_common.h"

// Scratch of rib_window_attn_bwd_static_scratch: device memory that exists from the moment the
// code object is loaded, so that the entry point has nothing to allocate.  In host code the
// array's name is only a handle for hipGetSymbolAddress; every GPU holds its own copy at its own
// address, looked up once per device and cached below.  (The host-side reference in
// static_scratch() is what makes the compiler export the symbol from the code object; no
// attribute may be added here: `used` turns it into a local symbol the runtime cannot find.)
static __device__ __align__(256) unsigned char scratch[RIB_STATIC_SCRATCH_BYTES];

namespace rib {
namespace {

constexpr int kMaxDevices = 64;
std::atomic<void *> scratch_ptr[kMaxDevices];

// Address of the current device's copy of `scratch` (nullptr and *err set on failure).
void *static_scratch(hipError_t *err)
{
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    void *ptr = scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (*err != hipSuccess) return nullptr;
        scratch_ptr[dev].store(ptr, std::memory_order_release);      // (racing threads store the same address)
    }
    return ptr;
}

// Validate everything that does not involve data pointers and fill Geo.
rib_status make_geo(const rib_params *p, Geo *g)
{
    if (p == nullptr) return RIB_ERR_NULL;
    if (p->B <= 0 || p->H <= 0 || p->W <= 0 || p->heads <= 0 || p->d <= 0 || p->r < 0 || p->window <= 0)
        return RIB_ERR_SHAPE;
    if (p->H % p->window != 0 || p->W % p->window != 0) return RIB_ERR_SHAPE;
    if (p->shift < 0 || p->shift >= p->window) return RIB_ERR_SHAPE;
    const int64_t C = (int64_t)p->heads * p->d;
    if (p->token_stride != 0 && p->token_stride < C) return RIB_ERR_SHAPE;
    if (!std::isfinite(p->scale_c) || !std::isfinite(p->scale_p)) return RIB_ERR_SHAPE;
    if (p->dtype != RIB_F32 && p->dtype != RIB_BF16) return RIB_ERR_DTYPE;
    if ((p->flags & ~(RIB_FLAG_FORCE_ROW_MAX | RIB_FLAG_WIDE | RIB_FLAG_VECTOR_ONLY)) != 0) return RIB_ERR_SHAPE;
    if (p->d > 64 || p->r > 64 || (int64_t)p->window * p->window > 65536 || C > (1 << 20))
        return RIB_ERR_UNSUPPORTED;
    g->B = p->B; g->H = p->H; g->W = p->W;
    g->heads = p->heads; g->d = p->d; g->r = p->r;
    g->M = p->window; g->s = p->shift;
    g->N = p->window * p->window;
    g->nwx = p->W / p->window; g->nwy = p->H / p->window;
    g->C = (int)C;
    g->tstride = p->token_stride != 0 ? p->token_stride : C;
    g->scale_c = p->scale_c; g->scale_p = p->scale_p;
    g->units = (int64_t)p->B * g->nwx * g->nwy * p->heads;
    g->gate = nullptr;
    g->out_raw = nullptr;
    g->flags = p->flags;
    g->inv_m = p->window > 1 ? (uint32_t)((((uint64_t)1 << 32) + p->window - 1) / p->window) : 0xffffffffu;
    // every kernel indexes workgroups with 32-bit block ids and tokens with int
    const int64_t blocks = g->units * ((g->N + 63) / 64);
    if (blocks > 0x7fffffffLL || (int64_t)p->B * p->H * p->W > 0x7fffffffLL ||
        g->units * g->N > ((int64_t)1 << 34))
        return RIB_ERR_UNSUPPORTED;
    return RIB_OK;
}

// The kernels read and write the tensors in 4-byte pieces (bf16 pairs, fp32 values): every
// data pointer must be 4-byte aligned (NULL passes; presence is checked separately).
bool aligned4(std::initializer_list<const void *> ptrs)
{
    for (const void *ptr : ptrs)
        if (((uintptr_t)ptr & 3) != 0) return false;
    return true;
}

rib_status check_bwd(const rib_params *p, Geo *g, const void *q, const void *k, const void *v, const void *f_q,
                     const void *f_k, const void *out, const void *d_out, const float *lse, void *dq, void *dk,
                     void *dv, float *df_q, float *df_k)
{
    rib_status st = make_geo(p, g);
    if (st != RIB_OK) return st;
    if (!q || !k || !v || !out || !d_out || !lse || !dq || !dk || !dv) return RIB_ERR_NULL;
    if (g->r > 0 && (!f_q || !f_k || !df_q || !df_k)) return RIB_ERR_NULL;
    if (!aligned4({q, k, v, f_q, f_k, out, d_out, lse, dq, dk, dv, df_q, df_k})) return RIB_ERR_SHAPE;
    return RIB_OK;
}

// The plain backward on whichever kernel family serves the problem; `ws` holds bwd_ws_layout(g).total bytes.
rib_status enqueue_bwd(const Geo &g, int dtype, const void *q, const void *k, const void *v, const void *f_q,
                       const void *f_k, const void *out, const void *d_out, const float *lse, void *dq, void *dk,
                       void *dv, float *df_q, float *df_k, void *ws, hipStream_t stream)
{
    hipError_t e;
    if (mfma_bwd_supported(g, dtype))
        e = launch_mfma_bwd(g, q, k, v, f_q, f_k, out, d_out, lse, dq, dk, dv, df_q, df_k, ws, stream);
    else if (mfma_f32_supported(g, dtype))
        e = launch_mfma_f32_bwd(g, q, k, v, f_q, f_k, out, d_out, lse, dq, dk, dv, df_q, df_k, ws, stream);
    else
        e = launch_valu_bwd(g, dtype, q, k, v, f_q, f_k, out, d_out, lse, dq, dk, dv, df_q, df_k, ws, stream);
    return e == hipSuccess ? RIB_OK : RIB_ERR_LAUNCH;
}

}  // namespace
}  // namespace rib

namespace rib {

hipError_t prepare_kernel(const void *kern, int *cus)
{
    static std::mutex mu;
    static std::set<std::pair<const void *, int>> raised;      // (kernel, device) pairs whose limit is set
    static int cu_count[kMaxDevices];                          // 0 = not looked up yet
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (cus != nullptr) {
        if (cu_count[dev] == 0) {
            int n = 0;
            e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
            if (e != hipSuccess) return e;
            cu_count[dev] = n;
        }
        *cus = cu_count[dev];
    }
    const auto key = std::make_pair(kern, dev);
    if (raised.find(key) == raised.end()) {
        e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynLds);
        if (e != hipSuccess) return e;
        raised.insert(key);
    }
    return hipSuccess;
}

}  // namespace rib

using namespace rib;

extern "C" {

const char *rib_status_string(rib_status st)
{
    switch (st) {
    case RIB_OK: return "ok";
    case RIB_ERR_NULL: return "a required pointer is NULL";
    case RIB_ERR_SHAPE: return "invalid shape, shift, stride or scale";
    case RIB_ERR_DTYPE: return "unknown dtype";
    case RIB_ERR_UNSUPPORTED: return "problem size outside what the kernels are built for";
    case RIB_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case RIB_ERR_LAUNCH: return "HIP kernel launch failed";
    }
    return "unknown status";
}

const char *rib_window_attn_kernel_name(const rib_params *p, int backward)
{
    Geo g;
    if (make_geo(p, &g) != RIB_OK) return nullptr;
    if (!backward && mfma_fwd_supported(g, p->dtype)) return "mfma-bf16";
    if (backward && mfma_bwd_supported(g, p->dtype)) return "mfma-bf16";
    if (mfma_f32_supported(g, p->dtype)) return "mfma-f32";
    return "valu-f32";
}

rib_status rib_window_attn_fwd(const rib_params *p, const void *q, const void *k, const void *v, const void *f_q,
                               const void *f_k, void *out, float *lse, void *stream)
{
    Geo g;
    rib_status st = make_geo(p, &g);
    if (st != RIB_OK) return st;
    if (!q || !k || !v || !out) return RIB_ERR_NULL;
    if (g.r > 0 && (!f_q || !f_k)) return RIB_ERR_NULL;
    if (!aligned4({q, k, v, f_q, f_k, out, lse})) return RIB_ERR_SHAPE;
    hipError_t e;
    if (mfma_fwd_supported(g, p->dtype))
        e = launch_mfma_fwd(g, (p->flags & RIB_FLAG_FORCE_ROW_MAX) != 0, q, k, v, f_q, f_k, out, lse,
                            (hipStream_t)stream);
    else if (mfma_f32_supported(g, p->dtype))
        e = launch_mfma_f32_fwd(g, q, k, v, f_q, f_k, out, lse, (hipStream_t)stream);
    else
        e = launch_valu_fwd(g, p->dtype, q, k, v, f_q, f_k, out, lse, (hipStream_t)stream);
    return e == hipSuccess ? RIB_OK : RIB_ERR_LAUNCH;
}

rib_status rib_window_attn_gated_fwd(const rib_params *p, const void *q, const void *k, const void *v, const void *f_q,
                                     const void *f_k, const void *gate, void *out_gated, void *out_raw, float *lse,
                                     void *stream)
{
    Geo g;
    rib_status st = make_geo(p, &g);
    if (st != RIB_OK) return st;
    if (!q || !k || !v || !gate || !out_gated) return RIB_ERR_NULL;
    if (g.r > 0 && (!f_q || !f_k)) return RIB_ERR_NULL;
    if (!aligned4({q, k, v, f_q, f_k, gate, out_gated, out_raw, lse})) return RIB_ERR_SHAPE;
    g.gate = gate;
    g.out_raw = out_raw;
    hipError_t e;
    if (mfma_fwd_supported(g, p->dtype))
        e = launch_mfma_fwd(g, (p->flags & RIB_FLAG_FORCE_ROW_MAX) != 0, q, k, v, f_q, f_k, out_gated, lse,
                            (hipStream_t)stream);
    else if (mfma_f32_supported(g, p->dtype))
        e = launch_mfma_f32_fwd(g, q, k, v, f_q, f_k, out_gated, lse, (hipStream_t)stream);
    else
        e = launch_valu_fwd(g, p->dtype, q, k, v, f_q, f_k, out_gated, lse, (hipStream_t)stream);
    return e == hipSuccess ? RIB_OK : RIB_ERR_LAUNCH;
}

size_t rib_window_attn_gated_bwd_workspace_bytes(const rib_params *p)
{
    Geo g;
    if (make_geo(p, &g) != RIB_OK) return 0;
    return valu_bwd_workspace(g) + gated_dout_bytes(g, p->dtype);
}

rib_status rib_window_attn_gated_bwd(const rib_params *p, const void *q, const void *k, const void *v, const void *f_q,
                                     const void *f_k, const void *gate, const void *out_raw, const void *d_out_gated,
                                     const float *lse, void *dq, void *dk, void *dv, void *dgate, float *df_q,
                                     float *df_k, void *workspace, size_t workspace_bytes, void *stream)
{
    Geo g;
    rib_status st = make_geo(p, &g);
    if (st != RIB_OK) return st;
    if (!q || !k || !v || !gate || !out_raw || !d_out_gated || !lse || !dq || !dk || !dv || !dgate) return RIB_ERR_NULL;
    if (g.r > 0 && (!f_q || !f_k || !df_q || !df_k)) return RIB_ERR_NULL;
    if (!aligned4({q, k, v, f_q, f_k, gate, out_raw, d_out_gated, lse, dq, dk, dv, dgate, df_q, df_k})) return RIB_ERR_SHAPE;
    const size_t base = valu_bwd_workspace(g);
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < base + gated_dout_bytes(g, p->dtype))
        return RIB_ERR_WORKSPACE;
    // dO = dO' * gate lives behind the plain backward's scratch; the delta pass writes it (and dgate),
    // the main kernels then run exactly as for the plain operator.
    void *d_out = (char *)workspace + base;
    g.gate = gate;
    hipError_t e;
    if (mfma_bwd_supported(g, p->dtype))
        e = launch_mfma_bwd(g, q, k, v, f_q, f_k, out_raw, d_out_gated, lse, dq, dk, dv, df_q, df_k, workspace,
                            (hipStream_t)stream, d_out, dgate);
    else if (mfma_f32_supported(g, p->dtype))
        e = launch_mfma_f32_bwd(g, q, k, v, f_q, f_k, out_raw, d_out_gated, lse, dq, dk, dv, df_q, df_k, workspace,
                                (hipStream_t)stream, d_out, dgate);
    else
        e = launch_valu_bwd(g, p->dtype, q, k, v, f_q, f_k, out_raw, d_out_gated, lse, dq, dk, dv, df_q, df_k, workspace,
                            (hipStream_t)stream, d_out, dgate);
    return e == hipSuccess ? RIB_OK : RIB_ERR_LAUNCH;
}

size_t rib_window_attn_bwd_workspace_bytes(const rib_params *p)
{
    Geo g;
    if (make_geo(p, &g) != RIB_OK) return 0;
    return valu_bwd_workspace(g);
}

rib_status rib_window_attn_bwd(const rib_params *p, const void *q, const void *k, const void *v, const void *f_q,
                               const void *f_k, const void *out, const void *d_out, const float *lse, void *dq,
                               void *dk, void *dv, float *df_q, float *df_k, void *workspace, size_t workspace_bytes,
                               void *stream)
{
    Geo g;
    rib_status st = check_bwd(p, &g, q, k, v, f_q, f_k, out, d_out, lse, dq, dk, dv, df_q, df_k);
    if (st != RIB_OK) return st;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < valu_bwd_workspace(g))
        return RIB_ERR_WORKSPACE;
    return enqueue_bwd(g, p->dtype, q, k, v, f_q, f_k, out, d_out, lse, dq, dk, dv, df_q, df_k, workspace,
                       (hipStream_t)stream);
}

rib_status rib_window_attn_bwd_static_scratch(const rib_params *p, const void *q, const void *k, const void *v,
                                              const void *f_q, const void *f_k, const void *out, const void *d_out,
                                              const float *lse, void *dq, void *dk, void *dv, float *df_q,
                                              float *df_k, void *stream)
{
    Geo g;
    rib_status st = check_bwd(p, &g, q, k, v, f_q, f_k, out, d_out, lse, dq, dk, dv, df_q, df_k);
    if (st != RIB_OK) return st;
    if (valu_bwd_workspace(g) > (size_t)RIB_STATIC_SCRATCH_BYTES) return RIB_ERR_WORKSPACE;
    hipError_t e;
    void *ws = static_scratch(&e);
    if (ws == nullptr) return RIB_ERR_LAUNCH;
    // Nothing in the scratch has to start at zero: the delta pass and the main kernels write every
    // element the later kernels of the same call read.
    return enqueue_bwd(g, p->dtype, q, k, v, f_q, f_k, out, d_out, lse, dq, dk, dv, df_q, df_k, ws,
                       (hipStream_t)stream);
}

}  // extern "C"
