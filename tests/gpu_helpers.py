"""Plumbing for the GPU parity tests: move seeded inputs to the device, call the
library through its C ABI (via the ctypes binding) and bring results back as
float64 numpy arrays.  No arithmetic of the method lives here."""
import numpy as np
import torch

from paper_2603_06738_amd import binding as rb

DEV = "cuda:0"
TOL = {"f32": 1e-4, "bf16": 2e-2}     # max-abs bound per output tensor, from the benchmark spec


def tdtype(wl):
    return torch.bfloat16 if wl.dtype == "bf16" else torch.float32


def device_inputs(wl, x, packed=False):
    """Dict of device tensors.  packed=True stores q, k, v interleaved per token
    ([B,H,W,3C]) and returns strided views, exercising token_stride."""
    t = {n: rb.to_device(a, wl.dtype, DEV) for n, a in x.items()}
    if packed:
        qkv = torch.cat([t["q"], t["k"], t["v"]], dim=-1).contiguous()
        C = wl.C
        t["_qkv"] = qkv
        t["q"], t["k"], t["v"] = qkv[..., :C], qkv[..., C:2 * C], qkv[..., 2 * C:]
    return t


def gpu_fwd(wl, t, flags=0, want_lse=True, packed=False):
    p = rb.params_of(wl, flags=flags, token_stride=3 * wl.C if packed else 0)
    out = torch.full((wl.B, wl.H, wl.W, wl.C), float("nan"), dtype=tdtype(wl), device=DEV)
    lse = torch.full((wl.n_windows, wl.heads, wl.N), float("nan"), dtype=torch.float32, device=DEV) \
        if want_lse else None
    rb.rib_window_attn_fwd(p, t["q"], t["k"], t["v"], t.get("f_q"), t.get("f_k"), out, lse)
    torch.cuda.synchronize()
    return out, lse


def gpu_bwd(wl, t, out, lse, flags=0, packed=False):
    p = rb.params_of(wl, flags=flags, token_stride=3 * wl.C if packed else 0)
    ws = rb.alloc_workspace(p, DEV)
    grid = (wl.B, wl.H, wl.W, wl.C)
    dq, dk, dv = (torch.full(grid, float("nan"), dtype=tdtype(wl), device=DEV) for _ in range(3))
    dfq, dfk = (torch.full((wl.heads, wl.N, wl.r), float("nan"), dtype=torch.float32, device=DEV)
                for _ in range(2))
    rb.rib_window_attn_bwd(p, t["q"], t["k"], t["v"], t.get("f_q"), t.get("f_k"), out, t["d_out"], lse,
                           dq, dk, dv, dfq, dfk, ws)
    torch.cuda.synchronize()
    return dq, dk, dv, dfq, dfk


def host(tensor):
    return tensor.detach().to(torch.float64).cpu().numpy()


def max_abs(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    if a.size == 0:
        return 0.0
    diff = np.abs(a - b)
    assert np.isfinite(a).all(), "non-finite values in the GPU result"
    return float(diff.max())


def gather_unit(oracle, g, arr, unit):
    """[B,H,W,C] array -> the [N,d] block of one (window, head) unit, window-local order."""
    b, y, x, hd = oracle.unit_token_index(g, unit)
    return arr[b, y, x, hd * g.d:(hd + 1) * g.d]
