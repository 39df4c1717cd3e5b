"""The backward entry point that allocates nothing (its scratch is a static device
array inside the library) against the ordinary backward, through the C ABI: same
kernels, same fixed summation order, so every output must agree bit for bit.  Two
calls in a row share the array; the second is the smaller problem."""
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2603_06738_amd import binding as rb
from paper_2603_06738_amd import workloads as wk


def _both(gh, wl):
    x = wk.make_inputs(wl)
    t = gh.device_inputs(wl, x)
    out, lse = gh.gpu_fwd(wl, t)
    ref = gh.gpu_bwd(wl, t, out, lse)
    p = rb.params_of(wl)
    assert rb.rib_window_attn_bwd_workspace_bytes(p) <= rb.RIB_STATIC_SCRATCH_BYTES
    grid = (wl.B, wl.H, wl.W, wl.C)
    dq, dk, dv = (torch.full(grid, float("nan"), dtype=gh.tdtype(wl), device=gh.DEV) for _ in range(3))
    dfq, dfk = (torch.full((wl.heads, wl.N, wl.r), float("nan"), dtype=torch.float32, device=gh.DEV)
                for _ in range(2))
    rb.rib_window_attn_bwd_static_scratch(p, t["q"], t["k"], t["v"], t["f_q"], t["f_k"], out, t["d_out"], lse,
                                          dq, dk, dv, dfq, dfk)
    torch.cuda.synchronize()
    for name, a, b in zip(("dQ", "dK", "dV", "dF_q", "dF_k"), (dq, dk, dv, dfq, dfk), ref):
        assert torch.equal(a, b), (wl.name, name)


def test_static_scratch_backward_matches_the_workspace_backward():
    import gpu_helpers as gh
    big = wk.custom("noalloc-big", "bf16", 2, 64, 64, 6, 30, 16, 32, 16, 501, backward=True)      # 25.9 MB of scratch
    small = wk.custom("noalloc-small", "bf16", 1, 16, 32, 2, 30, 16, 16, 3, 502, backward=True)   # 0.07 MB
    f32 = wk.custom("noalloc-f32", "f32", 1, 24, 12, 2, 30, 8, 12, 5, 503, backward=True)         # ragged window, fp32
    for wl in (big, small, f32):
        _both(gh, wl)


def test_static_scratch_rejects_what_does_not_fit():
    wl = wk.WORKLOADS["c5"]                                     # 117 MB of scratch
    p = rb.params_of(wl)
    assert rb.rib_window_attn_bwd_workspace_bytes(p) > rb.RIB_STATIC_SCRATCH_BYTES
    one = torch.zeros(64, device="cuda:0")
    st = rb.rib_window_attn_bwd_static_scratch_status(p, *([one] * 13))
    assert st == 5      # RIB_ERR_WORKSPACE, before any launch
