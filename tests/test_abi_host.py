"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the public header declares, and rejects bad arguments with the
documented status codes before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2603_06738_amd import binding as rb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000  # non-NULL dummy "device pointer"; validation must fail before it is ever used


def good(**kw):
    base = dict(B=2, H=8, W=8, heads=2, d=4, r=2, window=4, shift=1, scale_c=0.5, scale_p=0.5,
                dtype="f32")
    base.update(kw)
    return rb.make_params(**base)


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "rib_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(rib_[a-z_]+)\s*\(", text))
    assert declared == set(rb.EXPORTS)
    lib = rb.load()
    for name in declared:
        assert getattr(lib, name) is not None


def test_params_struct_layout_matches_header():
    # 8 int32 + 2 float + 2 int32 + int64, naturally aligned
    assert ctypes.sizeof(rb.RibParams) == 56
    assert rb.RibParams.token_stride.offset == 48


def test_status_strings():
    seen = {rb.status_string(i) for i in range(7)}
    assert len(seen) == 7 and all(seen)


def fwd_status(p, **ptrs):
    a = dict(q=FAKE, k=FAKE, v=FAKE, f_q=FAKE, f_k=FAKE, out=FAKE, lse=None)
    a.update(ptrs)
    return rb.rib_window_attn_fwd_status(p, a["q"], a["k"], a["v"], a["f_q"], a["f_k"], a["out"], a["lse"], stream=0)


@pytest.mark.parametrize("kw", [dict(B=0), dict(H=-8), dict(d=0), dict(r=-1), dict(window=0),
                                dict(H=10), dict(W=6), dict(shift=4), dict(shift=-1),
                                dict(token_stride=7), dict(scale_c=float("nan"))])
def test_shape_errors(kw):
    assert fwd_status(good(**kw)) == 2
    assert rb.rib_window_attn_bwd_workspace_bytes(good(**kw)) == 0
    assert rb.kernel_name(good(**kw)) is None


def test_dtype_and_unsupported_errors():
    assert fwd_status(good(dtype=7)) == 3
    assert fwd_status(good(d=65)) == 4
    assert fwd_status(good(r=65)) == 4
    assert fwd_status(good(H=512, W=512, window=512)) == 4


def test_unknown_flags_and_misaligned_pointers_are_rejected():
    assert fwd_status(good(flags=8)) == 2
    assert fwd_status(good(flags=1 << 20)) == 2
    for name in ("q", "k", "v", "f_q", "f_k", "out"):
        assert fwd_status(good(), **{name: FAKE + 2}) == 2
        assert fwd_status(good(dtype="bf16"), **{name: FAKE + 1}) == 2
    p = good()
    args = [FAKE] * 13
    for i in range(13):
        bad = list(args)
        bad[i] = FAKE + 2
        assert rb.rib_window_attn_bwd_status(p, *bad, FAKE, 1 << 30, stream=0) == 2


def test_null_pointer_errors():
    assert rb.rib_window_attn_fwd_status(None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, stream=0) == 1
    for name in ("q", "k", "v", "out", "f_q", "f_k"):
        assert fwd_status(good(), **{name: None}) == 1
    # r == 0 makes the RIB tables optional: validation passes and only the launch
    # fails (no GPU here) or succeeds (on a GPU machine this test is not given real memory)
    p0 = good(r=0, B=1, H=4, W=4)
    assert rb.kernel_name(p0) is not None


def test_backward_workspace_validation():
    p = good()
    need = rb.rib_window_attn_bwd_workspace_bytes(p)
    assert need > 0 and need % 256 == 0
    args = [FAKE] * 13

    def call(ws, nbytes, **kw):
        a = list(args)
        for i, n in enumerate(("q", "k", "v", "f_q", "f_k", "out", "d_out", "lse", "dq", "dk", "dv", "df_q", "df_k")):
            if n in kw:
                a[i] = kw[n]
        return rb.rib_window_attn_bwd_status(p, *a, ws, nbytes, stream=0)

    assert call(None, need) == 5
    assert call(0x1000, need - 1) == 5
    assert call(0x1010, need) == 5          # not 256-byte aligned
    assert call(0x1000, need, lse=None) == 1
    assert call(0x1000, need, df_q=None) == 1
    assert call(0x1000, need, d_out=None) == 1


def test_kernel_family_names():
    assert rb.kernel_name(good()) is not None
    assert rb.kernel_name(good(), backward=True) is not None


def test_generator_params_layout_and_validation():
    assert ctypes.sizeof(rb.RibGenParams) == 24
    ok = rb.make_gen_params(16, 6, 18)
    need = rb.rib_features_bwd_workspace_bytes(ok)
    assert need > 0 and need % 256 == 0
    ptrs = [FAKE] * 6
    for bad in (dict(window=0), dict(window=257), dict(heads=0), dict(r=0), dict(r=65), dict(L=-1), dict(L=17),
                dict(d_h=0), dict(d_h=65)):
        kw = dict(window=16, heads=6, r=18, L=10, d_h=32)
        kw.update(bad)
        p = rb.make_gen_params(**kw)
        assert rb.rib_features_fwd_status(p, *ptrs, stream=0) == 2, bad
        assert rb.rib_features_bwd_workspace_bytes(p) == 0
    assert rb.rib_features_fwd_status(rb.make_gen_params(16, 6, 18, dtype=5), *ptrs, stream=0) == 3
    assert rb.rib_features_fwd_status(None, *ptrs, stream=0) == 1
    for i in range(6):
        a = list(ptrs)
        a[i] = None
        assert rb.rib_features_fwd_status(ok, *a, stream=0) == 1
    b = [FAKE] * 10
    assert rb.rib_features_bwd_status(ok, *b, None, need, stream=0) == 5
    assert rb.rib_features_bwd_status(ok, *b, 0x1000, need - 1, stream=0) == 5
    assert rb.rib_features_bwd_status(ok, *b, 0x1010, need, stream=0) == 5
    for i in range(10):
        a = list(b)
        a[i] = None
        assert rb.rib_features_bwd_status(ok, *a, 0x1000, need, stream=0) == 1


def test_gated_entry_points_validate():
    p = good()
    ptrs = dict(q=FAKE, k=FAKE, v=FAKE, f_q=FAKE, f_k=FAKE, gate=FAKE, out_gated=FAKE, out_raw=None, lse=None)

    def fwd(**kw):
        a = dict(ptrs)
        a.update(kw)
        return rb.rib_window_attn_gated_fwd_status(p, *[a[n] for n in ("q", "k", "v", "f_q", "f_k", "gate", "out_gated",
                                                                        "out_raw", "lse")], stream=0)

    assert fwd(gate=None) == 1 and fwd(out_gated=None) == 1 and fwd(q=None) == 1
    assert rb.rib_window_attn_gated_fwd_status(good(H=10), *([FAKE] * 9), stream=0) == 2
    need = rb.rib_window_attn_gated_bwd_workspace_bytes(p)
    plain = rb.rib_window_attn_bwd_workspace_bytes(p)
    assert need % 256 == 0 and need >= plain + 2 * 8 * 8 * 8 * 4
    b = [FAKE] * 15
    assert rb.rib_window_attn_gated_bwd_status(p, *b, 0x1000, need - 1, stream=0) == 5
    assert rb.rib_window_attn_gated_bwd_status(p, *b, 0x1010, need, stream=0) == 5
    for i in range(15):
        a = list(b)
        a[i] = None
        assert rb.rib_window_attn_gated_bwd_status(p, *a, 0x1000, need, stream=0) == 1, i
    assert rb.rib_window_attn_gated_bwd_workspace_bytes(good(shift=9)) == 0


def test_kernel_family_selection_is_host_logic():
    """Which family serves a problem is decided on the host (no GPU needed): matrix-core kernels
    for d <= 32 and d + r <= 64 (bf16: even d and r, 64+ tokens; fp32: 32+ tokens), the vector ALU
    for everything else and for anything under RIB_FLAG_VECTOR_ONLY."""
    def name(back=False, **kw):
        base = dict(B=1, H=16, W=16, heads=2, d=30, r=16, window=16, shift=0, scale_c=0.1, scale_p=0.1, dtype="bf16")
        base.update(kw)
        return rb.kernel_name(rb.make_params(**base), backward=back)
    for back in (False, True):
        assert name(back) == "mfma-bf16"
        assert name(back, dtype="f32") == "mfma-f32"
        assert name(back, flags=rb.RIB_FLAG_VECTOR_ONLY) == "valu-f32"
        assert name(back, dtype="f32", flags=rb.RIB_FLAG_VECTOR_ONLY) == "valu-f32"
        assert name(back, d=40, r=8) == "valu-f32"                          # d > 32
        assert name(back, d=32, r=34) == "valu-f32"                         # d + r > 64
        assert name(back, d=32, r=34, dtype="f32") == "valu-f32"
        assert name(back, d=31, r=33, dtype="f32") == "mfma-f32"            # odd d and r are fine in fp32
        assert name(back, d=31, r=16) == "valu-f32"                         # ... not in bf16 (pairs of channels)
        assert name(back, H=5, W=5, window=5, dtype="f32") == "valu-f32"    # 25 tokens: below one 32-token block
        assert name(back, H=6, W=6, window=6, dtype="f32") == "mfma-f32"    # 36 tokens
        assert name(back, H=6, W=6, window=6) == "valu-f32"                 # bf16 kernels start at 64 tokens
    # offsets inside one image must fit 32 bits for the fp32 matrix-core kernels
    assert name(dtype="f32", H=8192, W=8192, heads=1, d=32, r=0, window=16) == "valu-f32"
