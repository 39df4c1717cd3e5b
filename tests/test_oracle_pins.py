"""Pins of the CPU oracle against things other than itself (all CPU, no GPU).

Each test states what would go wrong in the oracle if it failed: a dropped or
mis-scaled term, a wrong index map, a transposed operand, a wrong sign in the
backward pass, a missing sum over windows."""
import math

import numpy as np
import pytest

from paper_2603_06738_amd import workloads as wk
from helpers import (brute_force_fwd, concat_form_fwd, geometry, partition,
                     torch_sdpa_fwd_bwd, unpartition)

TINY = [
    # name, dtype, B, H, W, heads, d, r, M, s, seed
    wk.custom("t0", "f32", 1, 4, 4, 1, 2, 1, 2, 0, 11),
    wk.custom("t1", "f32", 2, 4, 6, 2, 3, 2, 2, 1, 12),               # H != W, shifted
    wk.custom("t2", "f32", 1, 6, 3, 2, 2, 3, 3, 2, 13, scale_c=0.7, scale_p=0.3),
]


def _run_fwd(oracle, wl, x):
    return oracle.fwd(geometry(oracle, wl), x["q"], x["k"], x["v"], x["f_q"], x["f_k"])


def _run_bwd(oracle, wl, x, d_out):
    return oracle.bwd(geometry(oracle, wl), x["q"], x["k"], x["v"], x["f_q"], x["f_k"], d_out)


@pytest.mark.parametrize("wl", TINY, ids=lambda w: w.name)
def test_brute_force_over_global_coordinates(oracle, wl):
    """Index maps (shift sign, partition, row-major local order, head-major
    channels) and both logit terms, against 7 nested loops over pixels."""
    x = wk.make_inputs(wl)
    O, _ = _run_fwd(oracle, wl, x)
    np.testing.assert_allclose(O, brute_force_fwd(wl, x), rtol=0, atol=1e-12)


def test_hand_computed_window():
    """One 2x2 window, d = r = 1, every k and f_k zero except token 0: then
    S[i][0] = sc*q_i*k_0 + sp*fq_i*fk_0 and S[i][j>0] = 0, so
    P[i][0] = 1 / (1 + 3 exp(-S[i][0])) and the rest share 1 - P[i][0] equally."""
    import oracle
    sc, sp = 0.5, 2.0
    wl = wk.custom("hand", "f32", 1, 2, 2, 1, 1, 1, 2, 0, 0, scale_c=sc, scale_p=sp)
    q = np.array([1.0, -2.0, 0.5, 3.0], np.float32).reshape(1, 2, 2, 1)
    k = np.array([2.0, 0, 0, 0], np.float32).reshape(1, 2, 2, 1)
    v = np.array([1.0, 10.0, 100.0, 1000.0], np.float32).reshape(1, 2, 2, 1)
    fq = np.array([0.25, 1.0, -1.0, 0.0], np.float32).reshape(1, 4, 1)
    fk = np.array([0.5, 0, 0, 0], np.float32).reshape(1, 4, 1)
    O, lse = oracle.fwd(geometry(oracle, wl), q, k, v, fq, fk)
    for i in range(4):
        s0 = sc * float(q.ravel()[i]) * 2.0 + sp * float(fq.ravel()[i]) * 0.5
        p0 = 1.0 / (1.0 + 3.0 * math.exp(-s0))
        want = p0 * 1.0 + (1.0 - p0) / 3.0 * 1110.0
        assert abs(O.ravel()[i] - want) < 1e-10 * max(1.0, abs(want))
        assert abs(lse.ravel()[i] - math.log(math.exp(s0) + 3.0)) < 1e-12


@pytest.mark.parametrize("wl", TINY + [wk.custom("t3", "f32", 2, 8, 8, 2, 5, 3, 4, 3, 14,
                                                 scale_c=1 / math.sqrt(5), scale_p=1 / math.sqrt(3))],
                         ids=lambda w: w.name)
def test_concat_form_equals_additive_bias(oracle, wl):
    """Eq. 6: one dot product of the concatenated, pre-scaled vectors of Eq. 5
    gives the same logits (hence O and LSE) as content term + bias term."""
    x = wk.make_inputs(wl)
    O, lse = _run_fwd(oracle, wl, x)
    O2, lse2 = concat_form_fwd(wl, x)
    np.testing.assert_allclose(O, O2, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, lse2, rtol=0, atol=1e-12)


def test_softmax_rows_sum_to_one_and_lse(oracle):
    """sum_j exp(S_ij - LSE_i) = 1 with S rebuilt independently; with v = 1 the
    output is exactly 1 (P >= 0 and rows sum to one)."""
    wl = wk.custom("sm", "f32", 2, 8, 4, 2, 4, 2, 4, 1, 21)
    x = wk.make_inputs(wl)
    _, lse = _run_fwd(oracle, wl, x)
    qs, ks = partition(x["q"].astype(np.float64), wl.M, wl.s), partition(x["k"].astype(np.float64), wl.M, wl.s)
    for hd in range(wl.heads):
        ch = slice(hd * wl.d, (hd + 1) * wl.d)
        S = wl.scale_c * qs[..., ch] @ ks[..., ch].transpose(0, 2, 1) \
            + wl.scale_p * (x["f_q"][hd].astype(np.float64) @ x["f_k"][hd].astype(np.float64).T)[None]
        rows = np.exp(S - lse[:, hd, :, None]).sum(-1)
        np.testing.assert_allclose(rows, 1.0, rtol=0, atol=1e-12)
    ones = dict(x, v=np.ones_like(x["v"]))
    O, _ = _run_fwd(oracle, wl, ones)
    np.testing.assert_allclose(O, 1.0, rtol=0, atol=1e-13)


def test_single_token_window(oracle):
    """M = 1: softmax over one logit is 1, so O = V, dV = dO and every other
    gradient vanishes."""
    wl = wk.custom("m1", "f32", 2, 3, 5, 2, 3, 2, 1, 0, 31, backward=True)
    x = wk.make_inputs(wl)
    O, lse = _run_fwd(oracle, wl, x)
    np.testing.assert_array_equal(O, x["v"].astype(np.float64))
    dQ, dK, dV, dFq, dFk = _run_bwd(oracle, wl, x, x["d_out"])
    np.testing.assert_array_equal(dV, x["d_out"].astype(np.float64))
    for g in (dQ, dK, dFq, dFk):
        assert np.abs(g).max() < 1e-15


def test_zero_queries_give_window_mean(oracle):
    """q = 0 and f_q = 0 make every logit 0: O[i] is the plain mean of V over
    the token's (shifted) window."""
    wl = wk.custom("mean", "f32", 1, 6, 6, 2, 3, 2, 3, 1, 41)
    x = wk.make_inputs(wl)
    x = dict(x, q=np.zeros_like(x["q"]), f_q=np.zeros_like(x["f_q"]))
    O, lse = _run_fwd(oracle, wl, x)
    vm = partition(x["v"].astype(np.float64), wl.M, wl.s).mean(1, keepdims=True)
    want = unpartition(np.broadcast_to(vm, (wl.n_windows, wl.N, wl.C)).copy(), wl.B, wl.H, wl.W, wl.M, wl.s)
    np.testing.assert_allclose(O, want, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, math.log(wl.N), rtol=0, atol=1e-13)


def test_row_constant_in_bias_is_invisible(oracle):
    """Appending a column c_i to f_q and a column of ones to f_k adds c_i to
    every logit of row i; softmax ignores it (O unchanged, LSE shifts by
    scale_p * c_i)."""
    wl = wk.custom("rc", "f32", 1, 4, 8, 2, 3, 2, 4, 2, 51)
    x = wk.make_inputs(wl)
    O, lse = _run_fwd(oracle, wl, x)
    c = np.random.default_rng(5).standard_normal((wl.heads, wl.N, 1)).astype(np.float32)
    wl2 = wk.custom("rc2", "f32", 1, 4, 8, 2, 3, 3, 4, 2, 51, scale_c=wl.scale_c, scale_p=wl.scale_p)
    x2 = dict(x, f_q=np.concatenate([x["f_q"], c], -1),
              f_k=np.concatenate([x["f_k"], np.ones_like(c)], -1))
    O2, lse2 = _run_fwd(oracle, wl2, x2)
    np.testing.assert_allclose(O2, O, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse2 - lse, wl.scale_p * c[None, :, :, 0].astype(np.float64)
                               * np.ones((wl.n_windows, 1, 1)), rtol=0, atol=1e-12)


def test_sharp_onehot_bias_selects_own_value(oracle):
    """f_q = f_k = lambda * identity (r = N) makes the diagonal logit dominate
    as lambda grows, so O -> V."""
    wl = wk.custom("hot", "f32", 1, 2, 4, 1, 2, 4, 2, 0, 61, scale_p=1.0)
    x = wk.make_inputs(wl)
    eye = (30.0 * np.eye(4, dtype=np.float32))[None]
    x = dict(x, f_q=eye, f_k=eye)
    O, _ = _run_fwd(oracle, wl, x)
    np.testing.assert_allclose(O, x["v"].astype(np.float64), rtol=0, atol=1e-9)


def test_window_permutation_equivariance(oracle):
    """With s = 0, windows are independent (Sec. 2.2): permuting whole MxM
    blocks of q, k, v permutes the blocks of O the same way and leaves the RIB
    gradients (sums over windows) unchanged."""
    wl = wk.custom("perm", "f32", 2, 8, 12, 2, 3, 2, 4, 0, 71, backward=True)
    x = wk.make_inputs(wl)
    perm = np.random.default_rng(3).permutation(wl.n_windows)

    def shuffle(a):
        return unpartition(partition(a, wl.M, 0)[perm], wl.B, wl.H, wl.W, wl.M, 0)

    xs = dict(x, **{n: shuffle(x[n]) for n in ("q", "k", "v", "d_out")})
    O, _ = _run_fwd(oracle, wl, x)
    Os, _ = _run_fwd(oracle, wl, xs)
    np.testing.assert_allclose(Os, shuffle(O), rtol=0, atol=1e-13)
    g = _run_bwd(oracle, wl, x, x["d_out"])
    gs = _run_bwd(oracle, wl, xs, xs["d_out"])
    for a, b in zip(g[:3], gs[:3]):
        np.testing.assert_allclose(b, shuffle(a), rtol=0, atol=1e-12)
    for a, b in zip(g[3:], gs[3:]):
        np.testing.assert_allclose(b, a, rtol=0, atol=1e-11)


def test_shift_invariants(oracle):
    """(i) shifting by s equals pre-rolling the inputs by (-s,-s), running
    unshifted and rolling the result back; (ii) s = M is s = 0; (iii) with one
    window per image and no RIB a shift only permutes the tokens of the window,
    so O does not change -- and with RIB it does, because f is indexed by the
    window-local position."""
    wl = wk.custom("sh", "f32", 2, 8, 12, 2, 3, 2, 4, 3, 81)
    x = wk.make_inputs(wl)
    O, _ = _run_fwd(oracle, wl, x)
    wl0 = wk.custom("sh0", "f32", 2, 8, 12, 2, 3, 2, 4, 0, 81)
    xr = dict(x, **{n: np.roll(x[n], (-wl.s, -wl.s), (1, 2)) for n in ("q", "k", "v")})
    O0, _ = _run_fwd(oracle, wl0, xr)
    np.testing.assert_allclose(np.roll(O0, (wl.s, wl.s), (1, 2)), O, rtol=0, atol=1e-13)

    wlM = wk.custom("shM", "f32", 2, 8, 12, 2, 3, 2, 4, 4, 81)
    Oa, _ = _run_fwd(oracle, wl0, x)
    Ob, _ = _run_fwd(oracle, wlM, x)
    np.testing.assert_allclose(Ob, Oa, rtol=0, atol=1e-13)

    one0 = wk.custom("one0", "f32", 1, 4, 4, 1, 3, 2, 4, 0, 82)
    one1 = wk.custom("one1", "f32", 1, 4, 4, 1, 3, 2, 4, 1, 82)
    y = wk.make_inputs(one0)
    nof = dict(y, f_q=np.zeros_like(y["f_q"]))
    np.testing.assert_allclose(_run_fwd(oracle, one1, nof)[0], _run_fwd(oracle, one0, nof)[0],
                               rtol=0, atol=1e-13)
    assert np.abs(_run_fwd(oracle, one1, y)[0] - _run_fwd(oracle, one0, y)[0]).max() > 1e-3


SDPA_CASES = [
    wk.custom("sd0", "f32", 2, 8, 8, 2, 6, 3, 4, 2, 91, backward=True),
    wk.custom("sd1", "f32", 1, 8, 16, 3, 5, 4, 8, 5, 92, scale_c=1 / math.sqrt(5), scale_p=0.5,
              backward=True),
]


@pytest.mark.parametrize("wl", SDPA_CASES, ids=lambda w: w.name)
def test_against_library_sdpa_and_autograd(oracle, wl):
    """Forward against torch's scaled_dot_product_attention with the bias as an
    additive float mask (after an explicit roll + partition); all five
    gradients against autograd through that same library call."""
    x = wk.make_inputs(wl)
    ref = torch_sdpa_fwd_bwd(wl, x, x["d_out"])
    O, _ = _run_fwd(oracle, wl, x)
    np.testing.assert_allclose(O, ref["O"], rtol=0, atol=1e-12)
    got = dict(zip(("dQ", "dK", "dV", "dF_q", "dF_k"), _run_bwd(oracle, wl, x, x["d_out"])))
    for n, a in got.items():
        np.testing.assert_allclose(a, ref[n], rtol=0, atol=1e-11, err_msg=n)


def test_without_rib_is_plain_window_attention(oracle):
    """f = 0: ordinary per-window attention with scale scale_c."""
    wl = wk.custom("norib", "f32", 1, 8, 8, 2, 4, 2, 4, 1, 93)
    x = wk.make_inputs(wl)
    x = dict(x, f_q=np.zeros_like(x["f_q"]))
    O, _ = _run_fwd(oracle, wl, x)
    np.testing.assert_allclose(O, torch_sdpa_fwd_bwd(wl, x)["O"], rtol=0, atol=1e-12)


def test_backward_by_finite_differences(oracle):
    """Central differences of the brute-force forward (global-coordinate loops,
    independent of the oracle) for the scalar loss sum(O * G): pins the sign,
    the scales and the index maps of all five gradients."""
    wl = wk.custom("fd", "f32", 1, 4, 4, 2, 2, 2, 2, 1, 101, scale_c=0.6, scale_p=0.9, backward=True)
    x = wk.make_inputs(wl)
    G = x["d_out"].astype(np.float64)
    grads = dict(zip(("q", "k", "v", "f_q", "f_k"), _run_bwd(oracle, wl, x, x["d_out"])))
    rng = np.random.default_rng(7)
    eps = 1e-3                       # inputs are float32: 1e-3 is exactly representable enough
    for name, g in grads.items():
        flat_idx = rng.choice(x[name].size, size=min(12, x[name].size), replace=False)
        for fi in flat_idx:
            idx = np.unravel_index(fi, x[name].shape)
            xp = {n: a.astype(np.float64) for n, a in x.items()}
            xm = {n: a.astype(np.float64) for n, a in x.items()}
            xp[name][idx] += eps
            xm[name][idx] -= eps
            fd = ((brute_force_fwd(wl, xp) - brute_force_fwd(wl, xm)) * G).sum() / (2 * eps)
            assert abs(fd - g[idx]) < 5e-6 * max(1.0, abs(fd)), (name, idx, fd, g[idx])


def test_rib_gradients_sum_over_batch(oracle):
    """f_q, f_k are shared by every window and image (Sec. 3.1), so stacking the
    batch twice doubles dF_q and dF_k and leaves per-token gradients alone."""
    wl = wk.custom("lin", "f32", 1, 4, 8, 2, 3, 2, 4, 1, 111, backward=True)
    x = wk.make_inputs(wl)
    g1 = _run_bwd(oracle, wl, x, x["d_out"])
    wl2 = wk.custom("lin2", "f32", 2, 4, 8, 2, 3, 2, 4, 1, 111, scale_c=wl.scale_c, scale_p=wl.scale_p)
    x2 = dict(x, **{n: np.concatenate([x[n], x[n]], 0) for n in ("q", "k", "v", "d_out")})
    g2 = _run_bwd(oracle, wl2, x2, x2["d_out"])
    np.testing.assert_allclose(g2[3], 2 * g1[3], rtol=0, atol=1e-12)
    np.testing.assert_allclose(g2[4], 2 * g1[4], rtol=0, atol=1e-12)
    np.testing.assert_allclose(g2[0][:1], g1[0], rtol=0, atol=1e-13)


def test_unit_entry_points_match_full(oracle):
    """The sampled-unit entry points return the same numbers as the full ones
    (they are what the full-size GPU parity tests call)."""
    wl = wk.custom("un", "f32", 2, 8, 8, 3, 4, 2, 4, 3, 121, backward=True)
    x = wk.make_inputs(wl)
    g = geometry(oracle, wl)
    O, lse = _run_fwd(oracle, wl, x)
    grads = _run_bwd(oracle, wl, x, x["d_out"])
    units = [0, 5, wl.n_units - 1]
    Ou, lu = oracle.fwd_units(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], units)
    bu = oracle.bwd_units(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"], units)
    for a, u in enumerate(units):
        b, y, xx, hd = oracle.unit_token_index(g, u)
        ch = slice(hd * wl.d, (hd + 1) * wl.d)
        np.testing.assert_array_equal(Ou[a], O[b, y, xx, ch])
        np.testing.assert_array_equal(lu[a], lse[u // wl.heads, hd])
        for j in range(3):
            np.testing.assert_array_equal(bu[j][a], grads[j][b, y, xx, ch])
    allu = list(range(wl.n_units))
    ball = oracle.bwd_units(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"], allu)
    for hd in range(wl.heads):
        np.testing.assert_allclose(ball[3][hd::wl.heads].sum(0), grads[3][hd], rtol=0, atol=1e-12)
        np.testing.assert_allclose(ball[4][hd::wl.heads].sum(0), grads[4][hd], rtol=0, atol=1e-12)


def test_bf16_input_rounding_is_shared_not_hidden(oracle):
    """The bf16 workloads hand both sides the same rounded values: they are
    exactly representable (rounding again changes nothing) and differ from the
    unrounded draw by at most half a bf16 ulp."""
    wl = wk.custom("bf", "bf16", 1, 8, 8, 2, 4, 2, 4, 1, 131)
    x = wk.make_inputs(wl)
    for a in x.values():
        np.testing.assert_array_equal(wk.round_to_bf16(a), a)
    raw = wk.make_inputs(wk.custom("bf", "f32", 1, 8, 8, 2, 4, 2, 4, 1, 131))
    for n in x:
        assert np.all(np.abs(x[n] - raw[n]) <= np.abs(raw[n]) * 2.0 ** -8)
    import torch
    np.testing.assert_array_equal(torch.tensor(raw["q"]).bfloat16().float().numpy(), x["q"])


def test_single_precision_evaluation_agrees_on_bf16_inputs(oracle):
    """The oracle in double against the plain definition (Eq. 5 concat form over explicit
    windows) evaluated entirely in float32, on bf16-rounded inputs of the paper's head shape:
    they agree to 1e-4, i.e. the arithmetic precision of the reference is not what the bf16
    tolerance of 2e-2 has to absorb -- the GPU's own bf16 operands are."""
    wl = wk.custom("p9", "bf16", 2, 32, 16, 2, 30, 16, 16, 5, 132)
    x = wk.make_inputs(wl)
    O, lse = oracle.fwd(geometry(oracle, wl), x["q"], x["k"], x["v"], x["f_q"], x["f_k"])
    O32, lse32 = concat_form_fwd(wl, x, dtype=np.float32)
    assert O32.dtype == np.float32 and lse32.dtype == np.float32
    assert np.abs(O - O32).max() <= 1e-4
    assert np.abs(lse - lse32).max() <= 1e-4


def test_gate_of_ones_is_the_plain_operator(oracle):
    wl = wk.custom("gate1", "f32", 1, 4, 8, 2, 3, 2, 4, 1, 121, backward=True)
    x = wk.make_inputs(wl)
    g = geometry(oracle, wl)
    ones = np.ones((wl.B, wl.H, wl.W, wl.C), np.float32)
    Og, O, lse = oracle.gated_fwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], ones)
    O_ref, lse_ref = oracle.fwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"])
    np.testing.assert_array_equal(Og, O_ref)
    np.testing.assert_array_equal(O, O_ref)
    np.testing.assert_array_equal(lse, lse_ref)
    got = oracle.gated_bwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], ones, x["d_out"])
    ref = _run_bwd(oracle, wl, x, x["d_out"])
    for a, b in zip(got[:5], ref):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)
    np.testing.assert_allclose(got[5], x["d_out"].astype(np.float64) * O_ref, rtol=0, atol=1e-14)


def test_gated_backward_by_finite_differences(oracle):
    """Eq. 9 (O' = O * G) chained behind the brute-force forward: central
    differences of sum(O' * R) in the gate itself and in q, k, v, f_q, f_k."""
    wl = wk.custom("gatefd", "f32", 1, 4, 4, 2, 2, 2, 2, 1, 131, scale_c=0.7, scale_p=0.8, backward=True)
    x = wk.make_inputs(wl)
    gate = wk.make_gate(wl).astype(np.float64)
    R = x["d_out"].astype(np.float64)
    g = geometry(oracle, wl)
    got = oracle.gated_bwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], gate, x["d_out"])
    grads = dict(zip(("q", "k", "v", "f_q", "f_k", "gate"), got))
    base = {n: a.astype(np.float64) for n, a in x.items()}
    base["gate"] = gate
    rng = np.random.default_rng(9)
    eps = 1e-3

    def loss(z):
        return float((brute_force_fwd(wl, z) * z["gate"] * R).sum())

    for name, gr in grads.items():
        for fi in rng.choice(base[name].size, size=min(8, base[name].size), replace=False):
            idx = np.unravel_index(fi, base[name].shape)
            zp = {n: a.copy() for n, a in base.items()}
            zm = {n: a.copy() for n, a in base.items()}
            zp[name][idx] += eps
            zm[name][idx] -= eps
            fd = (loss(zp) - loss(zm)) / (2 * eps)
            assert abs(fd - gr[idx]) < 5e-6 * max(1.0, abs(fd)), (name, idx, fd, gr[idx])
