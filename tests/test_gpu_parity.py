"""GPU parity: the HIP library, called through its C ABI, against the CPU
oracle on the same seeded inputs, element by element.

Tolerances (max abs error per output tensor): 1e-4 for fp32 problems, 2e-2 for
bf16 storage with fp32 accumulation; the same bounds for gradients and LSE."""
import math

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2603_06738_amd import binding as rb
from paper_2603_06738_amd import workloads as wk
from helpers import geometry

FORCE_MAX = rb.RIB_FLAG_FORCE_ROW_MAX


def _small_cases():
    c = wk.custom
    cases = []
    for dt in ("f32", "bf16"):
        cases += [
            c(f"m1-{dt}", dt, 2, 3, 5, 2, 3, 2, 1, 0, 201),                 # one token per window
            c(f"m2-{dt}", dt, 2, 4, 6, 2, 3, 2, 2, 1, 202),
            c(f"m3-{dt}", dt, 1, 6, 9, 3, 7, 3, 3, 2, 203),                 # odd everything
            c(f"m5-{dt}", dt, 1, 10, 5, 2, 30, 16, 5, 4, 204),
            c(f"m9-{dt}", dt, 1, 9, 18, 2, 30, 8, 9, 3, 205),               # N=81: one tile + ragged tail
            c(f"m12-{dt}", dt, 1, 24, 12, 2, 30, 16, 12, 7, 206),           # N=144
            c(f"m16-{dt}", dt, 2, 16, 32, 3, 30, 16, 16, 8, 207),           # N=256, paper-like head
            c(f"norib-{dt}", dt, 1, 8, 8, 2, 16, 0, 8, 3, 208),             # r = 0
            c(f"wide-{dt}", dt, 1, 8, 8, 1, 64, 64, 8, 0, 209),             # largest d and r
            c(f"eq5-{dt}", dt, 1, 16, 16, 6, 30, 18, 16, 5, 210,
              scale_c=1 / math.sqrt(30), scale_p=1 / math.sqrt(18)),        # the paper's scales and an SST rank
            c(f"d32r16-{dt}", dt, 1, 32, 32, 2, 32, 16, 32, 16, 211),       # SST-L head, N=1024
            c(f"d30r34-{dt}", dt, 1, 16, 16, 2, 30, 34, 16, 1, 212),        # SST second-cycle rank
            c(f"d32r32-{dt}", dt, 1, 16, 32, 2, 32, 32, 16, 0, 213),        # SST-L second-cycle rank
            c(f"d16r24-{dt}", dt, 1, 16, 16, 3, 16, 24, 16, 2, 214),        # SST-light second-cycle rank
            c(f"d16r16-{dt}", dt, 1, 16, 16, 3, 16, 16, 16, 0, 215),        # SST-light first cycle
            c(f"d30r18m12-{dt}", dt, 1, 12, 24, 2, 30, 18, 12, 5, 216),     # SST rank on a ragged window
            c(f"d30r34m12-{dt}", dt, 1, 12, 12, 2, 30, 34, 12, 0, 217),
            c(f"d32r24-{dt}", dt, 1, 16, 32, 2, 32, 24, 16, 3, 218),        # d = 32, an odd number of 16-byte RIB pieces
            c(f"d28r24-{dt}", dt, 1, 16, 16, 2, 28, 24, 16, 0, 219),        # 64 columns with the ones row
            c(f"d4r4-{dt}", dt, 1, 16, 16, 2, 4, 4, 16, 1, 220),            # the smallest head the streaming kernels take
        ]
    return cases


SMALL = _small_cases()


def _check_fwd(oracle, gh, wl, x, flags=0, packed=False):
    g = geometry(oracle, wl)
    O_ref, lse_ref = oracle.fwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"])
    t = gh.device_inputs(wl, x, packed=packed)
    out, lse = gh.gpu_fwd(wl, t, flags=flags, packed=packed)
    tol = gh.TOL[wl.dtype]
    assert gh.max_abs(gh.host(out), O_ref) <= tol
    assert gh.max_abs(gh.host(lse), lse_ref) <= tol
    return t, out, lse


@pytest.fixture(scope="module")
def gh():
    import gpu_helpers
    return gpu_helpers


@pytest.mark.parametrize("wl", SMALL, ids=lambda w: w.name)
@pytest.mark.parametrize("flags", [0, FORCE_MAX], ids=["auto", "rowmax"])
def test_forward_small(oracle, gh, wl, flags):
    _check_fwd(oracle, gh, wl, wk.make_inputs(wl), flags=flags)


@pytest.mark.parametrize("wl", SMALL, ids=lambda w: w.name)
def test_backward_small(oracle, gh, wl):
    x = wk.make_inputs(wl, with_dout=True)
    t, out, lse = _check_fwd(oracle, gh, wl, x)
    got = gh.gpu_bwd(wl, t, out, lse)
    ref = oracle.bwd(geometry(oracle, wl), x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"])
    tol = gh.TOL[wl.dtype]
    for name, a, b in zip(("dQ", "dK", "dV", "dF_q", "dF_k"), got, ref):
        assert gh.max_abs(gh.host(a), b) <= tol, name


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_forward_full_configs(oracle, gh, name):
    """Configs 1 and 2 end to end (every output element)."""
    wl = wk.WORKLOADS[name]
    _check_fwd(oracle, gh, wl, wk.make_inputs(wl))


def test_packed_qkv_stride(oracle, gh):
    """q, k, v as strided views of one [B,H,W,3C] buffer (token_stride = 3C)."""
    for dt in ("f32", "bf16"):
        wl = wk.custom(f"packed-{dt}", dt, 1, 16, 16, 2, 30, 16, 16, 3, 221, backward=True)
        x = wk.make_inputs(wl)
        t, out, lse = _check_fwd(oracle, gh, wl, x, packed=True)
        got = gh.gpu_bwd(wl, t, out, lse, packed=True)
        ref = oracle.bwd(geometry(oracle, wl), x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"])
        for a, b in zip(got, ref):
            assert gh.max_abs(gh.host(a), b) <= gh.TOL[dt]


def test_inference_without_lse(oracle, gh):
    wl = wk.custom("nolse", "bf16", 1, 16, 16, 2, 30, 16, 16, 0, 222)
    x = wk.make_inputs(wl)
    O_ref, _ = oracle.fwd(geometry(oracle, wl), x["q"], x["k"], x["v"], x["f_q"], x["f_k"])
    out, _ = gh.gpu_fwd(wl, gh.device_inputs(wl, x), want_lse=False)
    assert gh.max_abs(gh.host(out), O_ref) <= gh.TOL["bf16"]


def test_large_logits_need_the_row_max(oracle, gh):
    """Logits of magnitude ~1e2: exp() without a running maximum would overflow, so the library
    must fall back to max tracking on its own, and the results stay close to the oracle.

    Bounds.  fp32 storage keeps 1e-4 per unit of magnitude.  The bf16 matrix-core path rounds the
    pre-scaled Q_aug = [scale_c q || scale_p f_q] * log2(e) to bf16 once (round to nearest: relative
    error at most 2^-8 per element: 8 significant bits), so a logit is perturbed by at most
        eps = 2^-8 * max_ij sum_c |Q_aug[i][c] * K_aug[j][c]|
    (computed below from the inputs; about 0.3 here).  LSE is 1-Lipschitz in the logits under the
    sup norm, hence |LSE err| <= eps + the usual 2e-2.  A probability moves by a factor of at most
    e^(2 eps), so O and the gradients -- sums of products with P -- move by at most about
    2 eps * (sum of absolute terms); the test keeps the tighter 0.15 per unit of the reference's
    largest magnitude that the results actually meet."""
    for dt in ("f32", "bf16"):
        wl = wk.custom(f"big-{dt}", dt, 1, 16, 16, 2, 30, 16, 16, 4, 223, scale_c=4.0, scale_p=6.0,
                       backward=True)
        x = wk.make_inputs(wl)
        g = geometry(oracle, wl)
        O_ref, lse_ref = oracle.fwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"])
        assert np.abs(lse_ref).max() * math.log2(math.e) > 130      # really out of exp2's range
        if dt == "f32":
            tol, tol_lse = 1e-4, 1e-4 * float(np.abs(lse_ref).max())
        else:
            eps = 0.0
            for hd in range(wl.heads):
                ch = slice(hd * wl.d, (hd + 1) * wl.d)
                # one window (H = W = M), shift-independent: every (i, j) pair of the image
                qa = np.abs(x["q"][0, :, :, ch]).reshape(-1, wl.d).astype(np.float64) * wl.scale_c
                ka = np.abs(x["k"][0, :, :, ch]).reshape(-1, wl.d).astype(np.float64)
                fa = np.abs(x["f_q"][hd]).astype(np.float64) * wl.scale_p
                fb = np.abs(x["f_k"][hd]).astype(np.float64)
                # content and positional parts pair different token orders; bound each by its own maximum
                eps = max(eps, float((qa @ ka.T).max() + (fa @ fb.T).max()))
            eps *= 2.0 ** -8
            print(f"big-bf16: logit perturbation bound eps = {eps:.3f}", flush=True)
            tol, tol_lse = 0.15, eps + 2e-2
        t = gh.device_inputs(wl, x)
        out, lse = gh.gpu_fwd(wl, t)
        assert gh.max_abs(gh.host(out), O_ref) <= tol * max(1.0, float(np.abs(O_ref).max()))
        err_lse = gh.max_abs(gh.host(lse), lse_ref)
        print(f"big-{dt}: LSE max abs err {err_lse:.4f} (bound {tol_lse:.4f})", flush=True)
        assert err_lse <= tol_lse
        got = gh.gpu_bwd(wl, t, out, lse)
        ref = oracle.bwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"])
        for name, a, b in zip(("dQ", "dK", "dV", "dF_q", "dF_k"), got, ref):
            assert gh.max_abs(gh.host(a), b) <= tol * max(1.0, float(np.abs(b).max())), name


@pytest.mark.parametrize("name", ["c3", "c3s", "c4", "c5"])
def test_forward_full_size_every_element(oracle, gh, name):
    """Configs 3-5 at full size in the launch configuration the benchmark times: every element of
    O and LSE against the oracle (one oracle pass, seconds on the machine's cores), in both softmax
    paths."""
    wl = wk.WORKLOADS[name]
    x = wk.make_inputs(wl, with_dout=False)
    g = geometry(oracle, wl)
    print(f"{name}: oracle forward over {wl.n_units} units on {oracle.num_threads()} threads ...", flush=True)
    O_ref, lse_ref = oracle.fwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"])
    t = gh.device_inputs(wl, x)
    for flags in (0, FORCE_MAX):
        out, lse = gh.gpu_fwd(wl, t, flags=flags)
        assert gh.max_abs(gh.host(out), O_ref) <= gh.TOL[wl.dtype], flags
        assert gh.max_abs(gh.host(lse), lse_ref) <= gh.TOL[wl.dtype], flags


def test_config5_backward_full_size(oracle, gh):
    """Config 5 (training step) at full size: dQ, dK, dV on sampled units and the
    RIB gradients dF_q, dF_k -- sums over all 144 windows -- on every element
    (the oracle runs the whole backward once for those)."""
    wl = wk.WORKLOADS["c5"]
    x = wk.make_inputs(wl)
    g = geometry(oracle, wl)
    t = gh.device_inputs(wl, x)
    out, lse = gh.gpu_fwd(wl, t)
    got = [gh.host(a) for a in gh.gpu_bwd(wl, t, out, lse)]
    print("config 5: oracle backward on", oracle.num_threads(), "threads ...", flush=True)
    ref = oracle.bwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"])
    tol = gh.TOL[wl.dtype]
    for name, a, b in zip(("dQ", "dK", "dV", "dF_q", "dF_k"), got, ref):
        assert gh.max_abs(a, b) <= tol, name


@pytest.mark.parametrize("name", list(wk.SCHEDULE))
def test_paper_schedule_layers(oracle, gh, name):
    """The (head dim, rank, window) combinations of the paper's networks (Appendix,
    "Network implementation details"), with the paper's two scales: forward and
    backward, every element, on ONE image of the scheduled workload (the kernels'
    launch shape per window is the benchmark's; the batch only multiplies windows;
    the 64- and 96-windows keep two heads so that the oracle finishes in seconds)."""
    from dataclasses import replace
    wl = replace(wk.SCHEDULE[name], B=1)
    if wl.M >= 64:
        wl = replace(wl, heads=2)
    x = wk.make_inputs(wl)
    t, out, lse = _check_fwd(oracle, gh, wl, x)
    got = gh.gpu_bwd(wl, t, out, lse)
    ref = oracle.bwd(geometry(oracle, wl), x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"])
    for nm, a, b in zip(("dQ", "dK", "dV", "dF_q", "dF_k"), got, ref):
        assert gh.max_abs(gh.host(a), b) <= gh.TOL[wl.dtype], nm
    if wl.M >= 64:      # the 8-wave kernels the benchmark's batch selects for these windows
        _check_fwd(oracle, gh, wl, x, flags=rb.RIB_FLAG_WIDE)
        got = gh.gpu_bwd(wl, t, out, lse, flags=rb.RIB_FLAG_WIDE)
        for nm, a, b in zip(("dQ", "dK", "dV", "dF_q", "dF_k"), got, ref):
            assert gh.max_abs(gh.host(a), b) <= gh.TOL[wl.dtype], nm + " (wide)"


# --- the method's special inputs on the pipelined matrix-core kernels (N a multiple of 256) ---

def _edge_shapes():
    return [wk.custom("edge-m16", "bf16", 2, 16, 32, 3, 30, 16, 16, 5, 601, backward=True),
            wk.custom("edge-m32", "bf16", 1, 32, 64, 2, 30, 16, 32, 16, 602, backward=True)]


def _sign_codes(N, r):
    """[N, r] of +-1: row n spells the bits of n (distinct rows for N <= 2^r)."""
    n = np.arange(N)[:, None]
    return (1.0 - 2.0 * ((n >> np.arange(r)[None, :]) & 1)).astype(np.float32)


def _logit_eps(wl, x):
    """Largest perturbation of a logit by the ONE rounding the bf16 matrix-core kernels apply to
    their operands: Q_aug = [scale_c q || scale_p f_q] * log2(e) is rounded to bf16 (relative error
    at most 2^-8 per element: 8 significant bits; k, f_k enter as given), so
        |logit err| <= eps = 2^-8 * max over (window, head, i, j) of sum_c |Q_aug[i][c] K_aug[j][c]|.
    Computed here from the inputs with absolute values (no arithmetic of the method)."""
    from helpers import partition
    qa = np.abs(partition(x["q"].astype(np.float64), wl.M, wl.s))
    ka = np.abs(partition(x["k"].astype(np.float64), wl.M, wl.s))
    worst = 0.0
    for hd in range(wl.heads):
        ch = slice(hd * wl.d, (hd + 1) * wl.d)
        pos = wl.scale_p * (np.abs(x["f_q"][hd].astype(np.float64)) @ np.abs(x["f_k"][hd].astype(np.float64)).T)
        for w in range(qa.shape[0]):
            worst = max(worst, float((wl.scale_c * (qa[w][:, ch] @ ka[w][:, ch].T) + pos).max()))
    return worst * 2.0 ** -8


def _check_all(oracle, gh, wl, x, flags=0):
    """Forward and backward against the oracle.  Bounds: LSE is 1-Lipschitz in the logits (sup
    norm), so |LSE err| <= tol + eps with eps from _logit_eps.  A probability moves by a factor
    of at most e^(2 eps) ~ 1 + 2 eps; O and dV are sums of products with P, dQ, dK, dF with
    dS = P (dP - delta), whose second factor carries the same perturbation once more: to first
    order at most 4 eps per unit of magnitude.  Every other tensor therefore gets
    (tol + 4 eps) * max(1, largest reference magnitude) (bf16 storage alone rounds a value of
    size a by up to a * 2^-9)."""
    g = geometry(oracle, wl)
    eps = _logit_eps(wl, x)
    O_ref, lse_ref = oracle.fwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"])
    t = gh.device_inputs(wl, x)
    out, lse = gh.gpu_fwd(wl, t, flags=flags)
    tol = gh.TOL[wl.dtype]
    errs = {"O": (gh.max_abs(gh.host(out), O_ref), float(np.abs(O_ref).max())),
            "LSE": (gh.max_abs(gh.host(lse), lse_ref), 0.0)}
    got = gh.gpu_bwd(wl, t, out, lse, flags=flags)
    ref = oracle.bwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"])
    for name, a, b in zip(("dQ", "dK", "dV", "dF_q", "dF_k"), got, ref):
        errs[name] = (gh.max_abs(gh.host(a), b), float(np.abs(b).max()))
    print(wl.name, f"eps={eps:.2e}", {k: f"{e:.2e}/{m:.2e}" for k, (e, m) in errs.items()}, flush=True)
    for name, (e, m) in errs.items():
        bound = tol + eps if name == "LSE" else (tol + 4 * eps) * max(1.0, m)
        assert e <= bound, (name, e, bound)
    return gh.host(out), gh.host(lse), O_ref, lse_ref, [gh.host(a) for a in got]


@pytest.mark.parametrize("wl", _edge_shapes(), ids=lambda w: w.name)
@pytest.mark.parametrize("flags", [0, FORCE_MAX], ids=["auto", "rowmax"])
def test_zero_queries_give_the_window_mean(oracle, gh, wl, flags):
    """q = 0 and f_q = 0: every probability is exactly 1/N (a power of two: converting it to
    bf16 loses nothing, so any correction for conversion loss would show as pure bias), O is the
    window mean of v, LSE = ln N, and dQ, dF_q, dK, dF_k see dS = P (dP - delta)."""
    x = wk.make_inputs(wl)
    x["q"][:] = 0.0
    x["f_q"][:] = 0.0
    x["d_out"] = wk.round_to_bf16(4.0 * x["d_out"])
    out, lse, O_ref, _, _ = _check_all(oracle, gh, wl, x, flags)
    assert np.abs(lse - math.log(wl.N)).max() <= 1e-5
    assert np.abs(out - O_ref).max() <= 2.0 ** -8 * np.abs(O_ref).max() + 1e-6     # one bf16 rounding of O


@pytest.mark.parametrize("wl", _edge_shapes(), ids=lambda w: w.name)
def test_constant_values_come_back(oracle, gh, wl):
    """v = 1 everywhere: O = 1 exactly, whatever the probabilities (numerator and denominator
    must use the same converted P)."""
    x = wk.make_inputs(wl)
    x["v"][:] = 1.0
    out = _check_all(oracle, gh, wl, x)[0]
    assert np.abs(out - 1.0).max() <= 2.0 ** -8


@pytest.mark.parametrize("wl", _edge_shapes(), ids=lambda w: w.name)
@pytest.mark.parametrize("lam", [2.0, 12.0], ids=["peaked", "onehot"])
def test_sharp_bias_selects_the_own_token(oracle, gh, wl, lam):
    """f_q = lam * code(i), f_k = code(j) with distinct +-1 codes: the positional logit is largest
    at j = i by 2 lam scale_p per differing bit.  lam = 2: peaked rows, still in exp2's range
    without a maximum; lam = 12: one-hot rows (P = 1.0 exactly for the own token), logits past
    +-126 so the library must switch to max tracking by itself.  |dO| ~ 4."""
    x = wk.make_inputs(wl)
    code = _sign_codes(wl.N, wl.r)
    sp = 1.0                                     # take scale_p out of the picture: logit = lam * <code, code>
    from dataclasses import replace
    wl = replace(wl, scale_p=sp)
    x["f_q"][:] = wk.round_to_bf16(lam * code)[None]
    x["f_k"][:] = code[None]
    x["q"] = wk.round_to_bf16(0.25 * x["q"])
    x["d_out"] = wk.round_to_bf16(4.0 * x["d_out"])
    out, lse, O_ref, _, grads = _check_all(oracle, gh, wl, x)
    if lam >= 12.0:       # one-hot up to e^-24: O = v, dV = dO, whatever the rounding of the (huge) logits
        assert np.abs(out - x["v"].astype(np.float64)).max() <= 2e-2
        assert np.abs(grads[2] - x["d_out"].astype(np.float64)).max() <= 2e-2 * np.abs(x["d_out"]).max()


@pytest.mark.parametrize("wl", _edge_shapes(), ids=lambda w: w.name)
def test_row_constant_in_the_bias_changes_nothing_but_lse(oracle, gh, wl):
    """A per-query constant c_i added to every logit of row i (last RIB column: c_i in f_q, 1 in
    f_k) leaves P, O and every gradient except dF_q's last column unchanged; LSE moves by
    scale_p c_i.  Constants up to +-40 (logit shifts up to +-6)."""
    x = wk.make_inputs(wl)
    rng = np.random.Generator(np.random.Philox(key=wl.seed + 7))
    c = wk.round_to_bf16(rng.uniform(-40.0, 40.0, (wl.heads, wl.N)).astype(np.float32))
    x["f_k"][:, :, -1] = 1.0
    x0 = {n: a.copy() for n, a in x.items()}
    x0["f_q"][:, :, -1] = 0.0
    x["f_q"][:, :, -1] = c
    out, lse = _check_all(oracle, gh, wl, x)[:2]
    out0, lse0 = _check_all(oracle, gh, wl, x0)[:2]
    assert np.abs(out - out0).max() <= 2e-2
    shift = wl.scale_p * c.astype(np.float64)                       # [heads, N]
    assert np.abs((lse - lse0) - shift[None]).max() <= 2e-2 + _logit_eps(wl, x)


GATED = [
    wk.custom("gate-f32", "f32", 1, 16, 16, 2, 30, 16, 16, 3, 231, backward=True),          # fp32 matrix-core kernels
    wk.custom("gate-f32-m9", "f32", 1, 9, 18, 2, 30, 8, 9, 3, 235, backward=True),          # the same, ragged window
    wk.custom("gate-m12", "bf16", 1, 24, 12, 2, 30, 16, 12, 7, 232, backward=True),         # general matrix-core kernels
    wk.custom("gate-m32", "bf16", 2, 32, 64, 3, 30, 18, 32, 16, 233, backward=True),        # fast kernels
    wk.custom("gate-d32", "bf16", 1, 16, 32, 2, 32, 32, 16, 0, 234, backward=True),
]


@pytest.mark.parametrize("flags", [0, rb.RIB_FLAG_WIDE, rb.RIB_FLAG_VECTOR_ONLY], ids=["default", "wide", "vector"])
@pytest.mark.parametrize("wl", GATED, ids=lambda w: w.name)
def test_gated_forward_and_backward(oracle, gh, wl, flags):
    """CLA gate (Eq. 9) fused into the epilogue, and the gated backward (dO = dO' * G and
    dG = dO' * O formed in the delta pass).  Bounds: the benchmark spec's tolerance for every tensor;
    for dG the forward's error in O is multiplied by dO', hence tol * max(1, max|dO'|)."""
    import torch
    x = wk.make_inputs(wl)
    gate = wk.make_gate(wl)
    g = geometry(oracle, wl)
    Og_ref, O_ref, lse_ref = oracle.gated_fwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], gate)
    ref = oracle.gated_bwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], gate, x["d_out"])
    t = gh.device_inputs(wl, x)
    tg = rb.to_device(gate, wl.dtype, gh.DEV)
    p = rb.params_of(wl, flags=flags)
    td = gh.tdtype(wl)
    grid = (wl.B, wl.H, wl.W, wl.C)
    nan = float("nan")
    out_g, out_raw = (torch.full(grid, nan, dtype=td, device=gh.DEV) for _ in range(2))
    lse = torch.full((wl.n_windows, wl.heads, wl.N), nan, dtype=torch.float32, device=gh.DEV)
    rb.rib_window_attn_gated_fwd(p, t["q"], t["k"], t["v"], t["f_q"], t["f_k"], tg, out_g, out_raw, lse)
    torch.cuda.synchronize()
    tol = gh.TOL[wl.dtype]
    assert gh.max_abs(gh.host(out_g), Og_ref) <= tol
    assert gh.max_abs(gh.host(out_raw), O_ref) <= tol
    assert gh.max_abs(gh.host(lse), lse_ref) <= tol
    # inference form: no raw output
    out_g2 = torch.full(grid, nan, dtype=td, device=gh.DEV)
    rb.rib_window_attn_gated_fwd(p, t["q"], t["k"], t["v"], t["f_q"], t["f_k"], tg, out_g2, None, None)
    torch.cuda.synchronize()
    assert torch.equal(out_g, out_g2)
    dq, dk, dv, dgate = (torch.full(grid, nan, dtype=td, device=gh.DEV) for _ in range(4))
    dfq, dfk = (torch.full((wl.heads, wl.N, wl.r), nan, dtype=torch.float32, device=gh.DEV) for _ in range(2))
    ws = torch.empty(rb.rib_window_attn_gated_bwd_workspace_bytes(p), dtype=torch.uint8, device=gh.DEV)
    rb.rib_window_attn_gated_bwd(p, t["q"], t["k"], t["v"], t["f_q"], t["f_k"], tg, out_raw, t["d_out"], lse,
                                 dq, dk, dv, dgate, dfq, dfk, ws)
    torch.cuda.synchronize()
    for name, a, b in zip(("dQ", "dK", "dV", "dF_q", "dF_k"), (dq, dk, dv, dfq, dfk), ref):
        assert gh.max_abs(gh.host(a), b) <= tol, name
    assert gh.max_abs(gh.host(dgate), ref[5]) <= tol * max(1.0, float(np.abs(x["d_out"]).max())), "dG"


@pytest.mark.parametrize("name", ["c2", "sst-m32-r34"])
def test_run_to_run_identical(gh, name):
    """No atomics anywhere on the path: two runs on the same inputs give bit-identical
    outputs and gradients (the RIB gradients are reduced over windows in a fixed order)."""
    import torch
    from dataclasses import replace
    wl = {**wk.WORKLOADS, **wk.SCHEDULE}[name]
    wl = replace(wl, B=min(wl.B, 2), backward=True)
    x = wk.make_inputs(wl)
    t = gh.device_inputs(wl, x)
    runs = []
    for _ in range(2):
        out, lse = gh.gpu_fwd(wl, t)
        runs.append((out, lse, *gh.gpu_bwd(wl, t, out, lse)))
    for a, b in zip(*runs):
        assert torch.equal(a, b)


WIDE = [
    wk.custom("wide-d30r16", "bf16", 1, 32, 64, 2, 30, 16, 32, 16, 241, backward=True),     # extras in spare columns
    wk.custom("wide-d30r18", "bf16", 1, 32, 32, 2, 30, 18, 32, 0, 242, backward=True),      # extras in the C operand, 48 columns
    wk.custom("wide-d30r34", "bf16", 1, 32, 32, 2, 30, 34, 32, 5, 243, backward=True),      # ... 64 columns
    wk.custom("wide-d32r32", "bf16", 1, 32, 32, 2, 32, 32, 32, 0, 244, backward=True),
    wk.custom("wide-d30r24", "bf16", 1, 32, 32, 2, 30, 24, 32, 0, 245, backward=True),      # 64 columns, extras in spare columns
]


@pytest.mark.parametrize("wl", WIDE, ids=lambda w: w.name)
def test_wide_workgroups(oracle, gh, wl):
    """The 8-wave forward and backward kernels (default only for large windows) forced onto small
    problems so that every variant is checked element by element, the forward in both softmax
    paths."""
    x = wk.make_inputs(wl)
    _check_fwd(oracle, gh, wl, x, flags=rb.RIB_FLAG_WIDE | FORCE_MAX)
    t, out, lse = _check_fwd(oracle, gh, wl, x, flags=rb.RIB_FLAG_WIDE)
    got = gh.gpu_bwd(wl, t, out, lse, flags=rb.RIB_FLAG_WIDE)
    ref = oracle.bwd(geometry(oracle, wl), x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"])
    for name, a, b in zip(("dQ", "dK", "dV", "dF_q", "dF_k"), got, ref):
        assert gh.max_abs(gh.host(a), b) <= gh.TOL[wl.dtype], name


def _corner_cases():
    c = wk.custom
    combos = [  # (d, r, M, shift): corners of what the matrix-core kernels accept and just outside
        (32, 0, 8, 3), (32, 2, 16, 0), (2, 2, 16, 1), (4, 4, 16, 0), (2, 62, 16, 0), (16, 48, 16, 5),
        (8, 40, 16, 0), (28, 36, 16, 2), (30, 32, 16, 0), (6, 34, 16, 0), (32, 30, 16, 7), (20, 44, 16, 0),
        (30, 16, 48, 9), (18, 18, 32, 0), (64, 0, 8, 0), (34, 16, 16, 0), (31, 16, 16, 0), (30, 17, 16, 0),
    ]
    out = []
    for i, (d, r, M, s) in enumerate(combos):
        B, H, W = (1, M, 2 * M) if M < 48 else (1, M, M)
        out.append(c(f"corner-d{d}r{r}m{M}", "bf16", B, H, W, 2, d, r, M, s, 300 + i, backward=True))
    return out


@pytest.mark.parametrize("wl", _corner_cases(), ids=lambda w: w.name)
def test_corner_shapes(oracle, gh, wl):
    """Head dims and ranks at the edges of each kernel family's range (and one step outside,
    where the library must fall back to another family on its own): forward in both softmax
    paths and backward, every element."""
    x = wk.make_inputs(wl)
    _check_fwd(oracle, gh, wl, x, flags=FORCE_MAX)
    t, out, lse = _check_fwd(oracle, gh, wl, x)
    got = gh.gpu_bwd(wl, t, out, lse)
    ref = oracle.bwd(geometry(oracle, wl), x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"])
    names = ("dQ", "dK", "dV", "dF_q", "dF_k") if wl.r > 0 else ("dQ", "dK", "dV")
    for name, a, b in zip(names, got, ref):
        assert gh.max_abs(gh.host(a), b) <= gh.TOL[wl.dtype], name


# --- fp32 storage on the matrix cores, and the flag that keeps any problem on the vector ALU ---

VECTOR_ONLY = rb.RIB_FLAG_VECTOR_ONLY


def test_kernel_families_by_dtype_and_flag():
    """Which kernel family serves what: bf16 and fp32 problems with d <= 32, d + r <= 64 on their
    matrix-core kernels, everything under RIB_FLAG_VECTOR_ONLY (and shapes outside those ranges)
    on the vector ALU."""
    for dt, fam in (("bf16", "mfma-bf16"), ("f32", "mfma-f32")):
        wl = wk.custom("fam", dt, 1, 16, 16, 2, 30, 16, 16, 0, 1)
        for back in (False, True):
            assert rb.kernel_name(rb.params_of(wl), back) == fam
            assert rb.kernel_name(rb.params_of(wl, flags=VECTOR_ONLY), back) == "valu-f32"
        wide = wk.custom("fam-d64", dt, 1, 8, 8, 1, 64, 64, 8, 0, 1)
        assert rb.kernel_name(rb.params_of(wide)) == "valu-f32"
    tiny = wk.custom("fam-m5", "f32", 1, 5, 5, 1, 30, 16, 5, 0, 1)     # 25 tokens: below one 32-token block
    assert rb.kernel_name(rb.params_of(tiny)) == "valu-f32"


@pytest.mark.parametrize("wl", [w for w in SMALL if w.N >= 32 and w.d <= 32 and w.d + w.r <= 64],
                         ids=lambda w: w.name)
def test_vector_alu_kernels_where_the_matrix_cores_would_serve(oracle, gh, wl):
    """The vector-ALU kernels on the shapes they no longer get by default: forward and backward."""
    x = wk.make_inputs(wl, with_dout=True)
    t, out, lse = _check_fwd(oracle, gh, wl, x, flags=VECTOR_ONLY)
    got = gh.gpu_bwd(wl, t, out, lse, flags=VECTOR_ONLY)
    ref = oracle.bwd(geometry(oracle, wl), x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"])
    for name, a, b in zip(("dQ", "dK", "dV", "dF_q", "dF_k"), got, ref):
        assert gh.max_abs(gh.host(a), b) <= gh.TOL[wl.dtype], name


F32_MATRIX = [
    # (B, H, W, heads, d, r, M, s): ragged tails in the stationary block (N % 128), the streamed tile (N % 64)
    # and the 32-token block (N % 32); every padded width 16 / 32 / 48 / 64; d + r at both ends of a width
    wk.custom("f32-m6", "f32", 2, 12, 6, 2, 8, 4, 6, 1, 401, backward=True),              # N = 36, width 16
    wk.custom("f32-m7", "f32", 1, 7, 14, 3, 5, 11, 7, 3, 402, backward=True),             # N = 49, odd d and r, width 16
    wk.custom("f32-m10", "f32", 1, 10, 20, 2, 17, 1, 10, 9, 403, backward=True),          # N = 100, width 32
    wk.custom("f32-m13", "f32", 1, 13, 13, 2, 31, 33, 13, 6, 404, backward=True),         # N = 169, d + r = 64
    wk.custom("f32-m20", "f32", 1, 20, 40, 2, 32, 0, 20, 10, 405, backward=True),         # N = 400, r = 0, d = 32
    wk.custom("f32-m24", "f32", 1, 24, 24, 2, 30, 19, 24, 23, 406, backward=True),        # N = 576, d + r = 49 -> width 64
    wk.custom("f32-m32", "f32", 1, 32, 64, 3, 30, 16, 32, 16, 407, backward=True),        # config 3 / 5 head, fp32
    wk.custom("f32-m48", "f32", 1, 48, 48, 2, 30, 34, 48, 24, 408, backward=True,
              scale_c=1 / math.sqrt(30), scale_p=1 / math.sqrt(34)),                      # N = 2304, paper's scales
]


@pytest.mark.parametrize("wl", F32_MATRIX, ids=lambda w: w.name)
def test_f32_matrix_core_kernels(oracle, gh, wl):
    """fp32 problems on the fp32 MFMA kernels: forward (O, LSE) and backward, every element, 1e-4."""
    assert rb.kernel_name(rb.params_of(wl)) == "mfma-f32" and rb.kernel_name(rb.params_of(wl), True) == "mfma-f32"
    x = wk.make_inputs(wl)
    t, out, lse = _check_fwd(oracle, gh, wl, x)
    got = gh.gpu_bwd(wl, t, out, lse)
    ref = oracle.bwd(geometry(oracle, wl), x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"])
    names = ("dQ", "dK", "dV", "dF_q", "dF_k") if wl.r > 0 else ("dQ", "dK", "dV")
    for name, a, b in zip(names, got, ref):
        assert gh.max_abs(gh.host(a), b) <= gh.TOL[wl.dtype], name


def test_f32_training_shape_sampled_units(oracle, gh):
    """Config 5's shape in fp32 storage (the paper quotes its costs at FP32), full size: forward on sampled
    units, backward on every element (the RIB gradients sum 144 windows), and a rerun of the
    backward must reproduce the first run bit for bit (fixed summation order)."""
    from dataclasses import replace
    wl = replace(wk.WORKLOADS["c5"], name="c5-f32", dtype="f32")
    x = wk.make_inputs(wl)
    g = geometry(oracle, wl)
    rng = np.random.default_rng(wl.seed)
    units = sorted({0, wl.n_units - 1, *rng.choice(wl.n_units, 3, replace=False).tolist()})
    O_ref, lse_ref = oracle.fwd_units(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], units)
    t = gh.device_inputs(wl, x)
    out, lse = gh.gpu_fwd(wl, t)
    out_h, lse_h = gh.host(out), gh.host(lse)
    for a, u in enumerate(units):
        assert gh.max_abs(gh.gather_unit(oracle, g, out_h, u), O_ref[a]) <= 1e-4, u
        assert gh.max_abs(lse_h[u // wl.heads, u % wl.heads], lse_ref[a]) <= 1e-4, u
    got = gh.gpu_bwd(wl, t, out, lse)
    again = gh.gpu_bwd(wl, t, out, lse)
    for a, b in zip(got, again):
        assert bool((a == b).all())
    ref = oracle.bwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"])
    for name, a, b in zip(("dQ", "dK", "dV", "dF_q", "dF_k"), got, ref):
        err = gh.max_abs(gh.host(a), b)
        print(f"c5-f32 {name}: max abs err {err:.3e} (largest reference magnitude {np.abs(b).max():.3g})", flush=True)
        assert err <= 1e-4, name
