"""Pins of the RIB feature-generator oracle (oracle/features.py) against what the
paper's Sec. 3.1 Eq. 1-3 and plain mathematics fix: coordinate endpoints and
order, trigonometric identities that tie the Fourier bands to each other,
special weights that reduce the MLP to something known in closed form,
symmetries of the window, and central finite differences for the backward."""
import numpy as np
import pytest

from oracle import features as F
from paper_2603_06738_amd import workloads as wk


def test_coordinates_span_minus_one_to_one_row_major():
    x = F.coordinates(5)
    assert x.shape == (25, 2)
    np.testing.assert_allclose(x[0], [-1, -1])
    np.testing.assert_allclose(x[4], [-1, 1])          # token 4 = row 0, last column
    np.testing.assert_allclose(x[5], [-0.5, -1])       # token 5 = row 1, first column
    np.testing.assert_allclose(x[12], [0, 0])          # centre of an odd window
    np.testing.assert_allclose(x[24], [1, 1])
    np.testing.assert_allclose(F.coordinates(1), [[0, 0]])
    # equally spaced, both axes
    ax = F.coordinates(16)[:16, 1]
    np.testing.assert_allclose(np.diff(ax), 2 / 15)


def test_fourier_width_order_and_band_identities():
    L = 10
    x = F.coordinates(7)
    g = F.fourier(x, L)
    assert g.shape == (49, 2 + 4 * L)                                  # Eq. 1: width 2 + 4L
    np.testing.assert_array_equal(g[:, :2], x)                          # raw coordinates first
    np.testing.assert_array_equal(F.fourier(x, 0), x)
    s = lambda l: g[:, 2 + 4 * l: 4 + 4 * l]
    c = lambda l: g[:, 4 + 4 * l: 6 + 4 * l]
    np.testing.assert_allclose(s(0), np.sin(x), atol=1e-15)            # band 0 has frequency 2^0 = 1
    for l in range(L):
        np.testing.assert_allclose(s(l) ** 2 + c(l) ** 2, 1.0, atol=1e-12)
        if l + 1 < L:                                                   # consecutive bands: the frequency doubles
            np.testing.assert_allclose(s(l + 1), 2 * s(l) * c(l), atol=1e-10)
            np.testing.assert_allclose(c(l + 1), c(l) ** 2 - s(l) ** 2, atol=1e-10)
    centre = g[24]
    np.testing.assert_allclose(centre[2::4], 0, atol=1e-15)            # sin(0) = 0 in every band (row part)
    np.testing.assert_allclose(centre[4::4], 1, atol=1e-15)            # cos(0) = 1


def _params(heads=2, r=4, L=3, d_h=6, seed=7):
    return {k: v.astype(np.float64) for k, v in wk.make_generator_params(heads, r, L, d_h, seed).items()}


def test_selector_weights_expose_single_features():
    """W_h that copies feature a into hidden unit c, zero bias, identity-like head
    projection: f_q is ReLU of that Fourier feature."""
    M, L, d_h, r = 6, 2, 4, 4
    n_in = 2 + 4 * L
    g = F.fourier(F.coordinates(M), L)
    picks = [1, 2, 5, 9]                                # column coord, sin(row), cos(col) of band 0, cos(col) of band 1
    W_h = np.zeros((n_in, d_h))
    for cidx, a in enumerate(picks):
        W_h[a, cidx] = 1.0
    W_p = np.eye(d_h, r)[None]
    f_q, f_k = F.features_fwd(M, L, W_h, np.zeros(d_h), W_p, 2 * W_p)
    np.testing.assert_allclose(f_q[0], np.maximum(g[:, picks], 0), atol=1e-15)
    np.testing.assert_allclose(f_k[0], 2 * np.maximum(g[:, picks], 0), atol=1e-15)
    assert (f_q[0][:, 0] == 0).sum() >= M * M // 2 - M  # ReLU really clips the negative half of the column coordinate


def test_bias_only_network_is_constant_over_tokens():
    p = _params()
    W_h = np.zeros_like(p["W_h"])
    b_h = np.array([0.5, -1.0, 2.0, -0.1, 0.0, 1.5])
    f_q, _ = F.features_fwd(4, 3, W_h, b_h, p["W_pq"], p["W_pk"])
    expect = np.maximum(b_h, 0) @ p["W_pq"][1].astype(np.float64)
    np.testing.assert_allclose(f_q[1], np.broadcast_to(expect, (16, 4)), atol=1e-12)


def test_heads_are_independent_and_projection_is_linear():
    p = _params()
    f_q, f_k = F.features_fwd(5, 3, p["W_h"], p["b_h"], p["W_pq"], p["W_pk"])
    W2 = p["W_pq"].copy()
    W2[1] *= -3.0
    g_q, g_k = F.features_fwd(5, 3, p["W_h"], p["b_h"], W2, p["W_pk"])
    np.testing.assert_array_equal(g_q[0], f_q[0])
    np.testing.assert_allclose(g_q[1], -3.0 * f_q[1], rtol=1e-12)
    np.testing.assert_array_equal(g_k, f_k)             # f_k does not see W_pq


def test_vertical_flip_symmetry_identifies_row_features():
    """Reversing the rows of the window negates the row coordinate: the features
    must equal those of a network whose W_h rows for the ODD functions of the row
    coordinate (the coordinate itself and its sines) are negated."""
    M, L = 6, 3
    p = _params(L=L)
    f_q, _ = F.features_fwd(M, L, p["W_h"], p["b_h"], p["W_pq"], p["W_pk"])
    W_flip = p["W_h"].astype(np.float64).copy()
    odd_row = [0] + [2 + 4 * l for l in range(L)]
    W_flip[odd_row] *= -1.0
    g_q, _ = F.features_fwd(M, L, W_flip, p["b_h"], p["W_pq"], p["W_pk"])
    flipped = f_q.reshape(-1, M, M, f_q.shape[-1])[:, ::-1].reshape(f_q.shape)
    np.testing.assert_allclose(g_q, flipped, atol=1e-12)
    # and the analogous statement for the columns
    W_flip = p["W_h"].astype(np.float64).copy()
    W_flip[[1] + [3 + 4 * l for l in range(L)]] *= -1.0
    g_q, _ = F.features_fwd(M, L, W_flip, p["b_h"], p["W_pq"], p["W_pk"])
    flipped = f_q.reshape(-1, M, M, f_q.shape[-1])[:, :, ::-1].reshape(f_q.shape)
    np.testing.assert_allclose(g_q, flipped, atol=1e-12)


@pytest.mark.parametrize("M,L", [(4, 2), (5, 10)])
def test_backward_matches_central_differences(M, L):
    heads, r, d_h = 2, 3, 5
    p = {k: v.astype(np.float64) for k, v in wk.make_generator_params(heads, r, L, d_h, 11).items()}
    g = {k: v.astype(np.float64) for k, v in wk.make_feature_grads(heads, M, r, 12).items()}

    def loss(q):
        f_q, f_k = F.features_fwd(M, L, q["W_h"], q["b_h"], q["W_pq"], q["W_pk"])
        return float((f_q * g["df_q"]).sum() + (f_k * g["df_k"]).sum())

    grads = dict(zip(("W_h", "b_h", "W_pq", "W_pk"),
                     F.features_bwd(M, L, p["W_h"], p["b_h"], p["W_pq"], p["W_pk"], g["df_q"], g["df_k"])))
    rng = np.random.default_rng(3)
    eps = 1e-6
    for name in grads:
        assert grads[name].shape == p[name].shape
        for _ in range(4):
            direction = rng.standard_normal(p[name].shape)
            plus = dict(p); plus[name] = p[name] + eps * direction
            minus = dict(p); minus[name] = p[name] - eps * direction
            fd = (loss(plus) - loss(minus)) / (2 * eps)
            an = float((grads[name] * direction).sum())
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, fd, an)
