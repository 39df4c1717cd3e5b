"""Stored oracle samples of config 1 (tests/golden/c1_oracle_samples.txt, written by
tests/golden/make_golden.py from the oracle alone): the oracle must keep reproducing them, and
the GPU library must match them within the fp32 tolerance."""
import os

import numpy as np
import pytest

from paper_2603_06738_amd import workloads as wk
from helpers import geometry

PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "c1_oracle_samples.txt")


def _load():
    grid, feat = [], []
    for line in open(PATH):
        if line.startswith("#"):
            continue
        p = line.split()
        if p[0] == "L":
            feat.append((tuple(int(v) for v in p[1:5]), [float(v) for v in p[5:]]))
        else:
            grid.append((tuple(int(v) for v in p[:4]), [float(v) for v in p[4:]]))
    return grid, feat


def _compare(O, lse, dQ, dK, dV, dFq, dFk, tol):
    grid, feat = _load()
    assert len(grid) == 48 and len(feat) == 16
    for (b, y, x, c), (o, dq, dk, dv) in grid:
        for got, want in ((O, o), (dQ, dq), (dK, dk), (dV, dv)):
            assert abs(float(got[b, y, x, c]) - want) <= tol
    for (w, h, n, j), (l, gq, gk) in feat:
        assert abs(float(lse[w, h, n]) - l) <= tol
        assert abs(float(dFq[h, n, j]) - gq) <= tol and abs(float(dFk[h, n, j]) - gk) <= tol


def test_oracle_reproduces_stored_samples(oracle):
    wl = wk.WORKLOADS["c1"]
    x = wk.make_inputs(wl, with_dout=True)
    g = geometry(oracle, wl)
    O, lse = oracle.fwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"])
    grads = oracle.bwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"])
    _compare(O, lse, *grads, tol=1e-12)


@pytest.mark.gpu
def test_gpu_matches_stored_samples():
    import gpu_helpers as gh
    wl = wk.WORKLOADS["c1"]
    x = wk.make_inputs(wl, with_dout=True)
    t = gh.device_inputs(wl, x)
    out, lse = gh.gpu_fwd(wl, t)
    got = gh.gpu_bwd(wl, t, out, lse)
    _compare(gh.host(out), gh.host(lse), *[gh.host(a) for a in got], tol=gh.TOL["f32"])
