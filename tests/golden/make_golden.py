#!/usr/bin/env python3
"""Writes the stored expected values under tests/golden/ by calling ONLY the CPU oracle
(oracle/) on seeded inputs from paper_2603_06738_amd.workloads.  Nothing here touches the
GPU library.  Run from the repository root:  python tests/golden/make_golden.py

The paper (Sec. 3.1 Eq. 5-6, Sec. 2.2) prints no numeric worked example of the operator, so
there is no fixture quoted from it; these files freeze the oracle's own output at sampled
positions of config 1 (fp32, B=1, 48x48, 2 heads, d=30, r=8, 16x16 windows) so that a later
change to the oracle's arithmetic cannot pass unnoticed, and give the GPU tests a second,
file-based reference for the same launch.
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2603_06738_amd import workloads as wk  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def sample_positions(wl, n, seed):
    rng = np.random.default_rng(seed)
    return [(int(rng.integers(wl.B)), int(rng.integers(wl.H)), int(rng.integers(wl.W)), int(rng.integers(wl.C)))
            for _ in range(n)]


def main():
    wl = wk.WORKLOADS["c1"]
    x = wk.make_inputs(wl, with_dout=True)
    g = oracle.Geometry(wl.B, wl.H, wl.W, wl.heads, wl.d, wl.r, wl.M, wl.s, wl.scale_c, wl.scale_p)
    O, lse = oracle.fwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"])
    dQ, dK, dV, dFq, dFk = oracle.bwd(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"])
    pos = sample_positions(wl, 48, 20260306)
    with open(os.path.join(HERE, "c1_oracle_samples.txt"), "w") as f:
        f.write("# config 1, oracle output at sampled grid positions: b y x c  O dQ dK dV (float64, repr)\n")
        for (b, y, xx, c) in pos:
            f.write(f"{b} {y} {xx} {c} {float(O[b, y, xx, c])!r} {float(dQ[b, y, xx, c])!r} {float(dK[b, y, xx, c])!r} {float(dV[b, y, xx, c])!r}\n")
        f.write("# LSE at sampled (window, head, token) and RIB gradients at sampled (head, token, column)\n")
        rng = np.random.default_rng(7)
        for _ in range(16):
            w_, h_, n_ = int(rng.integers(lse.shape[0])), int(rng.integers(wl.heads)), int(rng.integers(wl.N))
            j = int(rng.integers(wl.r))
            f.write(f"L {w_} {h_} {n_} {j} {float(lse[w_, h_, n_])!r} {float(dFq[h_, n_, j])!r} {float(dFk[h_, n_, j])!r}\n")
    print("wrote c1_oracle_samples.txt")


if __name__ == "__main__":
    main()
