"""bench.py's command-line contract as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_workload_tables_are_consistent():
    from paper_2603_06738_amd import workloads as wk
    for name, wl in {**wk.WORKLOADS, **wk.SCHEDULE}.items():
        assert wl.H % wl.M == 0 and wl.W % wl.M == 0 and 0 <= wl.s < wl.M, name
        assert wl.fwd_flop == 2.0 * wl.N * wl.N * (2 * wl.d + wl.r) * wl.n_units
        assert wl.bwd_flop == 2.0 * wl.N * wl.N * (5 * wl.d + 3 * wl.r) * wl.n_units
    # config 5 is the benchmark's step: 137.7 GFLOP forward, 16 x 96 x 96 tokens
    c5 = wk.WORKLOADS["c5"]
    assert c5.backward and c5.tokens == 147456 and abs(c5.fwd_flop / 1e9 - 137.7) < 0.1
