#!/usr/bin/env python3
"""Benchmark of the RIB window-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5] [--all]

One "step" is one pass of the whole hot path over one batch of synthetic input:
forward (gather + RIB concat + scores + online softmax + PV + scatter) followed,
for the training workload, by the backward pass (delta, dQ/dK/dV, RIB gradient
reduction).  The default workload is the training-step configuration (config 5: fwd+bwd, bf16,
B=16, 96x96 grid, 32x32 windows, shift 16).  Inputs are resident in HBM before
the timed region starts.  Prints ONE JSON line.

`--all` adds a `configs` table with forward numbers for every named workload and a
`schedule` table (forward and backward) for the layer shapes of the paper's networks.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, vendor figure
PEAK_F32_VALU_TFLOPS = 157.3  # MI355X fp32 vector, vendor figure
PEAK_F32_MFMA_TFLOPS = 157.3  # MI355X dense fp32 MFMA, vendor figure
PEAK_HBM_GBS = 8000.0
# HBM bytes per launch are NOT measured by this script (that takes rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs,
# scaled by a plain copy of known size).  Where such a run of this very workload is committed under profiles/,
# `traffic` carries its figure and `traffic_from_profile` says which file it comes from; otherwise `traffic` is null.
PROFILED_TRAFFIC = {
    "c5": {"forward": {"bytes": 250.5e6, "source": "profiles/c5_step_hbm_traffic.md"},
           "backward": {"bytes": 1041.0e6, "source": "profiles/c5_step_hbm_traffic.md"},
           "kernels": {"mfma_fwd_stream_kernel": 250.5e6, "mfma_bwd_dq_fast_kernel": 451.5e6,
                       "mfma_bwd_dkv_fast_kernel": 475.4e6, "reduce_df_kernel": 114.1e6}},
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="c5")
    ap.add_argument("--dtype", choices=["bf16", "f32"], default=None,
                    help="run the workload in this storage type instead of its own (fp32: the fp32 MFMA kernels)")
    ap.add_argument("--all", action="store_true", help="also time the forward of every named workload")
    ap.add_argument("--rotate", type=int, default=1,
                    help="cycle the steps through this many distinct sets of buffers, so that a workload smaller than "
                         "the 256 MB Infinity Cache is read from HBM (for counter runs on the small-window configs)")
    ap.add_argument("--force-row-max", action="store_true", help="time the max-tracking softmax path")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-c3", action="store_true", help="skip the extra forward run of config 3")
    ap.add_argument("--no-kernel-table", action="store_true",
                    help="skip the torch.profiler pass (use under rocprofv3: two tracers in one process disagree)")
    ap.add_argument("--cpu-units", type=int, default=0, help="units in the CPU-oracle sample (0 = auto)")
    return ap.parse_args()


def family_peak(family):
    """(published peak in TFLOP/s, roofline bound) of a kernel family."""
    if family == "mfma-bf16":
        return PEAK_BF16_TFLOPS, "mfma"
    if family == "mfma-f32":
        return PEAK_F32_MFMA_TFLOPS, "mfma"
    return PEAK_F32_VALU_TFLOPS, "alu"


class Runner:
    """Device buffers of one workload plus closures that enqueue fwd / bwd."""

    def __init__(self, wl, flags=0):
        import torch
        from paper_2603_06738_amd import binding as rb
        from paper_2603_06738_amd import workloads as wk
        self.wl, self.rb, self.torch = wl, rb, torch
        x = wk.make_inputs(wl, with_dout=wl.backward)
        self.t = {n: rb.to_device(a, wl.dtype) for n, a in x.items()}
        del x
        td = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        dev = "cuda:0"
        grid = (wl.B, wl.H, wl.W, wl.C)
        self.p = rb.params_of(wl, flags=flags)
        self.out = torch.empty(grid, dtype=td, device=dev)
        self.lse = torch.empty((wl.n_windows, wl.heads, wl.N), dtype=torch.float32, device=dev)
        if wl.backward:
            self.dq, self.dk, self.dv = (torch.empty(grid, dtype=td, device=dev) for _ in range(3))
            self.dfq, self.dfk = (torch.empty((wl.heads, wl.N, wl.r), dtype=torch.float32, device=dev)
                                  for _ in range(2))
            self.ws = rb.alloc_workspace(self.p)

    def fwd(self):
        t = self.t
        self.rb.rib_window_attn_fwd(self.p, t["q"], t["k"], t["v"], t["f_q"], t["f_k"], self.out, self.lse)

    def bwd(self):
        t = self.t
        self.rb.rib_window_attn_bwd(self.p, t["q"], t["k"], t["v"], t["f_q"], t["f_k"], self.out, t["d_out"],
                                    self.lse, self.dq, self.dk, self.dv, self.dfq, self.dfk, self.ws)


def time_steps(r, steps, warmup, others=()):
    """Returns (wall ms per step, mean fwd ms, mean bwd ms) with HIP events on the launch stream.
    `others`: further Runners of the same workload; the steps then cycle through all of them."""
    torch = r.torch
    ring = (r,) + tuple(others)
    for i in range(warmup):
        ring[i % len(ring)].fwd()
        if r.wl.backward:
            ring[i % len(ring)].bwd()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    t0 = time.perf_counter()
    for s in range(steps):
        cur = ring[s % len(ring)]
        ev[s][0].record()
        cur.fwd()
        ev[s][1].record()
        if r.wl.backward:
            cur.bwd()
        ev[s][2].record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    f = sorted(e[0].elapsed_time(e[1]) for e in ev)
    b = sorted(e[1].elapsed_time(e[2]) for e in ev)
    r.last_stats = {"fwd_ms_median": round(f[len(f) // 2], 4), "fwd_ms_min": round(f[0], 4),
                    "bwd_ms_median": round(b[len(b) // 2], 4), "bwd_ms_min": round(b[0], 4)}
    return wall, sum(f) / steps, sum(b) / steps


def kernel_flop(name, wl):
    """(algorithmic flop per launch, note) of one of the library's kernels, by name.  The backward's
    5 contractions (2 N^2 (5d + 3r) per unit) are split without double counting: the dkv kernel gets the
    scores, dP, dV and dK_aug (4d + 2r), the dq kernel only dQ_aug (d + r): the scores and dP it
    recomputes are overhead of the two-kernel split, not algorithmic work."""
    per = 2.0 * wl.N * wl.N * wl.n_units
    if "fwd" in name:
        return wl.fwd_flop, "S, PV"
    if "dkv" in name:
        return per * (4 * wl.d + 2 * wl.r), "S, dP, dV, dK_aug"
    if "dq" in name:
        return per * (wl.d + wl.r), "dQ_aug (S and dP are recomputed: not counted)"
    return 0.0, "memory-bound helper"


PROFILE_STEPS = 20


def profile_kernels(r, steps=PROFILE_STEPS):
    """Device time per launch (mean, median, minimum) of every kernel of one step, from a torch.profiler
    (roctracer) pass over `steps` steps.  The pass is separate from the timed region: under the tracer the
    kernels run about a tenth slower, so the caller uses these figures for the split between kernels only."""
    try:
        from torch.profiler import profile, ProfilerActivity
        torch = r.torch
        with profile(activities=[ProfilerActivity.CUDA]) as prof:
            for _ in range(steps):
                r.fwd()
                if r.wl.backward:
                    r.bwd()
            torch.cuda.synchronize()
        per = {}
        for e in prof.events():
            if "rib::" not in e.name or "_kernel" not in e.name:
                continue
            m = re.search(r"(\w+_kernel)(<[^(]*>)?", e.name)
            short = (m.group(1) + (m.group(2) or "")) if m else e.name[:60]
            per.setdefault(short, []).append(e.time_range.elapsed_us())
        out = {}
        for short, us in per.items():
            us.sort()
            out[short] = {"avg_us": round(sum(us) / len(us), 2), "median_us": round(us[len(us) // 2], 2),
                          "min_us": round(us[0], 2), "calls": len(us)}
        return out
    except Exception as exc:       # no tracer in this build of torch: the aggregate figures still stand
        return {"error": repr(exc)}


def time_cold(wl, flags, sets=4, reps=40):
    """Forward time with the inputs rotated through `sets` distinct buffer sets, so that a small
    workload is not served from the 256 MB Infinity Cache: ms per launch."""
    import torch
    rs = [Runner(wl, flags) for _ in range(sets)]
    for r in rs:
        r.fwd()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps):
        rs[i % sets].fwd()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def time_generator(rb, torch, M=96, heads=6, r=34, L=10, d_h=32, reps=20):
    """RIB feature generator (Eq. 1-3) at the largest window of the paper's schedule: ms per call."""
    from paper_2603_06738_amd import workloads as wk
    dev = "cuda:0"
    w = {k: torch.from_numpy(v).to(dev) for k, v in wk.make_generator_params(heads, r, L, d_h).items()}
    g = {k: torch.from_numpy(v).to(dev) for k, v in wk.make_feature_grads(heads, M, r).items()}
    p = rb.make_gen_params(M, heads, r, L, d_h, "bf16")
    f_q = torch.empty((heads, M * M, r), dtype=torch.bfloat16, device=dev)
    f_k = torch.empty_like(f_q)
    grads = [torch.empty_like(w[n]) for n in ("W_h", "b_h", "W_pq", "W_pk")]
    ws = torch.empty(rb.rib_features_bwd_workspace_bytes(p), dtype=torch.uint8, device=dev)
    fwd = lambda: rb.rib_features_fwd(p, w["W_h"], w["b_h"], w["W_pq"], w["W_pk"], f_q, f_k)
    bwd = lambda: rb.rib_features_bwd(p, w["W_h"], w["b_h"], w["W_pq"], w["W_pk"], g["df_q"], g["df_k"], *grads, ws)
    out = {"window": M, "heads": heads, "r": r, "L": L, "d_h": d_h}
    for name, fn in (("fwd_ms", fwd), ("bwd_ms", bwd)):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name] = round(e0.elapsed_time(e1) / reps, 4)
    return out


def time_gated(rb, torch, wl, reps=30):
    """The same step with the CLA gate (Eq. 9) fused into the forward epilogue and the delta pass."""
    from paper_2603_06738_amd import workloads as wk
    r = Runner(wl)
    gate = rb.to_device(wk.make_gate(wl), wl.dtype)
    out_g, dgate = torch.empty_like(r.out), torch.empty_like(r.out)
    ws = torch.empty(rb.rib_window_attn_gated_bwd_workspace_bytes(r.p), dtype=torch.uint8, device="cuda:0")
    t = r.t

    def fwd():
        rb.rib_window_attn_gated_fwd(r.p, t["q"], t["k"], t["v"], t["f_q"], t["f_k"], gate, out_g, r.out, r.lse)

    def bwd():
        rb.rib_window_attn_gated_bwd(r.p, t["q"], t["k"], t["v"], t["f_q"], t["f_k"], gate, r.out, t["d_out"], r.lse,
                                     r.dq, r.dk, r.dv, dgate, r.dfq, r.dfk, ws)

    def fwd_infer():
        rb.rib_window_attn_gated_fwd(r.p, t["q"], t["k"], t["v"], t["f_q"], t["f_k"], gate, out_g, None, None)

    res = {}
    for name, fn in (("fwd_ms", fwd), ("fwd_inference_ms", fwd_infer), ("bwd_ms", bwd)):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        res[name] = round(e0.elapsed_time(e1) / reps, 4)
    return res


def cpu_baseline(wl, n_units):
    """The CPU oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np
    import oracle
    from paper_2603_06738_amd import workloads as wk
    g = oracle.Geometry(wl.B, wl.H, wl.W, wl.heads, wl.d, wl.r, wl.M, wl.s, wl.scale_c, wl.scale_p)
    x = wk.make_inputs(wl, with_dout=wl.backward)
    units = np.linspace(0, wl.n_units - 1, n_units).astype(np.int64)
    t0 = time.perf_counter()
    oracle.fwd_units(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], units)
    if wl.backward:
        oracle.bwd_units(g, x["q"], x["k"], x["v"], x["f_q"], x["f_k"], x["d_out"], units)
    dt = time.perf_counter() - t0
    flop = (wl.fwd_flop + (wl.bwd_flop if wl.backward else 0.0)) * n_units / wl.n_units
    return {"value": flop / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "seconds": round(dt, 3),
            "sample": f"{n_units} of {wl.n_units} (window, head) units of {wl.name}, "
                      f"{'fwd+bwd' if wl.backward else 'fwd'}, fp64"}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives are part of it); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2603_06738_amd import binding as rb
    from paper_2603_06738_amd import workloads as wk
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    rb.load()
    wl = {**wk.WORKLOADS, **wk.SCHEDULE}[a.workload]
    if a.dtype and a.dtype != wl.dtype:
        wl = wl.__class__(**{**wl.__dict__, "dtype": a.dtype, "name": wl.name + "-" + a.dtype})
    flags = rb.RIB_FLAG_FORCE_ROW_MAX if a.force_row_max else 0

    r = Runner(wl, flags)
    others = [Runner(wl, flags) for _ in range(max(1, a.rotate) - 1)]
    wall, fwd_ms, bwd_ms = time_steps(r, a.steps, a.warmup, others)
    del others
    step_flop = wl.fwd_flop + (wl.bwd_flop if wl.backward else 0.0)
    value = step_flop / (wall * 1e-3) / 1e12

    fwd_tflops = wl.fwd_flop / (fwd_ms * 1e-3) / 1e12
    res = {
        "metric": "RIB window-attention TFLOP/s fwd(+bwd) at 32x32 windows",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(wall, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: {'fwd+bwd' if wl.backward else 'fwd'} {wl.dtype} "
                               f"B={wl.B} H=W={wl.H} C={wl.C} heads={wl.heads} d={wl.d} r={wl.r} "
                               f"window={wl.M} shift={wl.s}",
                   "softmax_path": "row-max" if a.force_row_max else "auto", "buffer_sets": max(1, a.rotate),
                   "kernels": {"fwd": rb.kernel_name(r.p, False), "bwd": rb.kernel_name(r.p, True)}},
        "tokens_per_s": round(wl.tokens / (wall * 1e-3), 1),
        "fwd_ms": round(fwd_ms, 4), "fwd_tflops": round(fwd_tflops, 2),
        "fwd_pct_bf16_peak": round(100 * fwd_tflops / PEAK_BF16_TFLOPS, 2),
        "fwd_ms_median": r.last_stats["fwd_ms_median"], "fwd_ms_min": r.last_stats["fwd_ms_min"],
    }
    if wl.backward:
        bwd_tflops = wl.bwd_flop / (bwd_ms * 1e-3) / 1e12
        res.update(bwd_ms=round(bwd_ms, 4), bwd_tflops=round(bwd_tflops, 2),
                   bwd_pct_bf16_peak=round(100 * bwd_tflops / PEAK_BF16_TFLOPS, 2),
                   bwd_ms_median=r.last_stats["bwd_ms_median"], bwd_ms_min=r.last_stats["bwd_ms_min"])
    # Rooflines.  fwd / bwd: HIP events of this run around the library calls (the forward is ONE kernel launch,
    # the backward four).  `roofline` is the kernel that takes the largest share of the step, timed per launch by
    # a torch.profiler pass of this same process (events cannot separate launches made inside one library call).
    fam = rb.kernel_name(r.p, False)
    peak, bound = family_peak(fam)
    prof_traffic = PROFILED_TRAFFIC.get(wl.name, {})
    res["roofline_fwd"] = {"kernel": "forward (" + fam + "), one launch", "bound": bound, "achieved": round(fwd_tflops, 2),
                           "peak": peak, "unit": "TFLOP/s", "frac": round(fwd_tflops / peak, 4),
                           "traffic": (prof_traffic.get("forward") or {}).get("bytes"),
                           "traffic_from_profile": prof_traffic.get("forward"),
                           "algorithmic_flop": wl.fwd_flop, "algorithmic_bytes": wl.fwd_bytes,
                           "time_source": "HIP events on the launch stream, this run"}
    if wl.backward:
        bpeak, bbound = family_peak(rb.kernel_name(r.p, True))
        res["roofline_bwd"] = {"kernel": "backward (" + rb.kernel_name(r.p, True) + "), all its launches",
                               "bound": bbound, "achieved": round(bwd_tflops, 2),
                               "peak": bpeak, "unit": "TFLOP/s", "frac": round(bwd_tflops / bpeak, 4),
                               "traffic": (prof_traffic.get("backward") or {}).get("bytes"),
                               "traffic_from_profile": prof_traffic.get("backward"),
                               "algorithmic_flop": wl.bwd_flop, "time_source": "HIP events on the launch stream, this run"}
    kern = {} if a.no_kernel_table else profile_kernels(r)
    res["kernels"] = kern
    # The tracer's own overhead idles the GPU between launches and every kernel then runs about a tenth slower
    # than in the timed region.  The durations used below are therefore the event-timed phase (forward or
    # backward, this run) split in the proportions the tracer saw: launch_us = phase_ms * share.
    rows = {n: k for n, k in kern.items() if isinstance(k, dict) and "avg_us" in k}
    for is_bwd, phase_ms in ((False, fwd_ms), (True, bwd_ms)):
        names = [n for n in rows if ("fwd" not in n) == is_bwd]
        total = sum(rows[n]["avg_us"] * rows[n]["calls"] for n in names)
        for n in names:
            share = rows[n]["avg_us"] * rows[n]["calls"] / total
            rows[n].update(tracer_avg_us=rows[n].pop("avg_us"), tracer_median_us=rows[n].pop("median_us"),
                           tracer_min_us=rows[n].pop("min_us"), share_of_phase=round(share, 4),
                           launch_us=round(phase_ms * 1e3 * share * PROFILE_STEPS / rows[n]["calls"], 2))
    dominant = None
    for name, k in rows.items():
        flop, what = kernel_flop(name, wl)
        pk, bd = family_peak(rb.kernel_name(r.p, "fwd" not in name))
        k.update(algorithmic_flop=flop, counts=what)
        if flop > 0:
            tf = flop / (k["launch_us"] * 1e-6) / 1e12
            k.update(tflops=round(tf, 1), frac=round(tf / pk, 4), peak=pk, bound=bd)
        if dominant is None or k["launch_us"] * k["calls"] > rows[dominant]["launch_us"] * rows[dominant]["calls"]:
            dominant = name
    if dominant is not None and "frac" in rows[dominant]:
        k = rows[dominant]
        res["roofline"] = {"kernel": dominant, "bound": k["bound"], "achieved": k["tflops"], "peak": k["peak"],
                           "unit": "TFLOP/s", "frac": k["frac"], "algorithmic_flop": k["algorithmic_flop"],
                           "avg_launch_us": k["launch_us"],
                           "traffic_from_profile": next(({"bytes": b, "source": prof_traffic["forward"]["source"]}
                                                         for n, b in prof_traffic.get("kernels", {}).items()
                                                         if dominant.startswith(n)), None),
                           "time_source": "HIP events around the phase on the launch stream (this run), split between the "
                                          "phase's kernels in the proportions of a torch.profiler pass of 20 steps"}
        # HBM bytes per launch: the rocprofv3 FETCH_SIZE / WRITE_SIZE runs under profiles/ (not this run), else null
        res["roofline"]["traffic"] = (res["roofline"]["traffic_from_profile"] or {}).get("bytes")
    else:       # no per-kernel times: fall back to the phase that dominates the step
        res["roofline"] = dict(res["roofline_bwd"] if wl.backward and bwd_ms > fwd_ms else res["roofline_fwd"])
    # the headline shape of the forward target (config 3, 32x32 windows): a short run of its own
    if wl.name == "c5" and not a.no_c3:
        w3 = wk.WORKLOADS["c3"]
        r3 = Runner(w3, flags)
        _, f3, _ = time_steps(r3, min(100, max(20, a.steps)), min(a.warmup, 30))
        tf3 = w3.fwd_flop / (f3 * 1e-3) / 1e12
        res.update(fwd_c3_ms=round(f3, 4), fwd_c3_tflops=round(tf3, 2), fwd_c3_frac=round(tf3 / PEAK_BF16_TFLOPS, 4))
        del r3
    del r
    torch.cuda.empty_cache()

    if a.all:
        table = {}
        for name, w2 in wk.WORKLOADS.items():
            r2 = Runner(w2.__class__(**{**w2.__dict__, "backward": False}), flags)
            _, f_ms, _ = time_steps(r2, min(50, max(10, a.steps)), min(a.warmup, 10))
            tf = w2.fwd_flop / (f_ms * 1e-3) / 1e12
            pk = family_peak(rb.kernel_name(r2.p, False))[0]
            table[name] = {"fwd_ms": round(f_ms, 4), "fwd_tflops": round(tf, 2),
                           "tokens_per_s": round(w2.tokens / (f_ms * 1e-3), 1),
                           "frac_of_peak": round(tf / pk, 4), "peak_tflops": pk,
                           "hbm_gbs": round(w2.fwd_bytes / (f_ms * 1e-3) / 1e9, 1),
                           "kernel": rb.kernel_name(r2.p, False)}
            del r2
            torch.cuda.empty_cache()
            if w2.fwd_bytes < 128e6:       # fits the Infinity Cache: also time it with rotated buffers
                w2f = w2.__class__(**{**w2.__dict__, "backward": False})
                c_ms = time_cold(w2f, flags)
                table[name].update(fwd_ms_rotated_buffers=round(c_ms, 4),
                                   hbm_gbs_rotated_buffers=round(w2.fwd_bytes / (c_ms * 1e-3) / 1e9, 1))
                torch.cuda.empty_cache()
        res["configs"] = table
        sched = {}
        for name, w2 in wk.SCHEDULE.items():
            r2 = Runner(w2, flags)
            _, f_ms, b_ms = time_steps(r2, min(20, max(5, a.steps)), 3)
            ftf, btf = w2.fwd_flop / (f_ms * 1e-3) / 1e12, w2.bwd_flop / (b_ms * 1e-3) / 1e12
            sched[name] = {"d": w2.d, "r": w2.r, "window": w2.M, "fwd_ms": round(f_ms, 4), "fwd_tflops": round(ftf, 1),
                           "bwd_ms": round(b_ms, 4), "bwd_tflops": round(btf, 1),
                           "kernels": rb.kernel_name(r2.p, False) + "/" + rb.kernel_name(r2.p, True)}
            del r2
            torch.cuda.empty_cache()
        res["schedule"] = sched
        # one SST+ block = its six attention layers (windows 16, 32, 48, 32, 48, 96; ranks 18, 18, 18, 34, 34, 34)
        stack = ["sst-m16-r18", "sst-m32-r18", "sst-m48-r18", "sst-m32-r34", "sst-m48-r34", "sst-m96-r34"]
        f_ms = sum(sched[n]["fwd_ms"] for n in stack)
        b_ms = sum(sched[n]["bwd_ms"] for n in stack)
        flop = sum(wk.SCHEDULE[n].fwd_flop + wk.SCHEDULE[n].bwd_flop for n in stack)
        res["sst_plus_block"] = {"layers": stack, "fwd_ms": round(f_ms, 4), "bwd_ms": round(b_ms, 4),
                                 "tflops": round(flop / ((f_ms + b_ms) * 1e-3) / 1e12, 1),
                                 "tokens_per_s": round(wk.SCHEDULE[stack[0]].tokens / ((f_ms + b_ms) * 1e-3), 1)}
        # the same shapes in fp32 storage (the paper quotes its costs at FP32): fp32 MFMA kernels, fp32 peak
        f32 = {}
        for name in ("c2", "c3", "c4", "c5"):
            w2 = wk.WORKLOADS[name]
            w2 = w2.__class__(**{**w2.__dict__, "dtype": "f32", "name": name + "-f32"})
            r2 = Runner(w2, flags)
            _, f_ms, b_ms = time_steps(r2, 10, 3)
            pk = family_peak(rb.kernel_name(r2.p, False))[0]
            ftf = w2.fwd_flop / (f_ms * 1e-3) / 1e12
            f32[w2.name] = {"fwd_ms": round(f_ms, 4), "fwd_tflops": round(ftf, 1), "frac_of_peak": round(ftf / pk, 4),
                            "peak_tflops": pk, "kernel": rb.kernel_name(r2.p, False)}
            if w2.backward:
                btf = w2.bwd_flop / (b_ms * 1e-3) / 1e12
                f32[w2.name].update(bwd_ms=round(b_ms, 4), bwd_tflops=round(btf, 1), bwd_frac_of_peak=round(btf / pk, 4))
            del r2
            torch.cuda.empty_cache()
        res["configs_f32"] = f32
        res["generator"] = time_generator(rb, torch)
        res["gated_c5"] = time_gated(rb, torch, wk.WORKLOADS["c5"])

    if not a.no_cpu_baseline:
        n_units = a.cpu_units or min(wl.n_units, 864)
        res["cpu_baseline"] = cpu_baseline(wl, n_units)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
