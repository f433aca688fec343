#!/usr/bin/env python3
"""Benchmark of the ABS parameter-server round on one MI355X.

A "step" is one PS round of the whole hot path (select K^t uploads -> minibatch
gradients at stale model versions -> K-of-N reduction -> update -> snapshot -> adapt K)
on a synthetic workload; `value` is worker-gradients per second (sum of K^t over the
timed rounds / elapsed), with the dataset and the model ring resident in HBM.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5]

Prints ONE JSON line.  The CPU oracle is timed beside it on a bounded sample of the same
workload (reported baseline only).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_MFMA_BF16_TFLOPS = 2500.0  # dense bf16 MFMA

MFMA_KINDS = {"mlp_fwd_l1", "mlp_fwd_hidden", "mlp_dgrad", "mlp_wgrad_l1", "mlp_wgrad"}

# default (warmup, steps) per workload: short enough for a default run of about a minute
DEFAULT_STEPS = {1: (20, 180), 2: (200, 1800), 3: (200, 1800), 4: (200, 4800), 5: (100, 4900)}


def cpu_baseline(p, inputs, budget_s: float):
    """Time the oracle, as it stands, on the first rounds of the same workload."""
    from oracle.abs_sim import AbsOracle
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    o = AbsOracle(p, inputs["X"], inputs["y"], inputs["w0"], keep_models=False)
    t0 = time.perf_counter()
    grads = rounds = 0
    while True:
        rec = o.round()
        grads += rec["K"]
        rounds += 1
        el = time.perf_counter() - t0
        if el >= budget_s or rounds >= p["T"]:
            break
    return dict(value=grads / el, unit="worker-gradients/s", cores=int(threads), kind="oracle",
                sample=f"first {rounds} rounds ({grads} worker gradients) of {p['name']} in {el:.1f} s, "
                       f"NumPy fp64, {os.cpu_count()} host cpus visible")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=5, help="workload 1..5 (default: the largest)")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket kernels with events")
    ap.add_argument("--cpu-budget", type=float, default=15.0, help="seconds of oracle time (0: skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (one simulated parameter server per device); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads
    import paper_2301_08895_amd as lib

    p = workloads.preset(args.config)
    dw, ds = DEFAULT_STEPS[args.config]
    warmup = dw if args.warmup is None else args.warmup
    steps = ds if args.steps is None else args.steps
    inputs = workloads.make_inputs(p)

    sim = lib.Simulation(p, inputs, profile=0 if args.no_profile else 1)
    sim.round(warmup)
    torch.cuda.synchronize()
    stats0 = {s["name"]: s for s in sim.kernel_stats()}
    t0 = time.perf_counter()
    sim.round(steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    stats1 = {s["name"]: s for s in sim.kernel_stats()}
    tr = sim.trace(warmup, warmup + steps)
    final = sim.model()
    sim.close()
    assert np.all(np.isfinite(final)), "non-finite parameters after the timed run"
    grads = int(tr[:, 1].sum())
    value = grads / elapsed

    # per-kernel time inside the timed region (HIP events on the launch stream)
    kern = []
    for name, s1 in stats1.items():
        s0 = stats0.get(name, dict(launches=0, total_ms=0.0, flops=0.0, bytes=0.0))
        n = s1["launches"] - s0["launches"]
        if n <= 0:
            continue
        kern.append(dict(name=name, launches=n, ms=s1["total_ms"] - s0["total_ms"],
                         flops=s1["flops"] - s0["flops"], bytes=s1["bytes"] - s0["bytes"]))
    roofline = None
    if kern and not args.no_profile:
        dom = max(kern, key=lambda k: k["ms"])
        avg_s = dom["ms"] / dom["launches"] * 1e-3
        if dom["name"] in MFMA_KINDS:
            ach = dom["flops"] / dom["launches"] / avg_s / 1e12
            roofline = dict(bound="mfma", kernel=dom["name"], achieved=ach, peak=PEAK_MFMA_BF16_TFLOPS,
                            unit="TFLOP/s", frac=ach / PEAK_MFMA_BF16_TFLOPS, traffic=None,
                            avg_launch_us=avg_s * 1e6, launches=dom["launches"])
        else:
            ach = dom["bytes"] / dom["launches"] / avg_s / 1e9
            roofline = dict(bound="hbm", kernel=dom["name"], achieved=ach, peak=PEAK_HBM_GBS,
                            unit="GB/s", frac=ach / PEAK_HBM_GBS, traffic=None,
                            avg_launch_us=avg_s * 1e6, launches=dom["launches"])
    kernels = [dict(name=k["name"], launches=k["launches"], total_ms=round(k["ms"], 3),
                    avg_us=round(k["ms"] / k["launches"] * 1e3, 2),
                    tflops=round(k["flops"] / k["ms"] / 1e9, 1) if k["ms"] > 0 else None,
                    gbs=round(k["bytes"] / k["ms"] / 1e6, 1) if k["ms"] > 0 else None)
               for k in sorted(kern, key=lambda k: -k["ms"])]

    cpu = cpu_baseline(p, inputs, args.cpu_budget) if args.cpu_budget > 0 else None

    out = {
        "metric": "worker_gradients_per_sec",
        "value": value,
        "unit": "worker-gradients/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": elapsed / steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if p["x_dtype"] == 1 else "f32",
        "data": "synthetic",
        "config": {"workload": p["name"], "N": p["N"], "B": p["B"], "dims": p["dims"], "K0": p["K0"],
                   "tau_cap": p["tau_cap"], "a": p["a"], "lr": p["lr"], "sa_penalty": p["sa_penalty"],
                   "K_first": int(tr[0, 1]), "K_last": int(tr[-1, 1])},
        "samples_per_sec": value * p["B"],
        "rounds_per_sec": steps / elapsed,
        "kernels": kernels,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
