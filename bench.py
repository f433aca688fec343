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
PEAK_FP32_VECTOR_TFLOPS = 157.3  # fp32 vector ALUs: 256 CUs x 128 lanes x 2 flop x 2.4 GHz

MFMA_KINDS = {"mlp_fwd_l1", "mlp_fwd_hidden", "mlp_dgrad", "mlp_wgrad_l1", "mlp_wgrad"}

# rocprofv3 symbol (substring) of each kernel kind in the cfg 5 run, for the HBM-traffic import
KIND_SYMBOL = {
    "mlp_fwd_l1": "mlp_gemm256_kernel<0, true, true, 0>",
    "mlp_fwd_hidden": "mlp_gemm256_kernel<0, false, true, 3>",     # (A operand read from the transposed copy)
    "mlp_dgrad": "mlp_gemm256_kernel<2, false, true, 3>",
    "mlp_wgrad_l1": "mlp_gemm256_kernel<3, false, false, 2>",
}
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "cfg5_hbm_traffic.txt")
KERNEL_SOURCE = os.path.join(ROOT, "paper_2301_08895_amd", "csrc", "kernels_mlp.hip")
COPY_BYTES = 1 << 30          # --calibrate-copy moves this many bytes with a plain copy kernel


def source_hash():
    import hashlib
    return hashlib.sha256(open(KERNEL_SOURCE, "rb").read()).hexdigest()[:16]


def import_traffic(fetch_csv, write_csv, k):
    """Turn two rocprofv3 --pmc runs of `bench.py --config 5 --calibrate-copy` (FETCH_SIZE, then
    WRITE_SIZE; counters in KiB per dispatch) into profiles/cfg5_hbm_traffic.txt: HBM bytes
    per launch of each GEMM kind at K = `k` uploads per round, each counter scaled by what it
    reads for the 1 GiB copy.  Lines of other K taken from the same kernel source are kept."""
    import csv
    def per_kernel(path, counter):
        acc = {}
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] != counter:
                continue
            a = acc.setdefault(r["Kernel_Name"], [0.0, 0, 0.0])
            v = float(r["Counter_Value"]) * 1024.0
            a[0] += v
            a[1] += 1
            a[2] = max(a[2], v)
        return acc
    fetch, write = per_kernel(fetch_csv, "FETCH_SIZE"), per_kernel(write_csv, "WRITE_SIZE")
    def copy_factor(acc):
        # the calibration copy is the largest single dispatch of a copy kernel
        big = max([a[2] for name, a in acc.items() if "copy" in name.lower()] or [0.0])
        if big <= 0.0:
            raise SystemExit("no copy kernel in the counter file: run bench.py with --calibrate-copy")
        return COPY_BYTES / big
    ff, fw = copy_factor(fetch), copy_factor(write)
    kept = []
    if os.path.exists(TRAFFIC_FILE):
        old = open(TRAFFIC_FILE).read().splitlines()
        if f"source_hash {source_hash()}" in old:
            kept = [l for l in old if "@" in l.split(" ")[0] and not l.split(" ")[0].endswith(f"@{k}")]
    lines = [f"# HBM traffic per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch),",
             f"# scaled by the same counters' reading for a {COPY_BYTES >> 20} MiB copy kernel;",
             f"# kind@K = the launches of a round with K uploads (K * B stacked rows)",
             f"source_hash {source_hash()}"] + kept
    for kind, sym in KIND_SYMBOL.items():
        f = [v for n, v in fetch.items() if sym in n]
        w = [v for n, v in write.items() if sym in n]
        if not f or not w:
            continue
        fb, wb = f[0][0] / f[0][1] * ff, w[0][0] / w[0][1] * fw
        lines.append(f"{kind}@{k} launches {f[0][1]} fetch_bytes {fb:.0f} write_bytes {wb:.0f} "
                     f"fetch_factor {ff:.4f} write_factor {fw:.4f}")
    open(TRAFFIC_FILE, "w").write("\n".join(lines) + "\n")
    print("\n".join(lines))


def stored_traffic(kind, k_avg, k_full):
    """HBM bytes per launch of `kind` from the stored counters: the line taken at the launches'
    own K when there is one, else the line at K = N scaled by the rows.  None when there are no
    counters or the kernel source has changed since they were taken."""
    if not os.path.exists(TRAFFIC_FILE):
        return None
    rows = {}
    for line in open(TRAFFIC_FILE):
        t = line.split()
        if t and not t[0].startswith("#"):
            rows[t[0]] = t[1:]
    if rows.get("source_hash", [""])[0] != source_hash():
        return None
    def total(key):
        r = rows[key]
        d = dict(zip(r[0::2], r[1::2]))
        return float(d["fetch_bytes"]) + float(d["write_bytes"])
    own = f"{kind}@{int(round(k_avg))}"
    if abs(k_avg - round(k_avg)) < 1e-3 and own in rows:
        return total(own)
    full = f"{kind}@{k_full}"
    return total(full) * k_avg / k_full if full in rows else None


# default (warmup, steps) per workload: short enough for a default run of about a minute
DEFAULT_STEPS = {1: (20, 180), 2: (200, 1800), 3: (200, 1800), 4: (200, 4800), 5: (100, 4900), 6: (100, 1900)}


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
        grads += rec["K"] * p.get("U", 1)
        rounds += 1
        el = time.perf_counter() - t0
        if el >= budget_s or rounds >= p["T"]:
            break
    return dict(value=grads / el, unit="worker-gradients/s", cores=int(threads), kind="oracle",
                sample=f"first {rounds} rounds ({grads} worker gradients) of {p['name']} in {el:.1f} s, "
                       f"NumPy fp64, {os.cpu_count()} host cpus visible")


def _flops_at_full_k(p, kind):
    """Algorithmic flops of one launch of `kind` when all N workers upload."""
    d, rows = p["dims"], p["N"] * p["B"]
    if kind in ("mlp_fwd_l1", "mlp_wgrad_l1"):
        return 2.0 * rows * d[0] * d[1]
    if kind == "mlp_fwd_hidden":
        return sum(2.0 * rows * d[l] * d[l + 1] for l in range(1, len(d) - 2)) / max(1, len(d) - 3)
    if kind == "mlp_dgrad":
        return sum(2.0 * rows * d[l] * d[l + 1] for l in range(1, len(d) - 2)) / max(1, len(d) - 3)
    return sum(2.0 * rows * d[l] * d[l + 1] for l in range(1, len(d) - 1)) / max(1, len(d) - 2)


def kernel_deltas(stats0, stats1):
    """Per-kernel time and algorithmic work between two readings of abs_kernel_stats."""
    kern = []
    for name, s1 in stats1.items():
        s0 = stats0.get(name, dict(timed_launches=0, total_ms=0.0, timed_flops=0.0, timed_bytes=0.0))
        n = s1["timed_launches"] - s0["timed_launches"]      # the launches of the bracketed rounds
        if n <= 0:
            continue
        kern.append(dict(name=name, launches=n, ms=s1["total_ms"] - s0["total_ms"],
                         flops=s1["timed_flops"] - s0["timed_flops"], bytes=s1["timed_bytes"] - s0["timed_bytes"]))
    return kern


def roofline_of(kern, p, config):
    """The roofline block for the kernel kind with the largest total time."""
    if not kern:
        return None
    dom = max(kern, key=lambda k: k["ms"])
    avg_s = dom["ms"] / dom["launches"] * 1e-3
    if dom["name"] in MFMA_KINDS:
        ach = dom["flops"] / dom["launches"] / avg_s / 1e12
        k_avg = (dom["flops"] / dom["launches"]) / _flops_at_full_k(p, dom["name"]) * p["N"]
        traffic = stored_traffic(dom["name"], k_avg, p["N"]) if config == 5 else None
        return dict(bound="mfma", kernel=dom["name"], achieved=ach, peak=PEAK_MFMA_BF16_TFLOPS,
                    unit="TFLOP/s", frac=ach / PEAK_MFMA_BF16_TFLOPS, traffic=traffic,
                    avg_launch_us=avg_s * 1e6, launches=dom["launches"])
    if dom["name"].startswith("cnn_"):
        # the convolutional model's kernels are plain fp32 vector arithmetic on data that lives in LDS
        ach = dom["flops"] / dom["launches"] / avg_s / 1e12
        return dict(bound="alu", kernel=dom["name"], achieved=ach, peak=PEAK_FP32_VECTOR_TFLOPS,
                    unit="TFLOP/s", frac=ach / PEAK_FP32_VECTOR_TFLOPS, traffic=None,
                    avg_launch_us=avg_s * 1e6, launches=dom["launches"])
    ach = dom["bytes"] / dom["launches"] / avg_s / 1e9
    return dict(bound="hbm", kernel=dom["name"], achieved=ach, peak=PEAK_HBM_GBS,
                unit="GB/s", frac=ach / PEAK_HBM_GBS, traffic=None,
                avg_launch_us=avg_s * 1e6, launches=dom["launches"])


def calibrate_mfma(args):
    """The MFMA-only loop of the library (no memory traffic), constant and random operands: what the
    matrix cores sustain at the clock the chip settles at.  One JSON line."""
    import torch
    import paper_2301_08895_amd as lib
    wgs, iters = 512, args.calibrate_iters
    scratch = torch.zeros(wgs * 512, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    out = {"mode": "calibrate_mfma", "workgroups": wgs, "iters": iters, "peak_tflops": PEAK_MFMA_BF16_TFLOPS, "runs": []}
    for data_mode, label in ((0, "32x32x16, constant operands"), (1, "32x32x16, random bf16 operands"),
                             (2, "16x16x32, constant operands"), (3, "16x16x32, random bf16 operands")):
        best = None
        for _ in range(3):
            ms, tf = lib.abs_calibrate_mfma(data_mode, iters, wgs, scratch.data_ptr(), stream)
            best = (ms, tf) if best is None or tf > best[1] else best
        out["runs"].append({"operands": label, "ms": best[0], "tflops": best[1], "frac_of_peak": best[1] / PEAK_MFMA_BF16_TFLOPS})
    print(json.dumps(out))


def library_gemm(args):
    """Context only, not part of the library under test: the vendor BLAS (torch.matmul) on the shapes of the
    workload's large products - plain GEMMs, no gather, bias, ReLU, mask, second output orientation or per-upload
    weights - with operands distributed like the round's (ReLU'd unit normals times small normals).  One JSON line."""
    import torch
    import workloads
    p = workloads.preset(args.config)
    d = p["dims"]
    torch.manual_seed(0)
    dev = "cuda"
    out = {"mode": "library_gemm", "workload": p["name"], "note": "torch.matmul, bf16 in / bf16 out, 200 launches each after 50 warm-up launches", "products": []}

    def run(name, rows, m, n, k, transposed):
        if transposed:      # contraction over the leading dimension of both operands (a weight gradient)
            a = torch.relu(torch.randn(k, m, device=dev)).bfloat16()
            b = (torch.randn(k, n, device=dev) * 0.03).bfloat16()
            f = lambda: torch.matmul(a.t(), b)
        else:
            a = torch.relu(torch.randn(m, k, device=dev)).bfloat16()
            b = (torch.randn(n, k, device=dev) * 0.03).bfloat16()
            f = lambda: torch.matmul(a, b.t())
        for _ in range(50):
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(200):
            f()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 200 * 1e3
        out["products"].append({"product": name, "stacked_rows": rows, "m": m, "n": n, "k": k, "us": round(us, 1),
                                "tflops": round(2.0 * m * n * k / us / 1e6, 1)})

    for K in (p["K0"], p["N"]):
        rows = K * p["B"]
        run("first-layer forward", rows, rows, d[1], d[0], False)
        run("first-layer weight gradient", rows, d[0], d[1], rows, True)
        if len(d) > 3:
            run("hidden forward / input gradient", rows, rows, d[2], d[1], False)
            run("hidden weight gradient", rows, d[1], d[2], rows, True)
    print(json.dumps(out))


def bench_batch(args, p, inputs, warmup, steps):
    """S independent simulations (different simulation seeds) of a workload, advanced together by
    abs_batch_round: the sweep shape of the paper's experiments."""
    import numpy as np
    import torch
    import paper_2301_08895_amd as lib

    S = args.batch
    sims = [lib.Simulation(dict(p, seed_sim=p["seed_sim"] + 7919 * i), inputs) for i in range(S)]
    batch = lib.Batch(sims)
    batch.round(warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    batch.round(steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    grads = 0
    for sim in sims:
        tr = sim.trace(warmup, warmup + steps)
        grads += int(tr[:, 1].sum()) * p.get("U", 1)
        assert np.all(np.isfinite(sim.model())), "non-finite parameters after the timed run"
    batch.close()
    for sim in sims:
        sim.close()
    value = grads / elapsed
    mlp = p["model"] == 2
    if mlp:
        # algorithmic flops of a worker gradient: forward and weight gradient of every layer, input
        # gradient of every layer but the first
        dm = p["dims"]
        per = sum((2 if l == 0 else 3) * 2.0 * p["B"] * dm[l] * dm[l + 1] for l in range(len(dm) - 1))
        roof = {"bound": "mfma", "kernel": "whole round (all launches and the host, wall clock)",
                "achieved": grads * per / elapsed / 1e12, "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": grads * per / elapsed / 1e12 / PEAK_MFMA_BF16_TFLOPS, "traffic": None}
    else:
        # algorithmic bytes: every aggregated gradient reads B rows of d features and B targets once
        ach = grads * p["B"] * (p["dims"][0] + 1) * 4.0 / elapsed / 1e9
        roof = {"bound": "hbm", "kernel": "whole round (all launches and the host, wall clock)",
                "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS, "traffic": None}
    cpu = cpu_baseline(p, inputs, args.cpu_budget) if args.cpu_budget > 0 else None
    print(json.dumps({
        "metric": "worker_gradients_per_sec", "value": value, "unit": "worker-gradients/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": elapsed / steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if mlp else "f32", "data": "synthetic",
        "config": {"workload": f"{p['name']}_x{S}_simulations", "N": p["N"], "B": p["B"], "dims": p["dims"],
                   "K0": p["K0"], "tau_cap": p["tau_cap"], "a": p["a"], "lr": p["lr"], "U": p.get("U", 1),
                   "simulations": S},
        "samples_per_sec": value * p["B"], "rounds_per_sec": steps * S / elapsed,
        "roofline": roof,
        "cpu_baseline": cpu,
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=5, help="workload 1..5 (default: the largest); 6: the convolutional model of Section V-A")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket kernels with events")
    ap.add_argument("--profile-every", type=int, default=None, metavar="n",
                    help="bracket the kernels of every n-th round with HIP events (1: of every round; "
                         "default: 8, and 1 for runs shorter than 64 rounds so that the roofline figure "
                         "rests on every timed round)")
    ap.add_argument("--cpu-budget", type=float, default=15.0, help="seconds of oracle time (0: skip)")
    ap.add_argument("--fixed-k", action="store_true",
                    help="counter runs only: wait for all N workers every round (the steady state)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="counter runs only: end with a plain 1 GiB device copy to calibrate FETCH/WRITE_SIZE")
    ap.add_argument("--local-steps", type=int, default=1, metavar="U",
                    help="local SGD: U minibatch steps per job (Eq. 2); a worker gradient is one such step")
    ap.add_argument("--batch", type=int, default=0,
                    help="configs 1-2: advance this many independent simulations (seeds) per launch")
    ap.add_argument("--calibrate-mfma", action="store_true",
                    help="run the library's MFMA-only loop (constant and random operands), print its rate, exit")
    ap.add_argument("--library-gemm", action="store_true",
                    help="context only: time the vendor BLAS (torch.matmul) on the shapes of the workload's large products, exit")
    ap.add_argument("--calibrate-iters", type=int, default=4000, help="iterations of the MFMA-only loop")
    ap.add_argument("--full-k-rounds", type=int, default=8,
                    help="MLP workloads: extra rounds at K = N after the timed region for the roofline_full_k block (0: none)")
    ap.add_argument("--traffic-k", type=int, default=128,
                    help="uploads per round (K) of the run the --traffic-import counter files come from")
    ap.add_argument("--traffic-import", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="write profiles/cfg5_hbm_traffic.txt from two rocprofv3 --pmc counter files and exit")
    args = ap.parse_args()
    if args.traffic_import:
        import_traffic(*args.traffic_import, args.traffic_k)
        return
    if args.gpus != 1:
        print("bench.py: this library runs on ONE GPU only (one simulated parameter server per device); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    if args.calibrate_mfma:
        return calibrate_mfma(args)
    if args.library_gemm:
        return library_gemm(args)

    import numpy as np
    import torch
    import workloads
    import paper_2301_08895_amd as lib

    p = workloads.preset(args.config)
    mlp = p["model"] == 2
    if args.fixed_k:
        p["k_mode"], p["K0"] = 1, p["N"]
    if args.local_steps != 1:
        p["U"] = args.local_steps
        p["name"] += f"_U{args.local_steps}"
    dw, ds = DEFAULT_STEPS[args.config]
    warmup = dw if args.warmup is None else args.warmup
    steps = ds if args.steps is None else args.steps
    inputs = workloads.make_inputs(p)
    if args.profile_every is None:
        args.profile_every = 1 if steps < 64 else 8

    if args.batch:
        return bench_batch(args, p, inputs, warmup, steps)

    sim = lib.Simulation(p, inputs, profile=0 if args.no_profile else max(1, args.profile_every))
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
    if args.calibrate_copy:
        src = torch.ones(COPY_BYTES // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    assert np.all(np.isfinite(final)), "non-finite parameters after the timed run"
    grads = int(tr[:, 1].sum()) * p.get("U", 1)
    value = grads / elapsed

    kern = kernel_deltas(stats0, stats1)
    roofline = roofline_of(kern, p, args.config) if not args.no_profile else None

    # The steady state of the job, K = N, on a few extra rounds of a second handle AFTER the timed
    # region (the headline figures above are untouched): the wait count grows from K0 to N over the
    # job (Eq. 5), so a short run only ever sees K = K0, where every product is a quarter the size.
    roofline_full_k = None
    if mlp and not args.no_profile and not args.fixed_k and args.full_k_rounds > 0:
        q = dict(p, k_mode=1, K0=p["N"])
        sim2 = lib.Simulation(q, inputs, profile=1)
        sim2.round(3)
        torch.cuda.synchronize()
        a0 = {s_["name"]: s_ for s_ in sim2.kernel_stats()}
        t2 = time.perf_counter()
        sim2.round(args.full_k_rounds)
        torch.cuda.synchronize()
        el2 = time.perf_counter() - t2
        a1 = {s_["name"]: s_ for s_ in sim2.kernel_stats()}
        sim2.close()
        roofline_full_k = roofline_of(kernel_deltas(a0, a1), q, args.config)
        roofline_full_k.update(note=f"{args.full_k_rounds} extra rounds at fixed K = N = {p['N']} after the timed region; "
                                    "not part of value / ms_per_step / roofline",
                               ms_per_round=el2 / args.full_k_rounds * 1e3,
                               worker_gradients_per_sec=p["N"] * args.full_k_rounds / el2)
    # The same warm-up and timed rounds once more on a fresh handle WITHOUT per-kernel events, after
    # everything above: what the events cost (an event pair on every dispatch keeps consecutive
    # kernels from following each other directly).  Reported beside the headline, never in its place.
    no_events = None
    if not args.no_profile and steps <= 256:
        sim3 = lib.Simulation(p, inputs, profile=0)
        sim3.round(warmup)
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        sim3.round(steps)
        torch.cuda.synchronize()
        el3 = time.perf_counter() - t3
        tr3 = sim3.trace(warmup, warmup + steps)
        sim3.close()
        no_events = dict(value=int(tr3[:, 1].sum()) * p.get("U", 1) / el3, ms_per_step=el3 / steps * 1e3,
                         note=f"the same {warmup} + {steps} rounds again without per-kernel events, after the timed region; "
                              "not part of value / ms_per_step / roofline")
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
                   "U": p.get("U", 1), "K_first": int(tr[0, 1]), "K_last": int(tr[-1, 1])},
        "samples_per_sec": value * p["B"],
        "rounds_per_sec": steps / elapsed,
        "profile_every": 0 if args.no_profile else max(1, args.profile_every),
        "kernels": kernels,
        "roofline": roofline,
        "roofline_full_k": roofline_full_k,
        "no_events": no_events,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
