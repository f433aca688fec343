"""Read-outs of Section V-B for the paper's method and the systems it is compared with.

Runs each method (settings of the same simulated parameter-server round, see
workloads/methods.py) on one synthetic workload and prints, at regular checkpoints, the
simulated wall-clock time, the communication rounds (uploads + restart messages), the round's
training-loss estimate and the held-out loss and accuracy of the global model, followed by the
time and communication each method needed to reach a target held-out loss.

    python -m paper_2301_08895_amd.compare --config 2 --rounds 600 --every 100 --target 0.3

With --sweep-a the constant a of Eq. 4 is swept for the paper's method instead (the experiment
behind the discussion of a in Section V-B), every value over several simulation seeds; for the
regression workloads all these simulations advance together as one batch (abs_batch_round).

    python -m paper_2301_08895_amd.compare --config 2 --sweep-a 0,-1,-2,-3 --seeds 8 --rounds 600

Everything runs on the GPU through libabs (abs_round / abs_batch_round, abs_trace, abs_evaluate).
"""
from __future__ import annotations

import argparse
import json

import numpy as np

import workloads
from . import binding as lib

TICKS_PER_UNIT = float(1 << 20)       # the simulated clock counts 2^-20 time units


def run_method(p: dict, name: str, rounds: int, every: int, eval_rows: int, over: dict):
    q = workloads.method_preset(p, name, **over)
    train, Xe, ye = workloads.make_split(q, eval_rows)
    sim = lib.Simulation(q, train)
    rows = []
    done = 0
    while done < rounds:
        n = min(every, rounds - done)
        sim.round(n)
        done += n
        rec = sim.trace(done - 1, done)[0]
        now = (int(rec[3]) & 0xFFFFFFFF) | ((int(rec[4]) & 0xFFFFFFFF) << 32)
        uploads = (int(rec[6]) & 0xFFFFFFFF) | ((int(rec[7]) & 0xFFFFFFFF) << 32)
        restarts = (int(rec[8]) & 0xFFFFFFFF) | ((int(rec[9]) & 0xFFFFFFFF) << 32)
        loss, acc = sim.evaluate(Xe, ye)
        rows.append(dict(method=name, round=done, K=int(rec[1]), time=now / TICKS_PER_UNIT,
                         comm=uploads + restarts, restarts=restarts,
                         train_loss=float(rec[10:11].view(np.float32)[0]), eval_loss=loss, eval_acc=acc))
    sim.close()
    return rows


def _readout(sim, done, Xe, ye, **tags):
    rec = sim.trace(done - 1, done)[0]
    now = (int(rec[3]) & 0xFFFFFFFF) | ((int(rec[4]) & 0xFFFFFFFF) << 32)
    uploads = (int(rec[6]) & 0xFFFFFFFF) | ((int(rec[7]) & 0xFFFFFFFF) << 32)
    restarts = (int(rec[8]) & 0xFFFFFFFF) | ((int(rec[9]) & 0xFFFFFFFF) << 32)
    loss, acc = sim.evaluate(Xe, ye)
    return dict(round=done, K=int(rec[1]), time=now / TICKS_PER_UNIT, comm=uploads + restarts, restarts=restarts,
                train_loss=float(rec[10:11].view(np.float32)[0]), eval_loss=loss, eval_acc=acc, **tags)


def sweep_a(p: dict, values, seeds: int, rounds: int, every: int, eval_rows: int, target):
    """The paper's method for every a in `values` and `seeds` simulation seeds each; one dataset."""
    base = workloads.method_preset(p, "abs")
    train, Xe, ye = workloads.make_split(base, eval_rows)
    runs = [(av, sd, lib.Simulation(dict(base, a=av, seed_sim=base["seed_sim"] + 7919 * sd), train))
            for av in values for sd in range(seeds)]
    batch = lib.Batch([r[2] for r in runs]) if len(runs) > 1 else None
    rows, done = [], 0
    while done < rounds:
        n = min(every, rounds - done)
        if batch:
            batch.round(n)
        else:
            for _, _, sim in runs:
                sim.round(n)
        done += n
        rows += [_readout(sim, done, Xe, ye, a=av, seed=sd) for av, sd, sim in runs]
    if batch:
        batch.close()
    for _, _, sim in runs:
        sim.close()
    print(f"{'a':>4s} {'round':>6s} {'K':>6s} {'time':>10s} {'comm':>10s} {'restarts':>9s} {'eval loss':>10s} {'eval acc':>8s}"
          f"   (means over {seeds} seeds)")
    mean = lambda rs, k: float(np.mean([r[k] for r in rs]))
    for av in values:
        for rd in sorted({r["round"] for r in rows}):
            rs = [r for r in rows if r["a"] == av and r["round"] == rd]
            print(f"{av:4d} {rd:6d} {mean(rs, 'K'):6.1f} {mean(rs, 'time'):10.2f} {mean(rs, 'comm'):10.0f} "
                  f"{mean(rs, 'restarts'):9.1f} {mean(rs, 'eval_loss'):10.5f} {mean(rs, 'eval_acc'):8.4f}")
    if target is not None:
        print(f"\nfirst read-out with held-out loss <= {target} (mean over the seeds that reach it):")
        for av in values:
            hits = []
            for sd in range(seeds):
                hit = next((r for r in rows if r["a"] == av and r["seed"] == sd and r["eval_loss"] <= target), None)
                if hit:
                    hits.append(hit)
            print(f"  a = {av:3d}: " + (f"{len(hits)}/{seeds} seeds, time {mean(hits, 'time'):.2f}, comm {mean(hits, 'comm'):.0f}"
                                        if hits else "not reached"))
    return rows


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--config", type=int, default=2, help="workload 1..5; 6: the convolutional model of Section V-A")
    ap.add_argument("--methods", default="abs,adasync,sa_adasync,k_async,local_sgd")
    ap.add_argument("--rounds", type=int, default=600)
    ap.add_argument("--every", type=int, default=100, help="rounds between read-outs")
    ap.add_argument("--eval-rows", type=int, default=4096)
    ap.add_argument("--target", type=float, default=None, help="held-out loss to reach")
    ap.add_argument("--M", type=int, default=None, help="override the dataset size")
    ap.add_argument("--U", type=int, default=None, help="local steps (Eq. 2) for every method but sync_sgd")
    ap.add_argument("--a", type=int, default=None, help="constant of Eq. 4 for the abs variants")
    ap.add_argument("--json", action="store_true", help="one JSON object per read-out instead of the table")
    ap.add_argument("--sweep-a", default=None, help="comma-separated values of a: sweep Eq. 4's constant for the paper's method")
    ap.add_argument("--seeds", type=int, default=4, help="simulation seeds per value of --sweep-a")
    a = ap.parse_args(argv)
    p = workloads.preset(a.config)
    if a.M:
        p["M"] = a.M
    every = max(1, a.every)
    if a.sweep_a is not None:
        sweep_a(p, [int(v) for v in a.sweep_a.split(",")], max(1, a.seeds), a.rounds, every, a.eval_rows, a.target)
        return 0
    out = []
    for name in a.methods.split(","):
        over = {}
        if a.U and name != "sync_sgd":
            over["U"] = a.U
        if a.a is not None and name.startswith(("abs", "sa_abs")):
            over["a"] = a.a
        out += run_method(p, name, a.rounds, every, a.eval_rows, over)
    if a.json:
        for r in out:
            print(json.dumps(r))
        return 0
    print(f"{'method':14s} {'round':>6s} {'K':>4s} {'time':>10s} {'comm':>9s} {'restarts':>8s} {'train loss':>11s} "
          f"{'eval loss':>10s} {'eval acc':>8s}")
    for r in out:
        print(f"{r['method']:14s} {r['round']:6d} {r['K']:4d} {r['time']:10.2f} {r['comm']:9d} {r['restarts']:8d} "
              f"{r['train_loss']:11.5f} {r['eval_loss']:10.5f} {r['eval_acc']:8.4f}")
    if a.target is not None:
        print(f"\nfirst read-out with held-out loss <= {a.target}:")
        for name in a.methods.split(","):
            hit = next((r for r in out if r["method"] == name and r["eval_loss"] <= a.target), None)
            print(f"  {name:14s} " + (f"time {hit['time']:.2f}, comm {hit['comm']}, round {hit['round']}" if hit
                                      else "not reached"))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
