"""Shared by the GPU parity tests: run the oracle and libabs on the same seeded inputs
and compare trace (bit-exact, except the loss word) and parameters."""
import numpy as np

import workloads
import paper_2301_08895_amd as lib
from oracle.abs_sim import AbsOracle, trace_words

LOSS_WORD, KNEXT_WORD = 10, 11


def run_pair(p, T, checkpoints=(), emulate_bf16=None, inputs=None):
    """Returns dict(o=oracle, got_trace, want_trace, models={round: (gpu, oracle)}, flips)."""
    d = inputs if inputs is not None else workloads.make_inputs(p)
    o = AbsOracle(p, d["X"], d["y"], d["w0"], emulate_bf16=emulate_bf16, keep_models=True)
    sim = lib.Simulation(p, d)
    models = {}
    done = 0
    for cp in sorted(set(checkpoints) | {T}):
        o.run(cp - done)
        sim.round(cp - done)
        done = cp
        models[cp] = (sim.model(), o.model().copy())
    got = sim.trace()
    want = np.stack([trace_words(r, p["N"]) for r in o.trace])
    flips = [int(t) for t in np.nonzero(got[:, KNEXT_WORD] != want[:, KNEXT_WORD])[0]]
    if flips and p["k_mode"] in (0, 3):
        # an adaptive wait count decided on float losses flipped: report it and repeat with
        # the oracle's K sequence replayed
        sim.close()
        print(f"adaptive-K flips at rounds {flips[:8]}; repeating with the oracle's K replayed")
        q = dict(p, k_mode=2)
        sim = lib.Simulation(q, d, k_replay=[r["K"] for r in o.trace])
        done = 0
        for cp in sorted(set(checkpoints) | {T}):
            sim.round(cp - done)
            done = cp
            models[cp] = (sim.model(), o.models[cp].copy())
        got = sim.trace()
    stats = sim.kernel_stats()
    sim.close()
    return dict(o=o, got=got, want=want, models=models, flips=flips, stats=stats, sim_inputs=d)


def assert_trace_equal(res, loss_rtol):
    got, want = res["got"], res["want"]
    keep = np.ones(got.shape[1], bool)
    keep[LOSS_WORD] = False
    if res["flips"]:
        keep[KNEXT_WORD] = False
    bad = np.nonzero((got[:, keep] != want[:, keep]).any(axis=1))[0]
    assert bad.size == 0, f"integer trace differs first at round {bad[0]}"
    gl = got[:, LOSS_WORD].copy().view(np.float32).astype(np.float64)
    wl = want[:, LOSS_WORD].copy().view(np.float32).astype(np.float64)
    assert np.all(np.abs(gl - wl) <= loss_rtol * np.maximum(np.abs(wl), 1e-3)), \
        f"loss words differ: max rel {np.max(np.abs(gl - wl) / np.maximum(np.abs(wl), 1e-3))}"


def rel_err(got, want):
    return float(np.linalg.norm(got.astype(np.float64) - want) / max(np.linalg.norm(want), 1e-30))


def golden_path(name):
    import os
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)


def golden_lines(name):
    """Non-comment lines of a fixture under tests/golden/ (hand-worked or published values, each file
    carrying its citation)."""
    with open(golden_path(name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def hand_worked_schedule():
    """The hand-worked run of Algorithm 1 (tests/golden/abs_hand_worked_schedule.txt): its setting as
    overrides of a workload preset, and the records, finish times in ticks."""
    unit = 1 << 20
    setting = dict(N=4, K0=2, k_mode=1, tau_mode=1, tau_cap=1, time_dist=2, n_slow=1, slow_factor=3.0)
    ints = lambda s: [] if s == "-" else [int(v) for v in s.split(",")]
    recs = []
    for t, K, tmax, now, ids, vers, taus, rst, up, rs in golden_lines("abs_hand_worked_schedule.txt"):
        recs.append(dict(t=int(t), K=int(K), tau_max=int(tmax), now=int(now) * unit, ids=ints(ids), vers=ints(vers),
                         taus=ints(taus), restart_ids=ints(rst), comm_uploads=int(up), comm_restarts=int(rs)))
    return setting, recs


def hand_worked_updates(sa_penalty):
    """The hand-worked model updates (tests/golden/abs_hand_worked_updates.txt): the workload's
    settings and arrays, the models w^1 .. w^3 and the rounds' mean losses."""
    import workloads
    p = workloads.scaled_preset(1, M=3, N=3, B=1, dims=[2, 1], K0=2, k_mode=1, tau_mode=2, tau_cap=8, lr=0.5,
                                time_dist=2, n_slow=1, slow_factor=3.0, sa_penalty=sa_penalty)
    d = dict(X=np.array([[1, 0], [0, 1], [1, 1]], np.float32), y=np.array([1, 2, 0], np.float32),
             w0=np.zeros(2, np.float32))
    models, losses = {}, {}
    for row in golden_lines("abs_hand_worked_updates.txt"):
        if row[0] == "w" and int(row[1]) == sa_penalty:
            models[int(row[2])] = np.array([float(row[3]), float(row[4])])
        elif row[0] == "loss":
            losses[int(row[1])] = float(row[2])
    return p, d, models, losses


def softmax_hand_worked_first_round():
    """tests/golden/softmax_hand_worked_first_round.txt: settings, arrays and w^1."""
    import workloads
    p = workloads.scaled_preset(2, M=2, N=2, B=1, dims=[4, 4], n_classes=4, K0=2, k_mode=1, tau_mode=2, tau_cap=4,
                                lr=1.0, time_dist=2)
    d = dict(X=np.array([[1, 2, 0, 0], [-1, 0, 0, 0]], np.float32), y=np.array([1, 3], np.int32),
             w0=np.zeros(20, np.float32))
    w1 = np.array([float(r[0]) for r in golden_lines("softmax_hand_worked_first_round.txt")])
    assert w1.size == 20
    return p, d, w1


def mlp_hand_worked_first_round():
    """tests/golden/mlp_hand_worked_first_round.txt: settings, arrays (X as bf16 bit patterns) and w^1."""
    import workloads
    p = workloads.scaled_preset(3, M=2, N=2, B=1, dims=[8, 2, 4], n_classes=4, K0=2, k_mode=1, tau_mode=2, tau_cap=4,
                                lr=1.0, time_dist=2, n_slow=0)
    X = np.zeros((2, 8), np.float32)
    X[0, :2] = (1, 2)
    X[1, :2] = (-1, 3)
    w0 = np.zeros(30, np.float32)
    w0[0] = 1.0          # W_1[0][0]
    w0[3] = 1.0          # W_1[1][1]
    w0[17] = -1.0        # b_1[1]
    d = dict(X=(X.view(np.uint32) >> 16).astype(np.uint16), y=np.array([1, 3], np.int32), w0=w0)
    w1 = np.array([float(r[0]) for r in golden_lines("mlp_hand_worked_first_round.txt")])
    assert w1.size == 30
    return p, d, w1


def local_sgd_hand_worked():
    """tests/golden/local_sgd_hand_worked.txt: settings, arrays, models w^1, w^2 and round losses."""
    import workloads
    p = workloads.scaled_preset(1, M=2, N=2, B=1, dims=[2, 1], K0=2, k_mode=1, tau_mode=2, tau_cap=4, lr=0.5,
                                time_dist=2, U=2)
    d = dict(X=np.array([[1, 0], [0, 1]], np.float32), y=np.array([1, 2], np.float32), w0=np.zeros(2, np.float32))
    models, losses = {}, {}
    for row in golden_lines("local_sgd_hand_worked.txt"):
        if row[0] == "w":
            models[int(row[1])] = np.array([float(row[2]), float(row[3])])
        else:
            losses[int(row[1])] = float(row[2])
    return p, d, models, losses
