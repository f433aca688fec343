"""Shared by the GPU parity tests: run the oracle and libabs on the same seeded inputs
and compare trace (bit-exact, except the loss word) and parameters."""
import numpy as np

import workloads
import paper_2301_08895_amd as lib
from oracle.abs_sim import AbsOracle, trace_words
from progress import say, tick

LOSS_WORD, KNEXT_WORD = 10, 11


def _piece(p):
    """Rounds per call of the oracle: a few seconds of its work at the workload's size."""
    per_round = p["N"] * p["B"] * max(int(np.prod(p["dims"][:2])) if "dims" in p else 1, 1)
    return int(min(250, max(1, 2e10 // per_round)))


def run_pair(p, T, checkpoints=(), emulate_bf16=None, inputs=None):
    """Returns dict(o=oracle, got_trace, want_trace, models={round: (gpu, oracle)}, flips)."""
    d = inputs if inputs is not None else workloads.make_inputs(p)
    o = AbsOracle(p, d["X"], d["y"], d["w0"], emulate_bf16=emulate_bf16, keep_models=True)
    sim = lib.Simulation(p, d)
    models = {}
    done = 0
    for cp in sorted(set(checkpoints) | {T}):
        while o.t < cp:                  # in pieces, so that the output shows the run is alive
            o.run(min(_piece(p), cp - o.t))
            tick(f"  oracle at round {o.t}")
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
        say(f"adaptive-K flips at rounds {flips[:8]}; repeating with the oracle's K replayed")
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


def param_blocks(p):
    """(name, slice) of every tensor of the boundary layout: W_l [d_in, d_out] then b_l per layer
    (the linear model: w alone)."""
    d = p["dims"]
    if p["model"] == 0:
        return [("w", slice(0, d[0]))]
    out, o = [], 0
    if p["model"] == 3:              # convolutional model: conv1, conv2, dense1..3
        names = ["Wc1", "Wc2", "Wd1", "Wd2", "Wd3"]
        for name, (r, c) in zip(names, workloads.presets.cnn_layer_shapes(p)):
            out.append((name, slice(o, o + r * c))); o += r * c
            out.append(("b" + name[1:], slice(o, o + c))); o += c
        return out
    for l in range(len(d) - 1):
        out.append((f"W{l + 1}", slice(o, o + d[l] * d[l + 1]))); o += d[l] * d[l + 1]
        out.append((f"b{l + 1}", slice(o, o + d[l + 1]))); o += d[l + 1]
    return out


EPS32 = 2.0 ** -24      # half an ulp of the fp32 the library stores its models in
# Single elements are held to ELEM x the tolerance, in units of their tensor's largest update.  A ReLU
# is a discontinuity: a hidden pre-activation that lands within accumulation rounding of zero (cfg 5,
# first round: |z| = 3e-6 against a root mean square of 2) may fall on either side in fp32 and in fp64,
# which switches one term of one column of a weight gradient on or off - a few percent of the largest
# update when a round sums few terms (3.7e-2 measured at K = 1, B = 256), and nothing a norm notices.
# A mis-computed element is off by its own size, i.e. tens of percent of the largest update.
ELEM = 5.0

def compare_models(p, got, want, w0, rounds):
    """Per tensor of the model (every W_l and every b_l separately): the relative error of the tensor,
    of its update w - w^0, and the largest element error in units of the tensor's largest update.
    `slack` is what storing `rounds` updates in fp32 may cost (the oracle keeps fp64)."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    w0 = np.asarray(w0, np.float64)
    rows = []
    for name, sl in param_blocks(p):
        g, w, z = got[sl], want[sl], w0[sl]
        upd = w - z
        diff = np.abs(g - w)
        walk = EPS32 * (np.sqrt(rounds) + 1.0)
        rows.append(dict(name=name, finite=bool(np.all(np.isfinite(g))),
                         nw=float(np.linalg.norm(w)), nu=float(np.linalg.norm(upd)),
                         mw=float(np.max(np.abs(w))), mu=float(np.max(np.abs(upd))),
                         err=float(np.linalg.norm(g - w)), emax=float(diff.max()),
                         slack_norm=walk * float(np.linalg.norm(w)), slack_elem=2.0 * walk * float(np.max(np.abs(w))),
                         untouched_ok=bool(np.array_equal(g, z))))
    return rows


def assert_models_close(p, got, want, w0, tol, rounds, where=""):
    """The parity bar, tensor by tensor and element by element.  For every W_l and b_l:
      * ||g - w|| <= tol ||w||                      the stated tolerance on the parameters,
      * ||g - w|| <= tol ||w - w0|| + slack         ... and on the update the rounds produced,
      * max |g - w| <= ELEM tol max |w - w0| + slack   every element, in units of the tensor's largest update;
    a tensor the oracle leaves unchanged must be unchanged bit for bit.  Returns the worst ratios."""
    worst = dict(w=0.0, upd=0.0, elem=0.0)
    for r in compare_models(p, got, want, w0, rounds):
        tag = f"{where} {r['name']}"
        assert r["finite"], f"{tag}: non-finite parameters"
        if r["mu"] == 0.0:
            assert r["untouched_ok"], f"{tag}: the oracle leaves this tensor unchanged, the library does not"
            continue
        assert r["err"] <= tol * r["nw"], f"{tag}: ||g-w||/||w|| = {r['err'] / r['nw']:.3e} > {tol}"
        assert r["err"] <= tol * r["nu"] + r["slack_norm"], \
            f"{tag}: update differs, ||g-w||/||w-w0|| = {r['err'] / r['nu']:.3e} > {tol}"
        assert r["emax"] <= ELEM * tol * r["mu"] + r["slack_elem"], \
            f"{tag}: element error {r['emax']:.3e} > {ELEM * tol} x largest update {r['mu']:.3e}"
        worst["w"] = max(worst["w"], r["err"] / r["nw"])
        worst["upd"] = max(worst["upd"], max(0.0, r["err"] - r["slack_norm"]) / r["nu"])
        worst["elem"] = max(worst["elem"], max(0.0, r["emax"] - r["slack_elem"]) / r["mu"])
    return worst


def check_models(res, tol, label="", guard=None):
    """All checkpoints of a run_pair result against the oracle, tensor by tensor.  `guard`, if given,
    is a bound far inside the stated tolerance that the measured errors must also keep (both sides
    narrow the same quantities at the same points and differ only in accumulation width and order, so
    a kernel mistake of any size lands above it while rounding stays below)."""
    p = res["o"].cfg
    w0 = res["sim_inputs"]["w0"]
    for cp, (g, w) in sorted(res["models"].items()):
        worst = assert_models_close(p, g, w, w0, tol, cp, where=f"{label} round {cp}:")
        print(f"{label} round {cp}: worst tensor rel {worst['w']:.2e}, update rel {worst['upd']:.2e}, "
              f"element/max-update {worst['elem']:.2e}", flush=True)
        tick(f"  {label} round {cp} compared")
        if guard is not None:
            assert max(worst["w"], worst["upd"]) <= guard, f"{label} round {cp}: outside the guard band {guard}: {worst}"


def assert_matches_oracle(p, d, model, trace, T, tol, rerun, where=""):
    """A library run of T rounds (its final model and trace) against a fresh oracle run.  When an
    adaptive wait count flipped on a last-bit difference of a loss, the rounds up to the flip are
    compared and `rerun(settings, k_replay) -> (model, trace)` repeats the library run with the
    oracle's K sequence replayed; the comparison never falls away."""
    o = AbsOracle(p, d["X"], d["y"], d["w0"], keep_models=False)
    while o.t < T:
        o.run(min(_piece(p), T - o.t))
        tick(f"  {where}: oracle at round {o.t}")
    want = np.stack([trace_words(r, p["N"]) for r in o.trace])
    keep = np.ones(want.shape[1], bool)
    keep[LOSS_WORD] = False
    flips = np.nonzero(trace[:, KNEXT_WORD] != want[:, KNEXT_WORD])[0]
    if flips.size:
        assert p["k_mode"] in (0, 3), f"{where}: K^(t+1) differs although the wait count is not adaptive"
        first = int(flips[0])
        keep[KNEXT_WORD] = False
        assert np.array_equal(trace[:first + 1, keep], want[:first + 1, keep]), f"{where}: trace differs before the flip"
        say(f"{where}: adaptive-K flip at round {first}; repeating with the oracle's K replayed")
        model, trace = rerun(dict(p, k_mode=2), [r["K"] for r in o.trace])
    assert np.array_equal(trace[:, keep], want[:, keep]), f"{where}: integer trace differs from the oracle"
    worst = assert_models_close(p, model, o.model(), d["w0"], tol, T, where=where)
    print(f"{where}: worst tensor rel {worst['w']:.2e}, update rel {worst['upd']:.2e}, "
          f"element/max-update {worst['elem']:.2e}", flush=True)
    return worst


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
