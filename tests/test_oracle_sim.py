"""Pins for the oracle's event logic (CPU only): the reductions the paper states in
Section II-B, the invariants of Eq. 4-6, closed forms of the two adaptive rules,
and a brute-force re-derivation of the schedule from the full job history."""
from fractions import Fraction

import numpy as np
import pytest

import workloads
from oracle import counter_rng as crng
from oracle.abs_sim import (AbsOracle, next_wait_count, over_stale, threshold_floor,
                            trace_words, trace_stride, INT32_MAX)
from oracle.models import worker_update
from parity_util import (golden_lines, hand_worked_schedule, hand_worked_updates, softmax_hand_worked_first_round,
                         mlp_hand_worked_first_round, local_sgd_hand_worked)


def _small(model=0, **over):
    base = dict(M=400, N=4, B=8, T=30, tau_cap=2)
    if model == 0:
        base.update(dims=[12, 1])
        p = workloads.scaled_preset(1, **{**base, **over})
    elif model == 1:
        base.update(dims=[10, 3], n_classes=3)
        p = workloads.scaled_preset(2, **{**base, **over})
    else:
        base.update(dims=[16, 8, 3], n_classes=3, n_slow=1)
        p = workloads.scaled_preset(3, **{**base, **over})
    return p, workloads.make_inputs(p)


def _rows(p, d, idx):
    X = d["X"][idx]
    if p["x_dtype"] == 1:
        X = workloads.bf16_bits_to_f32(X)
    return X.astype(np.float64)


# ---------------------------------------------------------------- reductions

@pytest.mark.parametrize("model", [0, 1, 2])
def test_reduces_to_synchronous_sgd(model):
    """K^t = N, U = 1, tau = 0 is synchronous SGD (Section II-B): with constant
    execution times every worker uploads every round and the run must equal a
    plain minibatch-SGD loop w <- w - (eta/N) sum_n g_n(w)."""
    p, d = _small(model, k_mode=1, K0=4, time_dist=2, tau_mode=1, sa_penalty=0, n_slow=0)
    # wide arithmetic here; the bf16 rounding points are pinned in the gradient tests
    o = AbsOracle(p, d["X"], d["y"], d["w0"], emulate_bf16=False).run(12)
    lr = float(np.float32(p["lr"]))
    w = d["w0"].astype(np.float64)
    for t in range(12):
        acc = np.zeros_like(w)
        for n in range(4):
            idx = crng.batch_indices(p, n, t)
            g, _ = worker_update(p, w, _rows(p, d, idx), d["y"][idx], 1.0, False)
            acc += g
        w_next = w - (lr / 4) * acc
        assert np.allclose(o.model(t + 1), w_next, rtol=1e-12, atol=1e-15)
        w = o.model(t + 1).copy()
        assert o.trace[t]["taus"] == [0, 0, 0, 0] and o.trace[t]["ids"] == [0, 1, 2, 3]
        assert o.trace[t]["n_restart"] == 0


@pytest.mark.parametrize("K", [1, 2])
def test_reduces_to_asgd_and_k_async(K):
    """K^t = 1 without restarts is ASGD, fixed K without restarts is K-async SGD
    (Sections I and II-B).  Independent event loop: every worker holds the model
    it last read; the K earliest finishers are applied and re-issued."""
    p, d = _small(0, k_mode=1, K0=K, tau_mode=2, N=5, M=500)
    T = 25
    o = AbsOracle(p, d["X"], d["y"], d["w0"]).run(T)
    lr = float(np.float32(p["lr"]))
    w = d["w0"].astype(np.float64)
    held = [w.copy() for _ in range(5)]
    jobs = [0] * 5
    fin = [crng.compute_time_ticks(p, n, 0) for n in range(5)]
    for t in range(T):
        first = sorted(range(5), key=lambda n: (fin[n], n))[:K]
        now = fin[first[-1]]
        step = np.zeros_like(w)
        for n in first:
            idx = crng.batch_indices(p, n, jobs[n])
            g, _ = worker_update(p, held[n], d["X"][idx].astype(np.float64), d["y"][idx], 1.0)
            step += g
        w = w - (lr / K) * step
        for n in first:
            held[n] = w.copy(); jobs[n] += 1
            fin[n] = now + crng.compute_time_ticks(p, n, jobs[n])
        assert o.trace[t]["ids"] == first and o.trace[t]["now"] == now
        assert np.allclose(o.model(t + 1), w, rtol=1e-12, atol=1e-15)
    assert max(max(r["taus"]) for r in o.trace) > 2     # staleness is unbounded here


@pytest.mark.parametrize("model", [0, 1, 2])
def test_local_steps_reduce_to_model_averaging(model):
    """U > 1 with K^t = N and tau = 0 is classical (synchronous) local SGD (Section II-B):
    every worker takes U SGD steps of Eq. 2 from w^t on fresh minibatches and the server
    keeps the average of the N local models; the reported loss is the mean local loss."""
    U = 3
    p, d = _small(model, k_mode=1, K0=4, time_dist=2, tau_mode=1, sa_penalty=0, n_slow=0, U=U)
    o = AbsOracle(p, d["X"], d["y"], d["w0"], emulate_bf16=False).run(6)
    lr = float(np.float32(p["lr"]))
    w = d["w0"].astype(np.float64)
    for t in range(6):
        finals, losses = [], []
        for n in range(4):
            wn = w.copy()
            for u in range(U):
                idx = crng.batch_indices(p, n, t, u)
                g, l = worker_update(p, wn, _rows(p, d, idx), d["y"][idx], 1.0, False)
                wn = wn - lr * g
                losses.append(l)
            finals.append(wn)
        w_avg = np.mean(finals, axis=0)
        assert np.allclose(o.model(t + 1), w_avg, rtol=1e-12, atol=1e-15)
        assert np.isclose(o.trace[t]["loss"], np.mean(losses), rtol=1e-12)
        w = o.model(t + 1).copy()
    # the minibatches of different local steps differ, and differ from the next job's
    assert crng.batch_indices(p, 1, 0, 0) != crng.batch_indices(p, 1, 0, 1)
    assert crng.batch_indices(p, 1, 0, 1) != crng.batch_indices(p, 1, 1, 0)


def test_one_local_step_is_the_plain_update():
    """The U-step route at U = 1 (upload w^{t,0} - w^{t,1} = eta_k g_k) is Eq. 3's update."""
    p, d = _small(1, T=40, lr=0.05, sa_penalty=1)
    a = AbsOracle(p, d["X"], d["y"], d["w0"]).run(40)
    b = AbsOracle(p, d["X"], d["y"], d["w0"], local_path=True).run(40)
    assert [r["ids"] for r in a.trace] == [r["ids"] for r in b.trace]
    assert np.allclose(a.model(), b.model(), rtol=1e-11, atol=1e-14)


def test_staleness_aware_penalty_scales_the_stale_gradient():
    """SA: the step of a gradient with delay tau is eta / tau (Section I); one ASGD
    round with a stale upload must move the model by (eta/tau_k) g_k exactly."""
    p, d = _small(0, k_mode=1, K0=1, tau_mode=2, N=3, M=300, sa_penalty=1)
    o = AbsOracle(p, d["X"], d["y"], d["w0"]).run(15)
    lr = float(np.float32(p["lr"]))
    hit = 0
    for r in o.trace:
        (k,), (v,), (tau,) = r["ids"], r["vers"], r["taus"]
        job = sum(1 for q in o.trace[:r["t"]] if k in q["ids"])
        idx = crng.batch_indices(p, k, job)
        g, _ = worker_update(p, o.model(v), d["X"][idx].astype(np.float64), d["y"][idx], 1.0)
        want = o.model(r["t"]) - (lr / max(1, tau)) * g
        assert np.allclose(o.model(r["t"] + 1), want, rtol=1e-12, atol=1e-15)
        hit += tau >= 2
    assert hit > 0


# ---------------------------------------------------------------- closed forms

def test_threshold_rule_closed_forms():
    # Eq. 4: N = 8, K = 2, a = -1 -> 3;  K = 8 -> max{1, 0} = 1
    assert threshold_floor(2, 8, -1, 0, 99) == 3
    assert threshold_floor(8, 8, -1, 0, 99) == 1
    assert threshold_floor(2, 8, -1, 0, 2) == 2            # capped
    assert threshold_floor(3, 8, -1, 1, 5) == 5            # fixed mode
    assert threshold_floor(3, 8, -1, 2, 5) == INT32_MAX    # no threshold
    for N in (5, 8, 20):
        for K in range(1, N + 1):
            for a in range(-4, 4):
                tmax = max(Fraction(1), Fraction(N, K) + a)
                for tau in range(0, 12):
                    assert over_stale(tau, K, N, a, 0, 10 ** 6) == (tau > tmax)
                    assert over_stale(tau, K, N, a, 0, 3) == (tau > min(tmax, 3))
                    assert over_stale(tau, K, N, a, 1, 3) == (tau > 3)
                    assert not over_stale(tau, K, N, a, 2, 3)
                assert threshold_floor(K, N, a, 0, 10 ** 6) == int(tmax // 1)


def test_wait_count_rule_closed_forms():
    # Eq. 5: ratio f(w0)/f(wt) = 1 -> K0;  = 4 -> 2 K0;  = 2.25 -> 1.5 K0
    assert next_wait_count(5, 20, 5, 3.0, 3.0, 0) == 5
    assert next_wait_count(5, 20, 5, 4.0, 1.0, 0) == 10
    assert next_wait_count(4, 20, 4, 2.25, 1.0, 0) == 6
    assert next_wait_count(5, 20, 5, 4.0, 1.0 + 1e-12, 0) == 9       # floor
    assert next_wait_count(5, 20, 5, 1.0, 1e-9, 0) == 20             # clamp to N
    assert next_wait_count(5, 20, 5, 1.0, 0.0, 0) == 20
    assert next_wait_count(5, 20, 12, 1.0, 1.0, 0) == 12             # never decreases (k_mode 0)
    assert next_wait_count(5, 20, 12, 1.0, 1.0, 3) == 5              # free-running variant
    assert next_wait_count(5, 20, 12, 1.0, 9.0, 3) == 1              # floor(5/3) = 1
    assert next_wait_count(5, 20, 7, 4.0, 1.0, 1) == 5               # fixed K
    with pytest.raises(FloatingPointError):
        next_wait_count(5, 20, 5, 1.0, float("nan"), 0)
    for ratio in np.linspace(0.2, 30, 200):
        want = max([j for j in range(1, 21) if Fraction(j * j) <= 9 * Fraction(float(ratio))] or [1])
        assert next_wait_count(3, 20, 1, float(ratio), 1.0, 3) == want      # = floor(3 sqrt(ratio))
        assert want == min(20, max(1, int(np.floor(3 * np.sqrt(ratio)))))


def test_adaptive_rules_equal_the_hand_worked_values():
    """tests/golden/threshold_and_wait_count_values.txt: Eq. 4 and Eq. 5 evaluated by hand, among
    them the setting of Section V-B (N = 20, K^0 = 5, a = 0 .. -3)."""
    n_tau = n_k = 0
    for row in golden_lines("threshold_and_wait_count_values.txt"):
        if row[0] == "tau":
            N, K, a, want = (int(v) for v in row[1:])
            assert threshold_floor(K, N, a, 0, 10 ** 6) == want, row
            assert over_stale(want + 1, K, N, a, 0, 10 ** 6) and not over_stale(want, K, N, a, 0, 10 ** 6), row
            n_tau += 1
        else:
            K0, N, Kprev = (int(v) for v in row[1:4])
            assert next_wait_count(K0, N, Kprev, float(row[4]), float(row[5]), 0) == int(row[6]), row
            n_k += 1
    assert n_tau >= 10 and n_k >= 8


def test_schedule_equals_the_hand_worked_run():
    """tests/golden/abs_hand_worked_schedule.txt: seven rounds of Algorithm 1 on four workers worked
    out with pencil and paper (ties, a gradient of staleness tau_max + 1, a restart by Eq. 6)."""
    setting, want = hand_worked_schedule()
    p, d = _small(0, **setting)
    o = AbsOracle(p, d["X"], d["y"], d["w0"], keep_models=False).run(len(want))
    assert len(o.trace) == len(want)
    for got, w in zip(o.trace, want):
        for key, val in w.items():
            assert list(got[key]) == val if isinstance(val, list) else got[key] == val, (w["t"], key, got[key], val)
        assert got["n_restart"] == len(w["restart_ids"]) and got["K_next"] == w["K"]


@pytest.mark.parametrize("sa", [0, 1])
def test_updates_equal_the_hand_worked_run(sa):
    """tests/golden/abs_hand_worked_updates.txt: Eq. 2 / Eq. 3 on three rows by hand, with a gradient
    taken at a model two rounds old, plain and with the staleness-aware step."""
    p, d, models, losses = hand_worked_updates(sa)
    o = AbsOracle(p, d["X"], d["y"], d["w0"]).run(3)
    assert [r["ids"] for r in o.trace] == [[1, 2], [1, 2], [0, 1]] and o.trace[2]["taus"] == [2, 0]
    for v, w in models.items():
        assert np.array_equal(o.model(v), w), (v, o.model(v), w)         # every value is a dyadic fraction
    for t, l in losses.items():
        assert o.trace[t]["loss"] == l


def test_softmax_first_round_equals_the_hand_worked_values():
    """tests/golden/softmax_hand_worked_first_round.txt: from W = 0 every class has probability 1/C, so
    the gradient of Eq. 3's first round is an exact fraction; loss log C."""
    p, d, w1 = softmax_hand_worked_first_round()
    o = AbsOracle(p, d["X"], d["y"], d["w0"]).run(1)
    assert np.allclose(o.model(1), w1, rtol=0, atol=1e-15)
    assert abs(o.trace[0]["loss"] - np.log(4.0)) < 1e-12


def test_mlp_first_round_equals_the_hand_worked_values():
    """tests/golden/mlp_hand_worked_first_round.txt: ReLU forward, output-layer gradient H^T dZ and
    update by hand (exact fractions, also under the bf16 narrowing); the hidden layer must not move."""
    p, d, w1 = mlp_hand_worked_first_round()
    for emulate in (True, False):
        o = AbsOracle(p, d["X"], d["y"], d["w0"], emulate_bf16=emulate).run(1)
        assert np.allclose(o.model(1), w1, rtol=0, atol=1e-15), emulate
        assert abs(o.trace[0]["loss"] - np.log(4.0)) < 1e-12


def test_local_sgd_equals_the_hand_worked_run():
    """tests/golden/local_sgd_hand_worked.txt: U = 2 local steps per job, uploads w^{t,0} - w^{t,U},
    Eq. 3 over the uploads, average local loss; exact in binary."""
    p, d, models, losses = local_sgd_hand_worked()
    o = AbsOracle(p, d["X"], d["y"], d["w0"]).run(2)
    for v, w in models.items():
        assert np.array_equal(o.model(v), w), (v, o.model(v), w)
    for t, l in losses.items():
        assert o.trace[t]["loss"] == l


# ---------------------------------------------------------------- invariants

def _check_invariants(p, o):
    N, cap = p["N"], p["tau_cap"]
    tau = [0] * N
    prev_now, prevK = 0, None
    uploads = restarts = 0
    for r in o.trace:
        K, t = r["K"], r["t"]
        assert len(r["ids"]) == K == len(set(r["ids"]))                       # |K^t| = K^t
        assert all(v + s == t for v, s in zip(r["vers"], r["taus"]))          # tau = t - version
        assert [tau[k] for k in r["ids"]] == r["taus"]
        if p["tau_mode"] != 2:
            assert max(r["taus"]) <= cap + 1                                  # bounded staleness
            assert 1 <= r["tau_max"] <= cap                                   # Eq. 4 floor of 1
        assert r["now"] >= prev_now
        prev_now = r["now"]
        if p["k_mode"] == 0 and prevK is not None:
            assert p["K0"] <= prevK <= K <= N
        prevK = K
        must = {n for n in range(N) if n not in r["ids"] and
                over_stale(tau[n], K, N, p["a"], p["tau_mode"], cap)}
        assert set(r["restart_ids"]) == must and r["restart_ids"] == sorted(must)
        for n in range(N):                                                    # Eq. 6
            tau[n] = 0 if (n in r["ids"] or n in must) else tau[n] + 1
        if p["tau_mode"] != 2:
            assert max(tau) <= cap + 1
        uploads += K; restarts += len(must)
        assert (r["comm_uploads"], r["comm_restarts"]) == (uploads, restarts)
    assert o.trace[0]["K"] == p["K0"]
    if p["k_mode"] in (0, 3) and len(o.trace) > 1:
        assert o.trace[1]["K"] == p["K0"]            # ratio is 1 after round 0
    assert tau == o.tau
    assert all(f >= o.now for f in o.fin)


@pytest.mark.parametrize("which", range(6))
def test_invariants_on_varied_runs(which):
    over = [dict(), dict(tau_mode=1, tau_cap=1), dict(time_dist=1, time_param=1.5, N=8, M=800, tau_cap=3),
            dict(k_mode=3), dict(tau_mode=2), dict(N=7, M=700, K0=2, tau_cap=4, sa_penalty=1, seed_sim=77)][which]
    p, d = _small(0, T=120, lr=0.02, **over)
    o = AbsOracle(p, d["X"], d["y"], d["w0"]).run(120)
    _check_invariants(p, o)
    if which in (0, 1, 2):
        assert sum(r["n_restart"] for r in o.trace) > 0       # the restart rule is exercised


def test_invariants_classification_models():
    for model in (1, 2):
        p, d = _small(model, T=40, lr=0.02 if model == 1 else 2e-3)
        o = AbsOracle(p, d["X"], d["y"], d["w0"]).run(40)
        _check_invariants(p, o)


def test_schedule_rederived_from_job_history():
    """Brute force on tiny instances: recompute, from nothing but the list of past
    receiver sets and completion times, which model every worker holds, which job it
    runs and when it finishes; the K earliest must be the oracle's selection."""
    for seed in range(6):
        p, d = _small(0, N=4, M=400, T=8, tau_cap=1 + seed % 2, seed_sim=500 + seed, K0=1 + seed % 2)
        o = AbsOracle(p, d["X"], d["y"], d["w0"]).run(8)
        history = []                       # (receivers of w^{t+1}, completion tick of round t)
        for r in o.trace:
            t = r["t"]
            state = []
            for n in range(4):
                got = [(q + 1, now) for q, (recv, now) in enumerate(history) if n in recv]
                ver, start = got[-1] if got else (0, 0)
                job = len(got)
                state.append((start + crng.compute_time_ticks(p, n, job), n, ver, job))
            first = sorted(state)[:r["K"]]
            assert [s[1] for s in first] == r["ids"]
            assert [s[2] for s in first] == r["vers"]
            assert first[-1][0] == r["now"]
            stale = {n for (_, n, ver, _) in state if n not in r["ids"] and
                     over_stale(t - ver, r["K"], 4, p["a"], p["tau_mode"], p["tau_cap"])}
            assert sorted(stale) == r["restart_ids"]
            history.append((set(r["ids"]) | stale, r["now"]))


def test_large_a_discards_nothing():
    """With a large constant a the threshold is never hit and ABS behaves like the
    unbounded adaptive scheme (Section V-B): identical trace to tau_mode 2."""
    p, d = _small(0, T=60, tau_cap=10 ** 6, a=10 ** 6)
    q = dict(p, tau_mode=2)
    o1 = AbsOracle(p, d["X"], d["y"], d["w0"]).run(60)
    o2 = AbsOracle(q, d["X"], d["y"], d["w0"]).run(60)
    assert [r["ids"] for r in o1.trace] == [r["ids"] for r in o2.trace]
    assert np.array_equal(o1.model(), o2.model())
    assert sum(r["n_restart"] for r in o1.trace) == 0


def test_k_replay_reproduces_adaptive_run():
    p, d = _small(1, T=50, lr=0.05)
    o1 = AbsOracle(p, d["X"], d["y"], d["w0"]).run(50)
    Ks = [r["K"] for r in o1.trace]
    assert Ks[-1] > Ks[0]
    q = dict(p, k_mode=2, k_replay=Ks)
    o2 = AbsOracle(q, d["X"], d["y"], d["w0"]).run(50)
    assert np.array_equal(o1.model(), o2.model())
    assert [r["ids"] for r in o1.trace] == [r["ids"] for r in o2.trace]


def test_least_squares_converges_to_noise_floor():
    """Textbook sanity of data + step size: the iterate approaches w* and the minibatch
    loss approaches sigma^2 / 2 with sigma = 0.01."""
    p = workloads.preset(1)
    d = workloads.make_inputs(p)
    o = AbsOracle(p, d["X"], d["y"], d["w0"]).run(1500)
    err0 = np.linalg.norm(d["w0"] - d["w_star"])
    err = np.linalg.norm(o.model() - d["w_star"])
    assert err < 0.02 * err0
    assert np.mean([r["loss"] for r in o.trace[-50:]]) < 5e-3
    assert o.trace[-1]["K"] == p["N"]


def test_trace_word_layout():
    p, d = _small(0, T=5)
    o = AbsOracle(p, d["X"], d["y"], d["w0"]).run(5)
    r = o.trace[3]
    w = trace_words(r, 4)
    assert w.dtype == np.int32 and w.size == trace_stride(4) == 24
    assert (w[0], w[1], w[2]) == (3, r["K"], r["tau_max"])
    assert int(w[3]) & 0xFFFFFFFF | (int(w[4]) << 32) == r["now"]
    K = r["K"]
    assert list(w[12:12 + K]) == r["ids"] and list(w[12 + 2 * K:12 + 3 * K]) == r["taus"]
    assert w[11] == r["K_next"] and np.int32(w[10]).view(np.float32) == np.float32(r["loss"])
    assert all(x == -1 for x in w[12 + 3 * K + r["n_restart"]:])
