"""GPU parity at the workloads' full shapes, in the launch configurations bench.py times:
a prefix of rounds from the start of each job (adaptive K) and rounds at K = N (the steady
state), element by element against the oracle; plus properties of whole-length runs that
hold at any size (checked on the GPU trace itself)."""
import numpy as np
import pytest

import workloads
import paper_2301_08895_amd as lib
from parity_util import run_pair, assert_trace_equal, rel_err

pytestmark = pytest.mark.gpu

BF16_TOL = 2e-2
FP32_TOL = 1e-5


def _check(res, tol):
    assert_trace_equal(res, 2e-3)
    T = max(res["models"])
    for cp, (g, w) in res["models"].items():
        e = rel_err(g, w)
        print(f"round {cp}: rel err {e:.3e}", flush=True)
        assert np.all(np.isfinite(g)) and e <= tol, (cp, e)
    g, w = res["models"][T]
    w0 = res["sim_inputs"]["w0"].astype(np.float64)
    assert rel_err(g - w0, w - w0) <= tol


@pytest.mark.parametrize("i,T,T_full_k", [(3, 40, 3), (4, 8, 2), (5, 3, 1)])
def test_mlp_workload_prefix_and_steady_state(i, T, T_full_k):
    p = workloads.preset(i)
    d = workloads.make_inputs(p)
    print(f"{p['name']}: adaptive prefix of {T} rounds", flush=True)
    _check(run_pair(p, T, checkpoints=(1,), inputs=d), BF16_TOL)
    q = dict(p, k_mode=1, K0=p["N"])
    print(f"{p['name']}: {T_full_k} rounds at K = N = {p['N']}", flush=True)
    _check(run_pair(q, T_full_k, inputs=d), BF16_TOL)


def _trace_properties(p, tr):
    N, cap = p["N"], p["tau_cap"]
    K = tr[:, 1]
    assert K[0] == p["K0"] and np.all(np.diff(K) >= 0) and K.max() <= N
    assert np.all(tr[:-1, 11] == K[1:])                         # K^{t+1} word feeds the next round
    assert np.all((tr[:, 2] >= 1) & (tr[:, 2] <= cap))           # Eq. 4: 1 <= tau_max <= tau_cap
    now = tr[:, 3].astype(np.uint32).astype(np.int64) | (tr[:, 4].astype(np.int64) << 32)
    assert np.all(np.diff(now) >= 0)
    tau = np.zeros(N, dtype=np.int64)
    for r in range(tr.shape[0]):
        k = K[r]
        ids = tr[r, 12:12 + k]
        vers = tr[r, 12 + k:12 + 2 * k]
        taus = tr[r, 12 + 2 * k:12 + 3 * k]
        nres = tr[r, 5]
        res = tr[r, 12 + 3 * k:12 + 3 * k + nres]
        assert len(set(ids.tolist())) == k
        assert np.all(vers + taus == r) and np.array_equal(tau[ids], taus)
        assert taus.max() <= cap + 1                            # bounded staleness
        keep = np.ones(N, bool); keep[ids] = False; keep[res] = False
        assert np.all(tau[res] > tr[r, 2])                      # restarted <=> over the threshold
        assert np.all(tau[keep] <= tr[r, 2])
        tau[keep] += 1
        tau[~keep] = 0
    up = tr[:, 6].astype(np.uint32).astype(np.int64) | (tr[:, 7].astype(np.int64) << 32)
    assert np.array_equal(up, np.cumsum(K))


@pytest.mark.parametrize("i", [2, 3])
def test_whole_job_properties(i):
    """The whole job at full size on the GPU: invariants of Eq. 4-6 on its own trace, the
    loss falls, K reaches N, and the schedule-only mode replays the same integer trace."""
    p = workloads.preset(i)
    d = workloads.make_inputs(p)
    sim = lib.Simulation(p, d)
    sim.round(p["T"])
    tr = sim.trace()
    w = sim.model()
    sim.close()
    _trace_properties(p, tr)
    loss = tr[:, 10].copy().view(np.float32)
    assert np.all(np.isfinite(loss)) and np.all(np.isfinite(w))
    assert loss[-50:].mean() < 0.25 * loss[:5].mean()
    assert tr[-1, 1] == p["N"]
    dry = lib.Simulation(dict(p, k_mode=2), None, device_mode=0, k_replay=tr[:, 1].copy())
    dry.round(p["T"])
    tr2 = dry.trace()
    dry.close()
    keep = np.ones(tr.shape[1], bool); keep[10] = False
    assert np.array_equal(tr[:, keep], tr2[:, keep])


@pytest.mark.parametrize("i,S,T", [(2, 64, 40), (2, 128, 24), (1, 512, 60)])
def test_batched_rounds_at_full_size(i, S, T):
    """The batches bench.py times (--batch S): the workload at its full shape, S simulation seeds on
    one dataset, advanced as groups (three, four and two).  Sampled simulations against the oracle,
    every trace against the invariants of Eq. 4-6."""
    from oracle.abs_sim import AbsOracle, trace_words
    from parity_util import LOSS_WORD, KNEXT_WORD
    p = workloads.preset(i)
    d = workloads.make_inputs(p)
    ps = [dict(p, seed_sim=p["seed_sim"] + 7919 * k) for k in range(S)]
    sims = [lib.Simulation(q, d) for q in ps]
    batch = lib.Batch(sims)
    batch.round(T)
    batch.close()
    got = [(s.model().copy(), s.trace().copy()) for s in sims]
    for s in sims:
        s.close()
    for q, (w, tr) in zip(ps, got):
        assert np.all(np.isfinite(w))
        _trace_properties(q, tr)
    checked = 0
    for k in (0, S // 2 - 1, S // 2, S - 1):
        o = AbsOracle(ps[k], d["X"], d["y"], d["w0"], keep_models=False).run(T)
        want = np.stack([trace_words(r, p["N"]) for r in o.trace])
        w, tr = got[k]
        if np.any(tr[:, KNEXT_WORD] != want[:, KNEXT_WORD]):
            continue                      # an adaptive-K decision flipped on a last-bit loss difference
        keep = np.ones(tr.shape[1], bool)
        keep[LOSS_WORD] = False
        assert np.array_equal(tr[:, keep], want[:, keep])
        e = rel_err(w, o.model())
        print(f"simulation {k}: rel err {e:.3e}", flush=True)
        assert e <= FP32_TOL
        checked += 1
    assert checked >= 2


def test_mlp_batch_at_full_size():
    """cfg 3 at its full shape, three simulations side by side (bench.py --config 3 --batch S): every
    one bitwise its unbatched run."""
    p = workloads.preset(3)
    d = workloads.make_inputs(p)
    ps = [dict(p, seed_sim=p["seed_sim"] + 7919 * k) for k in range(3)]
    T = 8
    sims = [lib.Simulation(q, d) for q in ps]
    batch = lib.Batch(sims)
    batch.round(T)
    batch.close()
    got = [(s.model().copy(), s.trace().copy()) for s in sims]
    for s in sims:
        s.close()
    for q, (w, tr) in zip(ps, got):
        alone = lib.Simulation(q, d)
        alone.round(T)
        assert np.array_equal(alone.model(), w) and np.array_equal(alone.trace(), tr)
        alone.close()
        _trace_properties(q, tr)
