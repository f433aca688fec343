"""GPU parity of the convolutional model (Section V-A: two convolutional + three dense layers, fp32)
against the CPU oracle, through the C-ABI: trace bit-exact, every tensor of the model and every
element; held-out evaluation; the hand-worked gradient; run-to-run determinism."""
import numpy as np
import pytest

import workloads
import paper_2301_08895_amd as lib
from oracle.evaluate import evaluate
from parity_util import run_pair, assert_trace_equal, check_models, golden_lines

pytestmark = pytest.mark.gpu

# fp32 on the GPU against fp64 in the oracle.  A filter gradient is a sum of up to K B S1 S1 (thousands of)
# signed products that largely cancel, each rounded to 2^-24: the sum's error relative to its own size is
# some 1e-6 .. 1e-5 per round, and a pooling window or ReLU whose two candidates differ by less than the
# forward pass's rounding may pick the other one.  Stated bar 1e-4 on every tensor, its update and (x 5)
# every element; measured errors stay below the guard.
FP32_TOL = 1e-4
GUARD = 3e-5


def _small(**over):
    """A reduced geometry: C0 x S x S images, k x k filters."""
    g = dict(C0=2, S=14, k=3, C1=4, C2=5, F1=24, F2=12, C=4)
    g.update({k: over.pop(k) for k in list(over) if k in g})
    dims = [g["C0"] * g["S"] ** 2, g["C1"], g["C2"], g["F1"], g["F2"], g["C"], g["C0"], g["k"]]
    base = dict(M=2000, dims=dims, n_classes=g["C"], N=6, B=8, K0=2, tau_cap=2, lr=3e-3)
    base.update(over)
    return workloads.scaled_preset(6, **base)


@pytest.mark.parametrize("over,T", [
    (dict(), 40),
    (dict(C0=1, S=10, k=3, C1=2, C2=3, F1=7, F2=5, C=3, N=4, B=5, K0=1), 40),        # odd sizes, ragged everything
    (dict(C0=3, S=32, k=5, C1=6, C2=16, F1=120, F2=84, C=10, N=8, B=32, K0=2, M=4000), 12),   # the full network, fewer workers
    (dict(N=12, B=16, K0=3, tau_cap=3, sa_penalty=1, n_slow=2, slow_factor=4.0), 30),       # staleness-aware steps, stragglers
    (dict(k_mode=1, K0=6, N=6), 6),                                                      # every worker every round
])
def test_rounds_against_the_oracle(over, T):
    p = _small(**over)
    res = run_pair(p, T, checkpoints=(1, max(1, T // 2)))
    assert_trace_equal(res, 1e-4)
    check_models(res, FP32_TOL, label=p["name"], guard=GUARD)
    stale = sum(1 for r in res["o"].trace for tau in r["taus"] if tau > 0)
    print("stale uploads aggregated:", stale, flush=True)


def test_the_workload_itself():
    """Preset 6 at its own shape (N = 20, B = 32, 3 x 32 x 32 images): its first rounds."""
    p = workloads.scaled_preset(6, M=20_000)
    res = run_pair(p, 16, checkpoints=(1, 4))
    assert_trace_equal(res, 1e-4)
    check_models(res, FP32_TOL, label=p["name"], guard=GUARD)
    assert any(tau > 0 for r in res["o"].trace for tau in r["taus"])


def test_hand_worked_gradient_on_the_gpu():
    vals = {t[0]: [float(v) for v in t[1:]] for t in golden_lines("cnn_hand_worked_gradient.txt")}
    p = workloads.scaled_preset(6, M=1, dims=[16, 1, 1, 1, 1, 2, 1, 1], n_classes=2, N=1, B=1, K0=1, k_mode=1,
                                tau_cap=1, lr=0.5)
    x = np.array([[1, 2, 0, -1, 3, -2, 1, 0, 0, 1, -1, 2, -3, 0, 4, 1]], dtype=np.float32)
    w0 = np.array([2, -1, 0.5, -1, 2, -1, 0.5, 0, 0.5, -0.5, 0, 0], dtype=np.float32)
    d = dict(X=x, y=np.array([1], dtype=np.int32), w0=w0)
    sim = lib.Simulation(p, d)
    sim.round(1)
    w1 = sim.model().astype(np.float64)
    loss = sim.trace()[0, 10:11].copy().view(np.float32)[0]
    sim.close()
    q = vals["q"][0]
    assert abs(loss - vals["loss"][0]) < 1e-6
    np.testing.assert_allclose(w1, w0 - 0.5 * q * np.array(vals["gradient_over_q"]), rtol=2e-7, atol=1e-7)


def test_evaluation_against_the_oracle():
    p = _small(M=1500)
    d, Xe, ye = workloads.make_split(p, 333)
    sim = lib.Simulation(p, d)
    sim.round(20)
    for v in (-1, 19):
        w = sim.model(v).astype(np.float64)
        loss, acc = sim.evaluate(Xe, ye, v)
        want_loss, want_acc, margin = evaluate(p, w, Xe.astype(np.float64), ye)
        unsure = int(np.sum(margin < 1e-4 * max(1.0, float(np.abs(margin).max()))))
        print(f"version {v}: loss {loss:.6f} vs {want_loss:.6f}, accuracy {acc} vs {want_acc}", flush=True)
        assert loss == pytest.approx(want_loss, rel=1e-5)
        assert abs(acc - want_acc) * 333 <= unsure + 1e-9
    before = sim.model().copy()
    sim.round(2)
    after = sim.model().copy()
    sim.close()
    ref = lib.Simulation(p, d)
    ref.round(22)
    assert np.array_equal(ref.model(), after) and not np.array_equal(before, after)
    ref.close()


def test_two_runs_are_bitwise_identical_and_a_batch_equals_its_members():
    p = _small()
    d = workloads.make_inputs(p)
    runs = []
    for _ in range(2):
        sim = lib.Simulation(p, d)
        sim.round(15)
        runs.append((sim.model().copy(), sim.trace().copy()))
        sim.close()
    assert np.array_equal(runs[0][0], runs[1][0]) and np.array_equal(runs[0][1], runs[1][1])
    sims = [lib.Simulation(dict(p, seed_sim=p["seed_sim"] + i), d) for i in range(3)]
    batch = lib.Batch(sims)
    batch.round(15)
    assert np.array_equal(sims[0].model(), runs[0][0]) and np.array_equal(sims[0].trace(), runs[0][1])
    assert not np.array_equal(sims[1].model(), runs[0][0])
    batch.close()
    for s in sims:
        s.close()


@pytest.mark.parametrize("over,T", [
    (dict(U=3), 20),
    (dict(U=10, C0=3, S=32, k=5, C1=6, C2=16, F1=120, F2=84, C=10, N=6, B=32, K0=2, M=4000, lr=1e-3), 5),   # the paper's U
    (dict(U=2, sa_penalty=1, N=10, K0=2, tau_cap=3), 20),
])
def test_local_steps_against_the_oracle(over, T):
    """Eq. 2 with U > 1: every upload steps a private copy of its stale model U times."""
    p = _small(**over)
    res = run_pair(p, T, checkpoints=(1,))
    assert_trace_equal(res, 1e-4)
    check_models(res, FP32_TOL, label=f"{p['name']} U={p['U']}", guard=GUARD)


def test_unsupported_settings_are_refused():
    p = _small(S=15)           # 15 - 3 + 1 = 13 is odd: no 2 x 2 pooling
    with pytest.raises(lib.AbsError):
        lib.abs_workspace_size(lib.make_config(p))
