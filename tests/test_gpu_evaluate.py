"""GPU parity of the held-out evaluation (mean loss, accuracy of a model version) against the
CPU oracle, through the C-ABI."""
import numpy as np
import pytest

import workloads
import paper_2301_08895_amd as lib
from oracle.abs_sim import AbsOracle
from oracle.evaluate import evaluate

pytestmark = pytest.mark.gpu


def _check(p, T, rows, loss_rtol, versions=(-1,)):
    d, Xe, ye = workloads.make_split(p, rows)      # held-out rows of the same mixture / w*
    Xe64 = workloads.bf16_bits_to_f32(Xe).astype(np.float64) if Xe.dtype == np.uint16 else Xe.astype(np.float64)
    sim = lib.Simulation(p, d)
    sim.round(T)
    for v in versions:
        w = sim.model(v).astype(np.float64)          # the GPU's own model: isolates the evaluation
        loss, acc = sim.evaluate(Xe, ye, v)
        want_loss, want_acc, margin = evaluate(p, w, Xe64, ye)
        print(f"version {v}: loss {loss:.6f} vs {want_loss:.6f}, accuracy {acc} vs {want_acc}", flush=True)
        assert loss == pytest.approx(want_loss, rel=loss_rtol)
        if margin is None:
            assert np.isnan(acc)
        else:
            # a row whose two largest logits are closer than the forward pass's rounding may flip
            unsure = int(np.sum(margin < 1e-3 * max(1.0, float(np.abs(margin).max()))))
            assert abs(acc - want_acc) * rows <= unsure + 1e-9, (acc, want_acc, unsure)
    # the evaluation must not disturb the simulation
    before = sim.model().copy()
    sim.round(3)
    after_eval_then_rounds = sim.model().copy()
    sim.close()
    ref = lib.Simulation(p, d)
    ref.round(T + 3)
    assert np.array_equal(ref.model(), after_eval_then_rounds) and not np.array_equal(before, after_eval_then_rounds)
    ref.close()


def test_linear():
    _check(workloads.scaled_preset(1, M=4000), 60, 5001, 1e-5, versions=(-1, 58))


def test_softmax():
    _check(workloads.scaled_preset(2, M=6000), 80, 40_003, 1e-5, versions=(-1, 77))     # three passes of 16384 rows
    _check(workloads.scaled_preset(2, M=4000, dims=[52, 3], n_classes=3, N=6, B=10, K0=2, tau_cap=2, lr=5e-3), 50, 777, 1e-5)


@pytest.mark.parametrize("over,T,rows", [
    (dict(M=4096, dims=[200, 96, 10], N=8, B=40, n_slow=2, lr=1e-3), 30, 1500),           # several passes, ragged tail
    (dict(M=8192, dims=[256, 256, 512, 10], N=6, B=256, K0=2, n_slow=1, lr=5e-4), 12, 1000),  # 256-tile kernels, one partial pass
    (dict(M=8192, dims=[256, 128, 256, 100], n_classes=100, N=8, B=128, n_slow=0, lr=5e-4), 12, 2049),
    # 256 classes and passes of 128 * 256 rows: the logits product itself runs on the 256 x 256 tile kernel
    (dict(M=65536, dims=[128, 256, 256], n_classes=256, N=128, B=256, K0=4, n_slow=0, lr=2e-4), 3, 40_000),
])
def test_mlp(over, T, rows):
    _check(workloads.scaled_preset(3, **over), T, rows, 2e-3)


def test_version_outside_the_ring_is_an_error():
    p = workloads.scaled_preset(1, M=2000)
    d = workloads.make_inputs(p)
    sim = lib.Simulation(p, d)
    sim.round(20)
    with pytest.raises(lib.AbsError):
        sim.evaluate(d["X"], d["y"], 3)
    with pytest.raises(lib.AbsError):
        sim.evaluate(d["X"], d["y"], 21)
    sim.close()


def test_mlp_full_width_several_passes():
    """The 3072-512-10 workload's layer shapes, evaluation set larger than two passes of N * Bp rows."""
    _check(workloads.scaled_preset(3, M=6400), 10, 9001, 2e-3)
