"""GPU parity of the comparison systems (settings of the same round) against the CPU oracle."""
import numpy as np
import pytest

import workloads
from parity_util import run_pair, assert_trace_equal, check_models

pytestmark = pytest.mark.gpu

SOFTMAX = workloads.scaled_preset(2, M=3000, dims=[16, 4], n_classes=4, N=12, B=8, K0=3, lr=5e-2, n_slow=3,
                                  slow_factor=5.0)
LINEAR = workloads.scaled_preset(1, M=4000, N=8, B=16)
MLP = workloads.scaled_preset(3, M=4096, dims=[128, 64, 10], N=8, B=32, n_slow=2, lr=1e-3)
# the convolutional model at a reduced geometry: 2 x 14 x 14 images, 3 x 3 filters, 4 and 5 channels, 20-24-12-4
CNN = workloads.scaled_preset(6, M=2000, dims=[2 * 14 * 14, 4, 5, 24, 12, 4, 2, 3], n_classes=4, N=8, B=8, K0=2,
                              tau_cap=2, lr=3e-3, n_slow=2, slow_factor=4.0)


@pytest.mark.parametrize("name", workloads.METHODS)
@pytest.mark.parametrize("base,tol,loss_rtol", [(LINEAR, 1e-5, 1e-4), (SOFTMAX, 1e-5, 1e-4), (MLP, 2e-2, 2e-3),
                                                (CNN, 1e-4, 1e-4)],
                         ids=["linear", "softmax", "mlp", "cnn"])
def test_method(base, tol, loss_rtol, name):
    over = dict(U=3) if name == "local_sgd" else {}
    p = workloads.method_preset(base, name, **over)
    T = 25 if name in ("sync_sgd", "local_sgd") else 80
    if base is CNN:
        T = min(T, 30)               # the oracle's convolutions are plain loops
    res = run_pair(p, T, checkpoints=(1,))
    assert_trace_equal(res, loss_rtol)
    check_models(res, tol, label=name)
    tr = res["got"]
    if name in ("adasync", "sa_adasync", "k_async", "asgd", "sync_sgd", "local_sgd"):
        assert np.all(tr[:, 5] == 0)                       # no forced restarts without a threshold
    if name == "asgd":
        assert np.all(tr[:, 1] == 1)
    if name in ("sync_sgd", "local_sgd"):
        assert np.all(tr[:, 1] == p["N"])


def test_compare_tool_readouts(capsys):
    """The read-out tool end to end on a shortened cfg 2: per-method table, and the sweep of Eq. 4's
    constant a (Section V-B) run as one batch of simulations."""
    from paper_2301_08895_amd import compare
    assert compare.main(["--config", "2", "--M", "6000", "--methods", "abs,adasync", "--rounds", "60", "--every", "30",
                         "--eval-rows", "512", "--target", "5.0"]) == 0
    out = capsys.readouterr().out
    assert "adasync" in out and "first read-out with held-out loss" in out
    assert compare.main(["--config", "2", "--M", "6000", "--sweep-a", "0,-2", "--seeds", "3", "--rounds", "60",
                         "--every", "30", "--eval-rows", "512", "--target", "5.0"]) == 0
    out = capsys.readouterr().out
    assert "means over 3 seeds" in out and "a =  -2: 3/3 seeds" in out
    # a smaller a means a tighter staleness bound, hence at least as many restarts (same seeds, same times)
    rows = compare.sweep_a(dict(workloads.preset(2), M=6000), [0, -3], 2, 60, 60, 256, None)
    r0 = sum(r["restarts"] for r in rows if r["a"] == 0)
    r3 = sum(r["restarts"] for r in rows if r["a"] == -3)
    assert r3 >= r0
    # the sweep of an MLP workload runs its simulations side by side (a batch of MLP handles)
    pm = workloads.scaled_preset(3, M=4096, dims=[256, 128, 10], N=6, B=32, n_slow=1, K0=2, tau_cap=3)
    rows = compare.sweep_a(pm, [0, -1], 2, 12, 12, 256, None)
    assert len(rows) == 4 and all(np.isfinite(r["eval_loss"]) for r in rows)
