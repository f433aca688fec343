"""GPU parity of local SGD (U > 1 steps of Eq. 2 per job, uploads w^{t,0} - w^{t,U}) against
the CPU oracle, through the C-ABI."""
import numpy as np
import pytest

import workloads
from parity_util import run_pair, assert_trace_equal, check_models

pytestmark = pytest.mark.gpu


def _check(res, tol, loss_rtol):
    assert_trace_equal(res, loss_rtol)
    check_models(res, tol)


@pytest.mark.parametrize("over,T", [
    (dict(U=10), 120),                                                      # cfg 1 with the paper's U = 10
    (dict(U=3, dims=[37, 1], M=999, N=5, B=7, K0=2, tau_cap=2), 100),       # ragged sizes
    (dict(U=2, dims=[512, 1], M=4000, N=3, B=1, K0=1, sa_penalty=1, lr=1e-3), 40),
    (dict(U=4, N=128, B=8, M=12800, tau_cap=8, time_dist=1, time_param=1.5), 60),
])
def test_linear_local_steps(over, T):
    p = workloads.scaled_preset(1, **over)
    _check(run_pair(p, T, checkpoints=(1, 5)), 1e-5, 1e-4)


@pytest.mark.parametrize("over,T", [
    (dict(U=10, M=6000), 100),                                               # cfg 2 shape, U = 10
    (dict(U=3, M=4000, dims=[52, 3], n_classes=3, N=6, B=10, K0=2, tau_cap=2, lr=5e-3), 100),
    (dict(U=2, M=4000, dims=[1024, 16], n_classes=16, N=4, B=300, lr=2e-4), 20),    # two row batches
    (dict(U=5, M=2000, dims=[8, 2], n_classes=2, N=16, B=5, sa_penalty=1, lr=2e-2), 80),
    (dict(U=9, M=4000, dims=[16, 4], n_classes=4, N=3, B=250, lr=5e-3), 12),     # U B > 2048: the wavefront-per-row kernel
    (dict(U=2, M=6000, dims=[784, 10], N=4, B=1000, K0=2, lr=1e-3), 6),           # 2000 rows per job
    (dict(U=2, M=3000, dims=[1000, 4], n_classes=4, N=4, B=21, lr=2e-4), 10),     # model in LDS, 8-row tiles
    (dict(U=3, M=3000, dims=[256, 16], n_classes=16, N=5, B=19, lr=1e-3), 12),    # all 16 class columns in use
])
def test_softmax_local_steps(over, T):
    p = workloads.scaled_preset(2, **over)
    _check(run_pair(p, T, checkpoints=(1, 5)), 1e-5, 1e-4)


@pytest.mark.parametrize("over,T", [
    # two layers, ragged B and d_0, every upload's private copy in use from step 1 on
    (dict(U=3, M=4096, dims=[200, 96, 10], N=8, B=40, n_slow=2, lr=1e-3), 30),
    # three layers on the 256 x 256 tile kernel, uploads of two row tiles
    (dict(U=2, M=8192, dims=[256, 256, 512, 10], N=6, B=256, K0=2, n_slow=1, lr=5e-4), 12),
    # staleness-aware step, restarts, narrow layers, 3 classes
    (dict(U=4, M=4096, dims=[128, 64, 3], n_classes=3, N=16, B=16, n_slow=4, sa_penalty=1,
          tau_mode=1, tau_cap=1, lr=2e-3), 40),
    # 100 classes (128-wide logits), B = one tile
    (dict(U=2, M=8192, dims=[256, 128, 256, 100], n_classes=100, N=8, B=128, n_slow=0, lr=5e-4), 12),
])
def test_mlp_local_steps(over, T):
    p = workloads.scaled_preset(3, **over)
    _check(run_pair(p, T, checkpoints=(1, 5)), 2e-2, 2e-3)       # the bf16 workloads' tolerance


def test_cfg3_shape_local_steps():
    """The 3072-512-10 workload at its real layer and batch shapes (shorter dataset) with U = 2."""
    p = workloads.scaled_preset(3, M=6400, U=2)
    _check(run_pair(p, 8, checkpoints=(1,)), 2e-2, 2e-3)


def test_local_sgd_equals_the_hand_worked_run():
    """The HIP path against tests/golden/local_sgd_hand_worked.txt (two local steps per job, exact in fp32)."""
    import paper_2301_08895_amd as lib
    from parity_util import local_sgd_hand_worked
    p, d, models, losses = local_sgd_hand_worked()
    sim = lib.Simulation(p, d)
    for t in range(2):
        sim.round(1)
        assert np.array_equal(sim.model().astype(np.float64), models[t + 1]), (t, sim.model())
    tr = sim.trace()
    sim.close()
    for t, l in losses.items():
        assert np.int32(tr[t][10]).view(np.float32) == np.float32(l)
