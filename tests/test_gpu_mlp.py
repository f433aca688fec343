"""GPU parity of the MLP workloads (bf16 operands, fp32 accumulation) against the CPU
oracle with its bf16 rounding points switched on, through the C-ABI."""
import numpy as np
import pytest

import workloads
from parity_util import run_pair, assert_trace_equal, check_models

pytestmark = pytest.mark.gpu

BF16_TOL = 2e-2     # relative, stated for the bf16-input workloads
BF16_GUARD = 5e-3   # per-tensor norms; measured at most 1.2e-3 (K = 4 at the largest shape), typically 1e-5 .. 3e-4


def _check(res, tol=BF16_TOL):
    assert_trace_equal(res, 2e-3)
    # every W_l and b_l separately, element by element, weights and updates (w^T - w^0)
    check_models(res, tol, guard=BF16_GUARD)


@pytest.mark.parametrize("over,T", [
    # two layers, several row tiles per upload boundary, ragged B, d_0 not a tile multiple
    (dict(M=4096, dims=[200, 96, 10], N=8, B=40, n_slow=2, lr=1e-3), 40),
    # three layers, B = one tile, hidden = one and two tiles, 100 classes (128-wide logits)
    (dict(M=8192, dims=[256, 128, 256, 100], n_classes=100, N=8, B=128, n_slow=0, lr=5e-4), 30),
    # staleness-aware step, fixed threshold, many restarts
    (dict(M=4096, dims=[128, 64, 3], n_classes=3, N=16, B=16, n_slow=4, sa_penalty=1,
          tau_mode=1, tau_cap=1, lr=2e-3), 60),
    # everything a multiple of 256: all products take the 256 x 256 tile kernel
    (dict(M=8192, dims=[256, 256, 512, 10], N=6, B=256, K0=2, n_slow=1, lr=5e-4), 20),
    # mixed: 256-row uploads but a 128-wide hidden layer (both GEMM kernels in one round)
    (dict(M=8192, dims=[320, 128, 256, 10], N=4, B=256, n_slow=0, lr=5e-4), 15),
    # B > one tile (two row tiles per upload), Pareto times
    (dict(M=8192, dims=[384, 128, 10], N=4, B=200, n_slow=0, time_dist=1, time_param=1.5, lr=1e-3), 25),
])
def test_mlp_small(over, T):
    p = workloads.scaled_preset(3, **over)
    _check(run_pair(p, T, checkpoints=(1, 5)))


def test_cfg3_shape_prefix():
    """The 3072-512-10 workload at its real layer and batch shapes (shorter dataset), first rounds."""
    p = workloads.scaled_preset(3, M=6400)
    _check(run_pair(p, 12, checkpoints=(1,)))


def test_run_to_run_bitwise_determinism():
    import paper_2301_08895_amd as lib
    p = workloads.scaled_preset(3, M=4096, dims=[256, 128, 10], N=8, B=64, n_slow=2, lr=1e-3)
    d = workloads.make_inputs(p)
    outs = []
    for _ in range(2):
        sim = lib.Simulation(p, d)
        sim.round(30)
        outs.append((sim.model().copy(), sim.trace().copy()))
        sim.close()
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])


def test_mlp_first_round_equals_the_hand_worked_values():
    """The HIP path against tests/golden/mlp_hand_worked_first_round.txt (ReLU forward, H^T dZ, update,
    an untouched hidden layer; every value survives the bf16 narrowing exactly)."""
    import paper_2301_08895_amd as lib
    from parity_util import mlp_hand_worked_first_round
    p, d, w1 = mlp_hand_worked_first_round()
    sim = lib.Simulation(p, d)
    sim.round(1)
    got = sim.model()
    loss = float(np.int32(sim.trace()[0][10]).view(np.float32))
    sim.close()
    assert np.allclose(got, w1, rtol=0, atol=1e-7), (got, w1)
    assert abs(loss - np.log(4.0)) < 1e-6


def test_sampled_kernel_timing_changes_nothing():
    """profile = n brackets the kernels of every n-th round only: same results bit for bit, and the
    statistics say which launches the measured time covers."""
    import paper_2301_08895_amd as lib
    p = workloads.scaled_preset(3, M=2048, dims=[128, 64, 10], N=4, B=32, n_slow=1)
    d = workloads.make_inputs(p)
    runs = {}
    for prof in (0, 1, 4):
        sim = lib.Simulation(p, d, profile=prof)
        sim.round(21)
        runs[prof] = (sim.model().copy(), sim.trace().copy(), sim.kernel_stats())
        sim.close()
    for prof in (1, 4):
        assert np.array_equal(runs[prof][0], runs[0][0]) and np.array_equal(runs[prof][1], runs[0][1])
    for s0, s1, s4 in zip(*(runs[k][2] for k in (0, 1, 4))):
        assert s0["launches"] == s1["launches"] == s4["launches"] and s0["timed_launches"] == 0 and s0["total_ms"] == 0
        assert s1["timed_launches"] == s1["launches"] and s1["timed_flops"] == s1["flops"] and s1["total_ms"] > 0
        per_round = s4["launches"] // 21
        assert s4["timed_launches"] == 6 * per_round and s4["total_ms"] > 0      # rounds 0, 4, ..., 20
