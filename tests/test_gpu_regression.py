"""GPU parity of the two regression workloads against the CPU oracle (through the C-ABI)."""
import numpy as np
import pytest

import workloads
from parity_util import run_pair, assert_trace_equal, check_models

pytestmark = pytest.mark.gpu

FP32_TOL = 1e-5     # relative, stated for the fp32 workloads


@pytest.mark.parametrize("over,T", [
    (dict(), 200),                                              # the workload as specified
    (dict(dims=[100, 1], N=8, B=32, seed_sim=4001), 200),       # second simulation seed
    (dict(dims=[37, 1], M=999, N=5, B=7, K0=2, tau_cap=2), 150),   # ragged: odd d, B, shard remainder
    (dict(dims=[300, 1], M=5000, N=16, B=40, tau_cap=1, tau_mode=1), 100),
    (dict(dims=[512, 1], M=4000, N=3, B=1, K0=1, sa_penalty=1, lr=1e-3), 60),      # B = 1, SA step
    (dict(N=128, B=8, M=12800, tau_cap=8, time_dist=1, time_param=1.5), 120),      # N at its maximum
    (dict(N=1, K0=1, M=500, B=16), 50),                          # a single worker
])
def test_linear_least_squares(over, T):
    p = workloads.scaled_preset(1, **over)
    res = run_pair(p, T, checkpoints=(1, 10))
    assert_trace_equal(res, 1e-4)
    check_models(res, FP32_TOL)


@pytest.mark.parametrize("over,T", [
    (dict(M=6000), 300),                                          # real shape, shorter dataset
    (dict(M=4000, dims=[52, 3], n_classes=3, N=6, B=10, K0=2, tau_cap=2, lr=5e-3), 200),
    (dict(M=4000, dims=[1024, 16], n_classes=16, N=4, B=33, lr=2e-4), 60),
    (dict(M=2000, dims=[8, 2], n_classes=2, N=16, B=5, sa_penalty=1, lr=2e-2), 150),
])
def test_softmax_regression(over, T):
    p = workloads.scaled_preset(2, **over)
    res = run_pair(p, T, checkpoints=(1, 10))
    assert_trace_equal(res, 1e-4)
    check_models(res, FP32_TOL)


def test_softmax_full_workload():
    p = workloads.preset(2)
    res = run_pair(p, p["T"])
    assert_trace_equal(res, 1e-4)
    check_models(res, FP32_TOL)
    assert res["got"][-1, 1] == p["N"]          # K has grown to N


def test_run_to_run_bitwise_determinism():
    import paper_2301_08895_amd as lib
    p = workloads.scaled_preset(2, M=6000)
    d = workloads.make_inputs(p)
    outs = []
    for _ in range(2):
        sim = lib.Simulation(p, d)
        sim.round(150)
        outs.append((sim.model().copy(), sim.trace().copy()))
        sim.close()
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])


def test_get_model_versions_and_errors():
    import paper_2301_08895_amd as lib
    p = workloads.preset(1)
    d = workloads.make_inputs(p)
    sim = lib.Simulation(p, d)
    assert np.array_equal(sim.model(0), d["w0"])
    sim.round(10)
    R = p["tau_cap"] + 3
    assert np.array_equal(sim.model(-1), sim.model(10))
    sim.model(10 - R + 1)
    with pytest.raises(lib.AbsError) as e:
        sim.model(10 - R)
    assert e.value.code == -4
    with pytest.raises(lib.AbsError):
        sim.model(11)
    sim.close()


@pytest.mark.parametrize("sa", [0, 1])
def test_linear_round_equals_the_hand_worked_updates(sa):
    """The HIP path against values worked out by hand (tests/golden/abs_hand_worked_updates.txt): three
    rounds on three rows, one gradient taken at a model two rounds old, plain and staleness-aware
    step.  Every intermediate is a dyadic fraction, so fp32 reproduces the models exactly."""
    import paper_2301_08895_amd as lib
    from parity_util import hand_worked_updates
    p, d, models, losses = hand_worked_updates(sa)
    sim = lib.Simulation(p, d)
    for t in range(3):
        sim.round(1)
        assert np.array_equal(sim.model().astype(np.float64), models[t + 1]), (t, sim.model(), models[t + 1])
    tr = sim.trace()
    sim.close()
    assert [list(r[12:14]) for r in tr] == [[1, 2], [1, 2], [0, 1]] and list(tr[2][16:18]) == [2, 0]
    for t, l in losses.items():
        assert np.int32(tr[t][10]).view(np.float32) == np.float32(l)


def test_softmax_first_round_equals_the_hand_worked_values():
    """The HIP path (unbatched and batched kernels) against tests/golden/softmax_hand_worked_first_round.txt."""
    import paper_2301_08895_amd as lib
    from parity_util import softmax_hand_worked_first_round
    p, d, w1 = softmax_hand_worked_first_round()
    sim = lib.Simulation(p, d)
    sim.round(1)
    assert np.allclose(sim.model(), w1, rtol=0, atol=1e-7)
    assert abs(float(np.int32(sim.trace()[0][10]).view(np.float32)) - np.log(4.0)) < 1e-6
    sim.close()
    sim = lib.Simulation(p, d)
    batch = lib.Batch([sim])
    batch.round(1)
    batch.close()
    assert np.allclose(sim.model(), w1, rtol=0, atol=1e-7)
    sim.close()
