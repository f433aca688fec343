"""abs_evaluate_static (the evaluation for callers that cannot allocate: its scratch is a fixed array
inside the library, its result stays on the device) against abs_evaluate, through the C-ABI: the same
kernels in the same order, so the two doubles must be equal bit for bit; two calls in a row, the second
on fewer rows, so that what the first call left in the shared scratch would show."""
import numpy as np
import pytest
import torch

import workloads
import paper_2301_08895_amd as lib

pytestmark = pytest.mark.gpu


def _same(a, b):
    return a == b or (np.isnan(a) and np.isnan(b))


def _both(sim, Xe, ye, n_rows, version=-1):
    dev = sim.d_X.device
    xt = torch.from_numpy(Xe.view(np.int16) if Xe.dtype == np.uint16 else Xe).to(dev)
    yt = torch.from_numpy(ye).to(dev)
    out = torch.full((2,), -1.0, dtype=torch.float64, device=dev)
    want = lib.abs_evaluate(sim.handle, version, xt.data_ptr(), yt.data_ptr(), n_rows)
    lib.abs_evaluate_static(sim.handle, version, xt.data_ptr(), yt.data_ptr(), n_rows, out.data_ptr())
    torch.cuda.synchronize(dev)
    got = out.cpu().numpy()
    assert _same(got[0], want[0]) and _same(got[1], want[1]), (n_rows, got, want)
    return want


@pytest.mark.parametrize("p,T,rows", [
    (workloads.scaled_preset(2, M=6000), 40, (40_003, 1_001)),            # three passes of 16384 rows, then one
    (workloads.scaled_preset(1, M=4000), 30, (5_001, 77)),                 # linear model: accuracy is NaN
    (workloads.scaled_preset(3, M=4096, dims=[200, 96, 10], N=8, B=40, n_slow=2, lr=1e-3), 12, (1_500, 333)),
    # the convolutional model: passes of N B = 48 rows
    (workloads.scaled_preset(6, M=1500, dims=[2 * 14 * 14, 4, 5, 24, 12, 4, 2, 3], n_classes=4, N=6, B=8, K0=2,
                             tau_cap=2, lr=3e-3), 10, (500, 77)),
])
def test_static_evaluation_equals_abs_evaluate(p, T, rows):
    d, Xe, ye = workloads.make_split(p, max(rows))
    sim = lib.Simulation(p, d)
    sim.round(T)
    first = _both(sim, Xe, ye, rows[0])
    second = _both(sim, Xe, ye, rows[1])                  # smaller input right after the larger one
    assert first[0] != second[0]
    _both(sim, Xe, ye, rows[1], version=T - 1)            # an older version still in the ring
    # a second handle on the same GPU shares the scratch: calls one after the other stay exact
    other = lib.Simulation(dict(p, seed_sim=p["seed_sim"] + 1), d)
    other.round(3)
    _both(other, Xe, ye, rows[1])
    _both(sim, Xe, ye, rows[0])
    # the simulation is not disturbed
    before = sim.model().copy()
    sim.round(2)
    ref = lib.Simulation(p, d)
    ref.round(T + 2)
    assert np.array_equal(ref.model(), sim.model()) and not np.array_equal(before, sim.model())
    for s in (sim, other, ref):
        s.close()


def test_static_evaluation_rejects_what_does_not_fit():
    # 128 workers x 640 rows = 81920 rows per pass, more than the fixed scratch holds
    p = workloads.scaled_preset(3, M=128 * 700, dims=[64, 64, 4], n_classes=4, N=128, B=640, n_slow=0)
    d, Xe, ye = workloads.make_split(p, 256)
    sim = lib.Simulation(p, d)
    dev = sim.d_X.device
    xt = torch.from_numpy(Xe.view(np.int16)).to(dev)
    yt = torch.from_numpy(ye).to(dev)
    out = torch.zeros(2, dtype=torch.float64, device=dev)
    with pytest.raises(lib.AbsError) as e:
        lib.abs_evaluate_static(sim.handle, -1, xt.data_ptr(), yt.data_ptr(), 256, out.data_ptr())
    assert e.value.code == -2 and "ABS_STATIC_EVAL_ROWS" in str(e.value)
    lib.abs_evaluate(sim.handle, -1, xt.data_ptr(), yt.data_ptr(), 256)      # the allocating form still works
    with pytest.raises(lib.AbsError):
        lib.abs_evaluate_static(sim.handle, 5, xt.data_ptr(), yt.data_ptr(), 256, out.data_ptr())   # version not in the ring
    sim.close()
