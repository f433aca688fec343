"""Host-side checks of libabs that need no GPU: the library loads and exports every
symbol include/abs.h declares, the config mirror matches, and the host scheduler
(schedule-only mode) reproduces the oracle's integer event trace bit for bit."""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads
import paper_2301_08895_amd as lib
from oracle import counter_rng as crng
from oracle.abs_sim import AbsOracle, trace_words
from parity_util import hand_worked_schedule

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "abs.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(abs_[a-z_]+)\s*\(", header))
    assert {"abs_create", "abs_round", "abs_get_model", "abs_trace", "abs_destroy"} <= names
    dll = ctypes.CDLL(lib.library_path())
    for n in sorted(names):
        assert hasattr(dll, n), n
    assert lib.abs_config_bytes() == ctypes.sizeof(lib.AbsConfig) == 152


def _dry_vs_oracle(p, T):
    d = workloads.make_inputs(p)
    o = AbsOracle(p, d["X"], d["y"], d["w0"], keep_models=False).run(T)
    Ks = [r["K"] for r in o.trace]
    q = dict(p, k_mode=2)
    sim = lib.Simulation(q, None, device_mode=0, k_replay=Ks)
    sim.round(T)
    got = sim.trace()
    sim.close()
    want = np.stack([trace_words(r, p["N"]) for r in o.trace])
    keep = np.ones(got.shape[1], bool)
    keep[10] = False          # the loss word: there are no losses without a device
    keep[11] = False          # K^{t+1}: in replay mode the last record repeats K
    assert np.array_equal(got[:, keep], want[:, keep])
    assert np.array_equal(got[:-1, 11], want[:-1, 11])
    return o


@pytest.mark.parametrize("i,over,T", [
    (1, dict(), 200),
    (2, dict(M=3200, dims=[16, 10]), 300),
    (3, dict(M=3200, dims=[16, 8, 10], lr=2e-3), 120),                     # slow subset
    (4, dict(M=6400, dims=[16, 8, 8, 10], lr=2e-3), 80),                   # staleness-aware step
    (5, dict(M=12800, dims=[16, 8, 8, 100], n_classes=100, lr=2e-3), 60),  # Pareto times, N = 128
    (1, dict(tau_mode=1, tau_cap=1), 150),
    (1, dict(tau_mode=2, tau_cap=40, k_mode=1, K0=1), 150),
    (1, dict(k_mode=3), 150),
])
def test_scheduler_trace_equals_oracle(i, over, T):
    p = workloads.scaled_preset(i, **over)
    o = _dry_vs_oracle(p, T)
    if over.get("tau_mode", 0) != 2:
        assert sum(r["n_restart"] for r in o.trace) > 0


def test_scheduler_equals_the_hand_worked_run():
    """The C++ scheduler against tests/golden/abs_hand_worked_schedule.txt (pencil-and-paper run of
    Algorithm 1: ties, a gradient of staleness tau_max + 1, a restart by Eq. 6)."""
    setting, want = hand_worked_schedule()
    p = workloads.scaled_preset(1, M=400, B=8, dims=[12, 1], **setting)
    sim = lib.Simulation(p, None, device_mode=0)
    sim.round(len(want))
    got = sim.trace()
    sim.close()
    for row, w in zip(got, want):
        K = w["K"]
        assert [int(row[0]), int(row[1]), int(row[2])] == [w["t"], K, w["tau_max"]]
        assert (int(row[3]) & 0xFFFFFFFF) | (int(row[4]) << 32) == w["now"]
        assert int(row[5]) == len(w["restart_ids"]) and int(row[6]) == w["comm_uploads"] and int(row[8]) == w["comm_restarts"]
        assert list(row[12:12 + K]) == w["ids"] and list(row[12 + K:12 + 2 * K]) == w["vers"]
        assert list(row[12 + 2 * K:12 + 3 * K]) == w["taus"]
        assert list(row[12 + 3 * K:12 + 3 * K + len(w["restart_ids"])]) == w["restart_ids"]


def test_draws_equal_oracle():
    for i in (1, 3, 5):
        p = workloads.scaled_preset(i, M=12800)
        cfg = lib.make_config(p)
        for n in (0, 1, p["N"] - 1):
            for j in (0, 1, 7, 1000):
                assert lib.abs_draw_time_ticks(cfg, n, j) == crng.compute_time_ticks(p, n, j)
                assert list(lib.abs_draw_batch_rows(cfg, n, j)) == crng.batch_indices(p, n, j)


def test_argument_errors():
    p = workloads.preset(1)
    with pytest.raises(lib.AbsError) as e:
        lib.Simulation(p, None, device_mode=0)              # adaptive K has no losses to use
    assert e.value.code == -1
    for bad in (dict(N=0), dict(N=129), dict(K0=9), dict(dims=[100, 2]), dict(lr=-1.0), dict(tau_cap=-1),
                dict(M=4)):
        q = dict(p, k_mode=1, **bad)
        with pytest.raises(lib.AbsError):
            lib.Simulation(q, None, device_mode=0)
    # replay array exhausted -> ABS_E_REPLAY, earlier rounds stay readable
    q = dict(p, k_mode=2)
    sim = lib.Simulation(q, None, device_mode=0, k_replay=[2, 3, 3])
    with pytest.raises(lib.AbsError) as e:
        sim.round(5)
    assert e.value.code == -6 and lib.abs_rounds_done(sim.handle) == 3
    assert sim.trace().shape == (3, lib.trace_stride(8))
    with pytest.raises(lib.AbsError):
        lib.abs_trace(sim.handle, 0, 4, 8)
    sim.close()
    # a worker staler than the ring allows is refused (tau_mode 2 with a small tau_cap)
    q = dict(p, k_mode=1, K0=1, tau_mode=2, tau_cap=0)
    sim = lib.Simulation(q, None, device_mode=0)
    with pytest.raises(lib.AbsError) as e:
        sim.round(200)
    assert e.value.code == -4
    sim.close()


def test_batch_and_evaluate_argument_errors_without_a_gpu():
    """Schedule-only handles have no model: they can be neither evaluated nor batched."""
    p = dict(workloads.preset(1), k_mode=1)
    a = lib.Simulation(p, None, device_mode=0)
    b = lib.Simulation(dict(p, seed_sim=7), None, device_mode=0)
    with pytest.raises(lib.AbsError) as e:
        lib.abs_evaluate(a.handle, -1, None, None, 10)
    assert e.value.code == -1
    with pytest.raises(lib.AbsError) as e:
        lib.abs_batch_create([a.handle, b.handle])
    assert e.value.code == -1 and "schedule-only" in str(e.value)
    with pytest.raises(lib.AbsError):
        lib.abs_batch_create([])
    assert lib.abs_batch_workspace_size([a.handle, b.handle]) == 0     # no batch, no size
    a.close(); b.close()
