"""The comparison systems as settings of the oracle: what defines each of them must show in its trace."""
import numpy as np
import pytest

import workloads
from oracle.abs_sim import AbsOracle


def _run(p, T):
    d = workloads.make_inputs(p)
    return AbsOracle(p, d["X"], d["y"], d["w0"], keep_models=False).run(T)


BASE = workloads.scaled_preset(2, M=3000, dims=[16, 4], n_classes=4, N=12, B=8, K0=3, lr=5e-2, n_slow=3, slow_factor=5.0)


def test_sync_sgd_waits_for_everybody_with_no_staleness():
    o = _run(workloads.method_preset(BASE, "sync_sgd"), 40)
    for r in o.trace:
        assert r["K"] == 12 and r["n_restart"] == 0 and all(t == 0 for t in r["taus"])
    # one round lasts as long as the slowest worker: time per round exceeds the K-async one
    a = _run(workloads.method_preset(BASE, "k_async"), 40)
    assert o.trace[-1]["now"] > a.trace[-1]["now"]


def test_asgd_and_k_async_keep_k_constant_and_never_restart():
    o = _run(workloads.method_preset(BASE, "asgd"), 80)
    assert all(r["K"] == 1 and r["n_restart"] == 0 for r in o.trace)
    assert max(max(r["taus"]) for r in o.trace) > 3          # staleness is unbounded
    o = _run(workloads.method_preset(BASE, "k_async"), 80)
    assert all(r["K"] == 3 and r["n_restart"] == 0 for r in o.trace)


def test_adasync_grows_k_and_never_restarts_abs_does_restart():
    ada = _run(workloads.method_preset(BASE, "adasync"), 150)
    Ks = [r["K"] for r in ada.trace]
    assert all(b >= a for a, b in zip(Ks, Ks[1:])) and Ks[-1] > Ks[0]
    assert all(r["n_restart"] == 0 for r in ada.trace)
    ab = _run(workloads.method_preset(BASE, "abs", tau_cap=2, a=2 - 12 // 3), 150)
    assert sum(r["n_restart"] for r in ab.trace) > 0
    assert max(max(r["taus"]) for r in ab.trace) <= 3        # threshold + the round it is tested in


def test_abs_with_a_huge_constant_is_adasync():
    """Eq. 4 with a very large `a` never forces a restart: the two runs coincide (Section V-A)."""
    ada = _run(workloads.method_preset(BASE, "adasync"), 120)
    big = _run(workloads.method_preset(BASE, "abs", a=10 ** 6, tau_cap=10 ** 6), 120)
    for ra, rb in zip(ada.trace, big.trace):
        assert (ra["K"], ra["now"], list(ra["ids"]), list(ra["taus"]), ra["n_restart"]) == \
               (rb["K"], rb["now"], list(rb["ids"]), list(rb["taus"]), rb["n_restart"])
        assert ra["loss"] == rb["loss"]
    assert np.array_equal(ada.model(), big.model())


def test_staleness_aware_step_only_changes_stale_uploads():
    plain = _run(workloads.method_preset(BASE, "adasync"), 1)
    sa = _run(workloads.method_preset(BASE, "sa_adasync"), 1)
    assert np.array_equal(plain.model(), sa.model())        # round 0: every upload has staleness 0
    plain.run(30); sa.run(30)
    assert not np.array_equal(plain.model(), sa.model())


def test_local_sgd_is_synchronous_with_u_steps():
    o = _run(workloads.method_preset(BASE, "local_sgd", U=4), 20)
    assert o.U == 4 and all(r["K"] == 12 and all(t == 0 for t in r["taus"]) for r in o.trace)


def test_unknown_method():
    with pytest.raises(ValueError):
        workloads.method_preset(BASE, "nope")
