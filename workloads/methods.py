"""The paper's method and the systems it is compared with, as settings of one configuration.

All of them are the same server loop (Algorithm 1) with different rules for the wait count K^t,
the staleness threshold and the local steps, so each is a set of flags on a preset:

  abs            adaptive K^t (Eq. 5) and adaptive threshold tau_max^t = N/K^t + a (Eq. 4, 6)
  abs_fixed_tau  adaptive K^t, constant threshold tau_cap (the fixed-threshold runs of Section III)
  adasync        adaptive K^t, no threshold (Section V-A: ABS with a very large `a` behaves like it)
  sa_adasync     adasync with the staleness-aware step eta / tau (Section I; Section V-A)
  k_async        constant K = K0, no threshold (K-async SGD, Section I)
  asgd           K = 1, no threshold (fully asynchronous SGD)
  sync_sgd       K = N: every round waits for everybody, no staleness (synchronous SGD)
  local_sgd      K = N with U local steps (synchronous local SGD, Section II-B / V-A)

`sa_abs` (ABS with the staleness-aware step) is the combination workload 4 asks for.
"""
from __future__ import annotations

import copy

from .presets import K_ADAPTIVE, K_FIXED, TAU_ADAPTIVE, TAU_FIXED, TAU_INF

METHODS = ("abs", "sa_abs", "abs_fixed_tau", "adasync", "sa_adasync", "k_async", "asgd", "sync_sgd", "local_sgd")


def method_preset(p: dict, name: str, **over) -> dict:
    """Preset p run as `name`; `over` replaces fields afterwards (e.g. a=..., U=..., K0=...)."""
    q = copy.deepcopy(p)
    if name == "abs":
        q.update(k_mode=K_ADAPTIVE, tau_mode=TAU_ADAPTIVE, sa_penalty=0)
    elif name == "sa_abs":
        q.update(k_mode=K_ADAPTIVE, tau_mode=TAU_ADAPTIVE, sa_penalty=1)
    elif name == "abs_fixed_tau":
        q.update(k_mode=K_ADAPTIVE, tau_mode=TAU_FIXED, sa_penalty=0)
    elif name == "adasync":
        q.update(k_mode=K_ADAPTIVE, tau_mode=TAU_INF, sa_penalty=0)
    elif name == "sa_adasync":
        q.update(k_mode=K_ADAPTIVE, tau_mode=TAU_INF, sa_penalty=1)
    elif name == "k_async":
        q.update(k_mode=K_FIXED, tau_mode=TAU_INF, sa_penalty=0)
    elif name == "asgd":
        q.update(k_mode=K_FIXED, K0=1, tau_mode=TAU_INF, sa_penalty=0)
    elif name == "sync_sgd":
        q.update(k_mode=K_FIXED, K0=q["N"], tau_mode=TAU_INF, sa_penalty=0, U=1)
    elif name == "local_sgd":
        q.update(k_mode=K_FIXED, K0=q["N"], tau_mode=TAU_INF, sa_penalty=0, U=max(2, q.get("U", 1)))
    else:
        raise ValueError(f"unknown method {name!r}; one of {METHODS}")
    if q["tau_mode"] == TAU_INF:
        # without a threshold the staleness is unbounded in principle; tau_cap then only sizes the
        # device's ring of model versions (a selected worker staler than the ring is an error)
        q["tau_cap"] = min(1024, max(q["tau_cap"], 8 * q["N"]))
    q["method"] = name
    q.update(over)
    return q
