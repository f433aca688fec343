"""Oracle simulator of ABS (Algorithm 1 of the paper), U >= 1 local steps.

State kept by the parameter server (Section III): round t, wait count K,
the staleness vector tau (initialised to zero), plus what a simulation needs:
the model version each worker last received, its job counter, its finish
tick and the simulated clock.  Every past global model is kept (no ring).

One round, in the paper's order (server part of Algorithm 1):
  wait for the K^t fastest uploads  -> Eq. 3 update -> Eq. 5 wait-count update
  -> Eq. 6 staleness update with the threshold of Eq. 4 -> the K^t fastest and
  the over-stale workers receive w^{t+1} and start a new job.
A job that is cut short by a forced restart is never uploaded, so its gradient
is never formed.

With U > 1 (cfg key "U") a worker takes U local SGD steps of Eq. 2 on a private copy of the
model it received, each on a fresh minibatch, and uploads the accumulated change
w^{t,0} - w^{t,U} together with its average local loss (worker part of Algorithm 1); the
server averages the K^t uploads (Eq. 3).  At U = 1 this is the same update: the single
step's eta_k g_k.  (Algorithm 1 lists its local loop as u = 0..U, one more than Eq. 2's
u = 0..U-1; Eq. 2 is followed: exactly U steps.)

Readings taken where the paper is silent (each is repeated in the repository's
design notes): K^t is floor'ed and clamped to [1, N]; k_mode 0 keeps it
non-decreasing ("dynamically increase K^t", and the proof of Theorem 1 uses
K^0 <= K^t), k_mode 3 does not; the threshold of round t uses the K^t that the
round waited for (the index in Eq. 4), capped at tau_cap in tau_mode 0;
the loss of the global model is the mean of the K^t uploaded minibatch losses
and f(w^0) is that mean at t = 0; ties in finish time go to the lower worker
id; a restarted worker starts its new job at the round's completion time.
"""
from __future__ import annotations

import math

import numpy as np

from . import counter_rng as crng
from .bf16 import bits_to_f64
from .models import narrowed_weights, worker_update

K_ADAPTIVE, K_FIXED, K_REPLAY, K_ADAPTIVE_FREE = 0, 1, 2, 3
TAU_ADAPTIVE, TAU_FIXED, TAU_INF = 0, 1, 2
INT32_MAX = 2**31 - 1


def next_wait_count(K0: int, N: int, K_now: int, loss0: float, loss_t: float, k_mode: int) -> int:
    """Eq. 5: K = K0 * sqrt(f(w^0) / f(w^t)), floor'ed, evaluated without the square
    root as the largest j <= N with j^2 * f(w^t) <= K0^2 * f(w^0)."""
    if not math.isfinite(loss_t):
        raise FloatingPointError("non-finite loss")
    if k_mode == K_FIXED:
        return K0
    if loss_t <= 0.0:
        cand = N
    else:
        cand = 0
        rhs = float(K0 * K0) * loss0
        for j in range(1, N + 1):
            if float(j * j) * loss_t <= rhs:
                cand = j
    if k_mode == K_ADAPTIVE:
        cand = max(K_now, cand)
    return min(N, max(1, cand))


def over_stale(tau_n: int, K: int, N: int, a: int, tau_mode: int, tau_cap: int) -> bool:
    """tau_n > tau_max^t with tau_max^t = max{1, N/K^t + a} (Eq. 4), in exact integers;
    tau_mode 0 additionally caps the threshold at tau_cap, 1 fixes it at tau_cap,
    2 means no threshold."""
    if tau_mode == TAU_INF:
        return False
    if tau_mode == TAU_FIXED:
        return tau_n > tau_cap
    if tau_n > tau_cap:
        return True
    return tau_n > 1 and tau_n * K > N + a * K


def threshold_floor(K: int, N: int, a: int, tau_mode: int, tau_cap: int) -> int:
    """floor(tau_max^t) as recorded in the trace (INT32_MAX for 'no threshold')."""
    if tau_mode == TAU_INF:
        return INT32_MAX
    if tau_mode == TAU_FIXED:
        return tau_cap
    return min(tau_cap, max(1, (N + a * K) // K))


class AbsOracle:
    """cfg keys: model, dims, x_dtype, M, N, B, K0, k_mode, tau_mode, tau_cap, a, lr,
    sa_penalty, time_dist, time_param, n_slow, slow_factor, seed_sim, k_replay (opt)."""

    def __init__(self, cfg: dict, X, y, w0, emulate_bf16=None, keep_models=True, local_path=None):
        self.cfg = dict(cfg)
        self.N, self.B = cfg["N"], cfg["B"]
        self.U = int(cfg.get("U", 1))
        # U = 1 folds 1/K into the back-propagation seed (one rounding point fewer under bf16
        # emulation); local_path=True takes the general U-step route even for U = 1
        self.local_path = (self.U > 1) if local_path is None else local_path
        self.lr = float(np.float32(cfg["lr"]))   # the step size is handed over as fp32
        if cfg["x_dtype"] == 1:
            self.Xbits, self.X = np.asarray(X), None
        else:
            self.Xbits, self.X = None, np.asarray(X)
        self.y = np.asarray(y)
        self.emulate = (cfg["x_dtype"] == 1) if emulate_bf16 is None else emulate_bf16
        self.keep_models = keep_models
        # Algorithm 1, initialisation: w^0 is broadcast to all workers, tau = 0, K = K^0.
        self.t = 0
        self.K = cfg["K0"]
        self.loss0 = None
        self.now = 0
        self.tau = [0] * self.N
        self.ver = [0] * self.N
        self.job = [0] * self.N
        self.fin = [crng.compute_time_ticks(self.cfg, n, 0) for n in range(self.N)]
        self.models = {0: np.asarray(w0, dtype=np.float64).copy()}
        self._narrowed = {}     # version -> narrowed_weights(...), computed once per version
        self.comm_uploads = 0
        self.comm_restarts = 0
        self.trace = []

    def _rows(self, idx):
        if self.X is not None:
            return self.X[idx].astype(np.float64)
        return bits_to_f64(self.Xbits[idx])

    def round(self):
        cfg, N, B, t = self.cfg, self.N, self.B, self.t
        K = self.K
        if cfg["k_mode"] == K_REPLAY:
            K = int(cfg["k_replay"][t])
        # the K^t fastest uploads, in arrival order (Section II-A; Algorithm 1, server)
        order = sorted(range(N), key=lambda n: (self.fin[n], n))
        sel = order[:K]
        self.now = self.fin[sel[-1]]
        # Eq. 3 with U = 1: w^{t+1} = w^t - (1/K) sum_k eta_k g_k, g_k at the stale model
        w_next = self.models[t].copy()
        losses, vers, taus = [], [], []
        for k in sel:
            v = self.ver[k]
            tau_k = t - v
            assert tau_k == self.tau[k]
            idx = crng.batch_indices(cfg, k, self.job[k])
            eta_k = self.lr / max(1, tau_k) if cfg["sa_penalty"] else self.lr
            if not self.local_path:
                if v not in self._narrowed:
                    self._narrowed[v] = narrowed_weights(cfg, self.models[v], self.emulate)
                u_k, loss_k = worker_update(cfg, self.models[v], self._rows(idx), self.y[idx],
                                            eta_k / K, self.emulate, self._narrowed[v])
                w_next -= u_k
            else:
                # Eq. 2, U local steps on a private copy; the upload is w^{t,0} - w^{t,U}
                w_loc = self.models[v].copy()
                step_losses = []
                for u in range(self.U):
                    idx_u = crng.batch_indices(cfg, k, self.job[k], u)
                    step, loss_u = worker_update(cfg, w_loc, self._rows(idx_u), self.y[idx_u],
                                                 eta_k, self.emulate)
                    w_loc -= step
                    step_losses.append(loss_u)
                w_next -= (self.models[v] - w_loc) / K
                loss_k = sum(step_losses) / self.U
            losses.append(loss_k); vers.append(v); taus.append(tau_k)
        self.models[t + 1] = w_next
        # loss of the global model := mean of the uploaded minibatch losses (Section III)
        loss_t = sum(losses) / K
        if t == 0:
            self.loss0 = loss_t
        # Eq. 4 / Eq. 6: forced restarts among the workers that did not upload
        selset = set(sel)
        restart = [n for n in range(N) if n not in selset and
                   over_stale(self.tau[n], K, N, cfg["a"], cfg["tau_mode"], cfg["tau_cap"])]
        # Eq. 5
        if cfg["k_mode"] == K_REPLAY:
            rep = cfg["k_replay"]
            K_next = int(rep[t + 1]) if t + 1 < len(rep) else K
            if not math.isfinite(loss_t):
                raise FloatingPointError("non-finite loss")
        else:
            K_next = next_wait_count(cfg["K0"], N, K, self.loss0, loss_t, cfg["k_mode"])
        # receivers of w^{t+1}: ages to zero, new job; everybody else ages by one
        recv = selset | set(restart)
        for n in range(N):
            if n in recv:
                self.ver[n] = t + 1
                self.tau[n] = 0
                self.job[n] += 1
                self.fin[n] = self.now + crng.compute_time_ticks(cfg, n, self.job[n])
            else:
                self.tau[n] += 1
        self.comm_uploads += K
        self.comm_restarts += len(restart)
        rec = dict(t=t, K=K, tau_max=threshold_floor(K, N, cfg["a"], cfg["tau_mode"], cfg["tau_cap"]),
                   now=self.now, n_restart=len(restart), comm_uploads=self.comm_uploads,
                   comm_restarts=self.comm_restarts, loss=loss_t, K_next=K_next,
                   ids=list(sel), vers=vers, taus=taus, restart_ids=restart,
                   worker_losses=losses)
        self.trace.append(rec)
        if not self.keep_models:
            live = set(self.ver) | {t + 1}
            for v in [v for v in self.models if v not in live]:
                del self.models[v]
        for v in [v for v in self._narrowed if v not in set(self.ver)]:
            del self._narrowed[v]
        self.K = K_next
        self.t = t + 1
        return rec

    def run(self, T: int):
        for _ in range(T):
            self.round()
        return self

    def model(self, version: int = -1) -> np.ndarray:
        return self.models[self.t if version < 0 else version]


TRACE_HEADER_WORDS = 12


def trace_stride(N: int) -> int:
    return TRACE_HEADER_WORDS + 3 * N


def trace_words(rec: dict, N: int) -> np.ndarray:
    """One round's record in the library's int32 word layout:
    [t, K, floor(tau_max), now lo, now hi, n_restart, uploads lo, hi, restarts lo, hi,
     loss as fp32 bits, K_next, ids[K], vers[K], taus[K], restart_ids[...], -1 fill]."""
    w = np.full(trace_stride(N), -1, dtype=np.int64)
    lo = lambda v: v & 0xFFFFFFFF
    hi = lambda v: (v >> 32) & 0xFFFFFFFF
    w[0:12] = [rec["t"], rec["K"], rec["tau_max"], lo(rec["now"]), hi(rec["now"]),
               rec["n_restart"], lo(rec["comm_uploads"]), hi(rec["comm_uploads"]),
               lo(rec["comm_restarts"]), hi(rec["comm_restarts"]),
               int(np.float32(rec["loss"]).view(np.uint32)), rec["K_next"]]
    K = rec["K"]
    o = 12
    w[o:o + K] = rec["ids"]; o += K
    w[o:o + K] = rec["vers"]; o += K
    w[o:o + K] = rec["taus"]; o += K
    w[o:o + rec["n_restart"]] = rec["restart_ids"]
    return (w & 0xFFFFFFFF).astype(np.uint32).view(np.int32)
