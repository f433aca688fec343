"""Per-worker minibatch loss and gradient (oracle side).

The paper only asks for a smooth per-sample loss f(w; xi) (Eq. 1) and uses
the minibatch gradient g = (1/B) sum_b grad f(w; xi_b) (Eq. 2, Assumption 3).
The first three models are the synthetic workloads' own, the fourth is Section V-A's:
  linear   f = 1/2 (x.w - y)^2                       (no bias)
  softmax  f = -log softmax(x W + b)_y
  mlp      H_0 = x, Z_l = H_{l-1} W_l + b_l, H_l = relu(Z_l) (l < L),
           softmax cross-entropy on Z_L, relu'(0) = 0.
  cnn      two convolutional + three dense layers (cnn.py).
Parameter vector layout: per layer W_l [d_in, d_out] row-major then b_l.

`worker_update` returns s * g and the minibatch mean loss, where s is the
scalar eta_k / K that multiplies g in Eq. 3: by linearity s * g is the
gradient of s * (mean loss), so s is used as the seed of back-propagation.
With bf16 emulation on, the rounding points are: every weight matrix is
narrowed to bf16 for the forward and input-gradient products (biases stay
wide), hidden activations are narrowed after the ReLU, and every layer's
output gradient dZ_l (seed included) is narrowed before it is used; all
sums are wide.
"""
from __future__ import annotations

import numpy as np

from .bf16 import round_bf16

from . import cnn as _cnn

MODEL_LINEAR, MODEL_SOFTMAX, MODEL_MLP = 0, 1, 2
MODEL_CNN = _cnn.MODEL_CNN      # Section V-A's convolutional network: cnn.py


def unpack(cfg: dict, w: np.ndarray):
    """Flat parameter vector -> list of (W_l, b_l) views; b_l is None for the linear model."""
    d = cfg["dims"]
    if cfg["model"] == MODEL_LINEAR:
        return [(w.reshape(d[0], 1), None)]
    if cfg["model"] == MODEL_CNN:
        return _cnn.unpack(cfg, w)
    out, o = [], 0
    for l in range(len(d) - 1):
        W = w[o:o + d[l] * d[l + 1]].reshape(d[l], d[l + 1]); o += d[l] * d[l + 1]
        b = w[o:o + d[l + 1]]; o += d[l + 1]
        out.append((W, b))
    assert o == w.size
    return out


def _softmax_ce(Z: np.ndarray, y: np.ndarray):
    """Per-row loss and softmax probabilities, log-sum-exp with the max subtracted."""
    zmax = Z.max(axis=1, keepdims=True)
    E = np.exp(Z - zmax)
    ssum = E.sum(axis=1, keepdims=True)
    P = E / ssum
    rows = np.arange(Z.shape[0])
    loss = (np.log(ssum[:, 0]) + zmax[:, 0]) - Z[rows, y]
    return loss, P


def narrowed_weights(cfg: dict, w: np.ndarray, emulate_bf16: bool):
    """The weight matrices as the forward / input-gradient products see them
    (bf16-rounded when emulation is on).  A pure function of the model version,
    so a caller may compute it once per version and hand it to worker_update."""
    w = np.asarray(w, dtype=np.float64)
    if cfg["model"] in (MODEL_LINEAR, MODEL_CNN):
        return None
    return [round_bf16(W) if emulate_bf16 else W for (W, _) in unpack(cfg, w)]


def worker_update(cfg: dict, w: np.ndarray, X: np.ndarray, y: np.ndarray, s: float,
                  emulate_bf16: bool = False, Wq=None):
    """(s * g, mean loss) for one worker: g is the minibatch gradient of Eq. 2 at the
    model `w` (the worker's stale copy), X [B, d0] float64 rows, y targets.
    Wq, if given, must be narrowed_weights(cfg, w, emulate_bf16)."""
    B = X.shape[0]
    model = cfg["model"]
    if model == MODEL_CNN:
        return _cnn.worker_update(cfg, w, X, y, s)
    w = np.asarray(w, dtype=np.float64)
    u = np.zeros_like(w)
    if model == MODEL_LINEAR:
        r = X @ w - y
        loss = 0.5 * np.mean(r * r)
        dZ = (s / B) * r
        u[:] = X.T @ dZ
        return u, float(loss)

    rnd = round_bf16 if emulate_bf16 else (lambda a: a)
    layers = unpack(cfg, w)
    grads = unpack(cfg, u)
    L = len(layers)
    if Wq is None:
        Wq = narrowed_weights(cfg, w, emulate_bf16)
    H = [X]
    for l in range(L):
        Z = H[l] @ Wq[l] + layers[l][1]
        if l < L - 1:
            H.append(rnd(np.maximum(Z, 0.0)))
    per_row, P = _softmax_ce(Z, y)
    loss = float(np.mean(per_row))
    onehot = np.zeros_like(P)
    onehot[np.arange(B), y] = 1.0
    dZ = rnd((s / B) * (P - onehot))
    for l in range(L - 1, -1, -1):
        gW, gb = grads[l]
        gW[:, :] = H[l].T @ dZ
        gb[:] = dZ.sum(axis=0)
        if l > 0:
            dH = dZ @ Wq[l].T
            dZ = rnd(dH * (H[l] > 0.0))
    return u, loss


def mean_loss(cfg: dict, w: np.ndarray, X: np.ndarray, y: np.ndarray) -> float:
    """Minibatch mean loss only (used by the finite-difference pins)."""
    return worker_update(cfg, w, X, y, 0.0, False)[1]
