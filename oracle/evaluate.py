"""Held-out evaluation of a global model (oracle side; test infrastructure only).

The paper's read-outs are the loss of the global model and its test accuracy, plotted against
wall-clock time and against communication rounds (Section V-B).  `evaluate` gives both for one
model version on an evaluation set: the mean per-sample loss f(w; xi) of Eq. 1 and the fraction
of rows whose largest logit is the label (ties: the lowest class index).  The forward pass is the
training one (models.worker_update): with bf16 emulation the weights are narrowed per version and
the hidden activations after the ReLU.  The linear model has no accuracy (NaN).
"""
from __future__ import annotations

import numpy as np

from .bf16 import round_bf16
from .models import MODEL_LINEAR, MODEL_MLP, MODEL_CNN, unpack, narrowed_weights, _softmax_ce
from . import cnn as _cnn


def logits(cfg: dict, w: np.ndarray, X: np.ndarray, emulate_bf16: bool = False) -> np.ndarray:
    """Z_L [rows, C] (the linear model: the prediction x.w as one column)."""
    w = np.asarray(w, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    if cfg["model"] == MODEL_LINEAR:
        return (X @ w)[:, None]
    if cfg["model"] == MODEL_CNN:
        return _cnn.logits(cfg, w, X)
    rnd = round_bf16 if emulate_bf16 else (lambda a: a)
    layers = unpack(cfg, w)
    Wq = narrowed_weights(cfg, w, emulate_bf16)
    H = X
    for l in range(len(layers)):
        Z = H @ Wq[l] + layers[l][1]
        if l < len(layers) - 1:
            H = rnd(np.maximum(Z, 0.0))
    return Z


def evaluate(cfg: dict, w: np.ndarray, X: np.ndarray, y: np.ndarray, emulate_bf16=None):
    """(mean loss, accuracy, per-row margin) over the rows of X.

    margin = largest logit minus the runner-up (classification) - rows with a tiny margin are the
    ones whose argmax a lower-precision forward pass may decide differently."""
    if emulate_bf16 is None:
        emulate_bf16 = cfg["model"] == MODEL_MLP
    Z = logits(cfg, w, X, emulate_bf16)
    if cfg["model"] == MODEL_LINEAR:
        r = Z[:, 0] - np.asarray(y, dtype=np.float64)
        return float(0.5 * np.mean(r * r)), float("nan"), None
    y = np.asarray(y).astype(np.int64)
    per_row, _ = _softmax_ce(Z, y)
    pred = np.argmax(Z, axis=1)                       # first maximum = lowest class index
    part = np.partition(Z, -2, axis=1)
    margin = part[:, -1] - part[:, -2]
    return float(np.mean(per_row)), float(np.mean(pred == y)), margin
