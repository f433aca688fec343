"""Seeded dataset / initial-weight generators for the presets.

Linear least squares: X ~ N(0,1), w* ~ N(0,1), y = X w* + N(0, 0.01^2), w0 = 0.
Classification: a Gaussian mixture, class means ~ N(0, I), unit variance,
labels uniform; softmax starts from w0 = 0, MLP and CNN weights W_l ~ N(0, 2/fan_in), b = 0.
bf16 datasets are the fp32 draw rounded to nearest-even and handed over as the
uint16 payload (the dataset *is* bf16 for those workloads).
"""
from __future__ import annotations

import numpy as np

from .presets import MODEL_LINEAR, MODEL_SOFTMAX, MODEL_MLP, MODEL_CNN, X_BF16, cnn_layer_shapes


def to_bf16_bits(x32: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 bf16 payload, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_inputs(p: dict):
    """Returns dict(X, y, w0, w_star): X fp32 [M,d] or uint16 bf16 payload [M,d];
    y fp32 [M] (linear) or int32 [M]; w0 fp32 flat in the boundary layout
    (per layer: W[d_in, d_out] row-major, then b[d_out]; the linear model has no bias)."""
    M, d = p["M"], p["dims"][0]
    rng = np.random.Generator(np.random.PCG64(p["seed_data"]))
    out = {}
    if p["model"] == MODEL_LINEAR:
        X = rng.standard_normal((M, d), dtype=np.float32)
        w_star = rng.standard_normal(d, dtype=np.float32)
        noise = rng.standard_normal(M, dtype=np.float32) * np.float32(0.01)
        y = (X.astype(np.float64) @ w_star.astype(np.float64)).astype(np.float32) + noise
        out.update(X=X, y=y.astype(np.float32), w_star=w_star)
    else:
        C = p["n_classes"]
        mu = rng.standard_normal((C, d), dtype=np.float32)
        y = rng.integers(0, C, size=M, dtype=np.int32)
        X = np.empty((M, d), dtype=np.float32)
        step = 8192
        for lo in range(0, M, step):
            hi = min(M, lo + step)
            X[lo:hi] = rng.standard_normal((hi - lo, d), dtype=np.float32) + mu[y[lo:hi]]
        if p["x_dtype"] == X_BF16:
            X = to_bf16_bits(X)
        out.update(X=X, y=y, w_star=None)

    irng = np.random.Generator(np.random.PCG64(p["seed_init"]))
    dims = p["dims"]
    if p["model"] == MODEL_LINEAR:
        w0 = np.zeros(d, dtype=np.float32)
    elif p["model"] == MODEL_SOFTMAX:
        w0 = np.zeros(dims[0] * dims[1] + dims[1], dtype=np.float32)
    elif p["model"] == MODEL_CNN:
        parts = []
        for rows, cols in cnn_layer_shapes(p):       # fan-in = rows for both kinds of layer
            W = irng.standard_normal((rows, cols), dtype=np.float32)
            W *= np.float32(np.sqrt(2.0 / rows))
            parts += [W.ravel(), np.zeros(cols, dtype=np.float32)]
        w0 = np.concatenate(parts).astype(np.float32)
    else:
        parts = []
        for l in range(len(dims) - 1):
            W = irng.standard_normal((dims[l], dims[l + 1]), dtype=np.float32)
            W *= np.float32(np.sqrt(2.0 / dims[l]))
            parts += [W.ravel(), np.zeros(dims[l + 1], dtype=np.float32)]
        w0 = np.concatenate(parts).astype(np.float32)
    out["w0"] = w0
    return out


def make_split(p: dict, eval_rows: int):
    """(training inputs for p, X_eval, y_eval): one draw of p["M"] + eval_rows rows from the
    preset's generator (same w* / class means), the last eval_rows of them held out."""
    M = p["M"]
    d = make_inputs(dict(p, M=M + eval_rows))
    train = dict(X=np.ascontiguousarray(d["X"][:M]), y=np.ascontiguousarray(d["y"][:M]),
                 w0=d["w0"], w_star=d["w_star"])
    return train, np.ascontiguousarray(d["X"][M:]), np.ascontiguousarray(d["y"][M:])
