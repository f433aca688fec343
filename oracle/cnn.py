"""The convolutional model of Section V-A, oracle side (TEST INFRASTRUCTURE ONLY).

Section V-A says of the network only that it has two convolutional and three fully
connected layers and is trained on 32 x 32 colour images in 10 classes.  The reading
taken here (the paper gives no further shape):

  x [C0, S, S]
  conv k x k, stride 1, no padding, C0 -> C1 channels, + bias; ReLU; 2 x 2 max-pool, stride 2
  conv k x k, stride 1, no padding, C1 -> C2 channels, + bias; ReLU; 2 x 2 max-pool, stride 2
  flatten (channel, row, column) -> F0 = C2 * S2 * S2 features
  dense F0 -> F1, ReLU; dense F1 -> F2, ReLU; dense F2 -> C; softmax cross-entropy

with relu'(0) = 0 and the pooling gradient going to the first maximum of a window in the
order (0,0), (0,1), (1,0), (1,1).  cfg["dims"] = [C0*S*S, C1, C2, F1, F2, C, C0, k].

Parameter vector (boundary layout), per layer W then b:
  conv layer: W [C_in * k * k, C_out] row-major, row index (ci * k + u) * k + v
              (input channel, kernel row, kernel column); b [C_out]
  dense layer: W [d_in, d_out] row-major; b [d_out]

Everything is written out from the definitions: a convolution output is the sum over
(ci, u, v) of shifted input planes times one weight; nothing is blocked or fused.
`worker_update` returns s * g and the minibatch mean loss like models.worker_update:
s is the seed of back-propagation (Eq. 2's minibatch gradient times the upload's
coefficient in Eq. 3).
"""
from __future__ import annotations

import numpy as np

MODEL_CNN = 3


def geometry(cfg: dict) -> dict:
    d0, C1, C2, F1, F2, C, C0, k = cfg["dims"]
    S = int(round((d0 // C0) ** 0.5))
    assert C0 * S * S == d0, "dims[0] must be C0 * S * S"
    S1c = S - k + 1
    assert S1c > 0 and S1c % 2 == 0
    S1 = S1c // 2
    S2c = S1 - k + 1
    assert S2c > 0 and S2c % 2 == 0
    S2 = S2c // 2
    return dict(C0=C0, C1=C1, C2=C2, F0=C2 * S2 * S2, F1=F1, F2=F2, C=C, k=k, S=S, S1c=S1c, S1=S1,
                S2c=S2c, S2=S2)


def layer_shapes(cfg: dict):
    """[(rows, cols)] of the five weight matrices in the parameter vector."""
    g = geometry(cfg)
    kk = g["k"] * g["k"]
    return [(g["C0"] * kk, g["C1"]), (g["C1"] * kk, g["C2"]), (g["F0"], g["F1"]), (g["F1"], g["F2"]),
            (g["F2"], g["C"])]


def param_count(cfg: dict) -> int:
    return sum(r * c + c for r, c in layer_shapes(cfg))


def unpack(cfg: dict, w: np.ndarray):
    """Flat parameter vector -> [(W_l, b_l)] views, l = conv1, conv2, dense1, dense2, dense3."""
    out, o = [], 0
    for r, c in layer_shapes(cfg):
        W = w[o:o + r * c].reshape(r, c); o += r * c
        b = w[o:o + c]; o += c
        out.append((W, b))
    assert o == w.size
    return out


def conv_forward(x: np.ndarray, W: np.ndarray, b: np.ndarray, k: int) -> np.ndarray:
    """x [B, Cin, S, S] -> [B, Cout, S-k+1, S-k+1]: out[n,co,i,j] = b[co] + sum x[n,ci,i+u,j+v] W[(ci,u,v),co]."""
    B, Cin, S, _ = x.shape
    So = S - k + 1
    out = np.zeros((B, W.shape[1], So, So)) + b[None, :, None, None]
    for ci in range(Cin):
        for u in range(k):
            for v in range(k):
                out += x[:, ci, u:u + So, v:v + So][:, None, :, :] * W[(ci * k + u) * k + v][None, :, None, None]
    return out


def conv_backward(x: np.ndarray, W: np.ndarray, dout: np.ndarray, k: int):
    """Gradients of sum(out * dout): (dW [Cin*k*k, Cout], db [Cout], dx like x)."""
    B, Cin, S, _ = x.shape
    So = S - k + 1
    dW = np.zeros_like(W)
    dx = np.zeros_like(x)
    for ci in range(Cin):
        for u in range(k):
            for v in range(k):
                r = (ci * k + u) * k + v
                dW[r] = np.einsum("nij,ncij->c", x[:, ci, u:u + So, v:v + So], dout)
                dx[:, ci, u:u + So, v:v + So] += np.einsum("ncij,c->nij", dout, W[r])
    return dW, dout.sum(axis=(0, 2, 3)), dx


_WINDOW = ((0, 0), (0, 1), (1, 0), (1, 1))


def pool_forward(a: np.ndarray):
    """2 x 2 max-pool, stride 2: (pooled, index of the first maximum of each window in _WINDOW order)."""
    cand = np.stack([a[:, :, dy::2, dx::2] for dy, dx in _WINDOW])      # [4, B, C, S/2, S/2]
    arg = np.argmax(cand, axis=0)                                       # first maximum
    return np.take_along_axis(cand, arg[None], axis=0)[0], arg


def pool_backward(dp: np.ndarray, arg: np.ndarray, shape):
    da = np.zeros(shape)
    for q, (dy, dx) in enumerate(_WINDOW):
        da[:, :, dy::2, dx::2] = np.where(arg == q, dp, 0.0)
    return da


def _softmax_ce(Z: np.ndarray, y: np.ndarray):
    zmax = Z.max(axis=1, keepdims=True)
    E = np.exp(Z - zmax)
    ssum = E.sum(axis=1, keepdims=True)
    rows = np.arange(Z.shape[0])
    return (np.log(ssum[:, 0]) + zmax[:, 0]) - Z[rows, y], E / ssum


def forward(cfg: dict, w: np.ndarray, X: np.ndarray):
    """All intermediate activations of the forward pass; X [B, C0*S*S] rows (channel, row, column)."""
    g = geometry(cfg)
    L = unpack(cfg, np.asarray(w, dtype=np.float64))
    B = X.shape[0]
    x0 = np.asarray(X, dtype=np.float64).reshape(B, g["C0"], g["S"], g["S"])
    a1 = conv_forward(x0, L[0][0], L[0][1], g["k"])
    r1 = np.maximum(a1, 0.0)
    p1, arg1 = pool_forward(r1)
    a2 = conv_forward(p1, L[1][0], L[1][1], g["k"])
    r2 = np.maximum(a2, 0.0)
    p2, arg2 = pool_forward(r2)
    h0 = p2.reshape(B, g["F0"])
    z1 = h0 @ L[2][0] + L[2][1]
    h1 = np.maximum(z1, 0.0)
    z2 = h1 @ L[3][0] + L[3][1]
    h2 = np.maximum(z2, 0.0)
    z3 = h2 @ L[4][0] + L[4][1]
    return dict(x0=x0, a1=a1, p1=p1, arg1=arg1, a2=a2, p2=p2, arg2=arg2, h0=h0, h1=h1, h2=h2, z3=z3)


def logits(cfg: dict, w: np.ndarray, X: np.ndarray) -> np.ndarray:
    return forward(cfg, w, X)["z3"]


def worker_update(cfg: dict, w: np.ndarray, X: np.ndarray, y: np.ndarray, s: float):
    """(s * g, mean loss): g the minibatch gradient (Eq. 2) of the mean softmax cross-entropy at w."""
    g = geometry(cfg)
    w = np.asarray(w, dtype=np.float64)
    L = unpack(cfg, w)
    f = forward(cfg, w, X)
    B = X.shape[0]
    per_row, P = _softmax_ce(f["z3"], np.asarray(y).astype(np.int64))
    onehot = np.zeros_like(P)
    onehot[np.arange(B), np.asarray(y).astype(np.int64)] = 1.0
    u = np.zeros_like(w)
    G = unpack(cfg, u)
    dz3 = (s / B) * (P - onehot)
    G[4][0][:, :] = f["h2"].T @ dz3; G[4][1][:] = dz3.sum(axis=0)
    dz2 = (dz3 @ L[4][0].T) * (f["h2"] > 0.0)
    G[3][0][:, :] = f["h1"].T @ dz2; G[3][1][:] = dz2.sum(axis=0)
    dz1 = (dz2 @ L[3][0].T) * (f["h1"] > 0.0)
    G[2][0][:, :] = f["h0"].T @ dz1; G[2][1][:] = dz1.sum(axis=0)
    dp2 = (dz1 @ L[2][0].T).reshape(f["p2"].shape)
    da2 = pool_backward(dp2, f["arg2"], f["a2"].shape) * (f["a2"] > 0.0)
    dW2, db2, dp1 = conv_backward(f["p1"], L[1][0], da2, g["k"])
    G[1][0][:, :] = dW2; G[1][1][:] = db2
    da1 = pool_backward(dp1, f["arg1"], f["a1"].shape) * (f["a1"] > 0.0)
    dW1, db1, _ = conv_backward(f["x0"], L[0][0], da1, g["k"])
    G[0][0][:, :] = dW1; G[0][1][:] = db1
    return u, float(np.mean(per_row))
