"""Pins of the convolutional model of the oracle (oracle/cnn.py), CPU only."""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import cnn
from oracle import models
from oracle.abs_sim import AbsOracle
from oracle.evaluate import evaluate

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "cnn_hand_worked_gradient.txt")


def _cfg(C0=3, S=14, k=3, C1=4, C2=5, F1=7, F2=6, C=4):
    return dict(model=cnn.MODEL_CNN, dims=[C0 * S * S, C1, C2, F1, F2, C, C0, k])


def _random_case(cfg, B, seed):
    rng = np.random.default_rng(seed)
    w = rng.standard_normal(cnn.param_count(cfg)) * 0.3
    X = rng.standard_normal((B, cfg["dims"][0]))
    y = rng.integers(0, cfg["dims"][5], B)
    return w, X, y


def _torch_loss_and_grad(cfg, w, X, y):
    """The same network from library layers (conv2d, relu, max_pool2d, linear, cross_entropy) in fp64."""
    g = cnn.geometry(cfg)
    k = g["k"]
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    parts, o = [], 0
    for r, c in cnn.layer_shapes(cfg):
        parts.append((wt[o:o + r * c].reshape(r, c), wt[o + r * c:o + r * c + c])); o += r * c + c
    def conv_w(W, cin):          # [(ci,u,v), co] -> [co, ci, u, v]
        return W.reshape(cin, k, k, -1).permute(3, 0, 1, 2)
    x = torch.tensor(X, dtype=torch.float64).reshape(-1, g["C0"], g["S"], g["S"])
    h = F.max_pool2d(F.relu(F.conv2d(x, conv_w(parts[0][0], g["C0"]), parts[0][1])), 2)
    h = F.max_pool2d(F.relu(F.conv2d(h, conv_w(parts[1][0], g["C1"]), parts[1][1])), 2)
    h = h.reshape(h.shape[0], -1)
    h = F.relu(h @ parts[2][0] + parts[2][1])
    h = F.relu(h @ parts[3][0] + parts[3][1])
    z = h @ parts[4][0] + parts[4][1]
    loss = F.cross_entropy(z, torch.tensor(y, dtype=torch.int64))
    loss.backward()
    return loss.item(), wt.grad.numpy(), z.detach().numpy()


@pytest.mark.parametrize("shape", [dict(), dict(C0=1, S=10, k=3, C1=2, C2=3), dict(C0=3, S=32, k=5, C1=6, C2=16, F1=120, F2=84, C=10)])
def test_loss_logits_and_gradient_equal_the_library_layers(shape):
    cfg = _cfg(**shape)
    w, X, y = _random_case(cfg, 5, 11)
    u, loss = cnn.worker_update(cfg, w, X, y, 1.0)
    tl, tg, tz = _torch_loss_and_grad(cfg, w, X, y)
    assert abs(loss - tl) < 1e-12 * max(1.0, abs(tl))
    np.testing.assert_allclose(cnn.logits(cfg, w, X), tz, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(u, tg, rtol=1e-9, atol=1e-13)
    # every layer of the network receives a gradient in this case
    o = 0
    for r, c in cnn.layer_shapes(cfg):
        assert np.abs(u[o:o + r * c]).max() > 0 and np.abs(u[o + r * c:o + r * c + c]).max() > 0
        o += r * c + c


def test_gradient_against_central_differences():
    cfg = _cfg(C0=2, S=10, k=3, C1=3, C2=4, F1=5, F2=4, C=3)
    w, X, y = _random_case(cfg, 4, 5)
    u, _ = cnn.worker_update(cfg, w, X, y, 1.0)
    rng = np.random.default_rng(1)
    h = 1e-6
    worst = 0.0
    for i in rng.choice(w.size, 60, replace=False):
        e = np.zeros_like(w); e[i] = h
        fd = (cnn.worker_update(cfg, w + e, X, y, 0.0)[1] - cnn.worker_update(cfg, w - e, X, y, 0.0)[1]) / (2 * h)
        worst = max(worst, abs(fd - u[i]) / max(1e-6, abs(u[i])))
    assert worst < 1e-5, worst


def test_seed_scales_the_gradient_linearly():
    cfg = _cfg()
    w, X, y = _random_case(cfg, 3, 2)
    u1, l1 = cnn.worker_update(cfg, w, X, y, 1.0)
    u2, l2 = cnn.worker_update(cfg, w, X, y, 0.125)
    assert l1 == l2
    np.testing.assert_allclose(u2, 0.125 * u1, rtol=1e-14, atol=0)


def test_hand_worked_gradient():
    vals = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        t = line.split()
        vals[t[0]] = [float(v) for v in t[1:]]
    cfg = dict(model=cnn.MODEL_CNN, dims=[16, 1, 1, 1, 1, 2, 1, 1])
    x = np.array([[1, 2, 0, -1, 3, -2, 1, 0, 0, 1, -1, 2, -3, 0, 4, 1]], dtype=np.float64)
    w = np.array([2, -1, 0.5, -1, 2, -1, 0.5, 0, 0.5, -0.5, 0, 0], dtype=np.float64)
    u, loss = cnn.worker_update(cfg, w, x, np.array([1]), 1.0)
    q = vals["q"][0]
    assert abs(q - 1.0 / (1.0 + np.exp(-2.0))) < 1e-15
    assert abs(loss - vals["loss"][0]) < 1e-14
    np.testing.assert_allclose(u, q * np.array(vals["gradient_over_q"]), rtol=1e-14, atol=0)


def test_pooling_routes_to_the_first_maximum_and_dead_windows_pass_nothing():
    a = np.array([[[[3., 3., -1., -2.], [1., 3., -5., -1.]]]])            # windows {3,3,1,3} and {-1,-2,-5,-1}
    r = np.maximum(a, 0.0)
    p, arg = cnn.pool_forward(r)
    assert p.tolist() == [[[[3., 0.]]]] and arg.tolist() == [[[[0, 0]]]]
    da = cnn.pool_backward(np.array([[[[7., 9.]]]]), arg, a.shape) * (a > 0.0)
    assert da.tolist() == [[[[7., 0., 0., 0.], [0., 0., 0., 0.]]]]


def test_the_model_runs_inside_the_simulator_and_evaluates():
    cfg = dict(_cfg(C0=1, S=10, k=3, C1=2, C2=3, F1=6, F2=5, C=3), x_dtype=0, M=64, N=4, B=4, K0=1, k_mode=0,
               tau_mode=0, tau_cap=2, a=-2, lr=0.05, sa_penalty=0, time_dist=0, time_param=0.0, n_slow=0,
               slow_factor=1.0, seed_sim=9, U=1)
    rng = np.random.default_rng(3)
    y = rng.integers(0, 3, 64).astype(np.int32)
    X = (rng.standard_normal((64, 100)) + 2.0 * y[:, None]).astype(np.float32)
    w0 = (rng.standard_normal(cnn.param_count(cfg)) * 0.2).astype(np.float32)
    o = AbsOracle(cfg, X, y, w0).run(40)
    first = np.mean([r["loss"] for r in o.trace[:5]]); last = np.mean([r["loss"] for r in o.trace[-5:]])
    assert np.isfinite(last) and last < first
    loss, acc, margin = evaluate(cfg, o.model(), X, y)
    assert np.isfinite(loss) and 0.0 <= acc <= 1.0 and margin.shape == (64,)
    # local steps go through the same per-worker routine
    o2 = AbsOracle(dict(cfg, U=3), X, y, w0).run(5)
    assert np.isfinite(o2.trace[-1]["loss"])
    assert len(models.unpack(cfg, o.model())) == 5
