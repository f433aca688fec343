"""Pins of the oracle's held-out evaluation (mean loss of Eq. 1 and accuracy) against library
routines, brute force and closed forms."""
import numpy as np
import pytest
from scipy.special import log_softmax

import workloads
from oracle.evaluate import evaluate, logits
from oracle.bf16 import round_bf16


def _data(i, **over):
    p = workloads.scaled_preset(i, **over)
    return p, workloads.make_inputs(p)


def test_softmax_matches_library_log_softmax_and_argmax():
    p, d = _data(2, M=640, dims=[20, 5], n_classes=5, N=4)
    rng = np.random.default_rng(5)
    w = rng.normal(size=workloads.param_count(p)) * 0.3
    X, y = d["X"].astype(np.float64), d["y"].astype(np.int64)
    W, b = w[:100].reshape(20, 5), w[100:]
    Z = X @ W + b
    nll = -log_softmax(Z, axis=1)[np.arange(len(y)), y]
    loss, acc, margin = evaluate(p, w, X, y)
    assert loss == pytest.approx(nll.mean(), rel=1e-12)
    assert acc == np.mean(Z.argmax(1) == y)
    assert margin.shape == (640,) and np.all(margin >= 0)


def test_linear_at_the_generating_weights_leaves_the_noise():
    p, d = _data(1, M=4000)
    X, y = d["X"].astype(np.float64), d["y"].astype(np.float64)
    w_ls = np.linalg.lstsq(X, y, rcond=None)[0]
    loss, acc, _ = evaluate(p, w_ls, X, y)
    r = y - X @ w_ls
    assert loss == pytest.approx(0.5 * np.mean(r * r), rel=1e-12)
    assert np.isnan(acc)
    # any other point is worse than the least-squares solution
    assert evaluate(p, w_ls + 1e-3, X, y)[0] > loss


def test_mlp_against_a_per_sample_loop():
    p, d = _data(3, M=64, dims=[8, 6, 4], n_classes=4, N=4, B=4)
    rng = np.random.default_rng(1)
    w = rng.normal(size=workloads.param_count(p)) * 0.5
    X = workloads.bf16_bits_to_f32(d["X"]).astype(np.float64)
    y = d["y"].astype(np.int64)
    W1, b1 = w[:48].reshape(8, 6), w[48:54]
    W2, b2 = w[54:78].reshape(6, 4), w[78:82]
    tot, hits = 0.0, 0
    for i in range(64):
        h = [max(0.0, sum(X[i, a] * W1[a, j] for a in range(8)) + b1[j]) for j in range(6)]
        z = [sum(h[j] * W2[j, c] for j in range(6)) + b2[c] for c in range(4)]
        m = max(z)
        tot += m + np.log(sum(np.exp(v - m) for v in z)) - z[y[i]]
        hits += int(z.index(m) == y[i])
    loss, acc, _ = evaluate(p, w, X, y, emulate_bf16=False)
    assert loss == pytest.approx(tot / 64, rel=1e-12)
    assert acc == hits / 64


def test_mlp_bf16_emulation_rounds_weights_and_hidden_activations():
    p, d = _data(3, M=32, dims=[8, 6, 4], n_classes=4, N=4, B=4)
    rng = np.random.default_rng(2)
    w = rng.normal(size=workloads.param_count(p))
    X = workloads.bf16_bits_to_f32(d["X"]).astype(np.float64)
    W1, b1 = round_bf16(w[:48].reshape(8, 6)), w[48:54]
    W2, b2 = round_bf16(w[54:78].reshape(6, 4)), w[78:82]
    Z = round_bf16(np.maximum(X @ W1 + b1, 0)) @ W2 + b2
    assert np.array_equal(logits(p, w, X, emulate_bf16=True), Z)
    assert not np.array_equal(logits(p, w, X, emulate_bf16=False), Z)


def test_degenerate_models():
    p, d = _data(2, M=500, dims=[12, 4], n_classes=4, N=4)
    X, y = d["X"].astype(np.float64), d["y"].astype(np.int64)
    n = workloads.param_count(p)
    # all-zero model: uniform softmax, every argmax ties and resolves to class 0
    loss, acc, margin = evaluate(p, np.zeros(n), X, y)
    assert loss == pytest.approx(np.log(4), rel=1e-12)
    assert acc == np.mean(y == 0) and np.all(margin == 0)
    # a bias that always wins for class 2
    w = np.zeros(n); w[12 * 4 + 2] = 50.0
    loss, acc, _ = evaluate(p, w, X, y)
    assert acc == np.mean(y == 2)
    assert loss == pytest.approx(50.0 * np.mean(y != 2), rel=1e-9)
