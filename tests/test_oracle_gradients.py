"""Pins for the oracle's per-worker loss / gradient (CPU only): finite differences,
closed forms and an independent autograd library."""
import numpy as np
import pytest
import scipy.special
import torch

from oracle.models import worker_update, mean_loss, unpack, narrowed_weights
from oracle.bf16 import round_bf16


def _cfg(model, dims):
    return dict(model=model, dims=dims)


def _fd(cfg, w, X, y, eps=1e-6):
    g = np.zeros_like(w)
    for i in range(w.size):
        wp, wm = w.copy(), w.copy()
        wp[i] += eps; wm[i] -= eps
        g[i] = (mean_loss(cfg, wp, X, y) - mean_loss(cfg, wm, X, y)) / (2 * eps)
    return g


def _case(model, dims, B, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((B, dims[0]))
    if model == 0:
        y = rng.standard_normal(B)
        w = rng.standard_normal(dims[0])
    else:
        y = rng.integers(0, dims[-1], B)
        n = sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1))
        w = rng.standard_normal(n) * 0.7
    return X, y, w


@pytest.mark.parametrize("model,dims,B", [(0, [8, 1], 4), (1, [6, 3], 4), (2, [5, 4, 3], 4),
                                          (2, [6, 4, 4, 3], 3)])
def test_gradient_matches_central_differences(model, dims, B):
    cfg = _cfg(model, dims)
    X, y, w = _case(model, dims, B, 42 + model)
    g, loss = worker_update(cfg, w, X, y, 1.0)
    fd = _fd(cfg, w, X, y)
    assert np.linalg.norm(g - fd) <= 1e-6 * max(1.0, np.linalg.norm(fd))
    # the seed s multiplies the gradient and leaves the loss alone (linearity used in Eq. 3)
    g3, loss3 = worker_update(cfg, w, X, y, 0.37)
    assert np.allclose(g3, 0.37 * g, rtol=1e-13, atol=0) and loss3 == loss


def test_linear_closed_form():
    cfg = _cfg(0, [7, 1])
    X, y, w = _case(0, [7, 1], 5, 1)
    g, loss = worker_update(cfg, w, X, y, 1.0)
    assert np.allclose(g, X.T @ (X @ w - y) / 5, rtol=1e-13)
    assert np.isclose(loss, 0.5 * np.mean((X @ w - y) ** 2), rtol=1e-14)
    # at the least-squares solution of a consistent system the gradient vanishes
    w_star = np.arange(7.0)
    g0, l0 = worker_update(cfg, w_star, X, X @ w_star, 1.0)
    assert np.abs(g0).max() < 1e-12 and l0 < 1e-24


def test_softmax_output_gradient_and_loss_against_scipy():
    dims = [6, 4]
    cfg = _cfg(1, dims)
    X, y, w = _case(1, dims, 5, 3)
    (W, b), = unpack(cfg, w)
    Z = X @ W + b
    g, loss = worker_update(cfg, w, X, y, 1.0)
    want_loss = np.mean(scipy.special.logsumexp(Z, axis=1) - Z[np.arange(5), y])
    assert np.isclose(loss, want_loss, rtol=1e-13)
    P = scipy.special.softmax(Z, axis=1)
    P[np.arange(5), y] -= 1.0
    (gW, gb), = unpack(cfg, g)
    assert np.allclose(gb, P.mean(axis=0), rtol=1e-12, atol=1e-15)   # bias gradient = mean(softmax - onehot)
    assert np.allclose(gW, X.T @ P / 5, rtol=1e-12, atol=1e-15)
    # large logits do not overflow (max subtraction)
    big = worker_update(cfg, w * 1e4, X, y, 1.0)
    assert np.isfinite(big[1]) and np.all(np.isfinite(big[0]))


@pytest.mark.parametrize("dims", [[9, 5, 3], [7, 6, 5, 4]])
def test_mlp_against_autograd(dims):
    cfg = _cfg(2, dims)
    X, y, w = _case(2, dims, 6, 9)
    g, loss = worker_update(cfg, w, X, y, 1.0)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    h, o = torch.tensor(X), 0
    for l in range(len(dims) - 1):
        W = wt[o:o + dims[l] * dims[l + 1]].reshape(dims[l], dims[l + 1]); o += dims[l] * dims[l + 1]
        b = wt[o:o + dims[l + 1]]; o += dims[l + 1]
        h = h @ W + b
        if l < len(dims) - 2:
            h = torch.relu(h)
    lt = torch.nn.functional.cross_entropy(h, torch.tensor(y))
    lt.backward()
    assert np.isclose(loss, lt.item(), rtol=1e-13)
    assert np.allclose(g, wt.grad.numpy(), rtol=1e-11, atol=1e-14)


def test_relu_derivative_at_zero_is_zero():
    # one hidden unit whose pre-activation is exactly 0: no gradient flows through it
    cfg = _cfg(2, [2, 1, 2])
    w = np.array([1.0, -1.0, 0.0, 0.5, -0.5, 0.0, 0.0])   # W1=[1,-1]^T, b1=0, W2=[.5,-.5], b2=0
    X = np.array([[2.0, 2.0]])
    g, _ = worker_update(cfg, w, X, np.array([0]), 1.0)
    assert np.all(g[:3] == 0.0)


def test_bf16_emulation_is_exact_on_representable_values_and_close_otherwise():
    dims = [8, 4, 3]
    cfg = _cfg(2, dims)
    rng = np.random.default_rng(5)
    X = round_bf16(rng.standard_normal((4, 8)))
    y = rng.integers(0, 3, 4)
    w = rng.standard_normal(8 * 4 + 4 + 4 * 3 + 3) * 0.5
    g_wide, l_wide = worker_update(cfg, w, X, y, 1.0, emulate_bf16=False)
    g_emu, l_emu = worker_update(cfg, w, X, y, 1.0, emulate_bf16=True)
    # bf16 keeps 8 significant bits: the two must agree to a few 2^-8 and differ somewhere
    assert np.linalg.norm(g_emu - g_wide) < 0.05 * np.linalg.norm(g_wide)
    assert abs(l_emu - l_wide) < 0.05 * abs(l_wide)
    assert not np.array_equal(g_emu, g_wide)
    # the forward pass sees weights narrowed to bf16, biases wide
    Wq = narrowed_weights(cfg, w, True)
    (W1, b1), (W2, b2) = unpack(cfg, w)
    assert np.array_equal(Wq[0], round_bf16(W1)) and np.array_equal(Wq[1], round_bf16(W2))
    h1 = torch.relu(torch.tensor(X) @ torch.tensor(Wq[0]) + torch.tensor(b1))
    h1 = h1.to(torch.float32).to(torch.bfloat16).to(torch.float64)       # library narrowing
    z2 = (h1 @ torch.tensor(Wq[1]) + torch.tensor(b2)).numpy()
    want = np.mean(scipy.special.logsumexp(z2, axis=1) - z2[np.arange(4), y])
    assert np.isclose(l_emu, want, rtol=1e-13)
    # the output-layer gradient is the narrowed seed (s/B)(softmax - onehot) times H_1^T
    P = scipy.special.softmax(z2, axis=1); P[np.arange(4), y] -= 1.0
    dz = torch.tensor(0.25 * P).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    (_, _), (gW2, gb2) = unpack(cfg, g_emu)
    assert np.allclose(gW2, h1.numpy().T @ dz, rtol=1e-13, atol=1e-18)
    assert np.allclose(gb2, dz.sum(axis=0), rtol=1e-13, atol=1e-18)


def test_bf16_rounding_points_of_the_hidden_layers_against_a_library_narrowing():
    """Every rounding point of the bf16 reading below the output layer, re-derived with torch's own
    float32 -> bfloat16 conversion on a three-layer network: the input gradient uses the NARROWED
    weights (dH = dZ Wq^T), it is masked by the narrowed activation (H > 0) and narrowed again before
    it is used, and each weight gradient is H_{l-1}^T dZ_l of those narrowed factors, summed wide.  A
    mistake in any of them (wide weights in the input gradient, the mask taken from the pre-activation,
    a dZ_l used before narrowing, a transposed factor) moves the result by about 2^-8 of its size."""
    dims = [6, 5, 4, 3]
    cfg = _cfg(2, dims)
    rng = np.random.default_rng(11)
    B, s = 5, 0.37
    X = round_bf16(rng.standard_normal((B, dims[0])))
    y = rng.integers(0, dims[-1], B)
    n = sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(3))
    w = rng.standard_normal(n) * 0.6
    g, _ = worker_update(cfg, w, X, y, s, emulate_bf16=True)
    (W1, b1), (W2, b2), (W3, b3) = unpack(cfg, w)
    (gW1, gb1), (gW2, gb2), (gW3, gb3) = unpack(cfg, g)

    def narrow(a):                       # torch's conversion, not the oracle's helper
        return torch.tensor(np.asarray(a)).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()

    Wq = [narrow(W1), narrow(W2), narrow(W3)]
    h1 = narrow(np.maximum(X @ Wq[0] + b1, 0.0))
    h2 = narrow(np.maximum(h1 @ Wq[1] + b2, 0.0))
    z3 = h2 @ Wq[2] + b3
    P = scipy.special.softmax(z3, axis=1); P[np.arange(B), y] -= 1.0
    dz3 = narrow((s / B) * P)
    dz2 = narrow((dz3 @ Wq[2].T) * (h2 > 0.0))
    dz1 = narrow((dz2 @ Wq[1].T) * (h1 > 0.0))
    for got, want in ((gW3, h2.T @ dz3), (gb3, dz3.sum(0)), (gW2, h1.T @ dz2), (gb2, dz2.sum(0)),
                      (gW1, X.T @ dz1), (gb1, dz1.sum(0))):
        assert np.allclose(got, want, rtol=1e-12, atol=1e-18)
    # the variants a wrong reading would give differ by far more than that
    dz2_wide_w = narrow((dz3 @ W3.T) * (h2 > 0.0))
    dz2_unnarrowed = (dz3 @ Wq[2].T) * (h2 > 0.0)
    assert not np.allclose(gW2, h1.T @ dz2_wide_w, rtol=1e-6, atol=0)
    assert not np.allclose(gW2, h1.T @ dz2_unnarrowed, rtol=1e-6, atol=0)
