"""Pins for the oracle's loss and gradient, g = grad f(w; xi): numerical differences,
closed forms, and library routines on cases that reduce to them."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as W
from oracle.oracle import batch_loss_grad

TINY = {
    "softmax": W.softmax_model(5, 3, batch=4),
    "mlp": W.mlp_model(6, 4, 3, batch=3),
    "lenet": W.Model(2, 8, 8, [W.Layer(W.CONV, 3, 3, 0, 1), W.Layer(W.POOL),
                                W.Layer(W.CONV, 4, 2, 0, 1), W.Layer(W.DENSE, 5, relu=1),
                                W.Layer(W.DENSE, 3)], 3),
    "cnn": W.Model(3, 8, 8, [W.Layer(W.CONV, 4, 3, 1, 1), W.Layer(W.CONV, 4, 3, 1, 1),
                              W.Layer(W.POOL), W.Layer(W.CONV, 5, 3, 1, 1), W.Layer(W.POOL),
                              W.Layer(W.DENSE, 6, relu=1), W.Layer(W.DENSE, 4)], 2),
}


def _batch(model, B, seed):
    g = np.random.default_rng(seed)
    X = g.uniform(-1, 1, (B, model.in_size())).astype(np.float32)
    y = g.integers(0, model.n_classes(), B).astype(np.int32)
    w = g.uniform(-0.7, 0.7, model.n_params())
    return w, X, y


@pytest.mark.parametrize("name", list(TINY))
def test_gradient_matches_central_differences(oracle_libs, name):
    model = TINY[name]
    w, X, y = _batch(model, model.batch, 1)
    _, g = batch_loss_grad(model, w, X, y)
    h = 1e-6
    num = np.zeros_like(w)
    for p in range(w.size):
        wp, wm = w.copy(), w.copy()
        wp[p] += h
        wm[p] -= h
        lp, _ = batch_loss_grad(model, wp, X, y, want_grad=False)
        lm, _ = batch_loss_grad(model, wm, X, y, want_grad=False)
        num[p] = (lp - lm) / (2 * h)
    assert np.abs(g - num).max() <= 1e-6 * max(1.0, np.abs(num).max())
    assert np.abs(g).max() > 1e-3          # not a vacuous comparison


def _torch_loss_grad(model, w, X, y):
    """The same network through PyTorch's CPU ops and autograd, in float64."""
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    x = torch.tensor(X, dtype=torch.float64).reshape(-1, model.in_c, model.in_h, model.in_w)
    shp = model.shapes()
    for L, sl, (c, h, ww) in zip(model.layers, model.param_slices(), shp[:-1]):
        if L.type == W.CONV:
            Wt = wt[sl[0]:sl[0] + sl[1]].reshape(L.cout, c, L.k, L.k)
            x = F.conv2d(x, Wt, wt[sl[2]:sl[2] + sl[3]], padding=L.pad)
        elif L.type == W.POOL:
            x = F.max_pool2d(x, 2)
        else:
            x = x.reshape(x.shape[0], -1)
            Wt = wt[sl[0]:sl[0] + sl[1]].reshape(L.cout, c * h * ww)
            x = F.linear(x, Wt, wt[sl[2]:sl[2] + sl[3]])
        if L.relu:
            x = F.relu(x)
    loss = F.cross_entropy(x.reshape(x.shape[0], -1), torch.tensor(y, dtype=torch.long))
    loss.backward()
    return float(loss.detach()), wt.grad.numpy()


@pytest.mark.parametrize("name", list(TINY) + ["lenet_full", "cnn_16x16"])
def test_gradient_matches_library_autograd(oracle_libs, name):
    """Convolution (cross-correlation, weight layout [cout][cin][kh][kw]), padding, pooling,
    C-H-W flattening, bias and mean-over-batch all have to agree with the library."""
    if name == "lenet_full":
        model = W.lenet_model(4)
    elif name == "cnn_16x16":
        model = W.cnn32_model(2, hw=16, width=8, fc=32)
    else:
        model = TINY[name]
    w, X, y = _batch(model, model.batch, 2)
    if name in ("lenet_full", "cnn_16x16"):
        w = W.init_weights(model, 5).astype(np.float64)
    loss, g = batch_loss_grad(model, w, X, y)
    tl, tg = _torch_loss_grad(model, w, X, y)
    assert loss == pytest.approx(tl, rel=1e-12)
    assert np.abs(g - tg).max() <= 1e-11 * max(1.0, np.abs(tg).max())


def test_softmax_regression_textbook_form(oracle_libs):
    """One dense layer: grad_W = mean_b (p_b - onehot(y_b)) x_b^T, grad_b = mean_b (p_b - onehot)."""
    model = W.softmax_model(7, 4, batch=5)
    w, X, y = _batch(model, 5, 3)
    loss, g = batch_loss_grad(model, w, X, y)
    Wm, b = w[:28].reshape(4, 7), w[28:]
    z = X.astype(np.float64) @ Wm.T + b
    p = np.exp(z - z.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    oh = np.eye(4)[y]
    assert np.allclose(g[:28].reshape(4, 7), (p - oh).T @ X.astype(np.float64) / 5, rtol=0, atol=1e-14)
    assert np.allclose(g[28:], (p - oh).mean(0), rtol=0, atol=1e-14)
    assert loss == pytest.approx(-np.log(p[np.arange(5), y]).mean(), rel=1e-13)


@pytest.mark.parametrize("name", list(TINY))
def test_loss_at_zero_weights_is_log_classes(oracle_libs, name):
    model = TINY[name]
    _, X, y = _batch(model, model.batch, 4)
    loss, g = batch_loss_grad(model, np.zeros(model.n_params()), X, y)
    assert loss == pytest.approx(math.log(model.n_classes()), rel=1e-14)
    # the output bias gradient is (1/C - onehot) averaged over the batch
    C = model.n_classes()
    want = 1.0 / C - np.bincount(y, minlength=C) / y.size
    assert np.allclose(g[-C:], want, atol=1e-15)


def test_loss_is_shift_invariant_and_stable(oracle_libs):
    """Adding a constant to all output biases changes nothing; huge logits do not overflow."""
    model = W.softmax_model(5, 3, batch=4)
    w, X, y = _batch(model, 4, 5)
    l0, g0 = batch_loss_grad(model, w, X, y)
    w2 = w.copy()
    w2[-3:] += 1000.0
    l1, g1 = batch_loss_grad(model, w2, X, y)
    assert l1 == pytest.approx(l0, abs=1e-10)
    assert np.allclose(g0, g1, atol=1e-10)
    l2, g2 = batch_loss_grad(model, w * 1e4, X, y)
    assert np.isfinite(l2) and np.isfinite(g2).all()


def test_batch_gradient_is_mean_of_per_sample_gradients(oracle_libs):
    model = TINY["lenet"]
    w, X, y = _batch(model, 3, 6)
    loss, g = batch_loss_grad(model, w, X, y)
    per = [batch_loss_grad(model, w, X[j:j + 1], y[j:j + 1]) for j in range(3)]
    assert loss == pytest.approx(np.mean([p[0] for p in per]), rel=1e-14)
    assert np.allclose(g, np.mean([p[1] for p in per], axis=0), atol=1e-15)


def test_pool_routes_gradient_to_first_maximum(oracle_libs):
    """A 2x2 window of equal values: the whole gradient goes to the first element in
    row-major window order (and nowhere else)."""
    model = W.Model(1, 2, 2, [W.Layer(W.CONV, 1, 1, 0, 0), W.Layer(W.POOL), W.Layer(W.DENSE, 2)], 1)
    # conv 1x1 with weight 1, bias 0 copies the input; dense weights (1, -1)
    w = np.array([1.0, 0.0, 1.0, -1.0, 0.0, 0.0])
    X = np.full((1, 4), 0.5, dtype=np.float32)
    y = np.array([0], dtype=np.int32)
    _, g = batch_loss_grad(model, w, X, y)
    # d loss / d pooled = W_dense^T (p - onehot); conv weight gradient = that * x[first]
    z = np.array([0.5, -0.5])
    p = np.exp(z) / np.exp(z).sum()
    dpool = (p - np.array([1.0, 0.0])) @ np.array([1.0, -1.0])
    assert g[0] == pytest.approx(dpool * 0.5, rel=1e-14)      # exactly one element contributed
    assert g[1] == pytest.approx(dpool, rel=1e-14)


def test_f32_twin_agrees_with_f64(oracle_libs):
    model = TINY["cnn"]
    w, X, y = _batch(model, 2, 7)
    l64, g64 = batch_loss_grad(model, w, X, y, "f64")
    l32, g32 = batch_loss_grad(model, w, X, y, "f32")
    assert l32 == pytest.approx(l64, rel=1e-5)
    assert np.abs(g32 - g64).max() <= 1e-5 * np.abs(g64).max()
