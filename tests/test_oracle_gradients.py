"""Pins for oracle/gradients.py: closed forms, finite differences of the loss,
and autograd of an independently written loss (torch CPU, fp64)."""
import numpy as np
import pytest
import torch

from oracle import gradients as og

RNG = np.random.default_rng(7)


def _fd(loss, theta, eps=1e-6):
    g = np.zeros_like(theta)
    for i in range(theta.size):
        e = np.zeros_like(theta)
        e[i] = eps
        g[i] = (loss(theta + e) - loss(theta - e)) / (2 * eps)
    return g


def _data(rows=50, d=7):
    X = RNG.standard_normal((rows, d))
    th = RNG.standard_normal(d)
    return X, th


def test_lsq_at_zero_is_minus_XTy():
    X, _ = _data()
    y = RNG.standard_normal(50)
    g = og.lsq_gradient(X, y, np.zeros(7))
    expect = -sum(y[i] * X[i] for i in range(50))
    assert np.allclose(g, expect, rtol=1e-12, atol=1e-12)


def test_lsq_vanishes_at_normal_equation_solution():
    X, _ = _data()
    y = RNG.standard_normal(50)
    th = np.linalg.lstsq(X, y, rcond=None)[0]
    assert np.linalg.norm(og.lsq_gradient(X, y, th)) < 1e-10 * np.linalg.norm(X.T @ y)


def test_lsq_finite_differences():
    X, th = _data()
    y = RNG.standard_normal(50)
    fd = _fd(lambda t: og.lsq_loss(X, y, t), th)
    assert np.allclose(og.lsq_gradient(X, y, th), fd, rtol=1e-6, atol=1e-6)


def test_lsq_autograd():
    X, th = _data()
    y = RNG.standard_normal(50)
    t = torch.tensor(th, requires_grad=True)
    loss = 0.5 * ((torch.tensor(X) @ t - torch.tensor(y)) ** 2).sum()
    loss.backward()
    assert np.allclose(og.lsq_gradient(X, y, th), t.grad.numpy(), rtol=1e-11, atol=1e-11)


def test_logistic_at_zero_is_minus_half_sum_yx():
    X, _ = _data()
    y = np.where(RNG.standard_normal(50) > 0, 1.0, -1.0)
    g = og.logistic_gradient(X, y, np.zeros(7))
    expect = -0.5 * sum(y[i] * X[i] for i in range(50))
    assert np.allclose(g, expect, rtol=1e-12, atol=1e-12)


def test_logistic_finite_differences_and_autograd():
    X, th = _data()
    y = np.where(RNG.standard_normal(50) > 0, 1.0, -1.0)
    g = og.logistic_gradient(X, y, th)
    fd = _fd(lambda t: og.logistic_loss(X, y, t), th)
    assert np.allclose(g, fd, rtol=1e-6, atol=1e-6)
    t = torch.tensor(th, requires_grad=True)
    loss = torch.nn.functional.softplus(-torch.tensor(y) * (torch.tensor(X) @ t)).sum()
    loss.backward()
    assert np.allclose(g, t.grad.numpy(), rtol=1e-11, atol=1e-11)


def test_logistic_saturated_margins_do_not_overflow():
    X = np.array([[1000.0, 0.0], [-1000.0, 0.0]])
    y = np.array([1.0, 1.0])
    g = og.logistic_gradient(X, y, np.array([1.0, 0.0]))
    # first row: margin +1000 -> weight 0; second: margin -1000 -> weight 1
    assert np.all(np.isfinite(g))
    assert np.allclose(g, [1000.0, 0.0])


def _mlp_case(rows=12, d_in=8, hidden=6, classes=3):
    X = RNG.random((rows, d_in))
    labels = RNG.integers(0, classes, rows)
    th = 0.5 * RNG.standard_normal(d_in * hidden + hidden + hidden * classes + classes)
    return X, labels, th, hidden, classes


def test_mlp_finite_differences():
    X, labels, th, h, c = _mlp_case()
    g = og.mlp2_gradient(X, labels, th, h, c)
    fd = _fd(lambda t: og.mlp2_loss(X, labels, t, h, c), th)
    assert np.allclose(g, fd, rtol=1e-5, atol=1e-6)


def test_mlp_autograd_layout():
    X, labels, th, h, c = _mlp_case()
    d_in = X.shape[1]
    t = torch.tensor(th, requires_grad=True)
    o = 0
    W1 = t[o:o + d_in * h].reshape(d_in, h); o += d_in * h
    b1 = t[o:o + h]; o += h
    W2 = t[o:o + h * c].reshape(h, c); o += h * c
    b2 = t[o:o + c]
    H = torch.relu(torch.tensor(X) @ W1 + b1)
    loss = torch.nn.functional.cross_entropy(H @ W2 + b2, torch.tensor(labels), reduction="sum")
    loss.backward()
    assert np.allclose(og.mlp2_gradient(X, labels, th, h, c), t.grad.numpy(),
                       rtol=1e-10, atol=1e-11)
    assert np.isclose(og.mlp2_loss(X, labels, th, h, c), loss.item(), rtol=1e-12)


@pytest.mark.parametrize("loss", [0, 1, 2])
def test_partial_gradients_add_up_to_full_batch_gradient(loss):
    """g = sum_i g_i, a sum and not a mean (Sec. II-B eq. (1), Sec. II-C)."""
    k, rows = 4, 9
    if loss == 2:
        X, labels, th, h, c = _mlp_case(rows=k * rows)
        Y = labels
        full = og.mlp2_gradient(X, Y, th, h, c)
        fdl = lambda t: og.mlp2_loss(X, Y, t, h, c)
    else:
        X = RNG.standard_normal((k * rows, 5))
        th = RNG.standard_normal(5)
        Y = np.where(RNG.standard_normal(k * rows) > 0, 1.0, -1.0)
        h = c = 0
        full = (og.lsq_gradient if loss == 0 else og.logistic_gradient)(X, Y, th)
        fdl = lambda t: (og.lsq_loss if loss == 0 else og.logistic_loss)(X, Y, t)
    G = og.partial_gradients(loss, X.reshape(k, rows, -1), Y.reshape(k, rows), th, h, c)
    assert G.shape == (k, th.size)
    assert np.allclose(G.sum(axis=0), full, rtol=1e-11, atol=1e-11)
    # and the full-batch loss differentiates to it (no 1/m anywhere)
    assert np.allclose(G.sum(axis=0), _fd(fdl, th), rtol=1e-5, atol=1e-5)


def test_gd_update_rule():
    th = np.array([1.0, 2.0])
    g = np.array([10.0, -20.0])
    assert np.allclose(og.gd_update(th, g, eta=0.5, m=10), [0.5, 3.0])
