"""Pins for the oracle's local layer training step (loss and gradients of one
layer plus its temporary classifier, section "Lazy Message Passing").

Independent references: a hand-computed softmax example, closed forms, dense
matrix algebra with numpy's matmul, and numerical differentiation of the loss.
"""
import math

import numpy as np
import pytest

import oracle
from paper_2302_13053_amd import workloads as wl


def problem(n, d_in, h, c, seed, frac=0.7):
    rng = np.random.Generator(np.random.Philox(key=seed))
    X = wl.random_matrix(n, d_in, seed, ld=d_in + 3)
    X[:, d_in:] = 1e30
    y = rng.integers(0, c, n).astype(np.int32)
    y[rng.random(n) > frac] = -1
    W1 = (rng.standard_normal((d_in, h if h else c)) * 0.4).astype(np.float32)
    b1 = (rng.standard_normal(h if h else c) * 0.2).astype(np.float32)
    Wc = (rng.standard_normal((h, c)) * 0.4).astype(np.float32) if h else None
    bc = (rng.standard_normal(c) * 0.2).astype(np.float32) if h else None
    return X, y, W1, b1, Wc, bc


def test_hand_computed_single_node():
    # one node, no hidden layer, W = 0, bias = logits (1, 2, 3), label 2
    X = np.array([[0.5, -1.0]], np.float32)
    y = np.array([2], np.int32)
    W = np.zeros((2, 3), np.float32)
    b = np.array([1, 2, 3], np.float32)
    loss, gW, gb, _, _ = oracle.layer_grad(X, 2, y, W, b)
    e = [math.exp(1), math.exp(2), math.exp(3)]
    p = [t / sum(e) for t in e]
    assert abs(loss - (-math.log(p[2]))) < 1e-15 and abs(loss - 0.40760596444438046) < 1e-12
    assert np.allclose(gb, [p[0], p[1], p[2] - 1], rtol=1e-14)
    assert np.allclose(gW, np.outer([0.5, -1.0], [p[0], p[1], p[2] - 1]), rtol=1e-14)


def test_uniform_logits_give_log_c_and_unlabelled_nodes_do_not_count():
    X, y, W1, b1, Wc, bc = problem(50, 6, 5, 7, 1)
    loss, gW1, gb1, gWc, gbc = oracle.layer_grad(X, 6, y, W1, b1, np.zeros_like(Wc), np.zeros_like(bc))
    assert abs(loss - math.log(7)) < 1e-14
    assert np.all(gW1 == 0) and np.all(gb1 == 0)            # nothing flows back through a zero classifier
    # rows of unlabelled nodes may hold anything
    X2 = X.copy()
    X2[y < 0] = 123.0
    assert oracle.layer_grad(X2, 6, y, W1, b1, Wc, bc)[0] == oracle.layer_grad(X, 6, y, W1, b1, Wc, bc)[0]
    # no labelled node at all: zero loss and gradients
    none = np.full(50, -1, np.int32)
    out = oracle.layer_grad(X, 6, none, W1, b1, Wc, bc)
    assert out[0] == 0 and all(np.all(g == 0) for g in out[1:])


@pytest.mark.parametrize("h", [0, 5])
def test_matches_dense_matrix_algebra(h):
    n, d_in, c = 80, 9, 6
    X, y, W1, b1, Wc, bc = problem(n, d_in, h, c, 2)
    loss, gW1, gb1, gWc, gbc = oracle.layer_grad(X, d_in, y, W1, b1, Wc, bc)
    Xd = X[:, :d_in].astype(np.float64)
    lab = y >= 0
    Y = np.zeros((n, c))
    Y[lab, y[lab]] = 1
    if h:
        pre = Xd @ W1 + b1
        A = np.maximum(pre, 0)
        Z = A @ Wc + bc
    else:
        Z = Xd @ W1 + b1
    Z = Z - Z.max(1, keepdims=True)
    P = np.exp(Z) / np.exp(Z).sum(1, keepdims=True)
    nl = lab.sum()
    want_loss = -(np.log(P[lab, y[lab]])).sum() / nl
    dZ = (P - Y) * lab[:, None] / nl
    assert abs(loss - want_loss) < 1e-13
    if h:
        assert np.allclose(gWc, A.T @ dZ, atol=1e-14) and np.allclose(gbc, dZ.sum(0), atol=1e-14)
        dA = (dZ @ Wc.astype(np.float64).T) * (pre > 0)
        assert np.allclose(gW1, Xd.T @ dA, atol=1e-14) and np.allclose(gb1, dA.sum(0), atol=1e-14)
    else:
        assert np.allclose(gW1, Xd.T @ dZ, atol=1e-14) and np.allclose(gb1, dZ.sum(0), atol=1e-14)
        assert gWc is None and gbc is None


@pytest.mark.parametrize("h", [0, 4])
def test_gradient_is_the_derivative_of_the_loss(h):
    n, d_in, c = 30, 5, 3
    X, y, W1, b1, Wc, bc = problem(n, d_in, h, c, 3)
    _, gW1, gb1, gWc, gbc = oracle.layer_grad(X, d_in, y, W1, b1, Wc, bc)
    params = [W1.astype(np.float64), b1.astype(np.float64)]
    grads = [gW1, gb1]
    if h:
        params += [Wc.astype(np.float64), bc.astype(np.float64)]
        grads += [gWc, gbc]
    f = lambda ps: oracle.layer_loss(X, d_in, y, *ps) if h else oracle.layer_loss(X, d_in, y, ps[0], ps[1])
    eps = 1e-6
    for pi, (p, g) in enumerate(zip(params, grads)):
        for idx in np.ndindex(p.shape):
            hi = [q.copy() for q in params]
            lo = [q.copy() for q in params]
            hi[pi][idx] += eps
            lo[pi][idx] -= eps
            num = (f(hi) - f(lo)) / (2 * eps)
            assert abs(num - g[idx]) < 2e-8, (pi, idx, num, g[idx])


def test_structure_of_the_gradients():
    n, d_in, h, c = 120, 8, 6, 5
    X, y, W1, b1, Wc, bc = problem(n, d_in, h, c, 4)
    loss, gW1, gb1, gWc, gbc = oracle.layer_grad(X, d_in, y, W1, b1, Wc, bc)
    assert abs(gbc.sum()) < 1e-15                              # softmax minus one-hot sums to zero per node
    # all units dead (very negative bias): only the classifier bias learns
    dead = oracle.layer_grad(X, d_in, y, W1, np.full(h, -1e4, np.float32), Wc, bc)
    assert np.all(dead[1] == 0) and np.all(dead[2] == 0) and np.all(dead[3] == 0) and np.any(dead[4] != 0)
    # the mean is over labelled nodes: listing every node twice changes nothing
    X2 = np.concatenate([X, X])
    y2 = np.concatenate([y, y])
    twice = oracle.layer_grad(X2, d_in, y2, W1, b1, Wc, bc)
    assert abs(twice[0] - loss) < 1e-14 and np.allclose(twice[1], gW1, atol=1e-15)
    # a step against the gradient lowers the loss
    lr = 0.1
    new = oracle.layer_loss(X, d_in, y, W1 - lr * gW1, b1 - lr * gb1, Wc - lr * gWc, bc - lr * gbc)
    assert new < loss


@pytest.mark.parametrize("h", [0, 5])
def test_input_gradient_matches_dense_algebra_and_differences(h):
    """dL/dX, the gradient that flows back into an aggregation in front of the layer."""
    n, d_in, c = 40, 6, 4
    X, y, W1, b1, Wc, bc = problem(n, d_in, h, c, 6)
    out = oracle.layer_grad(X, d_in, y, W1, b1, Wc, bc, input_grad=True)
    gX = out[5]
    assert out[:1] == oracle.layer_grad(X, d_in, y, W1, b1, Wc, bc)[:1]
    Xd = X[:, :d_in].astype(np.float64)
    lab = y >= 0
    Y = np.zeros((n, c))
    Y[lab, y[lab]] = 1
    pre = Xd @ W1 + b1
    Z = (np.maximum(pre, 0) @ Wc + bc) if h else pre
    Z = Z - Z.max(1, keepdims=True)
    P = np.exp(Z) / np.exp(Z).sum(1, keepdims=True)
    dZ = (P - Y) * lab[:, None] / lab.sum()
    want = ((dZ @ Wc.astype(np.float64).T) * (pre > 0)) @ W1.astype(np.float64).T if h else dZ @ W1.astype(np.float64).T
    assert np.allclose(gX, want, atol=1e-14)
    assert np.all(gX[~lab] == 0) and np.abs(gX[lab]).min() > 0
    # central differences of the loss in perturbations that are exact in float32
    grid = np.float32(2.0 ** -12)
    Xq = X.copy()
    Xq[:, :d_in] = np.round(X[:, :d_in] / grid) * grid
    gXq = oracle.layer_grad(Xq, d_in, y, W1, b1, Wc, bc, input_grad=True)[5]
    f = lambda Xp: oracle.layer_loss(Xp, d_in, y, W1, b1, Wc, bc) if h else oracle.layer_loss(Xp, d_in, y, W1, b1)
    t = np.float32(2.0 ** -9)
    rng = np.random.Generator(np.random.Philox(key=4))
    for _ in range(4):
        D = np.zeros_like(Xq)
        D[:, :d_in] = rng.integers(-1, 2, (n, d_in))
        num = (f(Xq + t * D) - f(Xq - t * D)) / (2 * float(t))
        assert abs(num - (gXq * D[:, :d_in]).sum()) < 1e-6 * max(1.0, abs(num))


def test_transform_backward_is_the_transposed_product():
    n, d_in, d_out = 70, 9, 5
    H = wl.random_matrix(n, d_in, 1, ld=d_in + 2)
    dZ = wl.random_matrix(n, d_out, 2, ld=d_out + 3)
    H[:, d_in:] = 1e30
    dZ[:, d_out:] = 1e30
    gW, gb = oracle.transform_backward(H, d_in, dZ, d_out)
    assert np.allclose(gW, H[:, :d_in].astype(np.float64).T @ dZ[:, :d_out].astype(np.float64), rtol=1e-13, atol=1e-13)
    assert np.allclose(gb, dZ[:, :d_out].astype(np.float64).sum(0), rtol=1e-13, atol=1e-13)
    # adjoint of the oracle's own forward: <dZ, H W + b> = <gW, W> + <gb, b>
    W = wl.random_matrix(d_in, d_out, 3)
    b = wl.random_matrix(1, d_out, 4)[0]
    Z = oracle.transform(H, d_in, W, b)
    assert np.isclose((Z * dZ[:, :d_out]).sum(), (gW * W).sum() + (gb * b).sum(), rtol=1e-12)
