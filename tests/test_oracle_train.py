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


# ---------------------------------------------------------------------------
# dropout on the hidden units
# ---------------------------------------------------------------------------
def test_generator_reproduces_the_published_known_answers():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_known_answers.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        assert oracle.philox4x32_10(w[0:4], w[4:6]) == w[6:10]


def test_mask_is_a_function_of_seed_draw_node_and_unit():
    n, h = 300, 37                                    # 37: the last block of a row is used in part
    k = oracle.dropout_keep(n, h, 0.3, 1234, 5)
    assert k.dtype == np.uint8 and set(np.unique(k)) <= {0, 1}
    # definition, re-stated: word (j % 4) of block (v, j // 4, draw) under key seed, kept iff word >= floor(p 2^32)
    thr = int(np.float64(np.float32(0.3)) * 4294967296.0)
    for v, j in [(0, 0), (0, 3), (7, 4), (299, 36), (123, 18)]:
        word = oracle.philox4x32_10([v, j // 4, 5, 0], [1234, 0])[j % 4]
        assert k[v, j] == (word >= thr)
    # high words of seed and draw are used
    assert oracle.dropout_keep(4, 8, 0.5, (9 << 32) | 1234, 5)[0].tolist() == \
        [int(w >= 2 ** 31) for q in (0, 1) for w in oracle.philox4x32_10([0, q, 5, 0], [1234, 9])]
    assert oracle.dropout_keep(4, 8, 0.5, 1234, (3 << 32) | 5)[1].tolist() == \
        [int(w >= 2 ** 31) for q in (0, 1) for w in oracle.philox4x32_10([1, q, 5, 3], [1234, 0])]
    # a prefix of the nodes / another width leaves the shared blocks alone
    assert np.array_equal(oracle.dropout_keep(100, h, 0.3, 1234, 5), k[:100])
    assert np.array_equal(oracle.dropout_keep(n, 36, 0.3, 1234, 5), k[:, :36])
    # other draw or seed: another mask; p = 0 keeps all; the kept share is 1 - p
    assert not np.array_equal(oracle.dropout_keep(n, h, 0.3, 1234, 6), k)
    assert not np.array_equal(oracle.dropout_keep(n, h, 0.3, 1235, 5), k)
    assert oracle.dropout_keep(n, h, 0.0, 1234, 5).all()
    big = oracle.dropout_keep(4000, 64, 0.3, 77, 0)
    assert abs(big.mean() - 0.7) < 4 * math.sqrt(0.21 / big.size)
    assert abs(big.mean(0) - 0.7).max() < 0.04 and abs(big.mean(1) - 0.7).max() < 0.35
    # monotone in p: whoever survives p = 0.5 survives p = 0.3
    assert np.all(oracle.dropout_keep(n, h, 0.5, 1234, 5) <= k)


def test_dropout_matches_dense_matrix_algebra_with_the_same_mask():
    n, d_in, h, c = 90, 7, 10, 4
    X, y, W1, b1, Wc, bc = problem(n, d_in, h, c, 8)
    p = 0.4
    loss, gW1, gb1, gWc, gbc, gX = oracle.layer_grad(X, d_in, y, W1, b1, Wc, bc, input_grad=True,
                                                     dropout=(p, 42, 3))
    keep = oracle.dropout_keep(n, h, p, 42, 3).astype(np.float64)
    s = 1.0 / (1.0 - float(np.float32(p)))
    Xd = X[:, :d_in].astype(np.float64)
    lab = y >= 0
    Y = np.zeros((n, c))
    Y[lab, y[lab]] = 1
    pre = Xd @ W1 + b1
    A = np.maximum(pre, 0) * keep * s
    Z = A @ Wc + bc
    Z = Z - Z.max(1, keepdims=True)
    P = np.exp(Z) / np.exp(Z).sum(1, keepdims=True)
    nl = lab.sum()
    assert abs(loss - (-(np.log(P[lab, y[lab]])).sum() / nl)) < 1e-13
    dZ = (P - Y) * lab[:, None] / nl
    assert np.allclose(gWc, A.T @ dZ, atol=1e-14) and np.allclose(gbc, dZ.sum(0), atol=1e-14)
    dpre = (dZ @ Wc.astype(np.float64).T) * keep * s * (pre > 0)
    assert np.allclose(gW1, Xd.T @ dpre, atol=1e-14) and np.allclose(gb1, dpre.sum(0), atol=1e-14)
    assert np.allclose(gX, dpre @ W1.astype(np.float64).T, atol=1e-14)
    # p = 0 is the step without dropout, bit for bit
    plain = oracle.layer_grad(X, d_in, y, W1, b1, Wc, bc)
    zero = oracle.layer_grad(X, d_in, y, W1, b1, Wc, bc, dropout=(0.0, 42, 3))
    assert plain[0] == zero[0] and all(np.array_equal(a, b) for a, b in zip(plain[1:], zero[1:]))
    # ... and differs from it for p > 0
    assert abs(loss - plain[0]) > 1e-4


def test_dropout_gradient_is_the_derivative_of_the_loss_with_the_mask_held_fixed():
    n, d_in, h, c = 30, 5, 6, 3
    X, y, W1, b1, Wc, bc = problem(n, d_in, h, c, 9)
    drop = (0.5, 7, 11)
    _, gW1, gb1, gWc, gbc = oracle.layer_grad(X, d_in, y, W1, b1, Wc, bc, dropout=drop)
    params = [W1.astype(np.float64), b1.astype(np.float64), Wc.astype(np.float64), bc.astype(np.float64)]
    grads = [gW1, gb1, gWc, gbc]
    f = lambda ps: oracle.layer_loss(X, d_in, y, *ps, dropout=drop)
    eps = 1e-6
    for pi, (p, g) in enumerate(zip(params, grads)):
        for idx in np.ndindex(p.shape):
            hi = [q.copy() for q in params]
            lo = [q.copy() for q in params]
            hi[pi][idx] += eps
            lo[pi][idx] -= eps
            num = (f(hi) - f(lo)) / (2 * eps)
            assert abs(num - g[idx]) < 2e-8, (pi, idx, num, g[idx])


def test_dropout_keeps_the_expected_activation():
    # E[A] over the draws is the plain activation: the mean loss gradient of the classifier bias over many
    # draws approaches the one without dropout when the classifier is linear in A (zero Wc rows but one)
    n, d_in, h, c = 40, 4, 8, 3
    X, y, W1, b1, Wc, bc = problem(n, d_in, h, c, 10)
    keep = np.stack([oracle.dropout_keep(n, h, 0.25, 5, d) for d in range(400)]).astype(np.float64)
    s = 1.0 / (1.0 - 0.25)
    assert abs((keep * s).mean() - 1.0) < 0.01
    assert abs((keep * s).mean(0) - 1.0).max() < 0.15


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
