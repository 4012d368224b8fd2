"""Pins for the oracle's aggregation backward (no GPU).

None of these retypes the oracle's chain rule: they use torch's automatic differentiation of a
dense float64 formulation, numerical differencing of the oracle's own (separately pinned) forward,
hand-derived closed forms on a three-node star, dense transposed matrix algebra and invariants.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2302_13053_amd import workloads as wl

LINEAR = ["mean", "sum", "gcn_sym"]


def directed_csr(n, m, seed, self_loops=False):
    """A random *asymmetric* CSR (sorted unique columns): the backward must not lean on symmetry."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    A = np.zeros((n, n), bool)
    A[rng.integers(0, n, m), rng.integers(0, n, m)] = True
    np.fill_diagonal(A, self_loops)
    A[n // 2] = False                         # an empty row
    A[:, n // 3] = False                      # and a node nobody points at
    if self_loops:
        np.fill_diagonal(A, True)
    rp = np.concatenate([[0], np.cumsum(A.sum(1))]).astype(np.int64)
    ci = np.nonzero(A)[1].astype(np.int32)
    return A, rp, ci


def dense_forward_torch(mode, A, Z, a_src, a_dst, heads, slope, concat):
    """Dense float64 forward written with torch ops so that autograd can differentiate it."""
    At = torch.from_numpy(A.astype(np.float64))
    n, F = Z.shape
    deg = At.sum(1)
    if mode == "sum":
        agg = At @ Z
    elif mode == "mean":
        agg = (At @ Z) / torch.clamp(deg, min=1.0)[:, None]
    elif mode == "gcn_sym":
        # the oracle defines dinv as a float32 quantity; reproduce that rounding here
        dinv = np.where(deg.numpy() > 0, np.float32(1.0) / np.sqrt(deg.numpy().astype(np.float32)), 0).astype(np.float32)
        d = torch.from_numpy(dinv.astype(np.float64))
        agg = d[:, None] * (At @ (d[:, None] * Z))
    else:
        Dh = F // heads
        Zh = Z.view(n, heads, Dh)
        el = (Zh * a_src[None]).sum(-1)                       # [n, heads]  source score
        er = (Zh * a_dst[None]).sum(-1)                       # [n, heads]  destination score
        p = el[None, :, :] + er[:, None, :]                   # [v, u, h]
        e = torch.nn.functional.leaky_relu(p, slope)
        e = e.masked_fill(~torch.from_numpy(A)[:, :, None], -float("inf"))
        alpha = torch.softmax(e, dim=1)
        alpha = torch.nan_to_num(alpha, nan=0.0)              # empty rows
        agg = torch.einsum("vuh,uhd->vhd", alpha, Zh).reshape(n, F)
    return torch.cat([Z, agg], 1) if concat else agg


@pytest.mark.parametrize("mode", LINEAR + ["gat_softmax"])
@pytest.mark.parametrize("concat", [False, True])
def test_backward_matches_autograd_of_dense_formulation(mode, concat):
    n, F, heads, slope = 23, 12, 3, 0.2
    A, rp, ci = directed_csr(n, 90, seed=5, self_loops=(mode == "gcn_sym"))
    Z32 = wl.random_matrix(n, F, 11)
    G32 = wl.random_matrix(n, 2 * F if concat else F, 12)
    a_s = wl.random_matrix(heads, F // heads, 13) * np.float32(0.7)
    a_d = wl.random_matrix(heads, F // heads, 14) * np.float32(0.7)
    Z = torch.from_numpy(Z32.astype(np.float64)).requires_grad_(True)
    ts = torch.from_numpy(a_s.astype(np.float64)).requires_grad_(True)
    td = torch.from_numpy(a_d.astype(np.float64)).requires_grad_(True)
    out = dense_forward_torch(mode, A, Z, ts, td, heads, slope, concat)
    # the dense forward itself agrees with the oracle's forward
    want_fwd = oracle.aggregate(mode, rp, ci, Z32, F, heads=heads, a_src=a_s, a_dst=a_d, slope=slope, self_concat=concat)
    assert np.allclose(out.detach().numpy(), want_fwd, rtol=1e-12, atol=1e-12)
    (out * torch.from_numpy(G32.astype(np.float64))).sum().backward()
    got = oracle.aggregate_backward(mode, rp, ci, Z32, F, G32, heads=heads, a_src=a_s, a_dst=a_d,
                                    slope=slope, self_concat=concat)
    if mode == "gat_softmax":
        dZ, das, dad = got
        assert np.allclose(das, ts.grad.numpy(), rtol=1e-11, atol=1e-12)
        assert np.allclose(dad, td.grad.numpy(), rtol=1e-11, atol=1e-12)
        assert np.abs(das).max() > 1e-3 and np.abs(dad).max() > 1e-3
    else:
        dZ = got
    assert np.allclose(dZ, Z.grad.numpy(), rtol=1e-11, atol=1e-12)
    # a subset of rows gives the same rows
    rows = np.array([0, n // 3, n // 2, n - 1], np.int64)
    sub = oracle.aggregate_backward(mode, rp, ci, Z32, F, G32, heads=heads, a_src=a_s, a_dst=a_d,
                                    slope=slope, self_concat=concat, rows=rows)
    sub = sub[0] if mode == "gat_softmax" else sub
    assert np.array_equal(sub, dZ[rows])


def test_gat_backward_matches_differences_of_the_oracle_forward():
    """Directional derivatives of L = <G, forward(Z, a_src, a_dst)> by Richardson-extrapolated central
    differences of the oracle's forward, with perturbations that are exact in float32."""
    n, F, heads, slope = 40, 8, 2, 0.2
    src, dst = wl.random_pairs(n, 120, 3, skew=1.0)
    rp, ci = oracle.csr_from_coo(src, dst, n, False)
    grid = np.float32(2.0 ** -10)
    q = lambda a: (np.round(a / grid) * grid).astype(np.float32)
    Z, G = q(wl.random_matrix(n, F, 21)), wl.random_matrix(n, F, 22)
    a_s, a_d = q(wl.random_matrix(heads, F // heads, 23)), q(wl.random_matrix(heads, F // heads, 24))
    dZ, das, dad = oracle.aggregate_backward("gat_softmax", rp, ci, Z, F, G, heads=heads, a_src=a_s, a_dst=a_d, slope=slope)

    def loss(Zp, sp, dp):
        out = oracle.aggregate("gat_softmax", rp, ci, Zp, F, heads=heads, a_src=sp, a_dst=dp, slope=slope)
        return float((out * G.astype(np.float64)).sum())

    rng = np.random.Generator(np.random.Philox(key=8))
    for trial in range(3):
        dirZ = rng.integers(-2, 3, Z.shape).astype(np.float32)
        dirs = rng.integers(-2, 3, a_s.shape).astype(np.float32)
        dird = rng.integers(-2, 3, a_d.shape).astype(np.float32)
        want = float((dZ * dirZ).sum() + (das * dirs).sum() + (dad * dird).sum())
        est = []
        for t in (np.float32(2.0 ** -15), np.float32(2.0 ** -16)):   # small: the score has a kink at zero
            up = loss(Z + t * dirZ, a_s + t * dirs, a_d + t * dird)
            dn = loss(Z - t * dirZ, a_s - t * dirs, a_d - t * dird)
            est.append((up - dn) / (2.0 * float(t)))
        rich = (4.0 * est[1] - est[0]) / 3.0
        assert abs(rich - want) <= 2e-6 * max(1.0, abs(want)), (trial, rich, want)


def test_closed_form_on_a_three_node_star():
    """Centre 0 with leaves 1, 2, one head of width one.  Leaves have a single neighbour, so their
    softmax is constant; the centre's two-way softmax is a logistic function, whose derivative
    alpha_1 alpha_2 is written out by hand below."""
    rp = np.array([0, 2, 3, 4], np.int64)
    ci = np.array([1, 2, 0, 0], np.int32)
    z = np.array([[0.5], [-1.25], [0.75]], np.float32)
    g = np.array([[2.0], [-3.0], [0.5]], np.float32)
    a, b, slope = np.float32(0.8), np.float32(-0.6), 0.1
    dZ, da, db = oracle.aggregate_backward("gat_softmax", rp, ci, z, 1, g, heads=1, a_src=np.array([[a]]),
                                           a_dst=np.array([[b]]), slope=slope)
    z0, z1, z2 = (float(x) for x in z[:, 0])
    g0, g1, g2 = (float(x) for x in g[:, 0])
    a, b = float(a), float(b)
    p1, p2 = a * z1 + b * z0, a * z2 + b * z0             # -1.3 and 0.3: one on each side of the kink
    assert p1 < 0 < p2
    l1, l2 = slope, 1.0
    e1, e2 = slope * p1, p2
    al1 = 1.0 / (1.0 + np.exp(e2 - e1))
    al2 = 1.0 - al1
    k = g0 * (z1 - z2) * al1 * al2
    want_dz = [g1 + g2 + k * (l1 - l2) * b, g0 * al1 + k * l1 * a, g0 * al2 - k * l2 * a]
    assert np.allclose(dZ[:, 0], want_dz, rtol=1e-13, atol=0)
    assert np.isclose(da[0, 0], k * (l1 * z1 - l2 * z2), rtol=1e-13)
    assert np.isclose(db[0, 0], k * (l1 - l2) * z0, rtol=1e-13)


@pytest.mark.parametrize("mode", LINEAR)
@pytest.mark.parametrize("concat", [False, True])
def test_linear_backward_is_the_transposed_operator(mode, concat):
    n, F = 31, 7
    A, rp, ci = directed_csr(n, 140, seed=9, self_loops=(mode == "gcn_sym"))
    G = wl.random_matrix(n, 2 * F if concat else F, 5)
    Z = wl.random_matrix(n, F, 6)
    deg = A.sum(1).astype(np.float64)
    M = A.astype(np.float64)
    if mode == "mean":
        M = M / np.maximum(deg, 1.0)[:, None]
    elif mode == "gcn_sym":
        _, dinv = oracle.degree(rp)
        M = dinv.astype(np.float64)[:, None] * M * dinv.astype(np.float64)[None, :]
    Ga = G[:, F:] if concat else G
    want = M.T @ Ga.astype(np.float64) + (G[:, :F].astype(np.float64) if concat else 0.0)
    got = oracle.aggregate_backward(mode, rp, ci, Z, F, G, self_concat=concat)
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13)
    assert not np.allclose(M, M.T)                              # the graph really is asymmetric
    # adjoint identity against the oracle's own forward: <G, forward(Z)> = <backward(G), Z>
    fwd = oracle.aggregate(mode, rp, ci, Z, F, self_concat=concat)
    assert np.isclose((fwd * G.astype(np.float64)).sum(), (got * Z.astype(np.float64)).sum(), rtol=1e-12)


def test_gat_invariants():
    n, F, heads = 60, 12, 3
    src, dst = wl.random_pairs(n, 200, 4, skew=1.5)
    rp, ci = oracle.csr_from_coo(src, dst, n, False)
    deg = np.diff(rp)
    Z, G = wl.random_matrix(n, F, 1), wl.random_matrix(n, F, 2)
    a_s, a_d = wl.random_matrix(heads, F // heads, 3), wl.random_matrix(heads, F // heads, 4)
    # slope 1 makes the score linear, and a softmax does not see a shift common to a row:
    # the destination vector then has no influence at all
    dZ1, das1, dad1 = oracle.aggregate_backward("gat_softmax", rp, ci, Z, F, G, heads=heads, a_src=a_s, a_dst=a_d, slope=1.0)
    assert np.abs(dad1).max() <= 1e-13 * np.abs(das1).max()
    dZ1b, das1b, _ = oracle.aggregate_backward("gat_softmax", rp, ci, Z, F, G, heads=heads, a_src=a_s, a_dst=3 * a_d, slope=1.0)
    assert np.allclose(dZ1, dZ1b, rtol=1e-10, atol=1e-12) and np.allclose(das1, das1b, rtol=1e-10, atol=1e-12)
    # the gradient is linear in G
    dZ, das, dad = oracle.aggregate_backward("gat_softmax", rp, ci, Z, F, G, heads=heads, a_src=a_s, a_dst=a_d)
    dZ2, das2, dad2 = oracle.aggregate_backward("gat_softmax", rp, ci, Z, F, 2 * G, heads=heads, a_src=a_s, a_dst=a_d)
    assert np.allclose(2 * dZ, dZ2, rtol=1e-12) and np.allclose(2 * das, das2, rtol=1e-12) and np.allclose(2 * dad, dad2, rtol=1e-12)
    # identical feature rows: every alpha is 1/deg and out does not move with the parameters,
    # so nothing reaches a_src, a_dst
    ones = np.ones((n, 3), np.float32)
    _, dsa, dda = oracle.aggregate_backward("gat_softmax", rp, ci, ones, 3, wl.random_matrix(n, 3, 8), heads=3,
                                            a_src=wl.random_matrix(3, 1, 9), a_dst=wl.random_matrix(3, 1, 10))
    assert np.abs(dsa).max() <= 1e-12 and np.abs(dda).max() <= 1e-12
    # zero attention vectors: alpha = 1/deg, so dZ is the mean's backward plus nothing through the scores
    zero = np.zeros((heads, F // heads), np.float32)
    dZ0, _, _ = oracle.aggregate_backward("gat_softmax", rp, ci, Z, F, G, heads=heads, a_src=zero, a_dst=zero)
    assert np.allclose(dZ0, oracle.aggregate_backward("mean", rp, ci, Z, F, G), rtol=1e-12, atol=1e-13)
    # nodes of degree zero receive nothing and send nothing
    assert (deg == 0).any()
    assert np.all(dZ[deg == 0] == 0.0)


def test_max_has_no_backward():
    rp = np.array([0, 1, 2], np.int64)
    ci = np.array([1, 0], np.int32)
    with pytest.raises(ValueError):
        oracle.aggregate_backward("max", rp, ci, np.ones((2, 2), np.float32), 2, np.ones((2, 2), np.float32))


def test_attention_layer_chain_matches_end_to_end_autograd():
    """A whole locally trained attention layer, composed from the oracle's pieces the way the GPU path
    composes its entry points — transform, edge-softmax aggregation, dense layer + temporary classifier
    + loss, and back: input gradient, aggregation backward, transform backward — against torch autograd
    of the same network written densely in float64.  (The pieces hand float32 tables to each other,
    hence the 1e-5 tolerance.)"""
    n, d_in, F, heads, Hd, C, slope = 30, 7, 12, 3, 6, 4, 0.2
    src, dst = wl.random_pairs(n, 80, 6, skew=1.0)
    rp, ci = oracle.csr_from_coo(src, dst, n, False)
    A = np.zeros((n, n), bool)
    A[np.repeat(np.arange(n), np.diff(rp)), ci] = True
    rng = np.random.Generator(np.random.Philox(key=12))
    Q = wl.random_matrix(n, d_in, 1)
    Wg = (rng.standard_normal((d_in, F)) * 0.4).astype(np.float32)
    bg = (rng.standard_normal(F) * 0.1).astype(np.float32)
    a_s = (rng.standard_normal((heads, F // heads)) * 0.5).astype(np.float32)
    a_d = (rng.standard_normal((heads, F // heads)) * 0.5).astype(np.float32)
    W1 = (rng.standard_normal((F, Hd)) * 0.4).astype(np.float32)
    b1 = (rng.standard_normal(Hd) * 0.1).astype(np.float32)
    Wc = (rng.standard_normal((Hd, C)) * 0.4).astype(np.float32)
    bc = (rng.standard_normal(C) * 0.1).astype(np.float32)
    y = rng.integers(0, C, n).astype(np.int32)
    y[rng.random(n) > 0.7] = -1
    # the oracle's chain
    Z = oracle.transform(Q, d_in, Wg, bg).astype(np.float32)
    X = oracle.aggregate("gat_softmax", rp, ci, Z, F, heads=heads, a_src=a_s, a_dst=a_d, slope=slope).astype(np.float32)
    loss, gW1, gb1, gWc, gbc, gX = oracle.layer_grad(X, F, y, W1, b1, Wc, bc, input_grad=True)
    dZ, das, dad = oracle.aggregate_backward("gat_softmax", rp, ci, Z, F, gX.astype(np.float32), heads=heads,
                                             a_src=a_s, a_dst=a_d, slope=slope)
    gWg, gbg = oracle.transform_backward(Q, d_in, dZ.astype(np.float32), F)
    # the same network, dense, float64, differentiated by torch
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64)).requires_grad_(True)
    tWg, tbg, tas, tad, tW1, tb1, tWc, tbc = (t(a) for a in (Wg, bg, a_s, a_d, W1, b1, Wc, bc))
    tZ = torch.from_numpy(Q.astype(np.float64)) @ tWg + tbg
    tX = dense_forward_torch("gat_softmax", A, tZ, tas, tad, heads, slope, False)
    logits = torch.relu(tX @ tW1 + tb1) @ tWc + tbc
    lab = torch.from_numpy(y >= 0)
    tl = torch.nn.functional.cross_entropy(logits[lab], torch.from_numpy(y.astype(np.int64))[lab])
    tl.backward()
    assert abs(loss - float(tl.detach())) < 1e-6
    for got, ref, name in ((gWg, tWg, "W_g"), (gbg, tbg, "b_g"), (das, tas, "a_src"), (dad, tad, "a_dst"),
                           (gW1, tW1, "W1"), (gb1, tb1, "b1"), (gWc, tWc, "Wc"), (gbc, tbc, "bc")):
        ref = ref.grad.numpy()
        assert np.abs(ref).max() > 1e-4, name
        assert np.abs(got - ref).max() <= 1e-5 * np.abs(ref).max(), name


def test_kink_slack_is_the_jump_across_the_leaky_relu_kink():
    """An entry whose score is exactly zero sits on the kink of LeakyReLU; the slack output must be the size of
    the jump dZ makes when that score moves from just below to just above zero, on the two rows the entry
    touches, and zero on every other row.  (Pins oracle_aggregate_backward_slack against the oracle's own
    gradient on perturbed inputs: the jump is a property of the definition, not of the slack code.)"""
    n, F = 7, 2
    src = np.array([0, 0, 1, 2, 3, 4, 5], np.int32)
    dst = np.array([1, 2, 2, 3, 4, 5, 6], np.int32)
    rp, ci = oracle.csr_from_coo(src, dst, n, False)
    rng = np.random.Generator(np.random.Philox(key=91))
    Z = rng.standard_normal((n, F)).astype(np.float32)
    G = rng.standard_normal((n, F)).astype(np.float32)
    a_src = np.array([[1.0, 0.0]], np.float32)
    a_dst = np.array([[0.0, 1.0]], np.float32)
    v, u = 2, 3                              # entry (v, u): p = z_u[0] + z_v[1]
    Z[v, 1] = -0.5
    Z[u, 0] = 0.5
    kw = dict(heads=1, a_src=a_src, a_dst=a_dst, slope=0.2)
    dZ, _, _, slack = oracle.aggregate_backward("gat_softmax", rp, ci, Z, F, G, kink_rel=1e-9, **kw)
    assert np.array_equal(dZ, oracle.aggregate_backward("gat_softmax", rp, ci, Z, F, G, **kw)[0])
    eps = np.float32(2.0 ** -20)
    Zp, Zm = Z.copy(), Z.copy()
    Zp[u, 0] += eps
    Zm[u, 0] -= eps
    jump = np.abs(oracle.aggregate_backward("gat_softmax", rp, ci, Zp, F, G, **kw)[0]
                  - oracle.aggregate_backward("gat_softmax", rp, ci, Zm, F, G, **kw)[0])
    touched = np.zeros(n, bool)
    touched[[u, v]] = True
    assert np.all(slack[~touched] == 0.0)
    assert slack[u, 0] > 1e-3 and slack[v, 1] > 1e-3          # through a_src into row u, through a_dst into row v
    assert slack[u, 1] == 0.0 and slack[v, 0] == 0.0          # the zero components of the attention vectors
    assert np.allclose(slack[touched], jump[touched], rtol=0, atol=2e-5)
    assert np.all(jump[~touched] <= 2e-5)
    # no undecided entry: no slack; a wide band makes every entry undecided; modes without a kink have none
    Z2 = Z.copy()
    Z2[u, 0] = 0.75
    assert np.all(oracle.aggregate_backward("gat_softmax", rp, ci, Z2, F, G, kink_rel=1e-9, **kw)[3] == 0.0)
    wide = oracle.aggregate_backward("gat_softmax", rp, ci, Z2, F, G, kink_rel=10.0, **kw)[3]
    assert np.all(wide[:, 0][np.diff(rp) > 0] > 0)
    lin = oracle.aggregate_backward("mean", rp, ci, Z, F, G, kink_rel=1.0)
    assert np.all(lin[1] == 0.0)
