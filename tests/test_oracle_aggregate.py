"""Pins for the oracle's aggregators (the AGGR of Eq. 1 in the four modes).

Independent references used here: a hand-computed worked example
(tests/golden/four_node_example.txt), dense-adjacency matrix algebra done with
numpy in float64, closed forms on regular graphs, and invariants.
"""
import os

import numpy as np
import pytest

import oracle
from paper_2302_13053_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "four_node_example.txt")
MODES = ["sum", "mean", "gcn_sym", "gat_softmax"]
ALL_MODES = MODES + ["max"]


def small_graph(n, pairs, seed, self_loops, skew=1.0):
    src, dst = wl.random_pairs(n, pairs, seed, skew=skew)
    return oracle.csr_from_coo(src, dst, n, self_loops)


def dense(row_ptr, col, n):
    a = np.zeros((n, n))
    for v in range(n):
        a[v, col[row_ptr[v]:row_ptr[v + 1]]] = 1.0
    return a


def leaky(x, s=0.2):
    return np.where(x > 0, x, s * x)


def dense_reference(mode, a, Z, heads=1, a_src=None, a_dst=None, slope=0.2):
    """Matrix-algebra form of each aggregator on a dense 0/1 adjacency ``a``."""
    Z = Z.astype(np.float64)
    deg = a.sum(1)
    if mode == "sum":
        return a @ Z
    if mode == "mean":
        return (a @ Z) / np.maximum(deg, 1)[:, None]
    if mode == "gcn_sym":
        s = np.where(deg > 0, 1 / np.sqrt(np.maximum(deg, 1)), 0)
        return (s[:, None] * a * s[None, :]) @ Z
    n, F = Z.shape
    dh = F // heads
    out = np.zeros((n, F))
    for h in range(heads):
        Zh = Z[:, h * dh:(h + 1) * dh]
        el = Zh @ a_src[h].astype(np.float64)
        er = Zh @ a_dst[h].astype(np.float64)
        e = leaky(er[:, None] + el[None, :], slope)          # e[v, u]
        e = np.where(a > 0, e, -np.inf)
        m = np.where(deg > 0, e.max(1, initial=-np.inf), 0)
        p = np.where(a > 0, np.exp(e - m[:, None]), 0)
        alpha = p / np.maximum(p.sum(1), 1e-300)[:, None]
        out[:, h * dh:(h + 1) * dh] = alpha @ Zh
    return out


def test_hand_computed_example():
    src = np.array([0, 0, 1, 2], np.int32)
    dst = np.array([1, 2, 2, 3], np.int32)
    Z = np.array([[1, 2], [3, -1], [0, 4], [-2, 1]], np.float32)
    a_src = np.array([[1, 0]], np.float32)
    a_dst = np.array([[0, 1]], np.float32)
    want = {}
    alpha = None
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        tok = line.split()
        if tok[0] == "alpha":
            alpha = (int(tok[1]), np.array([float(t) for t in tok[2:]]))
        else:
            want.setdefault(tok[0], {})[int(tok[1])] = [float(tok[2]), float(tok[3])]
    mags = {k[4:]: want.pop(k) for k in list(want) if k.startswith("abs_")}
    assert sorted(want) == sorted(MODES) and all(len(v) == 4 for v in want.values())
    # the size of the terms behind each element (oracle.aggregate_abs), rows the file lists
    assert sorted(mags) == sorted(MODES)
    for mode, rows in mags.items():
        rp, ci = oracle.csr_from_coo(src, dst, 4, mode == "gcn_sym")
        got = oracle.aggregate_abs(mode, rp, ci, Z, 2, heads=1, a_src=a_src, a_dst=a_dst)
        tol = 2e-7 if mode == "gcn_sym" else 1e-15
        for v, ref in rows.items():
            assert np.allclose(got[v], ref, rtol=tol, atol=tol), (mode, v)
    for mode in MODES:
        rp, ci = oracle.csr_from_coo(src, dst, 4, mode == "gcn_sym")
        got = oracle.aggregate(mode, rp, ci, Z, 2, heads=1, a_src=a_src, a_dst=a_dst)
        ref = np.array([want[mode][v] for v in range(4)])
        # gcn_sym's normaliser is single precision by definition, hence the looser bound there
        tol = 2e-7 if mode == "gcn_sym" else 1e-15
        assert np.allclose(got, ref, rtol=tol, atol=tol), mode
    rp, ci = oracle.csr_from_coo(src, dst, 4, False)
    got = oracle.gat_alpha(alpha[0], 0, rp, ci, Z, 2, 1, a_src, a_dst)
    assert np.allclose(got, alpha[1], rtol=1e-15, atol=1e-15)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("n,pairs,F,heads,seed", [(23, 60, 6, 2, 1), (40, 400, 12, 3, 2), (9, 3, 4, 1, 3)])
def test_matches_dense_matrix_algebra(mode, n, pairs, F, heads, seed):
    rp, ci = small_graph(n, pairs, seed, mode == "gcn_sym")
    Z = wl.random_matrix(n, F, seed + 10, ld=F + 3)
    Z[:, F:] = 1e30
    a_src = wl.random_matrix(heads, F // heads, seed + 20)
    a_dst = wl.random_matrix(heads, F // heads, seed + 30)
    got = oracle.aggregate(mode, rp, ci, Z, F, heads=heads, a_src=a_src, a_dst=a_dst)
    ref = dense_reference(mode, dense(rp, ci, n), Z[:, :F], heads, a_src, a_dst)
    tol = 3e-7 if mode == "gcn_sym" else 1e-12
    assert np.allclose(got, ref, rtol=tol, atol=tol * np.abs(ref).max())


def test_max_pool_aggregator():
    # hand example on the four-node graph 0-1, 0-2, 1-2, 2-3 (same rows as the golden file)
    src = np.array([0, 0, 1, 2], np.int32)
    dst = np.array([1, 2, 2, 3], np.int32)
    Z = np.array([[1, 2], [3, -1], [0, 4], [-2, 1]], np.float32)
    rp, ci = oracle.csr_from_coo(src, dst, 4, False)
    assert np.array_equal(oracle.aggregate("max", rp, ci, Z, 2), [[3, 4], [1, 4], [3, 2], [0, 4]])
    # dense masked maximum with numpy on random graphs; empty rows give zero
    n = 60
    rp, ci = small_graph(n, 150, 31, False, skew=2.0)
    Zr = wl.random_matrix(n, 5, 32, ld=7)
    Zr[:, 5:] = 1e30
    a = dense(rp, ci, n)
    got = oracle.aggregate("max", rp, ci, Zr, 5, self_concat=True)
    masked = np.where(a[:, :, None] > 0, Zr[None, :, :5].astype(np.float64), -np.inf).max(1)
    masked[a.sum(1) == 0] = 0.0
    assert (a.sum(1) == 0).any()
    assert np.array_equal(got[:, 5:], masked) and np.array_equal(got[:, :5], Zr[:, :5].astype(np.float64))
    # max dominates the mean, and relabelling the nodes permutes the result exactly
    assert np.all(oracle.aggregate("max", rp, ci, Zr, 5) >= oracle.aggregate("mean", rp, ci, Zr, 5) - 1e-12)
    # all-negative rows must not be clamped at zero
    neg = -np.abs(Zr) - 1
    out = oracle.aggregate("max", rp, ci, neg, 5)
    assert np.all(out[a.sum(1) > 0] < 0)


def test_mean_of_constant_is_that_constant_and_empty_rows_are_zero():
    n = 300
    rp, ci = small_graph(n, 500, 4, False, skew=2.0)
    deg = np.diff(rp)
    assert (deg == 0).any() and (deg > 0).any()
    Z = np.full((n, 5), np.float32(3.25))
    for mode in ("mean", "gat_softmax"):
        out = oracle.aggregate(mode, rp, ci, Z, 5, heads=1,
                               a_src=np.ones((1, 5), np.float32), a_dst=np.ones((1, 5), np.float32))
        assert np.allclose(out[deg > 0], 3.25, rtol=1e-15, atol=0)
        assert np.all(out[deg == 0] == 0)
    assert np.array_equal(oracle.aggregate("sum", rp, ci, np.ones((n, 2), np.float32), 2)[:, 0], deg)
    assert np.all(oracle.aggregate("gcn_sym", rp, ci, Z, 5)[deg == 0] == 0)


def test_mean_and_gat_are_convex_combinations():
    n = 120
    rp, ci = small_graph(n, 900, 5, False)
    Z = wl.random_matrix(n, 8, 6)
    a = wl.random_matrix(2, 4, 7)
    for mode in ("mean", "gat_softmax"):
        out = oracle.aggregate(mode, rp, ci, Z, 8, heads=2, a_src=a, a_dst=a)
        for v in range(n):
            nb = ci[rp[v]:rp[v + 1]]
            if nb.size:
                assert np.all(out[v] <= Z[nb].max(0) + 1e-12) and np.all(out[v] >= Z[nb].min(0) - 1e-12)


def test_gcn_on_regular_graphs_is_closed_neighbourhood_mean():
    # cycle: every closed degree is 3, so the normalised sum is (z_{v-1} + z_v + z_{v+1}) / 3
    n = 17
    src = np.arange(n, dtype=np.int32)
    dst = ((src + 1) % n).astype(np.int32)
    rp, ci = oracle.csr_from_coo(src, dst, n, True)
    Z = wl.random_matrix(n, 3, 8)
    want = (np.roll(Z, 1, 0).astype(np.float64) + Z + np.roll(Z, -1, 0)) / 3
    assert np.allclose(oracle.aggregate("gcn_sym", rp, ci, Z, 3), want, rtol=3e-7, atol=1e-7)
    # complete graph on 16 nodes with self loops: closed degree 16, normaliser exactly 1/16
    iu, ju = np.triu_indices(16, 1)
    rp, ci = oracle.csr_from_coo(iu.astype(np.int32), ju.astype(np.int32), 16, True)
    Zi = wl.random_matrix(16, 4, 9, kind="smallint")
    got = oracle.aggregate("gcn_sym", rp, ci, Zi, 4)
    assert np.array_equal(got, np.broadcast_to(Zi.astype(np.float64).sum(0) / 16, (16, 4)))


def test_gcn_operator_is_symmetric_and_uses_both_endpoint_degrees():
    n = 60
    rp, ci = small_graph(n, 200, 10, True, skew=2.0)
    x = wl.random_matrix(n, 1, 11)
    y = wl.random_matrix(n, 1, 12)
    ax = oracle.aggregate("gcn_sym", rp, ci, x, 1)
    ay = oracle.aggregate("gcn_sym", rp, ci, y, 1)
    assert abs(float((y * ax).sum() - (x * ay).sum())) < 1e-9
    # star with self loops: centre closed degree 16, leaves 2 -> weights are exact powers of two
    src = np.zeros(15, np.int32)
    dst = np.arange(1, 16, dtype=np.int32)
    rp, ci = oracle.csr_from_coo(src, dst, 16, True)
    onehot = np.zeros((16, 1), np.float32)
    onehot[0] = 1                                    # only the centre carries a value
    out = oracle.aggregate("gcn_sym", rp, ci, onehot, 1)[:, 0]
    dinv = oracle.degree(rp)[1].astype(np.float64)
    assert out[0] == 1 / 16 and np.allclose(out[1:], dinv[0] * dinv[1], rtol=1e-15)


def test_gat_special_cases():
    n = 80
    rp, ci = small_graph(n, 500, 13, False, skew=1.0)
    deg = np.diff(rp)
    Z = wl.random_matrix(n, 12, 14)
    a_src = wl.random_matrix(3, 4, 15)
    a_dst = wl.random_matrix(3, 4, 16)
    # weights of every non-empty row sum to one and are positive
    for v in range(n):
        for h in range(3):
            al = oracle.gat_alpha(v, h, rp, ci, Z, 12, 3, a_src, a_dst)
            if deg[v]:
                assert abs(al.sum() - 1) < 1e-14 and np.all(al > 0)
    # zero attention vectors make every score equal: softmax is uniform, i.e. the mean
    zero = np.zeros((3, 4), np.float32)
    assert np.allclose(oracle.aggregate("gat_softmax", rp, ci, Z, 12, heads=3, a_src=zero, a_dst=zero),
                       oracle.aggregate("mean", rp, ci, Z, 12), rtol=1e-14, atol=1e-15)
    # a_src = 0: scores do not depend on the neighbour, again the mean, whatever a_dst is
    assert np.allclose(oracle.aggregate("gat_softmax", rp, ci, Z, 12, heads=3, a_src=zero, a_dst=a_dst),
                       oracle.aggregate("mean", rp, ci, Z, 12), rtol=1e-14, atol=1e-15)
    # a row with one neighbour returns that neighbour's row exactly
    out = oracle.aggregate("gat_softmax", rp, ci, Z, 12, heads=3, a_src=a_src, a_dst=a_dst)
    for v in np.flatnonzero(deg == 1):
        assert np.array_equal(out[v], Z[ci[rp[v]]].astype(np.float64))
    # scores near +-80 neither overflow nor vanish to NaN
    big = np.full((3, 4), np.float32(20))
    Zs = np.sign(Z).astype(np.float32)
    out = oracle.aggregate("gat_softmax", rp, ci, Zs, 12, heads=3, a_src=big, a_dst=big)
    assert np.all(np.isfinite(out))
    # the softmax really sharpens: huge a_src picks the neighbour with the largest <a_src, z>
    sharp = oracle.aggregate("gat_softmax", rp, ci, Z, 12, heads=1,
                             a_src=np.full((1, 12), np.float32(0)) + np.eye(1, 12, 0, dtype=np.float32) * 1e4,
                             a_dst=np.zeros((1, 12), np.float32), slope=1.0)
    for v in np.flatnonzero(deg > 0):
        nb = ci[rp[v]:rp[v + 1]]
        assert np.allclose(sharp[v], Z[nb[np.argmax(Z[nb, 0])]], rtol=1e-12, atol=1e-12)


def test_gat_slope_and_direction_of_src_dst():
    # two nodes, one edge, asymmetric vectors: e_01 (into row 1 from 0) uses a_src on z0 and a_dst on z1
    src = np.array([0, 0], np.int32)
    dst = np.array([1, 2], np.int32)
    rp, ci = oracle.csr_from_coo(src, dst, 3, False)     # row 0 has neighbours 1 and 2
    Z = np.array([[5.0], [1.0], [-1.0]], np.float32)
    a_src = np.array([[2.0]], np.float32)
    a_dst = np.array([[-1.0]], np.float32)
    # row 0: scores leaky(2*1 - 5) = leaky(-3), leaky(2*(-1) - 5) = leaky(-7)
    for slope in (0.2, 0.5):
        al = oracle.gat_alpha(0, 0, rp, ci, Z, 1, 1, a_src, a_dst, slope=slope)
        e = np.array([-3 * slope, -7 * slope])
        want = np.exp(e) / np.exp(e).sum()
        assert np.allclose(al, want, rtol=1e-14)


@pytest.mark.parametrize("mode", ALL_MODES)
def test_permutation_equivariance(mode):
    n = 70
    src, dst = wl.random_pairs(n, 400, 17, skew=1.0)
    sl = mode == "gcn_sym"
    rp, ci = oracle.csr_from_coo(src, dst, n, sl)
    Z = wl.random_matrix(n, 6, 18, kind="smallint")
    a = wl.random_matrix(2, 3, 19)
    perm = np.random.Generator(np.random.Philox(key=3)).permutation(n).astype(np.int32)
    rp2, ci2 = oracle.csr_from_coo(perm[src], perm[dst], n, sl)
    Z2 = np.empty_like(Z)
    Z2[perm] = Z
    out = oracle.aggregate(mode, rp, ci, Z, 6, heads=2, a_src=a, a_dst=a)
    out2 = oracle.aggregate(mode, rp2, ci2, Z2, 6, heads=2, a_src=a, a_dst=a)
    if mode in ("sum", "mean", "max"):
        assert np.array_equal(out2[perm], out)           # small integers: exact in any order
    else:
        assert np.allclose(out2[perm], out, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("mode", ["sum", "mean", "gcn_sym"])
def test_linearity(mode):
    n = 50
    rp, ci = small_graph(n, 300, 20, mode == "gcn_sym")
    A = wl.random_matrix(n, 4, 21, kind="smallint")
    B = wl.random_matrix(n, 4, 22, kind="smallint")
    f = lambda z: oracle.aggregate(mode, rp, ci, z, 4)
    assert np.allclose(f(A + 2 * B), f(A) + 2 * f(B), rtol=1e-14, atol=1e-14)


@pytest.mark.parametrize("mode", ALL_MODES)
def test_self_concat_layout_and_row_subsets(mode):
    n = 45
    rp, ci = small_graph(n, 200, 23, mode == "gcn_sym")
    Z = wl.random_matrix(n, 6, 24, ld=8)
    a = wl.random_matrix(3, 2, 25)
    kw = dict(heads=3, a_src=a, a_dst=a)
    plain = oracle.aggregate(mode, rp, ci, Z, 6, **kw)
    cat = oracle.aggregate(mode, rp, ci, Z, 6, self_concat=True, **kw)
    assert cat.shape == (n, 12)
    assert np.array_equal(cat[:, :6], Z[:, :6].astype(np.float64)) and np.array_equal(cat[:, 6:], plain)
    rows = np.array([44, 3, 3, 0], np.int64)
    assert np.array_equal(oracle.aggregate(mode, rp, ci, Z, 6, rows=rows, self_concat=True, **kw), cat[rows])


def test_round_is_transform_rounded_to_float_then_aggregate():
    n = 60
    rp, ci = small_graph(n, 300, 26, False)
    H = wl.random_matrix(n, 10, 27)
    W = wl.random_matrix(10, 6, 28)
    b = wl.random_matrix(1, 6, 29)[0]
    Z = oracle.transform(H, 10, W, b, relu=True).astype(np.float32)
    want = oracle.aggregate("mean", rp, ci, Z, 6, self_concat=True)
    got = oracle.round_("mean", rp, ci, H, 10, W, b, relu=True, self_concat=True)
    assert np.array_equal(got, want)
    rows = np.array([7, 59, 0], np.int64)
    assert np.array_equal(oracle.round_("mean", rp, ci, H, 10, W, b, relu=True, self_concat=True, rows=rows),
                          want[rows])
    # identity round (first message-passing round is over the raw features)
    assert np.array_equal(oracle.round_("mean", rp, ci, H, 10, None, None),
                          oracle.aggregate("mean", rp, ci, H, 10))


def test_head_mean_hand_example_and_single_head_identity():
    # two nodes, heads = 3, two classes: columns are [h0c0 h0c1 | h1c0 h1c1 | h2c0 h2c1 | padding]
    X = np.array([[1.0, 10.0, 2.0, 20.0, 6.0, 60.0, 99.0],
                  [-3.0, 0.5, 3.0, 0.25, 0.0, 0.0, 99.0]], np.float32)
    got = oracle.head_mean(X, 3, 2)
    assert np.array_equal(got, np.array([[3.0, 30.0], [0.0, 0.25]]))
    # one head: the class scores themselves; the padding column never enters
    assert np.array_equal(oracle.head_mean(X, 1, 6), X[:, :6].astype(np.float64))
    # averaging commutes with the layout: reshaping to [n, heads, classes] and taking the mean over heads
    rng = np.random.Generator(np.random.Philox(key=77))
    Y = rng.standard_normal((50, 4 * 47 + 4)).astype(np.float32)
    want = Y[:, :188].astype(np.float64).reshape(50, 4, 47).mean(axis=1)
    assert np.allclose(oracle.head_mean(Y, 4, 47), want, rtol=0, atol=1e-15)


@pytest.mark.parametrize("mode", ALL_MODES)
@pytest.mark.parametrize("concat", [False, True])
def test_term_magnitudes_against_dense_algebra_and_sign_flips(mode, concat):
    """oracle.aggregate_abs is sum_u |c_vu z_uj|.  Pins: for non-negative Z it is the aggregate itself; for the
    modes whose coefficients do not depend on Z it is the aggregate of |Z|; for the edge softmax it is the dense
    alpha (masked softmax written with numpy) times |Z|; the maximum has a single term."""
    n, F, heads = 31, 8, 2
    rp, ci = small_graph(n, 150, 5, mode == "gcn_sym", skew=2.0)
    Z = wl.random_matrix(n, F, 6, ld=F + 2)
    a_src = wl.random_matrix(heads, F // heads, 7)
    a_dst = wl.random_matrix(heads, F // heads, 8)
    kw = dict(heads=heads, a_src=a_src, a_dst=a_dst, self_concat=concat)
    mag = oracle.aggregate_abs(mode, rp, ci, Z, F, **kw)
    val = oracle.aggregate(mode, rp, ci, Z, F, **kw)
    assert mag.shape == val.shape and np.all(mag >= np.abs(val) - 1e-12)
    Zp = np.abs(Z)
    if mode != "gat_softmax":
        # coefficients independent of Z
        if mode == "max":
            assert np.array_equal(mag, np.abs(val))
        else:
            assert np.allclose(mag, oracle.aggregate(mode, rp, ci, Zp, F, **kw), rtol=1e-13, atol=0)
    else:
        a = dense(rp, ci, n)
        Zd = Z[:, :F].astype(np.float64)
        dh = F // heads
        ref = np.zeros((n, F))
        for h in range(heads):
            Zh = Zd[:, h * dh:(h + 1) * dh]
            e = leaky((Zh @ a_dst[h].astype(np.float64))[:, None] + (Zh @ a_src[h].astype(np.float64))[None, :])
            e = np.where(a > 0, e, -np.inf)
            m = np.where(a.sum(1) > 0, e.max(1, initial=-np.inf), 0)
            p = np.where(a > 0, np.exp(e - m[:, None]), 0)
            ref[:, h * dh:(h + 1) * dh] = (p / np.maximum(p.sum(1), 1e-300)[:, None]) @ np.abs(Zh)
        agg = mag[:, F:] if concat else mag
        assert np.allclose(agg, ref, rtol=1e-12, atol=1e-14)
    if concat:
        assert np.array_equal(mag[:, :F], np.abs(Z[:, :F]).astype(np.float64))
    # non-negative input: the magnitudes are the values
    assert np.allclose(oracle.aggregate_abs(mode, rp, ci, Zp, F, **kw), oracle.aggregate(mode, rp, ci, Zp, F, **kw),
                       rtol=1e-13, atol=0)
