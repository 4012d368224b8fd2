"""Pins for the oracle's CSR construction and degree/normaliser arrays.

The CSR of an undirected simple graph (paper: section "Edge-partitioned
Distributed Setup" — graphs are undirected) is checked against a dense boolean
adjacency matrix built independently here, plus structural properties.
"""
import numpy as np
import pytest

import oracle
from paper_2302_13053_amd import workloads as wl


def dense_adjacency(src, dst, n, self_loops):
    a = np.zeros((n, n), bool)
    for u, v in zip(src.tolist(), dst.tolist()):
        if u != v:
            a[u, v] = True
            a[v, u] = True
    if self_loops:
        a[np.arange(n), np.arange(n)] = True
    return a


def csr_to_dense(row_ptr, col, n):
    a = np.zeros((n, n), np.int64)
    for v in range(n):
        for e in range(row_ptr[v], row_ptr[v + 1]):
            a[v, col[e]] += 1
    return a


@pytest.mark.parametrize("n,pairs,seed", [(1, 5, 0), (7, 30, 1), (40, 300, 2), (64, 90, 3), (33, 0, 4)])
@pytest.mark.parametrize("self_loops", [False, True])
def test_csr_matches_dense_bruteforce(n, pairs, seed, self_loops):
    src, dst = wl.random_pairs(n, pairs, seed, skew=1.0)
    row_ptr, col = oracle.csr_from_coo(src, dst, n, self_loops)
    want = dense_adjacency(src, dst, n, self_loops)
    got = csr_to_dense(row_ptr, col, n)
    assert got.max(initial=0) <= 1                     # no repeated entry survives
    assert np.array_equal(got.astype(bool), want)
    assert row_ptr[0] == 0 and row_ptr[-1] == col.size == want.sum()
    for v in range(n):
        seg = col[row_ptr[v]:row_ptr[v + 1]]
        assert np.all(np.diff(seg) > 0)                # strictly ascending columns


def test_csr_is_structurally_symmetric_and_loop_free():
    n = 500
    src, dst = wl.random_pairs(n, 4000, 11, skew=2.0)
    row_ptr, col = oracle.csr_from_coo(src, dst, n, False)
    rows = np.repeat(np.arange(n), np.diff(row_ptr))
    fwd = set(zip(rows.tolist(), col.tolist()))
    assert all((c, r) in fwd for r, c in fwd)
    assert not np.any(rows == col)
    # with self loops: exactly one diagonal entry per row and nothing else changes
    row_ptr2, col2 = oracle.csr_from_coo(src, dst, n, True)
    rows2 = np.repeat(np.arange(n), np.diff(row_ptr2))
    assert np.array_equal(np.bincount(rows2[rows2 == col2], minlength=n), np.ones(n, np.int64))
    off = rows2 != col2
    assert np.array_equal(rows2[off], rows) and np.array_equal(col2[off], col)


def test_csr_relabelling_commutes():
    n = 200
    src, dst = wl.random_pairs(n, 1500, 5, skew=1.5)
    perm = np.random.Generator(np.random.Philox(key=9)).permutation(n).astype(np.int32)
    rp, ci = oracle.csr_from_coo(src, dst, n, True)
    rp2, ci2 = oracle.csr_from_coo(perm[src], perm[dst], n, True)
    for v in range(n):
        a = np.sort(perm[ci[rp[v]:rp[v + 1]]])
        b = ci2[rp2[perm[v]]:rp2[perm[v] + 1]]
        assert np.array_equal(a, b)


def test_csr_order_of_pairs_and_orientation_do_not_matter():
    n = 90
    src, dst = wl.random_pairs(n, 700, 6)
    rp, ci = oracle.csr_from_coo(src, dst, n, False)
    rp2, ci2 = oracle.csr_from_coo(dst[::-1], src[::-1], n, False)
    assert np.array_equal(rp, rp2) and np.array_equal(ci, ci2)


def test_csr_rejects_out_of_range_ids():
    with pytest.raises(ValueError):
        oracle.csr_from_coo(np.array([0, 5], np.int32), np.array([1, 2], np.int32), 5, False)
    with pytest.raises(ValueError):
        oracle.csr_from_coo(np.array([0, -1], np.int32), np.array([1, 2], np.int32), 5, False)


def test_empty_graph_and_pure_self_loops():
    rp, ci = oracle.csr_from_coo(np.empty(0, np.int32), np.empty(0, np.int32), 6, False)
    assert np.array_equal(rp, np.zeros(7, np.int64)) and ci.size == 0
    rp, ci = oracle.csr_from_coo(np.array([2, 3], np.int32), np.array([2, 3], np.int32), 6, True)
    assert np.array_equal(rp, np.arange(7)) and np.array_equal(ci, np.arange(6))


def test_degree_and_dinv():
    # star with centre 0 and 15 leaves, plus self loops: closed degrees 16 and 2
    src = np.zeros(15, np.int32)
    dst = np.arange(1, 16, dtype=np.int32)
    rp, _ = oracle.csr_from_coo(src, dst, 16, True)
    deg, dinv = oracle.degree(rp)
    assert deg[0] == 16 and np.all(deg[1:] == 2)
    assert dinv[0] == np.float32(0.25)                     # exact power of two
    assert dinv[1] == np.float32(1) / np.sqrt(np.float32(2))
    # without self loops an isolated node has degree 0 and normaliser 0 (no inf)
    rp, _ = oracle.csr_from_coo(np.array([0], np.int32), np.array([1], np.int32), 3, False)
    deg, dinv = oracle.degree(rp)
    assert deg.tolist() == [1, 1, 0] and dinv.tolist() == [1.0, 1.0, 0.0]


def test_dinv_is_correctly_rounded_float_for_every_degree_up_to_25000():
    # numpy's float32 sqrt and divide are IEEE correctly rounded: an independent routine
    d = np.arange(1, 25001, dtype=np.int64)
    rp = np.concatenate([[0], np.cumsum(d)]).astype(np.int64)
    deg, dinv = oracle.degree(rp)
    assert np.array_equal(deg, d.astype(np.int32))
    want = np.float32(1) / np.sqrt(d.astype(np.float32))
    assert want.dtype == np.float32 and np.array_equal(dinv, want)


def test_workload_shapes_small():
    # the three small workloads produce exactly the entry counts their recipes state
    for idx, nnz in ((0, 2 * 5429), (1, 2 * 44338 + 19717), (2, 2 * 171002)):
        w = wl.workload(idx)
        src, dst = wl.make_graph(w)
        rp, ci = oracle.csr_from_coo(src, dst, w.n_nodes, w.self_loops)
        assert rp[-1] == nnz == ci.size
