"""Pins for the partition oracle: brute force on a dense adjacency, cross-worker consistency, and the
property the set-up exists for — every worker's local aggregation over [own rows | received boundary
rows] reproduces the global aggregation on its inner nodes."""
import numpy as np
import pytest

import oracle
from oracle import partition as op
from paper_2302_13053_amd import workloads as wl


def small_graph(n=60, pairs=150, seed=3, self_loops=False):
    src, dst = wl.random_pairs(n, pairs, seed, skew=1.0)
    return oracle.csr_from_coo(src, dst, n, self_loops)


def parts_of(n, P, seed):
    return np.random.Generator(np.random.Philox(key=seed)).integers(0, P, n).astype(np.int32)


@pytest.mark.parametrize("P", [1, 2, 3, 5])
def test_share_against_dense_brute_force(P):
    n = 60
    rp, ci = small_graph(n)
    A = np.zeros((n, n), bool)
    A[np.repeat(np.arange(n), np.diff(rp)), ci] = True
    part = parts_of(n, P, 7)
    for p in range(P):
        s = op.share(rp, ci, part, P, p)
        inner = [v for v in range(n) if part[v] == p]
        halo = [u for u in range(n) if part[u] != p and any(A[v, u] for v in inner)]
        assert s.n_inner == len(inner) and s.n_halo == len(halo)
        assert list(s.local_ids) == inner + halo
        assert list(s.global_deg) == [int(A[v].sum()) for v in inner + halo]
        for i, v in enumerate(inner):
            row = s.col_idx[s.row_ptr[i]:s.row_ptr[i + 1]]
            assert np.all(np.diff(row) > 0)                                   # ascending, unique
            assert sorted(s.local_ids[row]) == [u for u in range(n) if A[v, u]]
        assert np.all(np.diff(s.row_ptr[s.n_inner:]) == 0)                   # boundary rows are empty
        for q in range(P):
            want_send = [v for v in inner if any(A[v, u] and part[u] == q for u in range(n))] if q != p else []
            assert list(s.local_ids[s.send_ids[q]]) == want_send
            assert list(s.local_ids[s.recv_ids[q]]) == [u for u in halo if part[u] == q]
            assert np.all(s.send_ids[q] < s.n_inner) and np.all(s.recv_ids[q] >= s.n_inner)


def test_send_and_receive_lists_line_up_across_workers():
    n, P = 200, 4
    rp, ci = small_graph(n, 700, seed=5)
    part = parts_of(n, P, 9)
    shares = [op.share(rp, ci, part, P, p) for p in range(P)]
    for p in range(P):
        for q in range(P):
            a = shares[p].local_ids[shares[p].send_ids[q]]
            b = shares[q].local_ids[shares[q].recv_ids[p]]
            assert np.array_equal(a, b)
        assert sum(r.size for r in shares[p].recv_ids) == shares[p].n_halo
    assert sum(s.n_inner for s in shares) == n


@pytest.mark.parametrize("mode,self_loops", [("mean", False), ("sum", False), ("gcn_sym", True), ("gat_softmax", False)])
def test_local_aggregation_with_exchanged_rows_equals_global(mode, self_loops):
    n, P, F, heads = 150, 3, 8, 2
    rp, ci = small_graph(n, 500, seed=11, self_loops=self_loops)
    part = parts_of(n, P, 13)
    Z = wl.random_matrix(n, F, 17)
    a_s, a_d = wl.random_matrix(heads, F // heads, 18), wl.random_matrix(heads, F // heads, 19)
    want = oracle.aggregate(mode, rp, ci, Z, F, heads=heads, a_src=a_s, a_dst=a_d)
    shares = [op.share(rp, ci, part, P, p) for p in range(P)]
    # every worker starts with its own rows only; boundary rows arrive through the send/receive lists
    tables = [np.full((s.n_inner + s.n_halo, F), np.nan, np.float32) for s in shares]
    for p, s in enumerate(shares):
        tables[p][:s.n_inner] = Z[s.local_ids[:s.n_inner]]
    for p, s in enumerate(shares):
        for q in range(P):
            buf = tables[p][s.send_ids[q]]                    # pack on p
            tables[q][shares[q].recv_ids[p]] = buf            # unpack on q
    for p, s in enumerate(shares):
        assert not np.isnan(tables[p]).any()
        if mode == "gcn_sym":
            # a boundary node's local row is empty: its normalisation must come from the global degree
            dinv = (np.float32(1.0) / np.sqrt(s.global_deg.astype(np.float32))).astype(np.float64)
            out = np.zeros((s.n_inner, F))
            for i in range(s.n_inner):
                cols = s.col_idx[s.row_ptr[i]:s.row_ptr[i + 1]]
                out[i] = dinv[i] * (dinv[cols, None] * tables[p][cols].astype(np.float64)).sum(0)
        else:
            out = oracle.aggregate(mode, s.row_ptr, s.col_idx, tables[p], F, heads=heads, a_src=a_s, a_dst=a_d)[:s.n_inner]
        assert np.allclose(out, want[s.local_ids[:s.n_inner]], rtol=1e-12, atol=1e-13), (mode, p)


def test_degenerate_partitions():
    rp, ci = small_graph(30, 60, seed=2)
    part = np.zeros(30, np.int32)
    s = op.share(rp, ci, part, 2, 1)                          # a worker that owns nothing
    assert s.n_inner == 0 and s.n_halo == 0 and s.col_idx.size == 0 and s.row_ptr.tolist() == [0]
    s = op.share(rp, ci, part, 2, 0)                          # a worker that owns everything
    assert s.n_halo == 0 and np.array_equal(s.row_ptr, rp) and np.array_equal(s.col_idx, ci)
    assert all(x.size == 0 for x in s.send_ids + s.recv_ids)
