"""GPU CSR construction and plan arrays against the oracle: bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from paper_2302_13053_amd import binding as B
from paper_2302_13053_amd import harness as Hn
from paper_2302_13053_amd import workloads as wl

pytestmark = pytest.mark.gpu


def gpu_csr(src, dst, n, self_loops, validate=True):
    g = Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, self_loops)
    Hn.make_plan(g, validate=validate)
    torch.cuda.synchronize()
    rp = g.row_ptr.cpu().numpy()
    ci = g.col_idx[:g.nnz].cpu().numpy()
    return g, rp, ci


def check_against_oracle(src, dst, n, self_loops):
    g, rp, ci = gpu_csr(src, dst, n, self_loops)
    try:
        orp, oci = oracle.csr_from_coo(src, dst, n, self_loops)
        assert g.nnz == orp[-1] == B.retexo_plan_nnz(g.plan)
        assert np.array_equal(rp, orp)
        assert np.array_equal(ci, oci)
        deg, dinv, order = Hn.plan_arrays(g)
        odeg, odinv = oracle.degree(orp)
        assert np.array_equal(deg, odeg)
        assert np.array_equal(dinv.view(np.uint32), odinv.view(np.uint32))     # bit for bit
        assert B.retexo_plan_max_degree(g.plan) == (odeg.max() if n else 0)
        assert B.retexo_plan_num_nodes(g.plan) == n
        # schedule: a permutation of the rows, longest first, ties in id order
        assert np.array_equal(np.sort(order), np.arange(n))
        key = odeg[order].astype(np.int64) * (n + 1) - order
        assert np.all(np.diff(key) < 0) if n > 1 else True
    finally:
        g.destroy()


@pytest.mark.parametrize("n,pairs,skew,seed", [
    (1, 3, 0.0, 0), (2, 1, 0.0, 1), (64, 500, 1.0, 2), (1000, 300, 0.0, 3),
    (5000, 60000, 3.0, 4), (100003, 400000, 1.0, 5), (4096, 9000, 0.5, 6),
])
@pytest.mark.parametrize("self_loops", [False, True])
def test_csr_bit_exact_random(n, pairs, skew, seed, self_loops):
    src, dst = wl.random_pairs(n, pairs, seed, skew=skew)
    check_against_oracle(src, dst, n, self_loops)


@pytest.mark.parametrize("self_loops", [False, True])
def test_csr_empty_pair_list(self_loops):
    check_against_oracle(np.empty(0, np.int32), np.empty(0, np.int32), 37, self_loops)


@pytest.mark.parametrize("idx", [0, 1, 2])
def test_csr_small_workloads(idx):
    w = wl.workload(idx)
    src, dst = wl.make_graph(w)
    check_against_oracle(src, dst, w.n_nodes, w.self_loops)


def test_csr_rejects_bad_ids_and_small_capacity():
    n = 50
    src, dst = wl.random_pairs(n, 200, 7)
    bad = src.copy()
    bad[17] = n
    ws = Hn.ws_tensor(B.retexo_csr_workspace_bytes(200, n, False))
    d_src, d_dst = Hn.dev(src), Hn.dev(dst)      # named so that the device buffers stay alive
    rp = torch.full((n + 1,), -7, dtype=torch.int64, device="cuda")
    ci = torch.full((400,), -7, dtype=torch.int32, device="cuda")
    d_bad = Hn.dev(bad)
    st, _ = B.retexo_csr_from_coo(200, d_bad.data_ptr(), d_dst.data_ptr(), n, False,
                                  rp.data_ptr(), ci.data_ptr(), 400, ws.data_ptr(), ws.numel())
    assert st == B.E_CSR
    neg = src.copy()
    neg[3] = -1
    d_neg = Hn.dev(neg)
    st, _ = B.retexo_csr_from_coo(200, d_neg.data_ptr(), d_dst.data_ptr(), n, False,
                                  rp.data_ptr(), ci.data_ptr(), 400, ws.data_ptr(), ws.numel())
    assert st == B.E_CSR
    st, nnz = B.retexo_csr_from_coo(200, d_src.data_ptr(), d_dst.data_ptr(), n, False,
                                    rp.data_ptr(), ci.data_ptr(), 10, ws.data_ptr(), ws.numel())
    assert st == B.E_CAPACITY and nnz == oracle.csr_from_coo(src, dst, n, False)[0][-1]
    torch.cuda.synchronize()
    assert bool((rp == -7).all()) and bool((ci == -7).all())      # nothing was written
    st, _ = B.retexo_csr_from_coo(200, d_src.data_ptr(), d_dst.data_ptr(), n, False,
                                  rp.data_ptr(), ci.data_ptr(), 400, ws.data_ptr(), 64)
    assert st == B.E_WORKSPACE


def test_plan_validation_catches_malformed_csr():
    rp = Hn.dev(np.array([0, 2, 1, 3], np.int64))             # decreasing
    ci = Hn.dev(np.array([0, 1, 2], np.int32))
    st, plan = B.retexo_plan_create(3, rp.data_ptr(), ci.data_ptr(), B.F_VALIDATE)
    assert st == B.E_CSR and plan is None
    rp = Hn.dev(np.array([1, 2, 3, 3], np.int64))             # does not start at 0
    st, plan = B.retexo_plan_create(3, rp.data_ptr(), ci.data_ptr(), B.F_VALIDATE)
    assert st == B.E_CSR and plan is None
    rp = Hn.dev(np.array([0, 1, 2, 3], np.int64))
    ci = Hn.dev(np.array([0, 3, 2], np.int32))                # column out of range
    st, plan = B.retexo_plan_create(3, rp.data_ptr(), ci.data_ptr(), B.F_VALIDATE)
    assert st == B.E_CSR and plan is None
    ci = Hn.dev(np.array([0, 1, 2], np.int32))
    st, plan = B.retexo_plan_create(3, rp.data_ptr(), ci.data_ptr(), B.F_VALIDATE)
    assert st == B.OK and plan
    B.retexo_plan_destroy(plan)


def _split_positions(g):
    n = g.n_nodes
    pos = torch.empty((B.SPLIT_PARTS + 1) * n, dtype=torch.int32, device="cuda")
    span = B.retexo_plan_export_split(g.plan, pos.data_ptr(), Hn._stream_ptr())
    torch.cuda.synchronize()
    return span, pos.cpu().numpy().reshape(B.SPLIT_PARTS + 1, n)


@pytest.mark.parametrize("n,pairs,skew,seed", [(3000, 60000, 1.2, 1), (1000, 90000, 0.0, 2), (70, 40, 0.0, 3)])
def test_plan_row_split_is_the_first_position_per_source_range(n, pairs, skew, seed):
    # every row cut at the first entry whose column reaches k * span: integer work, compared exactly with
    # a search over the (ascending) columns of the row
    src, dst = wl.graph_power_law(n, pairs, 2.0 + skew, 20.0, 400.0, seed) if skew else wl.graph_er(n, pairs, seed)
    g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, False), validate=True, split_rows=True)
    rp = g.row_ptr.cpu().numpy()
    ci = g.col_idx.cpu().numpy()[: g.nnz]
    _, _, order = Hn.plan_arrays(g)
    span, pos = _split_positions(g)
    assert span == (n + B.SPLIT_PARTS - 1) // B.SPLIT_PARTS
    for s in range(n):
        v = int(order[s])
        row = ci[rp[v]:rp[v + 1]]
        want = rp[v] + np.searchsorted(row, np.arange(B.SPLIT_PARTS + 1) * span, side="left")
        want[-1] = rp[v + 1]
        assert np.array_equal(pos[:, s], want), (s, v)
    g.destroy()
    # a plan without the split says so
    g2 = Hn.make_plan(Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, False))
    assert B.retexo_plan_export_split(g2.plan, 0) == 0
    g2.destroy()


def test_row_split_of_unsorted_columns_still_cuts_every_row_into_consecutive_pieces():
    # columns shuffled inside each row (a caller's own CSR): the positions stay a monotone chain from row
    # start to row end, so sums over the pieces are sums over the row
    n = 800
    src, dst = wl.graph_er(n, 30000, 5)
    rp, ci = oracle.csr_from_coo(src, dst, n, False)
    rng = np.random.Generator(np.random.Philox(key=9))
    ci = ci.copy()
    for v in range(n):
        rng.shuffle(ci[rp[v]:rp[v + 1]])
    g = Hn.DeviceGraph(n, int(rp[-1]), Hn.dev(rp.astype(np.int64)), Hn.dev(ci.astype(np.int32)))
    Hn.make_plan(g, validate=True, split_rows=True)
    _, _, order = Hn.plan_arrays(g)
    span, pos = _split_positions(g)
    assert span > 0
    assert np.array_equal(pos[0], rp[order]) and np.array_equal(pos[-1], rp[order + 1])
    assert bool((np.diff(pos.astype(np.int64), axis=0) >= 0).all())
    Z = wl.random_matrix(n, 40, 6, kind="smallint")
    out = Hn.aggregate(g, "sum", Hn.dev(Z), 40)
    assert np.array_equal(out.cpu().numpy()[:, :40].astype(np.float64), oracle.aggregate("sum", rp, ci, Z, 40))
    g.destroy()


@pytest.mark.parametrize("self_loops", [False, True])
def test_csr_with_exactly_sized_columns_gives_the_same_arrays(self_loops):
    # a column array that can hold every key lets the builder write columns and row offsets in the scan
    # itself; a smaller one (here: exactly nnz, after a size query) makes it count first.  Same result.
    n = 3000
    src, dst = wl.random_pairs(n, 40000, 11, skew=2.0)
    rp_o, ci_o = oracle.csr_from_coo(src, dst, n, self_loops)
    d_src, d_dst = Hn.dev(src), Hn.dev(dst)
    ws = Hn.ws_tensor(B.retexo_csr_workspace_bytes(src.size, n, self_loops))
    rp = torch.full((n + 1,), -7, dtype=torch.int64, device="cuda")
    st, nnz = B.retexo_csr_from_coo(src.size, d_src.data_ptr(), d_dst.data_ptr(), n, self_loops,
                                    rp.data_ptr(), 0, 0, ws.data_ptr(), ws.numel())
    assert st == B.E_CAPACITY and nnz == rp_o[-1] and bool((rp == -7).all())
    ci = torch.full((nnz + 5,), -7, dtype=torch.int32, device="cuda")
    st, nnz2 = B.retexo_csr_from_coo(src.size, d_src.data_ptr(), d_dst.data_ptr(), n, self_loops,
                                     rp.data_ptr(), ci.data_ptr(), nnz, ws.data_ptr(), ws.numel())
    torch.cuda.synchronize()
    assert st == B.OK and nnz2 == nnz
    assert np.array_equal(rp.cpu().numpy(), rp_o) and np.array_equal(ci.cpu().numpy()[:nnz], ci_o)
    assert bool((ci[nnz:] == -7).all())
    big = Hn.csr_from_coo(d_src, d_dst, n, self_loops)            # roomy column array: the one-pass path
    assert np.array_equal(big.row_ptr.cpu().numpy(), rp_o) and np.array_equal(big.col_idx.cpu().numpy()[:nnz], ci_o)


@pytest.mark.parametrize("n", [37, 1000, 70000])
@pytest.mark.parametrize("self_loops", [False, True])
def test_csr_of_heavily_repeated_and_clustered_pairs(n, self_loops):
    # neighbours within a window of 16 ids, one pair given thousands of times in both orders, one self
    # pair given thousands of times: the clean-up (repeats, self pairs, both directions) is all there is
    rng = np.random.Generator(np.random.Philox(key=n))
    m = 20 * n
    a = rng.integers(0, n, m)
    b = (a + rng.integers(-8, 9, m)) % n
    rep = np.full(3000, n // 3), np.full(3000, (n // 3 + 5) % n)
    selfs = np.full(2000, n // 2)
    src = np.concatenate([a, rep[0], rep[1], selfs, rng.integers(0, n, m // 4)]).astype(np.int32)
    dst = np.concatenate([b, rep[1], rep[0], selfs, rng.integers(0, n, m // 4)]).astype(np.int32)
    perm = rng.permutation(src.size)
    check_against_oracle(src[perm], dst[perm], n, self_loops)


def _star_and_repeats(n, seed):
    """A node joined to most others (one row far beyond what a bucket holds in LDS), a narrow id window with
    heavy traffic (a bucket whose keys cluster), one pair and one self pair given far more often than a bucket
    holds entries, plus background pairs."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    hub = n // 7
    spokes = rng.permutation(n)[: min(n - 1, 60000)]
    win = rng.integers(n // 2, min(n, n // 2 + 40), (2, 50000))
    rep_a, rep_b = np.full(30000, n // 3), np.full(30000, (n // 3 + 11) % n)
    selfs = np.full(20000, n // 5)
    bg = rng.integers(0, n, (2, 4 * n))
    src = np.concatenate([np.full(spokes.size, hub), win[0], rep_a, rep_b, selfs, bg[0]]).astype(np.int32)
    dst = np.concatenate([spokes, win[1], rep_b, rep_a, selfs, bg[1]]).astype(np.int32)
    perm = rng.permutation(src.size)
    return src[perm], dst[perm]


@pytest.mark.parametrize("n", [300, 70001, 1 << 20])
@pytest.mark.parametrize("self_loops", [False, True])
def test_csr_buckets_that_do_not_fit(n, self_loops):
    # rows, row ranges and repeated keys with more entries than the local data share holds take the construction's
    # key-range path; the result is the same function of the pair set
    src, dst = _star_and_repeats(n, 100 + n % 97)
    check_against_oracle(src, dst, n, self_loops)


@pytest.mark.parametrize("self_loops", [False, True])
def test_csr_both_constructions_give_the_same_arrays(self_loops):
    # the bucketing construction (graphs of up to 2^23 nodes) and the sorted-key construction (larger graphs, or
    # on request) are two routes to one result
    n = 50000
    src, dst = _star_and_repeats(n, 5)
    try:
        B.retexo_set_option("csr_sorted_keys", 1)
        check_against_oracle(src, dst, n, self_loops)
        a = Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, self_loops)
    finally:
        B.retexo_set_option("csr_sorted_keys", 0)
    b = Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, self_loops)
    torch.cuda.synchronize()
    assert a.nnz == b.nnz and torch.equal(a.row_ptr, b.row_ptr) and torch.equal(a.col_idx[:a.nnz], b.col_idx[:b.nnz])


def test_csr_of_a_graph_beyond_the_bucketing_range():
    # more than 2^23 nodes: the sorted-key construction runs by itself
    n = (1 << 23) + 12345
    src, dst = wl.random_pairs(n, 200000, 17, skew=1.0)
    g = Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, False)
    torch.cuda.synchronize()
    orp, oci = oracle.csr_from_coo(src, dst, n, False)
    assert g.nnz == orp[-1]
    assert np.array_equal(g.row_ptr.cpu().numpy(), orp) and np.array_equal(g.col_idx[:g.nnz].cpu().numpy(), oci)


@pytest.mark.parametrize("split_rows", [False, True])
def test_plan_in_caller_memory_equals_the_allocating_plan(split_rows):
    # retexo_plan_create_in: same arrays, no allocation, the entry count stated by the caller
    n = 3000
    src, dst = wl.graph_power_law(n, 60000, 2.2, 20.0, 400.0, 3)
    g = Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, False)
    a = Hn.make_plan(Hn.DeviceGraph(n, g.nnz, g.row_ptr, g.col_idx), validate=True, split_rows=split_rows)
    flags = B.F_VALIDATE | (B.F_SPLIT_ROWS if split_rows else 0)
    need = B.retexo_plan_workspace_bytes(n, g.nnz, flags)
    assert need > 0
    ws = Hn.ws_tensor(need)
    b = Hn.make_plan(Hn.DeviceGraph(n, g.nnz, g.row_ptr, g.col_idx), validate=True, split_rows=split_rows, workspace=ws)
    for x, y in zip(Hn.plan_arrays(a), Hn.plan_arrays(b)):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    assert B.retexo_plan_max_degree(a.plan) == B.retexo_plan_max_degree(b.plan)
    assert B.retexo_plan_nnz(b.plan) == g.nnz
    if split_rows:
        sa, pa = _split_positions(a)
        sb, pb = _split_positions(b)
        assert sa == sb and np.array_equal(pa, pb)
    Z = Hn.dev(wl.random_matrix(n, 40, 6))
    assert torch.equal(Hn.aggregate(a, "mean", Z, 40)[:, :40], Hn.aggregate(b, "mean", Z, 40)[:, :40])
    # argument errors: wrong entry count, workspace too small or misaligned
    rp, ci = g.row_ptr.data_ptr(), g.col_idx.data_ptr()
    st, plan = B.retexo_plan_create_in(n, g.nnz + 1, rp, ci, flags, ws.data_ptr(), ws.numel())
    assert st == B.E_CSR and plan is None
    st, plan = B.retexo_plan_create_in(n, g.nnz, rp, ci, flags, ws.data_ptr(), need - 1)
    assert st == B.E_WORKSPACE and plan is None
    st, plan = B.retexo_plan_create_in(n, g.nnz, rp, ci, flags, ws.data_ptr() + 64, ws.numel())
    assert st == B.E_WORKSPACE and plan is None
    st, plan = B.retexo_plan_create_in(n, g.nnz, 0, ci, flags, ws.data_ptr(), ws.numel())
    assert st == B.E_NULL and plan is None
    a.destroy()
    b.destroy()
