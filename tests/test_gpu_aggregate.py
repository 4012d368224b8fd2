"""GPU neighbourhood aggregation against the fp64 oracle, all four modes."""
import numpy as np
import pytest
import torch

import oracle
from paper_2302_13053_amd import binding as B
from paper_2302_13053_amd import harness as Hn
from paper_2302_13053_amd import workloads as wl
from parity import assert_close, assert_cond_close, row_rel_err

pytestmark = pytest.mark.gpu

MODES = ["sum", "mean", "gcn_sym", "gat_softmax"]


@pytest.fixture(scope="module")
def graphs():
    """name -> (DeviceGraph, row_ptr, col_idx) for a few shapes; gcn variants carry self loops."""
    specs = {
        "skewed": (5000, 60000, 3.0, 4),     # a few rows far above the heavy threshold, many empty
        "flat": (3000, 20000, 0.0, 5),
        "tiny": (3, 2, 0.0, 6),
    }
    out = {}
    for name, (n, pairs, skew, seed) in specs.items():
        src, dst = wl.random_pairs(n, pairs, seed, skew=skew)
        for sl in (False, True):
            g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, sl), validate=True, split_rows=(name == "skewed"))
            rp, ci = oracle.csr_from_coo(src, dst, n, sl)
            out[(name, sl)] = (g, rp, ci)
    deg = np.diff(out[("skewed", False)][1])
    assert deg.max() >= 2048 and (deg == 0).any()
    yield out
    for g, _, _ in out.values():
        g.destroy()


def run_case(graphs, name, mode, F, ld, heads, concat, seed, kind="normal", base_offset=0, with_mag=False):
    g, rp, ci = graphs[(name, mode == "gcn_sym")]
    n = g.n_nodes
    Zh = wl.random_matrix(n, F, seed, ld=ld, kind=kind)
    Zh[:, F:] = 0.0
    a_src = a_dst = None
    kw = {}
    if mode == "gat_softmax":
        a_src = wl.random_matrix(heads, F // heads, seed + 1) * np.float32(0.3)
        a_dst = wl.random_matrix(heads, F // heads, seed + 2) * np.float32(0.3)
        kw = dict(heads=heads, a_src=Hn.dev(a_src), a_dst=Hn.dev(a_dst))
    if base_offset:
        # shift the matrix start by a few floats to break 16-byte alignment
        buf = torch.zeros(n * ld + base_offset, dtype=torch.float32, device="cuda")
        Zd = buf[base_offset:].view(n, ld)
        Zd.copy_(torch.from_numpy(Zh))
    else:
        Zd = Hn.dev(Zh)
    ow = 2 * F if concat else F
    out = torch.full((n, ow + 3), 555.0, dtype=torch.float32, device="cuda")
    Hn.aggregate(g, mode, Zd, F, concat=concat, out=out, **kw)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.all(got[:, ow:] == 555.0)
    want = oracle.aggregate(mode, rp, ci, Zh, F, heads=heads, a_src=a_src, a_dst=a_dst, self_concat=concat)
    if with_mag:
        # size of the terms behind every element: the yardstick of the condition-aware measure
        mag = oracle.aggregate_abs(mode, rp, ci, Zh, F, heads=heads, a_src=a_src, a_dst=a_dst, self_concat=concat)
        return got[:, :ow], want, mag
    return got[:, :ow], want


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("F,ld,heads,concat,offset", [
    (256, 256, 4, False, 0),      # one float4 chunk per lane
    (602, 608, 1, True, 0),       # float4 gathers with a ragged last vector, 3 chunks
    (602, 602, 2, True, 0),       # float2 gathers
    (1433, 1433, 1, True, 0),     # scalar gathers, several slabs
    (1432, 1440, 4, False, 0),    # float4, two slabs
    (188, 192, 4, False, 0),      # heads of 47 columns: lanes straddle heads
    (100, 100, 4, True, 0),
    (64, 64, 8, False, 0),
    (7, 7, 1, True, 0),
    (1, 1, 1, False, 0),
    (128, 128, 2, False, 1),      # misaligned base pointer
])
def test_modes_match_oracle_on_skewed_graph(graphs, mode, F, ld, heads, concat, offset):
    if mode == "gat_softmax" and F % heads:
        heads = 1
    # signed data at every width.  Every element is held to 1e-5 of the size of its terms; rows of at least 64
    # columns are also held to 1e-5 of the row's largest magnitude (a row of one or a few signed columns can
    # cancel to nothing as a whole, so it has no robust magnitude of its own)
    got, want, mag = run_case(graphs, "skewed", mode, F, ld, heads, concat, seed=F + 17, base_offset=offset,
                              with_mag=True)
    assert_cond_close(got, want, mag, what="%s F=%d" % (mode, F))
    if F >= 64:
        assert_close(got, want, what="%s F=%d" % (mode, F))
    if concat:
        assert np.array_equal(got[:, :F].astype(np.float64), want[:, :F])      # self copy is a bit copy


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("name", ["flat", "tiny"])
def test_modes_match_oracle_other_graphs(graphs, mode, name):
    got, want = run_case(graphs, name, mode, 96, 96, 3, True, seed=3)
    assert_close(got, want, what="%s %s" % (mode, name))


@pytest.mark.parametrize("F,ld,concat,offset", [
    (256, 256, False, 0), (602, 608, True, 0), (602, 602, True, 0), (1433, 1433, True, 0),
    (1432, 1440, False, 0), (100, 100, True, 0), (7, 7, True, 0), (1, 1, False, 0), (128, 128, False, 1),
])
def test_max_pooling_is_bit_exact(graphs, F, ld, concat, offset):
    # a maximum does not depend on the order it is taken in, so every element must match exactly:
    # heavy rows (combined across waves), empty rows (zero, not -inf), all-negative rows (not clamped)
    got, want = run_case(graphs, "skewed", "max", F, ld, 1, concat, seed=F + 5, base_offset=offset)
    assert np.array_equal(got.astype(np.float64), want), "max F=%d" % F
    deg = np.diff(graphs[("skewed", False)][1])
    agg = got[:, F:] if concat else got
    assert np.all(agg[deg == 0] == 0.0) and (agg[deg == 1] < 0).any()
    for name in ("flat", "tiny"):
        got, want = run_case(graphs, name, "max", 96, 96, 1, True, seed=4)
        assert np.array_equal(got.astype(np.float64), want)
    defaults = {"agg_slab_cols": 0, "agg_max_vec": 4, "agg_heavy_degree": 2048, "agg_slab_major": -1}
    got, _ = run_case(graphs, "skewed", "max", F, ld, 1, concat, seed=F + 5, base_offset=offset)
    try:   # other slab widths, gather widths and heavy-row thresholds give the same bits
        for k, v in (("agg_slab_cols", 32), ("agg_max_vec", 1), ("agg_heavy_degree", 64), ("agg_slab_major", 1)):
            B.retexo_set_option(k, v)
            got2, _ = run_case(graphs, "skewed", "max", F, ld, 1, concat, seed=F + 5, base_offset=offset)
            assert np.array_equal(got2, got), k
            B.retexo_set_option(k, defaults[k])
    finally:
        for k, v in defaults.items():
            B.retexo_set_option(k, v)


def test_integer_features_are_bit_exact_and_ones_give_degree(graphs):
    g, rp, ci = graphs[("skewed", False)]
    deg = np.diff(rp)
    got, want = run_case(graphs, "skewed", "sum", 40, 40, 1, False, seed=1, kind="smallint")
    assert np.array_equal(got.astype(np.float64), want)     # any wrong, missed or repeated neighbour shows
    ones = torch.ones((g.n_nodes, 4), dtype=torch.float32, device="cuda")
    out = Hn.aggregate(g, "sum", ones, 4, ld_out=4)
    assert np.array_equal(out.cpu().numpy()[:, 0], deg.astype(np.float32))
    out = Hn.aggregate(g, "mean", ones, 4, ld_out=4).cpu().numpy()
    assert np.all(out[deg > 0] == 1.0) and np.all(out[deg == 0] == 0.0)


def test_gcn_indexing_exact_on_power_of_four_degrees():
    # disjoint stars whose closed degrees are 4, 16 and 64 (leaves: 2 -> not a power of 4, so
    # leaves get closed degree 4 by joining triangles instead): use complete graphs K4, K16, K64
    blocks, src, dst, off = [4, 16, 64, 4, 16], [], [], 0
    for k in blocks:
        iu, ju = np.triu_indices(k, 1)
        src.append(iu + off)
        dst.append(ju + off)
        off += k
    src = np.concatenate(src).astype(np.int32)
    dst = np.concatenate(dst).astype(np.int32)
    n = off
    g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, True))
    rp, ci = oracle.csr_from_coo(src, dst, n, True)
    Z = wl.random_matrix(n, 12, 2, kind="smallint")
    out = Hn.aggregate(g, "gcn_sym", Hn.dev(Z), 12, ld_out=12).cpu().numpy()
    want = oracle.aggregate("gcn_sym", rp, ci, Z, 12)
    assert np.array_equal(out.astype(np.float64), want)     # all weights are powers of two: exact
    g.destroy()


def test_gat_properties(graphs):
    g, rp, ci = graphs[("skewed", False)]
    n, F, heads = g.n_nodes, 64, 4
    deg = np.diff(rp)
    Zh = wl.random_matrix(n, F, 8)
    Z = Hn.dev(Zh)
    zero = torch.zeros((heads, F // heads), dtype=torch.float32, device="cuda")
    # zero attention vectors: uniform softmax == mean
    a = Hn.aggregate(g, "gat_softmax", Z, F, heads=heads, a_src=zero, a_dst=zero).cpu().numpy()[:, :F]
    assert_close(a, oracle.aggregate("mean", rp, ci, Zh, F), what="gat(a=0) vs mean")
    # constant rows stay constant (weights sum to one), empty rows give zero
    const = torch.full((n, F), 2.5, dtype=torch.float32, device="cuda")
    asrc = Hn.dev(wl.random_matrix(heads, F // heads, 9))
    c = Hn.aggregate(g, "gat_softmax", const, F, heads=heads, a_src=asrc, a_dst=asrc).cpu().numpy()[:, :F]
    assert np.abs(c[deg > 0] - 2.5).max() <= 2.5 * 1e-5 and np.all(c[deg == 0] == 0)
    # scores of magnitude ~80: finite, still matches
    big = np.full((heads, F // heads), 5.0, np.float32)
    Zs = np.sign(Zh).astype(np.float32)
    o = Hn.aggregate(g, "gat_softmax", Hn.dev(Zs), F, heads=heads, a_src=Hn.dev(big), a_dst=Hn.dev(big))
    want = oracle.aggregate("gat_softmax", rp, ci, Zs, F, heads=heads, a_src=big, a_dst=big)
    assert_close(o.cpu().numpy()[:, :F], want, what="gat large scores")
    # a row with a single neighbour returns that neighbour's row exactly
    o = Hn.aggregate(g, "gat_softmax", Z, F, heads=heads, a_src=asrc, a_dst=asrc).cpu().numpy()[:, :F]
    one = np.flatnonzero(deg == 1)
    assert one.size and np.array_equal(o[one], Zh[ci[rp[one]]])


@pytest.mark.parametrize("mode", MODES)
def test_bitwise_reproducible_and_option_sweep(graphs, mode):
    g, rp, ci = graphs[("skewed", mode == "gcn_sym")]
    n, F, heads = g.n_nodes, 512, 4
    Zh = wl.random_matrix(n, F, 10)
    Z = Hn.dev(Zh)
    kw = {}
    a = None
    if mode == "gat_softmax":
        a = wl.random_matrix(heads, F // heads, 11) * np.float32(0.2)
        kw = dict(heads=heads, a_src=Hn.dev(a), a_dst=Hn.dev(a))
    want = oracle.aggregate(mode, rp, ci, Zh, F, heads=heads, a_src=a, a_dst=a)
    first = Hn.aggregate(g, mode, Z, F, **kw).clone()
    again = Hn.aggregate(g, mode, Z, F, **kw)
    assert torch.equal(first, again)
    try:
        for slab, major, heavy, parts in [(64, 0, 2048, 1), (256, 1, 256, 1), (512, 0, 1 << 20, 1),
                                          (256, 1, 8192, 1), (32, 1, 2048, 1), (128, 1, 512, 1),
                                          (32, 1, 2048, 2), (64, 1, 2048, 4), (32, 0, 2048, 8),
                                          (128, 1, 2048, 16), (64, 0, 512, 1)]:
            B.retexo_set_option("agg_slab_cols", slab)
            B.retexo_set_option("agg_slab_major", major)
            B.retexo_set_option("agg_heavy_degree", heavy)
            B.retexo_set_option("agg_parts", parts)
            got = Hn.aggregate(g, mode, Z, F, **kw).cpu().numpy()[:, :F]
            assert_close(got, want, what="%s slab=%d major=%d heavy=%d parts=%d" % (mode, slab, major, heavy, parts))
            again = Hn.aggregate(g, mode, Z, F, **kw).cpu().numpy()[:, :F]
            assert np.array_equal(got, again)
    finally:
        B.retexo_set_option("agg_slab_cols", 0)
        B.retexo_set_option("agg_slab_major", -1)
        B.retexo_set_option("agg_heavy_degree", 2048)
        B.retexo_set_option("agg_parts", -1)


@pytest.mark.parametrize("mode", ["mean", "gcn_sym", "sum"])
def test_source_range_walk_with_concat_and_ragged_width(graphs, mode):
    """Narrow slabs + several source ranges, with the self half written and a width (602) whose
    last slab is ragged; also the in-place form where Z already sits in out's first F columns."""
    g, rp, ci = graphs[("skewed", mode == "gcn_sym")]
    n, F = g.n_nodes, 602
    Zh = wl.random_matrix(n, F, 31, ld=608)
    want = oracle.aggregate(mode, rp, ci, Zh, F, self_concat=True)
    try:
        for slab, parts in [(32, 4), (64, 8), (128, 2), (32, 16)]:
            B.retexo_set_option("agg_slab_cols", slab)
            B.retexo_set_option("agg_parts", parts)
            got = Hn.aggregate(g, mode, Hn.dev(Zh), F, concat=True).cpu().numpy()[:, :2 * F]
            assert_close(got, want, what="%s concat slab=%d parts=%d" % (mode, slab, parts))
            assert np.array_equal(got[:, :F], Zh[:, :F])
            buf = torch.zeros((n, 1216), dtype=torch.float32, device="cuda")
            buf[:, :F] = torch.from_numpy(Zh[:, :F]).cuda()
            st = B.retexo_aggregate(g.plan, B.MODES[mode], F, 1, buf.data_ptr(), 1216, 0, 0, 0.2,
                                    B.F_SELF_CONCAT, buf.data_ptr(), 1216, 0, 0)
            assert st == B.OK
            assert_close(buf.cpu().numpy()[:, :2 * F], want, what="in place, slab=%d parts=%d" % (slab, parts))
    finally:
        B.retexo_set_option("agg_slab_cols", 0)
        B.retexo_set_option("agg_parts", -1)


@pytest.mark.parametrize("mode", MODES)
def test_code_paths_for_tables_above_4_gib_and_plain_softmax_kernel(graphs, mode):
    """Tables of 4 GiB and more use 64-bit row offsets, and the pipelined edge-softmax kernel falls
    back to the plain one; force those paths on a small table and compare with the oracle."""
    g, rp, ci = graphs[("skewed", mode == "gcn_sym")]
    n, F, heads = g.n_nodes, 188, 4
    Zh = wl.random_matrix(n, F, 41, ld=192)
    a = wl.random_matrix(heads, F // heads, 42) * np.float32(0.2)
    kw = dict(heads=heads, a_src=Hn.dev(a), a_dst=Hn.dev(a)) if mode == "gat_softmax" else {}
    want = oracle.aggregate(mode, rp, ci, Zh, F, heads=heads, a_src=a, a_dst=a, self_concat=True)
    try:
        for wide, fast, slab, parts in [(1, 1, 0, -1), (1, 1, 32, 4), (1, 1, 64, 1), (0, 0, 0, -1), (1, 0, 256, 1)]:
            B.retexo_set_option("agg_wide_offsets", wide)
            B.retexo_set_option("agg_gat_fast", fast)
            B.retexo_set_option("agg_slab_cols", slab)
            B.retexo_set_option("agg_parts", parts)
            got = Hn.aggregate(g, mode, Hn.dev(Zh), F, concat=True, **kw).cpu().numpy()[:, :2 * F]
            assert_close(got, want, what="%s wide=%d fast=%d slab=%d parts=%d" % (mode, wide, fast, slab, parts))
    finally:
        B.retexo_set_option("agg_wide_offsets", 0)
        B.retexo_set_option("agg_gat_fast", 1)
        B.retexo_set_option("agg_slab_cols", 0)
        B.retexo_set_option("agg_parts", -1)


def test_empty_graph_and_zero_width(graphs):
    # a graph without any entry: every aggregate is zero, the self half is still copied
    n = 70
    g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(np.empty(0, np.int32)), Hn.dev(np.empty(0, np.int32)), n, False),
                     validate=True)
    Zh = wl.random_matrix(n, 40, 32)
    a = wl.random_matrix(2, 20, 33)
    for mode in MODES:
        out = Hn.aggregate(g, mode, Hn.dev(Zh), 40, heads=2, a_src=Hn.dev(a), a_dst=Hn.dev(a), concat=True)
        got = out.cpu().numpy()
        assert np.array_equal(got[:, :40], Zh) and np.all(got[:, 40:80] == 0)
    # zero feature width and the zero-node plan are no-ops that succeed
    assert B.retexo_aggregate(g.plan, B.MEAN, 0, 1, 0, 0, 0, 0, 0.2, 0, 0, 0, 0, 0) == B.OK
    g.destroy()
    rp0 = torch.zeros(1, dtype=torch.int64, device="cuda")
    st, plan = B.retexo_plan_create(0, rp0.data_ptr(), 0)
    assert st == B.OK and B.retexo_plan_nnz(plan) == 0
    assert B.retexo_aggregate(plan, B.MEAN, 8, 1, 0, 8, 0, 0, 0.2, 0, 0, 8, 0, 0) == B.OK
    B.retexo_plan_destroy(plan)


def test_in_place_concat_and_argument_errors(graphs):
    g, rp, ci = graphs[("flat", False)]
    n, F = g.n_nodes, 80
    Zh = wl.random_matrix(n, F, 12)
    buf = torch.zeros((n, 2 * F), dtype=torch.float32, device="cuda")
    buf[:, :F] = torch.from_numpy(Zh).cuda()
    st = B.retexo_aggregate(g.plan, B.MEAN, F, 1, buf.data_ptr(), 2 * F, 0, 0, 0.2, B.F_SELF_CONCAT,
                            buf.data_ptr(), 2 * F, 0, 0)
    assert st == B.OK
    assert_close(buf.cpu().numpy(), oracle.aggregate("mean", rp, ci, Zh, F, self_concat=True), what="in place")
    Z = Hn.dev(Zh)
    out = torch.empty((n, 2 * F), dtype=torch.float32, device="cuda")
    args = lambda **k: B.retexo_aggregate(
        k.get("plan", g.plan), k.get("mode", B.MEAN), k.get("F", F), k.get("heads", 1),
        k.get("Z", Z.data_ptr()), k.get("ldz", F), k.get("a", 0), k.get("a", 0), 0.2,
        k.get("flags", 0), k.get("out", out.data_ptr()), k.get("ldo", 2 * F),
        k.get("ws", 0), k.get("wsb", 0))
    assert args() == B.OK
    assert args(mode=9) == B.E_MODE
    assert args(heads=0) == B.E_HEADS
    assert args(mode=B.GAT_SOFTMAX, heads=3, a=Z.data_ptr()) == B.E_HEADS       # 3 does not divide 80
    assert args(mode=B.GAT_SOFTMAX, heads=4) == B.E_NULL                         # attention vectors missing
    assert args(mode=B.GAT_SOFTMAX, heads=4, a=Z.data_ptr()) == B.E_WORKSPACE
    assert args(ldz=F - 1) == B.E_LD
    assert args(flags=B.F_SELF_CONCAT, ldo=2 * F - 1) == B.E_LD
    assert args(flags=B.F_RELU) == B.E_FLAGS
    assert args(out=Z.data_ptr() + 64, ldo=F) == B.E_ALIAS
    assert args(Z=0) == B.E_NULL


@pytest.mark.parametrize("n,heads,C,ldi,ldo", [(1000, 4, 47, 188, 47), (513, 8, 7, 64, 9), (3, 1, 5, 5, 5), (0, 2, 3, 6, 3),
                                              (50, 2, 300, 608, 300), (77, 4, 64, 256, 64),
                                              (100, 3, 7, 24, 8),            # 21 input columns staged as 24
                                              (20, 4, 300, 1200, 304)])      # rows too wide for the staging kernel
def test_head_mean(n, heads, C, ldi, ldo):
    """The last attention round's heads are averaged: plain definition (float64 mean over the head axis)."""
    X = wl.random_matrix(max(n, 1), heads * C, 5, ld=ldi)[:n]
    out = torch.full((max(n, 1), ldo + 2), 9.0, dtype=torch.float32, device="cuda")
    Xd = Hn.dev(np.ascontiguousarray(X)) if n else torch.zeros((1, ldi), dtype=torch.float32, device="cuda")
    B.check(B.retexo_head_mean(n, heads, C, Xd.data_ptr(), ldi, out.data_ptr(), out.stride(0)), "retexo_head_mean")
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = X[:, :heads * C].astype(np.float64).reshape(n, heads, C).mean(axis=1)
    if n:
        assert_close(got[:n, :C], want, what="head mean")
    assert np.all(got[:, C:] == 9.0) and np.all(got[n:] == 9.0)
    assert B.retexo_head_mean(5, 9, C, Xd.data_ptr(), ldi, out.data_ptr(), ldo) == -6
    assert B.retexo_head_mean(5, heads, C, Xd.data_ptr(), heads * C - 1, out.data_ptr(), ldo) == -3


@pytest.mark.parametrize("F,heads", [
    (256, 1),     # one head over the whole wave
    (256, 2),     # 32 lanes per head
    (256, 4),     # 16
    (192, 3),     # 16, last quarter of the lanes idle
    (96, 3),      # 8
    (96, 6),      # 4
    (64, 8),      # 2
    (32, 8),      # one lane per head
    (24, 2),      # heads of three lanes: not a power of two, stays on the score table
])
@pytest.mark.parametrize("concat", [False, True])
def test_edge_softmax_with_scores_from_gathered_rows(graphs, F, heads, concat):
    # ordinary rows compute <a_src, z_u> from the row they gather anyway; long rows and odd head widths read
    # the score table.  Both must match the oracle, and each other to rounding.
    wide = F >= 64          # narrow signed rows are judged element by element against the size of their terms
    results, mags = {}, {}
    try:
        for flash in (1, 0):
            B.retexo_set_option("agg_gat_flash", flash)
            for name in ("skewed", "flat", "tiny"):
                got, want, mag = run_case(graphs, name, "gat_softmax", F, F, heads, concat, seed=F + heads,
                                          with_mag=True)
                what = "gat F=%d heads=%d flash=%d %s" % (F, heads, flash, name)
                assert_cond_close(got, want, mag, what=what)
                if wide:
                    assert_close(got, want, what=what)
                results[(flash, name)] = got
                mags[name] = mag
    finally:
        B.retexo_set_option("agg_gat_flash", 1)
    for name in ("skewed", "flat", "tiny"):
        assert_cond_close(results[(1, name)], results[(0, name)].astype(np.float64), mags[name],
                          what="flash vs table " + name)
    # long rows take the same kernel with eight waves per row: lower the threshold so that many rows do
    try:
        B.retexo_set_option("agg_heavy_degree", 64)
        for name in ("skewed", "flat"):
            got, want, mag = run_case(graphs, name, "gat_softmax", F, F, heads, concat, seed=F + heads, with_mag=True)
            what = "gat F=%d heads=%d, eight waves per row, %s" % (F, heads, name)
            assert_cond_close(got, want, mag, what=what)
            if wide:
                assert_close(got, want, what=what)
            again, _ = run_case(graphs, name, "gat_softmax", F, F, heads, concat, seed=F + heads)
            assert np.array_equal(got, again)
    finally:
        B.retexo_set_option("agg_heavy_degree", 2048)
