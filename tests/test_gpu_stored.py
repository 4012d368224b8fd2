"""Aggregation over a table in 16-bit storage (retexo_store_rows, retexo_aggregate_stored).

The rounding to bf16 / fp16 is integer work and must match the oracle bit for bit; the aggregation is
then compared with the oracle run on exactly the stored values, to the fp32 path's bound."""
import numpy as np
import pytest
import torch

import oracle
from oracle import storage as ost
from paper_2302_13053_amd import binding as B
from paper_2302_13053_amd import harness as Hn
from paper_2302_13053_amd import workloads as wl
from parity import assert_close, assert_cond_close

pytestmark = pytest.mark.gpu

FORMATS = ["bf16", "fp16"]


@pytest.fixture(scope="module")
def graphs():
    specs = {"skewed": (5000, 60000, 3.0, 4), "flat": (3000, 20000, 0.0, 5), "tiny": (3, 2, 0.0, 6)}
    out = {}
    for name, (n, pairs, skew, seed) in specs.items():
        src, dst = wl.random_pairs(n, pairs, seed, skew=skew)
        for sl in (False, True):
            g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, sl), validate=True, split_rows=(name == "skewed"))
            out[(name, sl)] = (g, *oracle.csr_from_coo(src, dst, n, sl))
    yield out
    for g, _, _ in out.values():
        g.destroy()


@pytest.mark.parametrize("fmt", FORMATS)
def test_store_rows_is_bit_exact(fmt):
    f = np.float32
    special = np.array([0.0, -0.0, 1.0, 65504.0, 65520.0, 65536.0, 6e-8, 2.98e-8, 2.99e-8, 1e-40, 3.4e38, np.inf, -np.inf,
                        np.nan, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 2.0 ** -24, 2.0 ** -25,
                        1.5 * 2.0 ** -25, -0.3, 2.0 ** -133, 0.1], f)
    rows, F, ld = 700, 37, 41
    X = wl.random_matrix(rows, F, 3, ld=ld) * f(2.5)
    X[:special.size, 0] = special
    X[:, 1] *= f(1e-6)
    X[:, 2] *= f(3e4)
    got = Hn.store_rows(Hn.dev(X), F, fmt, ld=40).cpu().numpy().view(np.uint16)
    want = ost.store(X[:, :F], fmt)
    assert np.array_equal(got[:, :F], want)
    assert np.all(got[:, F:] == 0)                      # nothing written past the F columns
    assert B.retexo_store_rows(3, 1, 1, 1, 1, 1, 1) == -4 and B.retexo_store_rows(1, 5, 9, 1, 8, 1, 9) == -3


def run_case(graphs, name, mode, fmt, F, ld16, heads, concat, seed, kind="normal", with_mag=False):
    g, rp, ci = graphs[(name, mode == "gcn_sym")]
    n = g.n_nodes
    Zh = wl.random_matrix(n, F, seed, kind=kind)
    Z16 = Hn.store_rows(Hn.dev(Zh), F, fmt, ld=ld16)
    stored = ost.load(ost.store(Zh, fmt), fmt)          # the values the table stands for
    a_s = a_d = None
    kw = {}
    if mode == "gat_softmax":
        a_s = wl.random_matrix(heads, F // heads, seed + 1) * np.float32(0.3)
        a_d = wl.random_matrix(heads, F // heads, seed + 2) * np.float32(0.3)
        kw = dict(heads=heads, a_src=Hn.dev(a_s), a_dst=Hn.dev(a_d))
    ow = 2 * F if concat else F
    out = torch.full((n, ow + 3), 555.0, dtype=torch.float32, device="cuda")
    Hn.aggregate_stored(g, mode, Z16, F, fmt, concat=concat, out=out, **kw)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.all(got[:, ow:] == 555.0)
    want = oracle.aggregate(mode, rp, ci, stored, F, heads=heads, a_src=a_s, a_dst=a_d, self_concat=concat)
    if with_mag:
        mag = oracle.aggregate_abs(mode, rp, ci, stored, F, heads=heads, a_src=a_s, a_dst=a_d, self_concat=concat)
        return got[:, :ow], want, mag
    return got[:, :ow], want


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("mode", ["sum", "mean", "gcn_sym", "gat_softmax", "max"])
@pytest.mark.parametrize("F,ld16,heads,concat", [
    (256, 256, 4, False),      # 16-byte gathers, 32 lanes
    (602, 608, 1, True),       # ragged last vector, two chunks
    (1432, 1432, 4, False),    # two slabs of 1024 columns
    (188, 192, 4, False),      # heads of 47 columns straddle lanes
    (100, 100, 4, True),       # rows not a multiple of 16 bytes: two-byte gathers
    (64, 64, 8, False),
    (7, 8, 1, True),
    (1, 1, 1, False),
])
def test_stored_modes_match_oracle_on_skewed_graph(graphs, fmt, mode, F, ld16, heads, concat):
    if mode == "gat_softmax" and F % heads:
        heads = 1
    # signed data at every width: each element within 1e-5 of the size of its terms, and rows of at least 64
    # columns also within 1e-5 of the row's largest magnitude
    got, want, mag = run_case(graphs, "skewed", mode, fmt, F, ld16, heads, concat, seed=F + 31, with_mag=True)
    if mode == "max":
        assert np.array_equal(got.astype(np.float64), want)
    else:
        assert_cond_close(got, want, mag, what="%s %s F=%d" % (fmt, mode, F))
        if F >= 64:
            assert_close(got, want, what="%s %s F=%d" % (fmt, mode, F))
    if concat:
        assert np.array_equal(got[:, :F].astype(np.float64), want[:, :F])      # self half: the stored value, widened


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("mode", ["mean", "gcn_sym", "gat_softmax"])
def test_stored_other_graphs(graphs, fmt, mode):
    for name in ("flat", "tiny"):
        got, want = run_case(graphs, name, mode, fmt, 96, 96, 3, True, seed=5)
        assert_close(got, want, what="%s %s %s" % (fmt, mode, name))


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("mode", ["sum", "mean", "gcn_sym"])
def test_narrow_slabs_and_source_ranges(graphs, fmt, mode):
    """The 64-column slab path with the rows walked range by range (forced here; chosen automatically for
    dense graphs), with a ragged last slab and the self half written."""
    try:
        B.retexo_set_option("agg_slab_cols", 64)
        for parts in (1, 4, 16):
            B.retexo_set_option("agg_parts", parts)
            got, want = run_case(graphs, "skewed", mode, fmt, 602, 608, 1, True, seed=9)
            assert_close(got, want, what="%s %s narrow parts=%d" % (fmt, mode, parts))
            again, _ = run_case(graphs, "skewed", mode, fmt, 602, 608, 1, True, seed=9)
            assert np.array_equal(got, again)
    finally:
        B.retexo_set_option("agg_slab_cols", 0)
        B.retexo_set_option("agg_parts", -1)


def test_stored_argument_errors(graphs):
    g, _, _ = graphs[("flat", False)]
    n = g.n_nodes
    Z16 = torch.zeros((n, 64), dtype=torch.int16, device="cuda")
    out = torch.zeros((n, 64), dtype=torch.float32, device="cuda")
    call = lambda **k: B.retexo_aggregate_stored(**dict(dict(plan=g.plan, mode=0, storage=1, F=64, heads=1, d_Z=Z16.data_ptr(),
                                                             ldz=64, d_attn_src=0, d_attn_dst=0, negative_slope=0.2, flags=0,
                                                             d_out=out.data_ptr(), ldo=64, d_workspace=0, workspace_bytes=0), **k))
    assert call() == 0
    assert call(storage=3) == -4 and call(ldz=63) == -3 and call(flags=B.F_RELU) == -5
    assert call(mode=3) == -1                           # edge softmax without attention vectors
    assert call(d_out=Z16.data_ptr()) == -9
    torch.cuda.synchronize()


@pytest.mark.parametrize("idx", [3, 4])
def test_full_size_stored_first_round(idx):
    """The first round's aggregation of the two large workloads on a bf16 table at full size (the launch
    configuration chosen automatically), every row against the oracle on the stored values."""
    w = wl.workload(idx)
    print("generating workload", idx, flush=True)
    src, dst = wl.make_graph(w)
    n = w.n_nodes
    g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, w.self_loops))
    print("oracle csr", flush=True)
    rp, ci = oracle.csr_from_coo(src, dst, n, w.self_loops)
    del src, dst
    st = w.stages[0]
    F = st.d_out
    p_ = wl.make_params(w)[0]
    Zh = wl.random_matrix(n, F, 90 + idx, ld=wl.pad_ld(F))
    Zd = Hn.dev(Zh)
    Z16 = Hn.store_rows(Zd, F, "bf16")
    kw = {}
    if st.mode == "gat_softmax":
        kw = dict(heads=st.heads, a_src=Hn.dev(p_.a_src), a_dst=Hn.dev(p_.a_dst))
    out = Hn.aggregate_stored(g, st.mode, Z16, F, "bf16", concat=st.concat, **kw)
    torch.cuda.synchronize()
    print("oracle: all %d rows" % n, flush=True)
    stored = ost.load(ost.store(Zh[:, :F], "bf16"), "bf16")
    worst = 0.0
    for lo in range(0, n, 1 << 17):
        rows = np.arange(lo, min(n, lo + (1 << 17)), dtype=np.int64)
        ref = oracle.aggregate(st.mode, rp, ci, stored, F, heads=st.heads, a_src=p_.a_src, a_dst=p_.a_dst,
                               self_concat=st.concat, rows=rows)
        got = out[lo:lo + rows.size, :ref.shape[1]].cpu().numpy()
        worst = max(worst, assert_close(got, ref, what="workload %d bf16 first round, rows %d.." % (idx, lo)))
    print("workload %d bf16 table: all %d rows, worst row-normwise error %.2e" % (idx, n, worst), flush=True)
    # timing beside the fp32 path (printed with -s)
    ws = Hn.ws_tensor(max(B.retexo_workspace_bytes(g.plan, F, B.MODES[st.mode], st.heads, 0), 256))
    o32 = torch.empty_like(out)

    def t(fn, reps=5):
        fn(); torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    t32 = t(lambda: Hn.aggregate(g, st.mode, Zd, F, concat=st.concat, out=o32, workspace=ws, **kw))
    t16 = t(lambda: Hn.aggregate_stored(g, st.mode, Z16, F, "bf16", concat=st.concat, out=out, workspace=ws, **kw))
    Zh16 = Hn.store_rows(Zd, F, "fp16")
    th = t(lambda: Hn.aggregate_stored(g, st.mode, Zh16, F, "fp16", concat=st.concat, out=out, workspace=ws, **kw))
    print("workload %d first-round aggregation: fp32 table %.2f ms, bf16 table %.2f ms, fp16 table %.2f ms"
          % (idx, t32, t16, th), flush=True)
    g.destroy()


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("F,heads", [(256, 1), (256, 2), (256, 4), (192, 3), (96, 3), (96, 6), (64, 8), (32, 8), (24, 2)])
@pytest.mark.parametrize("concat", [False, True])
def test_stored_edge_softmax_with_scores_from_gathered_rows(graphs, fmt, F, heads, concat):
    # ordinary rows compute <a_src, z_u> from the stored row they gather; long rows and head widths that are
    # not a power-of-two number of lanes read the score table: both against the oracle, and each other
    wide = F >= 64
    results, mags = {}, {}
    try:
        for flash in (1, 0):
            B.retexo_set_option("agg_gat_flash", flash)
            for name in ("skewed", "flat", "tiny"):
                got, want, mag = run_case(graphs, name, "gat_softmax", fmt, F, F, heads, concat, seed=F + heads,
                                          with_mag=True)
                what = "%s gat F=%d heads=%d flash=%d %s" % (fmt, F, heads, flash, name)
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
