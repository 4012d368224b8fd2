"""Whole rounds (retexo_round / retexo_transform chained as the workloads
prescribe) against the oracle: the three small workloads end to end, and the
two large ones stage by stage on every row at full size."""
import numpy as np
import pytest
import torch

import oracle
from paper_2302_13053_amd import binding as B
from paper_2302_13053_amd import harness as Hn
from paper_2302_13053_amd import workloads as wl
from parity import assert_close, assert_cond_close

pytestmark = pytest.mark.gpu


def oracle_stage(st, rp, ci, H, p, rows=None):
    if st.kind == "transform":
        return oracle.transform(H, st.d_in, p.W, p.b, st.relu, rows=rows)
    if st.kind == "head_mean":
        return oracle.head_mean(H if rows is None else H[rows], st.heads, st.d_out)
    return oracle.round_(st.mode, rp, ci, H, st.d_in, p.W, p.b, relu=st.relu, heads=st.heads,
                         a_src=p.a_src, a_dst=p.a_dst, self_concat=st.concat, rows=rows)


@pytest.mark.parametrize("idx", [0, 1, 2])
def test_small_workloads_end_to_end(idx):
    w = wl.workload(idx)
    src, dst = wl.make_graph(w)
    feats = wl.make_features(w, ld=wl.pad_ld(w.feat_dim))
    params = wl.make_params(w)
    pipe = Hn.Pipeline(w, src, dst, feats, params)
    outs = pipe.run()
    torch.cuda.synchronize()
    rp, ci = oracle.csr_from_coo(src, dst, w.n_nodes, w.self_loops)
    assert np.array_equal(pipe.row_ptr.cpu().numpy(), rp)
    assert np.array_equal(pipe.col_idx[:pipe.graph.nnz].cpu().numpy(), ci)
    H = feats
    for i, st in enumerate(w.stages):
        want = oracle_stage(st, rp, ci, H, params[i])
        got = outs[i].cpu().numpy()[:, :st.out_width]
        assert_close(got, want, what="workload %d stage %d (%s)" % (idx, i, st.kind))
        H = want.astype(np.float32)          # the oracle feeds itself, never the GPU's values
    # second pass over the same buffers reproduces the first bit for bit
    keep = [o[:, :st.out_width].clone() for o, st in zip(outs, w.stages)]
    outs = pipe.run()
    torch.cuda.synchronize()
    assert all(torch.equal(a, b[:, :st.out_width]) for a, b, st in zip(keep, outs, w.stages))
    pipe.close()


def test_round_separately_equals_fused_and_gcn_gat_modes():
    n = 4000
    src, dst = wl.random_pairs(n, 30000, 21, skew=2.0)
    H = wl.random_matrix(n, 150, 22, ld=160)
    W = wl.glorot(np.random.Generator(np.random.Philox(key=23)), 150, 192, (150, 192))
    b = wl.random_matrix(1, 192, 24)[0] * np.float32(0.1)
    a_s = wl.random_matrix(4, 48, 25) * np.float32(0.2)
    a_d = wl.random_matrix(4, 48, 26) * np.float32(0.2)
    for mode, concat, relu, sl in [("gcn_sym", False, True, True), ("gat_softmax", False, False, False),
                                   ("mean", True, True, False), ("sum", False, False, False)]:
        g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, sl))
        rp, ci = oracle.csr_from_coo(src, dst, n, sl)
        st = wl.Stage("round", 150, 192, relu=relu, mode=mode, concat=concat, heads=4)
        out = torch.empty((n, wl.pad_ld(st.out_width)), dtype=torch.float32, device="cuda")
        ws = Hn.ws_tensor(B.retexo_workspace_bytes(g.plan, 192, B.MODES[mode], 4,
                                                   B.F_SELF_CONCAT if concat else 0))
        gat = mode == "gat_softmax"
        Hn.round_(g, st, Hn.dev(H), Hn.dev(W), Hn.dev(b), Hn.dev(a_s) if gat else None,
                  Hn.dev(a_d) if gat else None, out, ws)
        want = oracle.round_(mode, rp, ci, H, 150, W, b, relu=relu, heads=4, a_src=a_s, a_dst=a_d,
                             self_concat=concat)
        assert_close(out.cpu().numpy()[:, :st.out_width], want, what="round " + mode)
        # the two-call form gives the same bits as the fused call
        Z = Hn.transform(Hn.dev(H), 150, Hn.dev(W), Hn.dev(b), relu)
        out2 = Hn.aggregate(g, mode, Z, 192, heads=4, a_src=Hn.dev(a_s) if gat else None,
                            a_dst=Hn.dev(a_d) if gat else None, concat=concat)
        assert torch.equal(out2[:, :st.out_width], out[:, :st.out_width])
        g.destroy()


@pytest.mark.parametrize("n,heads,dh,seed", [(5000, 4, 47, 1), (3000, 8, 27, 2), (2000, 2, 30, 3), (1500, 4, 7, 4),
                                             (1200, 4, 75, 5)])          # the last: two float4 per lane and row
def test_attention_round_with_the_source_scores_kept_in_the_rows_of_z(n, heads, dh, seed):
    # head widths that are not a power-of-two number of four-float lanes: retexo_round keeps <a_src, z_u> in
    # the unused columns of its own Z rows.  Written there by the score kernel: same bits as with the score
    # table.  Written there by the transform itself (as h_u (W a_src) + <b, a_src>, one more output column per
    # head; the destination scores then come from row v inside the aggregation kernel): the same scores up to
    # fp32 rounding.  All three: parity with the oracle.
    F = heads * dh
    assert F % 4 == 0 and F % 32 != 0
    src, dst = wl.graph_power_law(n, 12 * n, 2.2, 24.0, 3000.0, seed)
    g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, False))
    rp, ci = oracle.csr_from_coo(src, dst, n, False)
    H = wl.random_matrix(n, 60, seed + 10, ld=64)
    W = wl.glorot(np.random.Generator(np.random.Philox(key=seed + 20)), 60, F, (60, F))
    b = wl.random_matrix(1, F, seed + 30)[0] * np.float32(0.1)
    a_s = wl.random_matrix(heads, dh, seed + 40) * np.float32(0.3)
    a_d = wl.random_matrix(heads, dh, seed + 50) * np.float32(0.3)
    st = wl.Stage("round", 60, F, relu=False, mode="gat_softmax", concat=False, heads=heads)
    ws = Hn.ws_tensor(B.retexo_workspace_bytes(g.plan, F, B.GAT_SOFTMAX, heads, 0))
    outs = []
    try:
        for in_rows, fold in ((1, 0), (0, 0), (1, 1)):
            B.retexo_set_option("agg_gat_in_rows", in_rows)
            B.retexo_set_option("agg_gat_fold", fold)
            out = torch.full((n, wl.pad_ld(F)), -5.0, dtype=torch.float32, device="cuda")
            Hn.round_(g, st, Hn.dev(H), Hn.dev(W), Hn.dev(b), Hn.dev(a_s), Hn.dev(a_d), out, ws)
            torch.cuda.synchronize()
            outs.append(out)
    finally:
        B.retexo_set_option("agg_gat_in_rows", 1)
        B.retexo_set_option("agg_gat_fold", 1)
    assert torch.equal(outs[0], outs[1])
    want = oracle.round_("gat_softmax", rp, ci, H, 60, W, b, relu=False, heads=heads, a_src=a_s, a_dst=a_d)
    for out, what in ((outs[0], "score kernel"), (outs[2], "transform")):
        assert bool((out[:, F:] == -5.0).all())
        assert_close(out.cpu().numpy()[:, :F], want, what="attention round, scores in the rows by the " + what)
    g.destroy()


def test_round_argument_errors_leave_the_output_untouched():
    n, d_in, d_out = 300, 40, 64
    src, dst = wl.random_pairs(n, 2000, 31)
    g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, False))
    H = Hn.dev(wl.random_matrix(n, d_in, 32, ld=64))
    W = Hn.dev(wl.random_matrix(d_in, d_out, 33))
    b = Hn.dev(wl.random_matrix(1, d_out, 34)[0])
    out = torch.full((n, 128), -7.0, dtype=torch.float32, device="cuda")
    ws = Hn.ws_tensor(B.retexo_workspace_bytes(g.plan, d_out, B.GAT_SOFTMAX, 4, 0))

    def call(mode=B.MEAN, di=d_in, do=d_out, heads=1, h=H.data_ptr(), ldh=64, w=W.data_ptr(), bias=b.data_ptr(),
             a=0, flags=0, o=out.data_ptr(), ldo=128, wsp=ws.data_ptr(), wsb=ws.numel()):
        return B.retexo_round(g.plan, mode, di, do, heads, h, ldh, w, bias, a, a, 0.2, flags, o, ldo, wsp, wsb)

    assert call(di=-1) == B.E_SIZE
    assert call(di=1 << 31) == B.E_SIZE
    assert call(do=1 << 30) == B.E_SIZE
    assert call(mode=9) == B.E_MODE
    assert call(heads=0) == B.E_HEADS
    assert call(mode=B.GAT_SOFTMAX, heads=3, a=W.data_ptr()) == B.E_HEADS        # 64 columns, 3 heads
    assert call(flags=64) == B.E_FLAGS
    assert call(w=0, bias=0) == B.E_SIZE                                         # identity needs D_out == D_in
    assert call(w=0, do=d_in) == B.E_FLAGS                                       # a bias without a weight matrix
    assert call(w=0, bias=0, do=d_in, flags=B.F_RELU) == B.E_FLAGS
    assert call(h=0) == B.E_NULL
    assert call(o=0) == B.E_NULL
    assert call(mode=B.GAT_SOFTMAX, heads=4) == B.E_NULL                         # attention vectors missing
    assert call(ldh=d_in - 1) == B.E_LD
    assert call(flags=B.F_SELF_CONCAT, ldo=2 * d_out - 1) == B.E_LD
    assert call(o=H.data_ptr() + 128, ldo=64) == B.E_ALIAS
    assert call(wsp=0) == B.E_WORKSPACE
    assert call(wsp=ws.data_ptr() + 64) == B.E_WORKSPACE
    assert call(wsb=1024) == B.E_WORKSPACE
    assert call(wsp=out.data_ptr(), wsb=out.numel() * 4) == B.E_ALIAS             # Z staged on top of the output
    torch.cuda.synchronize()
    assert bool((out == -7.0).all())
    assert call() == B.OK
    torch.cuda.synchronize()
    assert not bool((out[:, :d_out] == -7.0).any()) and bool((out[:, d_out:] == -7.0).all())
    g.destroy()


def test_one_partitions_share_matches_the_global_result():
    """The edge-partitioned set-up of the paper on one GPU: a worker holds its inner nodes, its
    boundary nodes and the edges touching an inner node, numbered [inner | boundary].  Running
    the same entry points on that local graph must reproduce the global result on inner rows."""
    w = wl.workload(2)
    src, dst = wl.make_graph(w)
    n = w.n_nodes
    Z = wl.make_features(w, ld=wl.pad_ld(w.feat_dim))
    F = w.feat_dim
    rp, ci = oracle.csr_from_coo(src, dst, n, False)
    want = oracle.aggregate("mean", rp, ci, Z, F, self_concat=True)
    owner = (np.arange(n) * 2654435761 % 4294967296) >> 31          # two workers, scattered ownership
    for worker in (0, 1):
        inner = np.flatnonzero(owner == worker)
        keep = (owner[src] == worker) | (owner[dst] == worker)      # edges with an inner endpoint
        s, d = src[keep], dst[keep]
        boundary = np.setdiff1d(np.unique(np.concatenate([s, d])), inner)
        local_ids = np.concatenate([inner, boundary])
        to_local = np.full(n, -1, np.int64)
        to_local[local_ids] = np.arange(local_ids.size)
        g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(to_local[s].astype(np.int32)),
                                         Hn.dev(to_local[d].astype(np.int32)), local_ids.size, False))
        Zl = np.ascontiguousarray(Z[local_ids])                     # inner rows, then received boundary rows
        out = Hn.aggregate(g, "mean", Hn.dev(Zl), F, concat=True).cpu().numpy()[:inner.size, :2 * F]
        assert_close(out, want[inner], what="worker %d inner rows" % worker)
        g.destroy()


BLOCK = 1 << 17          # rows per comparison block: bounds the float64 temporaries at full size


def compare_all_rows(got_dev, st, want_rows, mag_rows, what):
    """Every row of one stage: ``got_dev`` (device, [n, ld]) against ``want_rows(block)`` (float64 rows of the
    oracle for the int64 row ids ``block``), block by block.  Returns the oracle's rows as float32 (the next
    stage's input), the worst row-normwise error and, when ``mag_rows`` is given, the worst element-wise error
    relative to the size of the element's terms."""
    n = got_dev.shape[0]
    nxt = np.zeros((n, wl.pad_ld(st.out_width)), np.float32)
    worst = worst_cond = 0.0
    for lo in range(0, n, BLOCK):
        block = np.arange(lo, min(n, lo + BLOCK), dtype=np.int64)
        want = want_rows(block)
        got = got_dev[lo:lo + block.size, :st.out_width].cpu().numpy()
        worst = max(worst, assert_close(got, want, what="%s rows %d.." % (what, lo)))
        if mag_rows is not None:
            worst_cond = max(worst_cond, assert_cond_close(got, want, mag_rows(block), what="%s rows %d.." % (what, lo)))
        nxt[lo:lo + block.size, :st.out_width] = want
    return nxt, worst, worst_cond


@pytest.mark.parametrize("idx", [3, 4])
def test_large_workloads_full_size_all_rows(idx):
    """Every row of every stage of the two large workloads at full size, in the launch configuration the
    benchmark uses.  The stages are chained through the oracle: stage i runs on the float32 copy of the
    oracle's own output of stage i-1 (uploaded), so no stage is judged on another stage's rounding.
    Then the exact pins on the same graph: a sum over ones is the degree, a sum over small integers is
    exact whatever the order, the self half of a concatenated output is a bit copy — for all rows."""
    w = wl.workload(idx)
    n = w.n_nodes
    print("generating workload", idx, flush=True)
    src, dst = wl.make_graph(w)
    feats = wl.make_features(w, ld=wl.pad_ld(w.feat_dim))
    params = wl.make_params(w)
    pipe = Hn.Pipeline(w, src, dst, feats, params)
    print("gpu csr + plan", flush=True)
    pipe.build_graph()
    torch.cuda.synchronize()
    print("oracle csr", flush=True)
    rp, ci = oracle.csr_from_coo(src, dst, n, w.self_loops)
    assert np.array_equal(pipe.row_ptr.cpu().numpy(), rp)
    assert np.array_equal(pipe.col_idx[:pipe.graph.nnz].cpu().numpy(), ci)
    deg, dinv, _ = Hn.plan_arrays(pipe.graph)
    odeg, odinv = oracle.degree(rp)
    assert np.array_equal(deg, odeg) and np.array_equal(dinv.view(np.uint32), odinv.view(np.uint32))
    del src, dst
    H = feats
    for i, st in enumerate(w.stages):
        p = params[i]
        if i > 0:
            pipe.outs[i - 1].copy_(torch.from_numpy(H))          # the oracle's previous output, as float32
        pipe.run_stage(i)
        torch.cuda.synchronize()
        what = "workload %d stage %d (%s)" % (idx, i, st.kind)
        mag_rows = None
        if st.kind == "transform":
            want_rows = lambda b: oracle.transform(H, st.d_in, p.W, p.b, st.relu, rows=b)
        elif st.kind == "head_mean":
            want_rows = lambda b: oracle.head_mean(H[b], st.heads, st.d_out)
        else:
            # the round as the pipeline stores it: Z rounded to float32 (all rows, once), then aggregated
            Z32 = H if p.W is None else oracle.transform(H, st.d_in, p.W, p.b, st.relu).astype(np.float32)
            kw = dict(heads=st.heads, a_src=p.a_src, a_dst=p.a_dst, self_concat=st.concat)
            want_rows = lambda b: oracle.aggregate(st.mode, rp, ci, Z32, st.d_out, rows=b, **kw)
            if i == 0:      # the size of every element's terms, for the first (widest) aggregation
                mag_rows = lambda b: oracle.aggregate_abs(st.mode, rp, ci, Z32, st.d_out, rows=b, **kw)
        H, worst, worst_cond = compare_all_rows(pipe.outs[i], st, want_rows, mag_rows, what)
        print("%s: all %d rows, worst row-normwise error %.2e, relative to the terms %.2e"
              % (what, n, worst, worst_cond), flush=True)
        if st.kind == "round" and st.concat:
            Zsrc = pipe.H0 if i == 0 else None
            if Zsrc is not None:     # identity round: the self half is a bit copy of the input, every row
                assert torch.equal(pipe.outs[i][:, :st.d_out], Zsrc[:, :st.d_out])
    del H
    # exact pins on this graph, all rows, through the kernels this graph's plan selects
    g = pipe.graph
    F1 = w.stages[0].d_out
    ones = torch.ones((n, wl.pad_ld(F1)), dtype=torch.float32, device="cuda")
    out = Hn.aggregate(g, "sum", ones, F1)
    torch.cuda.synchronize()
    assert torch.equal(out[:, :F1], torch.from_numpy(odeg.astype(np.float32)).cuda()[:, None].expand(n, F1))
    out = Hn.aggregate(g, "mean", ones, F1)
    torch.cuda.synchronize()
    assert torch.equal(out[:, :F1], torch.from_numpy((odeg > 0).astype(np.float32)).cuda()[:, None].expand(n, F1))
    del ones, out
    Fi = 64
    ints = wl.random_matrix(n, Fi, 900 + idx, ld=Fi, kind="smallint")
    out = Hn.aggregate(g, "sum", Hn.dev(ints), Fi, concat=True)
    torch.cuda.synchronize()
    for lo in range(0, n, BLOCK):
        block = np.arange(lo, min(n, lo + BLOCK), dtype=np.int64)
        want = oracle.aggregate("sum", rp, ci, ints, Fi, self_concat=True, rows=block)
        assert np.array_equal(out[lo:lo + block.size, :2 * Fi].cpu().numpy().astype(np.float64), want), lo
    print("exact pins: ones -> degree (F=%d), small integers bit-exact (F=%d), all %d rows" % (F1, Fi, n), flush=True)
    pipe.close()
