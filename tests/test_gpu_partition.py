"""A worker's share of an edge-partitioned graph on the GPU (retexo_partition_share, retexo_halo_pack /
retexo_halo_unpack, retexo_plan_set_degrees): bit-exact against the oracle, and partition-shaped
rounds on one GPU (several workers' shares side by side, rows exchanged through pack -> unpack)
against the oracle's global result."""
import numpy as np
import pytest
import torch

import oracle
from oracle import partition as op
from paper_2302_13053_amd import binding as B
from paper_2302_13053_amd import harness as Hn
from paper_2302_13053_amd import workloads as wl
from parity import assert_close

pytestmark = pytest.mark.gpu


def owner_map(n, P, seed):
    """Seeded balanced random ownership: the worst case for the boundary (no locality at all)."""
    return np.random.Generator(np.random.Philox(key=seed)).integers(0, P, n).astype(np.int32)


def check_share(ds: Hn.DeviceShare, want: op.Share, P: int):
    assert (ds.n_inner, ds.n_halo) == (want.n_inner, want.n_halo)
    assert np.array_equal(ds.local_ids.cpu().numpy(), want.local_ids)
    assert np.array_equal(ds.graph.row_ptr.cpu().numpy(), want.row_ptr)
    assert np.array_equal(ds.graph.col_idx[:ds.graph.nnz].cpu().numpy(), want.col_idx)
    assert np.array_equal(ds.global_deg.cpu().numpy(), want.global_deg)
    send, recv = ds.send_ids.cpu().numpy(), ds.recv_ids.cpu().numpy()
    assert ds.send_offsets[0] == 0 and ds.recv_offsets[0] == 0
    assert ds.send_offsets[P] == send.size and ds.recv_offsets[P] == recv.size == want.n_halo
    for q in range(P):
        assert np.array_equal(send[ds.send_offsets[q]:ds.send_offsets[q + 1]], want.send_ids[q])
        assert np.array_equal(recv[ds.recv_offsets[q]:ds.recv_offsets[q + 1]], want.recv_ids[q])


@pytest.mark.parametrize("n,pairs,skew,self_loops,P", [
    (5000, 60000, 3.0, False, 4),       # rows far longer than a wave, many empty rows
    (3000, 20000, 0.0, True, 3),
    (2000, 9000, 1.0, False, 64),       # the most workers the mask holds
    (700, 3000, 1.0, False, 1),         # a single worker owns everything
    (3, 2, 0.0, False, 2),
])
def test_share_is_bit_exact(n, pairs, skew, self_loops, P):
    src, dst = wl.random_pairs(n, pairs, n + P, skew=skew)
    g = Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, self_loops)
    rp, ci = oracle.csr_from_coo(src, dst, n, self_loops)
    part = owner_map(n, P, 5)
    dpart = Hn.dev(part)
    for p in sorted({0, P // 2, P - 1}):
        check_share(Hn.partition_share(g, dpart, P, p), op.share(rp, ci, part, P, p), P)
    # a worker that owns nothing
    part2 = np.where(part == 0, 1 % P, part).astype(np.int32)
    if P > 1:
        ds = Hn.partition_share(g, Hn.dev(part2), P, 0)
        assert (ds.n_inner, ds.n_halo, ds.graph.nnz) == (0, 0, 0)
        assert ds.graph.row_ptr.cpu().numpy().tolist() == [0]


def test_share_argument_errors():
    n, P = 100, 4
    src, dst = wl.random_pairs(n, 300, 1)
    g = Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, False)
    part = owner_map(n, P, 2)
    ws = Hn.ws_tensor(B.retexo_partition_workspace_bytes(n, P, 1000))
    big = torch.empty(4000, dtype=torch.int64, device="cuda")
    args = lambda **k: dict(dict(n_nodes=n, d_row_ptr=g.row_ptr.data_ptr(), d_col_idx=g.col_idx.data_ptr(),
                                 d_part=dpart.data_ptr(), n_parts=P, part=1, local_capacity=1000, col_capacity=4000,
                                 send_capacity=1000, d_local_ids=big.data_ptr(), d_local_row_ptr=big.data_ptr(),
                                 d_local_col_idx=big.data_ptr(), d_global_deg=big.data_ptr(), d_send_ids=big.data_ptr(),
                                 d_recv_ids=big.data_ptr(), d_workspace=ws.data_ptr(), workspace_bytes=ws.numel()), **k)
    dpart = Hn.dev(part)
    st, sizes, _, _ = B.retexo_partition_share(**args(local_capacity=0))
    assert st == -11 and sizes[0] > 0 and sizes[2] > 0                   # size query: capacity error, sizes filled
    assert B.retexo_partition_share(**args(col_capacity=sizes[2] - 1))[0] == -11
    assert B.retexo_partition_share(**args(send_capacity=sizes[3] - 1))[0] == -11
    assert B.retexo_partition_share(**args(part=4))[0] == -2
    assert B.retexo_partition_share(**args(n_parts=65))[0] == -2
    assert B.retexo_partition_share(**args(workspace_bytes=1024))[0] == -8
    bad = part.copy()
    bad[17] = 4
    dpart = Hn.dev(bad)
    assert B.retexo_partition_share(**args())[0] == -12                   # a worker id out of range
    bad[17] = -1
    dpart = Hn.dev(bad)
    assert B.retexo_partition_share(**args())[0] == -12
    assert B.retexo_partition_workspace_bytes(n, 0, 0) == -2


@pytest.mark.parametrize("F,ld,offset", [(256, 256, 0), (602, 608, 0), (7, 7, 0), (100, 100, 1), (1, 3, 0)])
def test_pack_and_unpack_rows(F, ld, offset):
    rows, n = 3000, 1100
    rng = np.random.Generator(np.random.Philox(key=F))
    ids = rng.permutation(rows)[:n].astype(np.int32)
    Hh = wl.random_matrix(rows, F, 3, ld=ld)
    buf_t = torch.full((rows * ld + 8,), 7.0, dtype=torch.float32, device="cuda")
    H = buf_t[offset:offset + rows * ld].view(rows, ld)
    H.copy_(torch.from_numpy(Hh))
    buf = torch.full((n, ld + 4), 5.0, dtype=torch.float32, device="cuda")
    Hn.halo_pack(Hn.dev(ids), H, F, buf=buf)
    got = buf.cpu().numpy()
    assert np.array_equal(got[:, :F], Hh[ids, :F]) and np.all(got[:, F:] == 5.0)
    # unpack into another table: only the listed rows and only their first F columns change
    T = torch.full((rows, ld), 9.0, dtype=torch.float32, device="cuda")
    Hn.halo_unpack(Hn.dev(ids), buf, T, F)
    want = np.full((rows, ld), 9.0, np.float32)
    want[ids, :F] = Hh[ids, :F]
    assert np.array_equal(T.cpu().numpy(), want)
    # ids outside the table are skipped, an empty list is a no-op
    wild = np.array([0, rows, -1, 5], np.int32)
    T.fill_(9.0)
    Hn.halo_unpack(Hn.dev(wild), buf, T, F)
    t = T.cpu().numpy()
    assert np.array_equal(t[0, :F], got[0, :F]) and np.array_equal(t[5, :F], got[3, :F]) and np.all(t[1:5] == 9.0)
    Hn.halo_pack(torch.empty(0, dtype=torch.int32, device="cuda"), H, F, buf=buf)
    assert B.retexo_halo_pack(4, Hn.dev(wild).data_ptr(), rows, F, H.data_ptr(), F - 1 if F > 1 else 0, buf.data_ptr(), ld + 4) == -3


class Worker:
    """One worker of a partition-shaped run held on this GPU: share, plan, feature table."""

    def __init__(self, g, dpart, P, p, gcn):
        self.share = Hn.partition_share(g, dpart, P, p)
        self.graph = Hn.make_plan(self.share.graph, validate=True)
        if gcn:
            B.check(B.retexo_plan_set_degrees(self.graph.plan, self.share.global_deg.data_ptr()), "set_degrees")
        self.n_local = self.share.n_inner + self.share.n_halo
        self.inner_ids = self.share.local_ids[:self.share.n_inner].cpu().numpy()


def exchange(workers, tables, F):
    """Every worker packs, for each peer, the rows that peer needs; the peer unpacks them into its
    boundary rows.  (One GPU: the transfer itself is the buffer changing hands.)"""
    P = len(workers)
    for p, wp in enumerate(workers):
        for q, wq in enumerate(workers):
            a, b = wp.share.send_offsets[q], wp.share.send_offsets[q + 1]
            c, d = wq.share.recv_offsets[p], wq.share.recv_offsets[p + 1]
            assert b - a == d - c
            if b > a:
                buf = Hn.halo_pack(wp.share.send_ids[a:b], tables[p], F)
                Hn.halo_unpack(wq.share.recv_ids[c:d], buf, tables[q], F)
    assert P == len(tables)


@pytest.mark.parametrize("idx,P", [(2, 4), (1, 3), (0, 2)])
def test_partition_shaped_pipeline_matches_global_oracle(idx, P):
    """The small workloads end to end with P workers: per round each worker transforms its inner rows,
    the boundary rows are exchanged, and each worker aggregates over its local graph.  Every worker's
    inner rows must equal the oracle's global result, stage by stage (the oracle feeds itself)."""
    w = wl.workload(idx)
    src, dst = wl.make_graph(w)
    n = w.n_nodes
    feats = wl.make_features(w, ld=wl.pad_ld(w.feat_dim))
    params = wl.make_params(w)
    rp, ci = oracle.csr_from_coo(src, dst, n, w.self_loops)
    g = Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, w.self_loops)
    part = owner_map(n, P, 40 + idx)
    dpart = Hn.dev(part)
    workers = [Worker(g, dpart, P, p, w.family == "gcn") for p in range(P)]
    assert sum(wk.share.n_inner for wk in workers) == n
    H_glob = feats                                             # oracle side, global numbering
    H_loc = [Hn.dev(np.ascontiguousarray(feats[wk.inner_ids])) for wk in workers]     # inner rows only
    for i, st in enumerate(w.stages):
        p_ = params[i]
        if st.kind == "transform":
            want = oracle.transform(H_glob, st.d_in, p_.W, p_.b, st.relu)
            outs = [Hn.transform(H_loc[k], st.d_in, Hn.dev(p_.W), Hn.dev(p_.b) if p_.b is not None else None, st.relu)
                    for k in range(P)]
        else:
            want = oracle.round_(st.mode, rp, ci, H_glob, st.d_in, p_.W, p_.b, relu=st.relu, heads=st.heads,
                                 a_src=p_.a_src, a_dst=p_.a_dst, self_concat=st.concat)
            F = st.d_out
            tables = []
            for k, wk in enumerate(workers):
                T = torch.full((wk.n_local, wl.pad_ld(F)), float("nan"), dtype=torch.float32, device="cuda")
                if p_.W is None:
                    T[:wk.share.n_inner, :F] = H_loc[k][:, :F]
                else:
                    Hn.transform(H_loc[k], st.d_in, Hn.dev(p_.W), Hn.dev(p_.b) if p_.b is not None else None, st.relu,
                                 out=T[:wk.share.n_inner])
                tables.append(T)
            exchange(workers, tables, F)
            outs = []
            for k, wk in enumerate(workers):
                assert not torch.isnan(tables[k][:, :F]).any()
                kw = {}
                if st.mode == "gat_softmax":
                    kw = dict(heads=st.heads, a_src=Hn.dev(p_.a_src), a_dst=Hn.dev(p_.a_dst))
                outs.append(Hn.aggregate(wk.graph, st.mode, tables[k], F, concat=st.concat, **kw)[:wk.share.n_inner])
        torch.cuda.synchronize()
        for k, wk in enumerate(workers):
            got = outs[k].cpu().numpy()[:, :st.out_width]
            assert_close(got, want[wk.inner_ids], what="workload %d stage %d worker %d" % (idx, i, k))
        H_glob = want.astype(np.float32)
        H_loc = [Hn.dev(np.ascontiguousarray(H_glob[wk.inner_ids])) for wk in workers]
    for wk in workers:
        wk.graph.destroy()


@pytest.mark.parametrize("idx,P", [(3, 4), (4, 2)])
def test_full_size_share_and_one_round(idx, P):
    """The shapes the paper distributes: the dense social graph over 4 workers and the large sparse
    graph over 2 (synthetic stand-ins, seeded random ownership).  Worker 0's share is compared bit for
    bit with the oracle's; then its first round runs on the local graph, with the boundary rows packed
    out of a table that plays the peers, and every inner row is compared with the global oracle."""
    w = wl.workload(idx)
    print("generating workload", idx, flush=True)
    src, dst = wl.make_graph(w)
    n = w.n_nodes
    g = Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, w.self_loops)
    print("oracle csr", flush=True)
    rp, ci = oracle.csr_from_coo(src, dst, n, w.self_loops)
    del src, dst
    part = owner_map(n, P, 70 + idx)
    print("gpu share", flush=True)
    ds = Hn.partition_share(g, Hn.dev(part), P, 0)
    torch.cuda.synchronize()
    print("oracle share: inner %d halo %d entries %d" % (ds.n_inner, ds.n_halo, ds.graph.nnz), flush=True)
    want = op.share(rp, ci, part, P, 0)
    check_share(ds, want, P)
    del want
    st = w.stages[0]
    F = st.d_out if st.w else st.d_in
    p_ = wl.make_params(w)[0]
    print("one round on the local graph", flush=True)
    Zh = wl.random_matrix(n, F, 90 + idx, ld=wl.pad_ld(F))         # the round's (already transformed) features
    Zg = Hn.dev(Zh)
    local = Hn.make_plan(ds.graph)
    T = torch.empty((ds.n_inner + ds.n_halo, wl.pad_ld(F)), dtype=torch.float32, device="cuda")
    Hn.halo_pack(ds.local_ids[:ds.n_inner], Zg, F, buf=T[:ds.n_inner])          # own rows
    peers = Hn.halo_pack(ds.local_ids[ds.n_inner:], Zg, F)                       # what the peers would send,
    order = ds.recv_ids                                                         # in receive-list order:
    sent = Hn.halo_pack((order - ds.n_inner).to(torch.int32), peers, F)          # grouped by owner
    Hn.halo_unpack(order, sent, T, F)
    kw = {}
    if st.mode == "gat_softmax":
        kw = dict(heads=st.heads, a_src=Hn.dev(p_.a_src), a_dst=Hn.dev(p_.a_dst))
    out = Hn.aggregate(local, st.mode, T, F, concat=st.concat, **kw)
    torch.cuda.synchronize()
    inner = np.flatnonzero(part == 0).astype(np.int64)            # local row k is global row inner[k]
    print("oracle: all %d inner rows" % inner.size, flush=True)
    worst = 0.0
    for lo in range(0, inner.size, 1 << 16):
        rows = inner[lo:lo + (1 << 16)]
        ref = oracle.aggregate(st.mode, rp, ci, Zh, F, heads=st.heads, a_src=p_.a_src, a_dst=p_.a_dst,
                               self_concat=st.concat, rows=rows)
        got = out[lo:lo + rows.size, :ref.shape[1]].cpu().numpy()
        worst = max(worst, assert_close(got, ref, what="workload %d worker 0 of %d, first round, rows %d.." % (idx, P, lo)))
    print("worker 0 of %d: all %d inner rows, worst row-normwise error %.2e" % (P, inner.size, worst), flush=True)
    local.destroy()
