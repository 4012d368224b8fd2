"""retexo_aggregate_noalloc (the entry point for callers that cannot allocate): same bits as
retexo_aggregate, on two calls in a row that share the library's fixed scratch array, the
second on a smaller graph; sizes beyond the array are rejected."""
import numpy as np
import pytest
import torch

import oracle
from paper_2302_13053_amd import binding as B
from paper_2302_13053_amd import harness as Hn
from paper_2302_13053_amd import workloads as wl
from parity import assert_close

pytestmark = pytest.mark.gpu


def _case(n, heads, dh, seed):
    F = heads * dh
    src, dst = wl.graph_power_law(n, 10 * n, 2.2, 20.0, 3000.0, seed)
    g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, False))
    Z = wl.random_matrix(n, F, seed + 1, ld=wl.pad_ld(F))
    a_s = wl.random_matrix(heads, dh, seed + 2) * np.float32(0.3)
    a_d = wl.random_matrix(heads, dh, seed + 3) * np.float32(0.3)
    return g, (src, dst), Z, a_s, a_d, F


def _noalloc(g, mode, Z, F, heads, a_s, a_d, concat=False):
    out = torch.full((g.n_nodes, wl.pad_ld(2 * F if concat else F)), -3.0, dtype=torch.float32, device="cuda")
    st = B.retexo_aggregate_noalloc(g.plan, B.MODES[mode], F, heads, Z.data_ptr(), Z.stride(0),
                                    a_s.data_ptr() if a_s is not None else 0,
                                    a_d.data_ptr() if a_d is not None else 0, 0.2,
                                    B.F_SELF_CONCAT if concat else 0, out.data_ptr(), out.stride(0),
                                    Hn._stream_ptr())
    B.check(st, "retexo_aggregate_noalloc")
    return out


def test_noalloc_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    # head width 47: the kernels read the score table, which here lives in the library's own array
    big = _case(20000, 4, 47, 11)
    small = _case(6000, 4, 47, 12)
    outs = []
    for g, _, Z, a_s, a_d, F in (big, small):           # back to back on one stream, no synchronisation between
        outs.append(_noalloc(g, "gat_softmax", Hn.dev(Z), F, 4, Hn.dev(a_s), Hn.dev(a_d)))
    torch.cuda.synchronize()
    for (g, (src, dst), Z, a_s, a_d, F), got in zip((big, small), outs):
        want = Hn.aggregate(g, "gat_softmax", Hn.dev(Z), F, heads=4, a_src=Hn.dev(a_s), a_dst=Hn.dev(a_d))
        torch.cuda.synchronize()
        assert torch.equal(got[:, :F], want[:, :F])
        assert bool((got[:, F:] == -3.0).all())
        rp, ci = oracle.csr_from_coo(src, dst, g.n_nodes, False)
        ref = oracle.aggregate("gat_softmax", rp, ci, Z, F, heads=4, a_src=a_s, a_dst=a_d)
        assert_close(got.cpu().numpy()[:, :F], ref, what="noalloc edge softmax, %d nodes" % g.n_nodes)
    # the other head layouts and modes go through the same entry point (8 heads: the wider table)
    g, (src, dst), Z, a_s, a_d, F = _case(5000, 8, 27, 13)
    got = _noalloc(g, "gat_softmax", Hn.dev(Z), F, 8, Hn.dev(a_s), Hn.dev(a_d))
    want = Hn.aggregate(g, "gat_softmax", Hn.dev(Z), F, heads=8, a_src=Hn.dev(a_s), a_dst=Hn.dev(a_d))
    assert torch.equal(got[:, :F], want[:, :F])
    g2, _, Z2, a_s2, a_d2, F2 = _case(4000, 4, 64, 14)                    # scores from the gathered rows: no table
    got = _noalloc(g2, "gat_softmax", Hn.dev(Z2), F2, 4, Hn.dev(a_s2), Hn.dev(a_d2))
    want = Hn.aggregate(g2, "gat_softmax", Hn.dev(Z2), F2, heads=4, a_src=Hn.dev(a_s2), a_dst=Hn.dev(a_d2))
    assert torch.equal(got[:, :F2], want[:, :F2])
    got = _noalloc(g2, "mean", Hn.dev(Z2), F2, 1, None, None, concat=True)
    want = Hn.aggregate(g2, "mean", Hn.dev(Z2), F2, concat=True)
    assert torch.equal(got[:, :2 * F2], want[:, :2 * F2])
    for gg in (big[0], small[0], g, g2):
        gg.destroy()


def test_noalloc_rejects_what_does_not_fit_and_save_mode():
    n = B.NOALLOC_SCRATCH_BYTES // 32 + 1            # one node more than the array holds with 4 heads
    rp = torch.zeros(n + 1, dtype=torch.int64, device="cuda")
    ci = torch.zeros(1, dtype=torch.int32, device="cuda")
    g = Hn.make_plan(Hn.DeviceGraph(n, 0, rp, ci))
    Z = torch.zeros((n, 8), dtype=torch.float32, device="cuda")
    out = torch.full((n, 8), -3.0, dtype=torch.float32, device="cuda")
    a = torch.zeros(8, dtype=torch.float32, device="cuda")

    def call(mode=B.GAT_SOFTMAX, heads=4, flags=0):
        return B.retexo_aggregate_noalloc(g.plan, mode, 8, heads, Z.data_ptr(), 8, a.data_ptr(), a.data_ptr(), 0.2,
                                          flags, out.data_ptr(), 8, Hn._stream_ptr())
    assert call() == B.E_WORKSPACE
    assert call(flags=B.F_SAVE) == B.E_FLAGS
    assert call(mode=9) == B.E_MODE
    assert call(heads=9) == B.E_HEADS
    torch.cuda.synchronize()
    assert bool((out == -3.0).all())
    assert call(mode=B.SUM, heads=1) == B.OK         # no workspace needed: any size goes
    torch.cuda.synchronize()
    assert bool((out == 0.0).all())
    g.destroy()
