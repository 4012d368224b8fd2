"""GPU backward of the aggregation (retexo_aggregate_backward) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2302_13053_amd import binding as B
from paper_2302_13053_amd import harness as Hn
from paper_2302_13053_amd import workloads as wl
from parity import assert_close, assert_cond_close

pytestmark = pytest.mark.gpu

LINEAR = ["sum", "mean", "gcn_sym"]


@pytest.fixture(scope="module")
def graphs():
    """name -> (DeviceGraph, row_ptr, col_idx); undirected graphs, hence symmetric CSRs."""
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


def offset_tensor(a: np.ndarray, offset: int) -> torch.Tensor:
    """Device copy of ``a`` whose first element sits ``offset`` floats past an aligned address."""
    if not offset:
        return Hn.dev(a)
    buf = torch.zeros(a.size + offset, dtype=torch.float32, device="cuda")
    t = buf[offset:].view(a.shape)
    t.copy_(torch.from_numpy(a))
    return t


def run_case(graphs, name, mode, F, ld, heads, concat, seed, offset=0, slope=0.2):
    g, rp, ci = graphs[(name, mode == "gcn_sym")]
    n = g.n_nodes
    gw = 2 * F if concat else F
    ldg = ld if not concat else ld + F
    Zh = wl.random_matrix(n, F, seed, ld=ld)
    Gh = wl.random_matrix(n, gw, seed + 1, ld=ldg)
    a_s = a_d = None
    kw = {}
    if mode == "gat_softmax":
        # attention vectors at an initialisation-like scale: scores of a few units whatever the head width
        # (far larger scores make the softmax one-hot, and the gradient through it a difference of
        # nearly equal inner products that no fp32 evaluation resolves to 1e-5 of the row)
        scale = np.float32(min(0.3, 2.4 / np.sqrt(F // heads)))
        a_s = wl.random_matrix(heads, F // heads, seed + 2) * scale
        a_d = wl.random_matrix(heads, F // heads, seed + 3) * scale
        kw = dict(Z=offset_tensor(Zh, offset), heads=heads, a_src=Hn.dev(a_s), a_dst=Hn.dev(a_d), slope=slope)
    dZ = torch.full((n, ld + 3), 777.0, dtype=torch.float32, device="cuda")
    if ld % 4 == 0:
        dZ = torch.full((n, ld + 4), 777.0, dtype=torch.float32, device="cuda")
    out = Hn.aggregate_backward(g, mode, F, offset_tensor(Gh, offset), concat=concat, dZ=dZ, **kw)
    torch.cuda.synchronize()
    got = out[0].cpu().numpy()
    assert np.all(got[:, F:] == 777.0)                      # nothing written past the F columns
    want = oracle.aggregate_backward(mode, rp, ci, Zh, F, Gh, heads=heads, a_src=a_s, a_dst=a_d,
                                     slope=slope, self_concat=concat)
    return got[:, :F], out[1], out[2], want


def check_params(das, dad, want, what):
    # one row-normwise ratio over each whole parameter gradient
    for got, ref, name in ((das, want[1], " da_src"), (dad, want[2], " da_dst")):
        got = got.cpu().numpy().reshape(1, -1)
        if np.abs(ref).max() == 0.0:
            # a gradient that vanishes by structure (every softmax over a single entry) is a difference
            # of two equal inner products on the GPU: rounding noise, not an exact zero
            assert np.abs(got).max() <= 1e-5, what + name
        else:
            assert_close(got, ref.reshape(1, -1), what=what + name)


@pytest.mark.parametrize("mode", LINEAR)
@pytest.mark.parametrize("F,ld,concat,offset", [
    (256, 256, False, 0), (602, 608, True, 0), (602, 602, False, 0), (1433, 1433, True, 0),
    (100, 100, True, 0), (7, 7, True, 0), (128, 128, False, 1),
])
def test_linear_modes_match_oracle(graphs, mode, F, ld, concat, offset):
    got, _, _, want = run_case(graphs, "skewed", mode, F, ld, 1, concat, seed=F + 3, offset=offset)
    # every element within 1e-5 of the size of its terms.  The graph is symmetric, so dZ_u = sum_v c_vu G_v is
    # again an aggregate of G: sum and gcn_sym with the same coefficients, mean with 1/deg of the destination
    g, rp, ci = graphs[("skewed", mode == "gcn_sym")]
    Gh = wl.random_matrix(g.n_nodes, 2 * F if concat else F, F + 3 + 1, ld=ld if not concat else ld + F)
    Ga = np.ascontiguousarray(Gh[:, F:2 * F] if concat else Gh[:, :F])
    if mode == "mean":
        Ga = (Ga / np.maximum(np.diff(rp), 1)[:, None]).astype(np.float32)
    mag = oracle.aggregate_abs("sum" if mode == "mean" else mode, rp, ci, Ga, F)
    if concat:
        mag = mag + np.abs(Gh[:, :F].astype(np.float64))
    assert_cond_close(got, want, mag, what="%s backward F=%d" % (mode, F))
    # rows of at least 64 columns also within 1e-5 of the row's largest magnitude
    if F >= 64:
        assert_close(got, want, what="%s backward F=%d" % (mode, F))
    for name in ("flat", "tiny"):
        got, _, _, want = run_case(graphs, name, mode, 96, 96, 1, concat, seed=5)
        assert_close(got, want, what="%s backward %s" % (mode, name))


@pytest.mark.parametrize("F,ld,heads,concat,offset", [
    (256, 256, 4, False, 0),      # the benchmark shape: 16 lanes per head
    (256, 256, 4, True, 0),
    (188, 192, 4, False, 0),      # heads of 47 columns: a lane's four columns straddle heads
    (512, 512, 8, False, 0),      # two chunks per lane, eight heads
    (1024, 1024, 8, True, 0),     # widest supported
    (768, 768, 1, False, 0),      # three chunks
    (100, 100, 4, True, 0),
    (94, 94, 2, False, 0),        # width not a multiple of four: scalar gathers
    (702, 702, 2, False, 0),      # scalar gathers, 11 chunks
    (301, 304, 7, False, 0),      # seven heads of 43, scalar gathers
    (7, 7, 7, True, 0),
    (1, 1, 1, False, 0),
    (128, 128, 2, False, 1),      # misaligned base pointers
])
def test_edge_softmax_backward_matches_oracle(graphs, F, ld, heads, concat, offset):
    got, das, dad, want = run_case(graphs, "skewed", "gat_softmax", F, ld, heads, concat, seed=F + 9, offset=offset)
    what = "gat backward F=%d heads=%d" % (F, heads)
    # narrow rows: a handful of signed terms has no robust magnitude to measure against
    assert_close(got, want[0], tol=1e-5 if F >= 64 else 5e-4, what=what)
    check_params(das, dad, want, what)


@pytest.mark.parametrize("name", ["flat", "tiny"])
def test_edge_softmax_backward_other_graphs(graphs, name):
    got, das, dad, want = run_case(graphs, name, "gat_softmax", 96, 96, 3, True, seed=3)
    assert_close(got, want[0], what="gat backward " + name)
    check_params(das, dad, want, "gat backward " + name)


def test_heavy_row_threshold_and_reproducibility(graphs):
    """Every row through the one-wave kernel, or many rows through the eight-wave kernel: same
    result within the bound, and each configuration reproduces itself bit for bit."""
    g, rp, ci = graphs[("skewed", False)]
    n, F, heads = g.n_nodes, 192, 3
    Zh, Gh = wl.random_matrix(n, F, 41), wl.random_matrix(n, F, 42)
    a_s, a_d = wl.random_matrix(heads, F // heads, 43) * np.float32(0.3), wl.random_matrix(heads, F // heads, 44) * np.float32(0.3)
    want = oracle.aggregate_backward("gat_softmax", rp, ci, Zh, F, Gh, heads=heads, a_src=a_s, a_dst=a_d)
    Z, G, As, Ad = Hn.dev(Zh), Hn.dev(Gh), Hn.dev(a_s), Hn.dev(a_d)
    try:
        for heavy in (1 << 20, 256, 2048):
            B.retexo_set_option("agg_heavy_degree", heavy)
            for vec in (4, 1):
                B.retexo_set_option("agg_max_vec", vec)
                a = Hn.aggregate_backward(g, "gat_softmax", F, G, Z=Z, heads=heads, a_src=As, a_dst=Ad)
                a = [t.clone() for t in a]
                b = Hn.aggregate_backward(g, "gat_softmax", F, G, Z=Z, heads=heads, a_src=As, a_dst=Ad)
                assert all(torch.equal(x, y) for x, y in zip(a, b))
                what = "gat backward heavy=%d vec=%d" % (heavy, vec)
                assert_close(a[0].cpu().numpy()[:, :F], want[0], what=what)
                check_params(a[1], a[2], want, what)
    finally:
        B.retexo_set_option("agg_heavy_degree", 2048)
        B.retexo_set_option("agg_max_vec", 4)


def test_slope_one_sends_nothing_to_the_destination_vector(graphs):
    """With slope 1 the score is linear and the softmax ignores a row-wide shift, so da_dst is zero up to
    rounding; the GPU must show that cancellation too (a property that holds at any size)."""
    got, das, dad, want = run_case(graphs, "flat", "gat_softmax", 128, 128, 4, False, seed=77, slope=1.0)
    assert_close(got, want[0], what="gat backward slope 1")
    assert np.abs(dad.cpu().numpy()).max() <= 1e-4 * np.abs(das.cpu().numpy()).max()


def test_argument_errors(graphs):
    g, _, _ = graphs[("flat", False)]
    n = g.n_nodes
    Z = torch.zeros((n, 64), dtype=torch.float32, device="cuda")
    G = torch.zeros((n, 64), dtype=torch.float32, device="cuda")
    a = torch.zeros((2, 32), dtype=torch.float32, device="cuda")
    with pytest.raises(B.RetexoError) as e:
        Hn.aggregate_backward(g, "max", 64, G)
    assert e.value.status == -4
    assert B.retexo_aggregate_backward_workspace_bytes(g.plan, B.MODES["gat_softmax"], 2048, 2) == -2      # too wide
    need = B.retexo_aggregate_backward_workspace_bytes(g.plan, B.MODES["gat_softmax"], 64, 2)
    ws = Hn.ws_tensor(need)
    p = lambda t: t.data_ptr()
    dZ, da1, da2 = torch.empty_like(Z), a.clone(), a.clone()
    args = lambda **k: dict(dict(plan=g.plan, mode=B.MODES["gat_softmax"], F=64, heads=2, d_Z=p(Z), ldz=64,
                                 d_attn_src=p(a), d_attn_dst=p(a), negative_slope=0.2, flags=0, d_G=p(G), ldg=64,
                                 d_dZ=p(dZ), lddz=64, d_dattn_src=p(da1), d_dattn_dst=p(da2),
                                 d_workspace=p(ws), workspace_bytes=need), **k)
    assert B.retexo_aggregate_backward(**args()) == 0
    assert B.retexo_aggregate_backward(**args(d_dZ=p(G))) == -9           # output over the gradient
    assert B.retexo_aggregate_backward(**args(d_dZ=p(Z))) == -9           # output over the forward input
    assert B.retexo_aggregate_backward(**args(workspace_bytes=need - 1)) == -8
    assert B.retexo_aggregate_backward(**args(d_dattn_src=0)) == -1
    assert B.retexo_aggregate_backward(**args(ldg=63)) == -3
    assert B.retexo_aggregate_backward(**args(heads=3)) == -6
    assert B.retexo_aggregate_backward(**args(flags=B.F_RELU)) == -5
    torch.cuda.synchronize()


def test_mid_size_graph_parameter_gradients():
    """A graph large enough for the two-stage parameter reduction to have many partial rows."""
    n, F, heads = 60000, 256, 4
    src, dst = wl.random_pairs(n, 600000, 51, skew=1.5)
    g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, False))
    rp, ci = oracle.csr_from_coo(src, dst, n, False)
    Zh, Gh = wl.random_matrix(n, F, 52), wl.random_matrix(n, F, 53)
    a_s, a_d = wl.random_matrix(heads, F // heads, 54) * np.float32(0.1), wl.random_matrix(heads, F // heads, 55) * np.float32(0.1)
    dZ, das, dad = Hn.aggregate_backward(g, "gat_softmax", F, Hn.dev(Gh), Z=Hn.dev(Zh), heads=heads,
                                         a_src=Hn.dev(a_s), a_dst=Hn.dev(a_d))
    torch.cuda.synchronize()
    want = oracle.aggregate_backward("gat_softmax", rp, ci, Zh, F, Gh, heads=heads, a_src=a_s, a_dst=a_d)
    assert_close(dZ.cpu().numpy()[:, :F], want[0], what="gat backward mid-size")
    check_params(das, dad, want, "gat backward mid-size")
    g.destroy()


def test_full_size_products_shape_all_rows():
    """The edge-softmax backward on the large attention workload's graph at full size (2.4 M nodes,
    124 M entries, 4 heads of 64), on every row of dZ.  The
    attention-vector gradients are sums over the whole graph that the oracle cannot produce at this
    size in test time; they are covered by the mid-size case above and here by a property that holds
    at any size: slope 1 leaves da_dst at rounding level."""
    w = wl.workload(4)
    print("generating workload 4", flush=True)
    src, dst = wl.make_graph(w)
    g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), w.n_nodes, False))
    print("oracle csr", flush=True)
    rp, ci = oracle.csr_from_coo(src, dst, w.n_nodes, False)
    del src, dst
    n, F, heads = w.n_nodes, 256, 4
    rows = np.arange(n, dtype=np.int64)        # every row of dZ (given as a list: the oracle then skips its
                                               # serial sum over the whole graph for the attention vectors)
    Zh, Gh = wl.random_matrix(n, F, 62), wl.random_matrix(n, F, 63)
    a_s = wl.random_matrix(heads, F // heads, 64) * np.float32(0.2)
    a_d = wl.random_matrix(heads, F // heads, 65) * np.float32(0.2)
    Z, G, As, Ad = Hn.dev(Zh), Hn.dev(Gh), Hn.dev(a_s), Hn.dev(a_d)
    print("gpu backward", flush=True)
    dZ, das, dad = Hn.aggregate_backward(g, "gat_softmax", F, G, Z=Z, heads=heads, a_src=As, a_dst=Ad)
    torch.cuda.synchronize()
    print("oracle: all %d rows of dZ" % n, flush=True)
    # The derivative of LeakyReLU jumps at a score of exactly zero.  Among the 5e8 (entry, head) scores of this
    # graph a few lie within float32 rounding of zero, where the kernel's float32 score and the oracle's float64
    # score can fall on different sides: both derivatives are then correct results of the method.  The oracle
    # reports, per element of dZ, how far such undecided entries can move it (zero for almost every row); rows
    # without any are held to the plain bound, the others to the bound plus that amount.
    # An entry counts as undecided within 4e-6 of the size of its score's terms (64-term float32 inner products).
    want, _, _, slack = oracle.aggregate_backward("gat_softmax", rp, ci, Zh, F, Gh, heads=heads, a_src=a_s, a_dst=a_d,
                                                  rows=rows, kink_rel=4e-6)
    worst = 0.0
    n_slack = n_moved = 0
    for lo in range(0, n, 1 << 18):
        got = dZ[lo:lo + (1 << 18), :F].cpu().numpy().astype(np.float64)
        w_, s_ = want[lo:lo + (1 << 18)], slack[lo:lo + (1 << 18)]
        free = s_.max(axis=1) == 0.0
        worst = max(worst, assert_close(got[free], w_[free], what="gat backward full size, rows %d.." % lo))
        den = np.abs(w_[~free]).max(axis=1, keepdims=True)
        over = np.abs(got[~free] - w_[~free]) - (1e-5 * den + s_[~free])
        assert over.max(initial=-1.0) <= 0.0, "rows %d..: an element beyond the bound plus the kink slack by %.3e" % (lo, over.max())
        n_slack += int((~free).sum())
        n_moved += int(((np.abs(got[~free] - w_[~free]).max(axis=1) / den[:, 0]) > 1e-5).sum())
    print("gat backward full size: all %d rows, worst row-normwise error %.2e on the %d rows without an undecided "
          "entry; %d rows touch one, %d of them differ by more than 1e-5 (within the slack)"
          % (n, worst, n - n_slack, n_slack, n_moved), flush=True)
    del slack
    del want
    assert np.all(np.isfinite(das.cpu().numpy())) and np.all(np.isfinite(dad.cpu().numpy()))
    _, das1, dad1 = Hn.aggregate_backward(g, "gat_softmax", F, G, Z=Z, heads=heads, a_src=As, a_dst=Ad, slope=1.0, dZ=dZ)
    torch.cuda.synchronize()
    assert np.abs(dad1.cpu().numpy()).max() <= 1e-4 * np.abs(das1.cpu().numpy()).max()
    g.destroy()


@pytest.mark.parametrize("flash", [1, 0])
@pytest.mark.parametrize("F,ld,heads,concat", [(256, 256, 4, False), (256, 256, 4, True), (188, 192, 4, False),
                                               (512, 512, 8, False), (1024, 1024, 8, True), (96, 96, 3, False),
                                               (256, 256, 1, False), (64, 64, 8, True), (32, 32, 8, False)])
def test_backward_after_a_forward_in_save_mode(graphs, F, ld, heads, concat, flash):
    """retexo_aggregate with RETEXO_F_SAVE leaves the statistics behind (its output stays within the forward's
    bound), and retexo_aggregate_backward_saved reaches the oracle's gradients with one gather pass.
    flash: ordinary rows compute the source scores from the gathered rows (where the head width allows it)
    or read them from the table."""
    B.retexo_set_option("agg_gat_flash", flash)
    try:
        _saved_forward_and_backward(graphs, F, ld, heads, concat)
    finally:
        B.retexo_set_option("agg_gat_flash", 1)


def _saved_forward_and_backward(graphs, F, ld, heads, concat):
    for name in ("skewed", "flat"):
        g, rp, ci = graphs[(name, False)]
        n = g.n_nodes
        Zh = wl.random_matrix(n, F, F + 21, ld=ld)
        Gh = wl.random_matrix(n, 2 * F if concat else F, F + 22)
        scale = np.float32(min(0.3, 2.4 / np.sqrt(F // heads)))
        a_s = wl.random_matrix(heads, F // heads, F + 23) * scale
        a_d = wl.random_matrix(heads, F // heads, F + 24) * scale
        Z, G, As, Ad = Hn.dev(Zh), Hn.dev(Gh), Hn.dev(a_s), Hn.dev(a_d)
        fwd = oracle.aggregate("gat_softmax", rp, ci, Zh, F, heads=heads, a_src=a_s, a_dst=a_d, self_concat=concat)
        flags = (B.F_SELF_CONCAT if concat else 0) | B.F_SAVE
        saved = Hn.ws_tensor(B.retexo_workspace_bytes(g.plan, F, B.MODES["gat_softmax"], heads, flags))
        out = Hn.aggregate(g, "gat_softmax", Z, F, heads=heads, a_src=As, a_dst=Ad, concat=concat, workspace=saved, save=True)
        ow = 2 * F if concat else F
        assert_close(out.cpu().numpy()[:, :ow], fwd, what="forward in save mode %s F=%d" % (name, F))
        dZ, das, dad = Hn.aggregate_backward(g, "gat_softmax", F, G, Z=Z, heads=heads, a_src=As, a_dst=Ad, concat=concat,
                                             saved=saved)
        torch.cuda.synchronize()
        want = oracle.aggregate_backward("gat_softmax", rp, ci, Zh, F, Gh, heads=heads, a_src=a_s, a_dst=a_d, self_concat=concat)
        what = "saved backward %s F=%d" % (name, F)
        assert_close(dZ.cpu().numpy()[:, :F], want[0], tol=1e-5 if F >= 64 else 5e-4, what=what)
        check_params(das, dad, want, what)
        again = Hn.aggregate_backward(g, "gat_softmax", F, G, Z=Z, heads=heads, a_src=As, a_dst=Ad, concat=concat,
                                      saved=saved)
        assert torch.equal(dZ[:, :F], again[0][:, :F]) and torch.equal(das, again[1]) and torch.equal(dad, again[2])


def test_save_mode_needs_aligned_rows(graphs):
    g, _, _ = graphs[("flat", False)]
    n, F, heads = g.n_nodes, 94, 2
    Z = Hn.dev(wl.random_matrix(n, F, 1, ld=94))                 # rows not a multiple of 16 bytes
    a = Hn.dev(wl.random_matrix(heads, F // heads, 2))
    ws = Hn.ws_tensor(B.retexo_workspace_bytes(g.plan, F, B.MODES["gat_softmax"], heads, B.F_SAVE))
    with pytest.raises(B.RetexoError) as e:
        Hn.aggregate(g, "gat_softmax", Z, F, heads=heads, a_src=a, a_dst=a, workspace=ws, save=True)
    assert e.value.status == -5
    assert B.retexo_workspace_bytes(g.plan, F, B.MODES["mean"], 1, B.F_SAVE) == -5      # only the edge softmax saves


@pytest.mark.parametrize("F,heads", [(256, 1), (256, 2), (256, 4), (192, 3), (96, 3), (96, 6), (64, 8), (32, 8), (24, 2)])
@pytest.mark.parametrize("concat", [False, True])
def test_edge_softmax_backward_with_scores_from_gathered_rows(graphs, F, heads, concat):
    # ordinary rows of the first gather pass compute <a_src, z_u> from the row they gather (1 to 64 lanes per
    # head); long rows and head widths that are not a power-of-two number of lanes read the score table.
    # Both against the oracle, and each other to rounding.
    res = {}
    try:
        for flash in (1, 0):
            B.retexo_set_option("agg_gat_flash", flash)
            for name in ("skewed", "flat", "tiny"):
                got, das, dad, want = run_case(graphs, name, "gat_softmax", F, F, heads, concat, seed=F + heads)
                what = "gat backward F=%d heads=%d flash=%d %s" % (F, heads, flash, name)
                assert_close(got, want[0], tol=1e-5 if F >= 64 else 5e-4, what=what)
                check_params(das, dad, want, what)
                res[(flash, name)] = got
    finally:
        B.retexo_set_option("agg_gat_flash", 1)
    for name in ("skewed", "flat", "tiny"):
        assert_close(res[(1, name)], res[(0, name)].astype(np.float64), tol=1e-5 if F >= 64 else 5e-4,
                     what="flash vs table " + name)
