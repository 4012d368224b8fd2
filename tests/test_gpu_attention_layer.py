"""One local training step of a layer whose aggregation has trainable parameters (edge softmax), chained
from the library's entry points on the GPU:

    Z = Q W_g + b_g  ->  X = AGGR_attention(Z)  ->  ReLU(X W1 + b1) Wc + bc  ->  loss
    and back:  dL/dX  ->  dL/dZ, dL/da_src, dL/da_dst  ->  dL/dW_g, dL/db_g

against the same chain made of the oracle's pieces (which is itself pinned to end-to-end autograd)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2302_13053_amd import binding as B
from paper_2302_13053_amd import harness as Hn
from paper_2302_13053_amd import workloads as wl
from parity import assert_close

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,pairs,d_in,F,heads,Hd,C", [(3000, 20000, 100, 256, 4, 64, 7), (1200, 6000, 33, 96, 3, 40, 5)])
def test_attention_layer_training_step(n, pairs, d_in, F, heads, Hd, C):
    src, dst = wl.random_pairs(n, pairs, 9, skew=1.5)
    rp, ci = oracle.csr_from_coo(src, dst, n, False)
    g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, False))
    rng = np.random.Generator(np.random.Philox(key=n))
    Q = wl.random_matrix(n, d_in, 1, ld=wl.pad_ld(d_in))
    Wg = wl.glorot(rng, d_in, F, (d_in, F))
    bg = rng.uniform(-0.1, 0.1, F).astype(np.float32)
    a_s = wl.glorot(rng, F // heads, 1, (heads, F // heads))
    a_d = wl.glorot(rng, F // heads, 1, (heads, F // heads))
    W1 = wl.glorot(rng, F, Hd, (F, Hd))
    b1 = rng.uniform(-0.1, 0.1, Hd).astype(np.float32)
    Wc = wl.glorot(rng, Hd, C, (Hd, C))
    bc = np.zeros(C, np.float32)
    y = rng.integers(0, C, n).astype(np.int32)
    y[rng.random(n) > 0.6] = -1

    # oracle chain (float32 tables between the pieces, as on the GPU)
    Z = oracle.transform(Q, d_in, Wg, bg).astype(np.float32)
    X = oracle.aggregate("gat_softmax", rp, ci, Z, F, heads=heads, a_src=a_s, a_dst=a_d).astype(np.float32)
    loss, gW1, gb1, gWc, gbc, gX = oracle.layer_grad(X, F, y, W1, b1, Wc, bc, input_grad=True)
    dZ, das, dad = oracle.aggregate_backward("gat_softmax", rp, ci, Z, F, gX.astype(np.float32), heads=heads,
                                             a_src=a_s, a_dst=a_d)
    gWg, gbg = oracle.transform_backward(Q, d_in, dZ.astype(np.float32), F)

    # GPU chain
    d = Hn.dev
    dQ, dWg, dbg, das_in, dad_in = d(Q), d(Wg), d(bg), d(a_s), d(a_d)
    Zd = Hn.transform(dQ, d_in, dWg, dbg, False)
    Xd = Hn.aggregate(g, "gat_softmax", Zd, F, heads=heads, a_src=das_in, a_dst=dad_in)
    gXd = torch.empty((n, wl.pad_ld(F)), dtype=torch.float32, device="cuda")
    lossd, gW1d, gb1d, gWcd, gbcd = Hn.layer_grad(Xd, F, d(y), d(W1), d(b1), d(Wc), d(bc), gX=gXd)
    dZd, dasd, dadd = Hn.aggregate_backward(g, "gat_softmax", F, gXd, Z=Zd, heads=heads, a_src=das_in, a_dst=dad_in)
    gWgd, gbgd = Hn.transform_backward(dQ, d_in, dZd, F)
    torch.cuda.synchronize()

    assert abs(float(lossd.cpu()[0]) - loss) <= 1e-5 * abs(loss)
    flat = lambda t: t.cpu().numpy().reshape(1, -1)
    # the chain hands float32 tables from one piece to the next on both sides, and the two sides' tables
    # differ in the last bits: the bound on the end of the chain is a few times that of a single piece
    tol = 5e-5
    for got, want, name in ((gW1d, gW1, "gW1"), (gWcd, gWc, "gWc"), (gWgd, gWg, "gW_g")):
        assert_close(got.cpu().numpy(), want, tol=tol, what=name)
    for got, want, name in ((gb1d, gb1, "gb1"), (gbcd, gbc, "gbc"), (gbgd, gbg, "gb_g"), (dasd, das, "ga_src"), (dadd, dad, "ga_dst")):
        assert_close(flat(got), want.reshape(1, -1), tol=tol, what=name)
    # a labelled node whose neighbours are all unlabelled and whose scores have one sign receives exactly
    # nothing; the oracle's float64 sum leaves a residue of 1e-17 there, the GPU an exact zero
    gotZ = dZd.cpu().numpy()[:, :F]
    residue = np.abs(dZ).max(axis=1) < 1e-12
    assert np.abs(gotZ[residue]).max(initial=0.0) <= 1e-7
    assert_close(gotZ[~residue], dZ[~residue], tol=tol, what="dL/dZ")

    # a few SGD steps on every parameter lower the loss
    params = [dWg, dbg, das_in, dad_in, d(W1), d(b1), d(Wc), d(bc)]
    first = None
    saved = Hn.ws_tensor(B.retexo_workspace_bytes(g.plan, F, B.MODES["gat_softmax"], heads, B.F_SAVE))
    for step in range(6):
        Zd = Hn.transform(dQ, d_in, params[0], params[1], False)
        # the forward keeps what the backward can reuse (one gather pass instead of two)
        Xd = Hn.aggregate(g, "gat_softmax", Zd, F, heads=heads, a_src=params[2], a_dst=params[3], workspace=saved, save=True)
        lossd, g1, g2, g3, g4 = Hn.layer_grad(Xd, F, d(y), params[4], params[5], params[6], params[7], gX=gXd)
        dZd, ga, gb_ = Hn.aggregate_backward(g, "gat_softmax", F, gXd, Z=Zd, heads=heads, a_src=params[2], a_dst=params[3],
                                             saved=saved)
        gw, gbias = Hn.transform_backward(dQ, d_in, dZd, F)
        for p_, g_ in zip(params, (gw, gbias, ga, gb_, g1, g2, g3, g4)):
            B.check(B.retexo_sgd_update(p_.numel(), p_.data_ptr(), g_.data_ptr(), 0.2, Hn._stream_ptr()), "sgd")
        val = float(lossd.cpu()[0])
        first = val if first is None else first
    assert val < first
    g.destroy()
