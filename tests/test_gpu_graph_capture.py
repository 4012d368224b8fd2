"""The stream-ordered entry points recorded into a HIP graph (by stream capture) and replayed.

A launch-bound loop — a round on a small graph followed by a local training step and its SGD updates —
is captured once and replayed several times, with the program's own eager work and synchronisations
between the replays; every replay must reproduce the eager result bit for bit."""
import numpy as np
import pytest
import torch

from paper_2302_13053_amd import binding as B
from paper_2302_13053_amd import harness as Hn
from paper_2302_13053_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_round_and_training_step_replay_from_a_graph():
    n, F0, Hd, C = 4000, 96, 64, 5
    src, dst = wl.random_pairs(n, 30000, 3, skew=1.5)
    g = Hn.make_plan(Hn.csr_from_coo(Hn.dev(src), Hn.dev(dst), n, False))
    rng = np.random.Generator(np.random.Philox(key=5))
    X0 = Hn.dev(wl.random_matrix(n, F0, 1, ld=wl.pad_ld(F0)))
    y = rng.integers(0, C, n).astype(np.int32)
    y[rng.random(n) > 0.5] = -1
    dy = Hn.dev(y)
    init = [wl.glorot(rng, 2 * F0, Hd, (2 * F0, Hd)), np.zeros(Hd, np.float32), wl.glorot(rng, Hd, C, (Hd, C)), np.zeros(C, np.float32)]
    params = [Hn.dev(p) for p in init]
    X1 = torch.empty((n, wl.pad_ld(2 * F0)), dtype=torch.float32, device="cuda")
    ws_a = Hn.ws_tensor(max(256, B.retexo_workspace_bytes(g.plan, F0, B.MODES["mean"], 1, B.F_SELF_CONCAT)))
    ws_t = Hn.ws_tensor(B.retexo_train_workspace_bytes(n, 2 * F0, Hd, C))
    grads = [torch.empty_like(p) for p in params]
    loss = torch.empty(1, dtype=torch.float32, device="cuda")

    def step():
        """One round (aggregate + self-concat) and one training step, pointers fixed so that it can be replayed."""
        Hn.aggregate(g, "mean", X0, F0, concat=True, out=X1, workspace=ws_a)
        st = B.retexo_layer_grad(n, 2 * F0, Hd, C, X1.data_ptr(), X1.stride(0), dy.data_ptr(), *[p.data_ptr() for p in params],
                                 *[q.data_ptr() for q in grads], loss.data_ptr(), ws_t.data_ptr(), ws_t.numel(), Hn._stream_ptr())
        B.check(st, "retexo_layer_grad")
        for p_, g_ in zip(params, grads):
            B.check(B.retexo_sgd_update(p_.numel(), p_.data_ptr(), g_.data_ptr(), 0.3, Hn._stream_ptr()), "sgd")

    def reset():
        for p_, v in zip(params, init):
            p_.copy_(torch.from_numpy(v))

    # eager reference: four steps, loss and parameters after each
    reset()
    want = []
    for _ in range(4):
        step()
        torch.cuda.synchronize()
        want.append((float(loss.cpu()[0]), [p.clone() for p in params]))
    assert want[3][0] < want[0][0]

    # capture one step, then replay it four times from the same start
    reset()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    reset()
    with torch.cuda.graph(graph, stream=side):
        step()
    reset()
    torch.cuda.synchronize()
    for k in range(4):
        graph.replay()
        torch.cuda.synchronize()
        assert float(loss.cpu()[0]) == want[k][0], k
        assert all(torch.equal(a, b) for a, b in zip(params, want[k][1])), k
        # unrelated eager work and a synchronisation between replays
        scratch = Hn.aggregate(g, "sum", X0, F0)
        assert torch.isfinite(scratch[:, :F0]).all()
        torch.cuda.synchronize()
    g.destroy()
