"""Device-side plumbing shared by the tests, the smoke check and the benchmark.

PyTorch is used only to own device memory and streams; every step of the path
is a call into libretexo.so through ``binding``.  Nothing here computes.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as B
from .workloads import Stage, StageParams, Workload, pad_ld


def _stream_ptr() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def ws_tensor(nbytes: int) -> torch.Tensor:
    """256-byte aligned byte buffer (torch's allocator aligns to 512)."""
    t = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")
    assert t.data_ptr() % 256 == 0
    return t


@dataclass
class DeviceGraph:
    n_nodes: int
    nnz: int
    row_ptr: torch.Tensor      # int64 [N+1]
    col_idx: torch.Tensor      # int32 [capacity], first nnz valid
    plan: Optional[int] = None

    def destroy(self) -> None:
        if self.plan:
            B.retexo_plan_destroy(self.plan)
            self.plan = None


def csr_from_coo(src: torch.Tensor, dst: torch.Tensor, n_nodes: int, self_loops: bool,
                 workspace: Optional[torch.Tensor] = None,
                 row_ptr: Optional[torch.Tensor] = None,
                 col_idx: Optional[torch.Tensor] = None) -> DeviceGraph:
    n_pairs = int(src.numel())
    need = B.retexo_csr_workspace_bytes(n_pairs, n_nodes, self_loops)
    if need < 0:
        raise B.RetexoError(need, "retexo_csr_workspace_bytes")
    if workspace is None or workspace.numel() < need:
        workspace = ws_tensor(need)
    cap = 2 * n_pairs + (n_nodes if self_loops else 0)
    if row_ptr is None:
        row_ptr = torch.empty(n_nodes + 1, dtype=torch.int64, device="cuda")
    if col_idx is None:
        col_idx = torch.empty(max(cap, 1), dtype=torch.int32, device="cuda")
    st, nnz = B.retexo_csr_from_coo(n_pairs, src.data_ptr() if n_pairs else 0,
                                    dst.data_ptr() if n_pairs else 0, n_nodes, self_loops,
                                    row_ptr.data_ptr(), col_idx.data_ptr(), col_idx.numel(),
                                    workspace.data_ptr(), workspace.numel(), _stream_ptr())
    B.check(st, "retexo_csr_from_coo")
    return DeviceGraph(n_nodes, nnz, row_ptr, col_idx)


def make_plan(g: DeviceGraph, validate: bool = False, split_rows: bool = False,
              workspace: Optional[torch.Tensor] = None) -> DeviceGraph:
    """``workspace``: caller memory the plan lives in (retexo_plan_create_in: no allocation, one synchronisation);
    it must stay untouched while the plan is in use."""
    flags = (B.F_VALIDATE if validate else 0) | (B.F_SPLIT_ROWS if split_rows else 0)
    if workspace is not None:
        st, plan = B.retexo_plan_create_in(g.n_nodes, g.nnz, g.row_ptr.data_ptr(), g.col_idx.data_ptr(), flags,
                                           workspace.data_ptr(), workspace.numel(), _stream_ptr())
        B.check(st, "retexo_plan_create_in")
    else:
        st, plan = B.retexo_plan_create(g.n_nodes, g.row_ptr.data_ptr(), g.col_idx.data_ptr(),
                                        flags, _stream_ptr())
        B.check(st, "retexo_plan_create")
    g.plan = plan
    return g


@dataclass
class DeviceShare:
    """One worker's share of an edge-partitioned graph (device arrays of retexo_partition_share)."""
    n_inner: int
    n_halo: int
    graph: DeviceGraph            # local CSR over n_inner + n_halo nodes (no plan yet)
    local_ids: torch.Tensor       # int32 [n_local] global ids
    global_deg: torch.Tensor      # int32 [n_local]
    send_ids: torch.Tensor        # int32 [n_send] local ids, grouped by peer
    recv_ids: torch.Tensor        # int32 [n_halo] local ids, grouped by owner
    send_offsets: list            # host, [n_parts + 1]
    recv_offsets: list


def partition_share(g: DeviceGraph, part: torch.Tensor, n_parts: int, p: int) -> DeviceShare:
    """Size query, allocation of exactly sized outputs, then the real call."""
    n = g.n_nodes
    nil = 0

    def call(cap_local, cap_col, cap_send, outs, ws):
        return B.retexo_partition_share(n, g.row_ptr.data_ptr(), g.col_idx.data_ptr(), part.data_ptr(), n_parts, p,
                                        cap_local, cap_col, cap_send, *outs, ws.data_ptr(), ws.numel(), _stream_ptr())
    need = B.retexo_partition_workspace_bytes(n, n_parts, 0)
    if need < 0:
        raise B.RetexoError(need, "retexo_partition_workspace_bytes")
    st, sizes, _, _ = call(0, 0, 0, (nil,) * 6, ws_tensor(need))
    if st != -11:                 # the size query always ends in the capacity error
        raise B.RetexoError(st, "retexo_partition_share (size query)")
    n_inner, n_halo, nnz_local, n_send = sizes
    n_local = n_inner + n_halo
    i32 = lambda k: torch.empty(max(k, 1), dtype=torch.int32, device="cuda")
    local_ids, col, gdeg, send, recv = i32(n_local), i32(nnz_local), i32(n_local), i32(n_send), i32(n_halo)
    rp = torch.empty(n_local + 1, dtype=torch.int64, device="cuda")
    ws = ws_tensor(B.retexo_partition_workspace_bytes(n, n_parts, n_send))
    st, sizes2, so, ro = call(n_local, nnz_local, n_send,
                              (local_ids.data_ptr(), rp.data_ptr(), col.data_ptr(), gdeg.data_ptr(),
                               send.data_ptr(), recv.data_ptr()), ws)
    B.check(st, "retexo_partition_share")
    assert sizes2 == sizes
    return DeviceShare(n_inner, n_halo, DeviceGraph(n_local, nnz_local, rp, col), local_ids[:n_local], gdeg[:n_local],
                       send[:n_send], recv[:n_halo], so, ro)


def halo_pack(ids: torch.Tensor, H: torch.Tensor, F: int, buf: Optional[torch.Tensor] = None) -> torch.Tensor:
    n = int(ids.numel())
    if buf is None:
        buf = torch.empty((max(n, 1), pad_ld(F)), dtype=torch.float32, device="cuda")
    B.check(B.retexo_halo_pack(n, ids.data_ptr() if n else 0, H.shape[0], F, H.data_ptr(), H.stride(0),
                               buf.data_ptr(), buf.stride(0), _stream_ptr()), "retexo_halo_pack")
    return buf


def halo_unpack(ids: torch.Tensor, buf: torch.Tensor, H: torch.Tensor, F: int) -> None:
    n = int(ids.numel())
    B.check(B.retexo_halo_unpack(n, ids.data_ptr() if n else 0, H.shape[0], F, buf.data_ptr(), buf.stride(0),
                                 H.data_ptr(), H.stride(0), _stream_ptr()), "retexo_halo_unpack")


def plan_arrays(g: DeviceGraph):
    """(deg int32[N], dinv float32[N], order int32[N]) copied out of the plan, as numpy."""
    n = g.n_nodes
    deg = torch.empty(max(n, 1), dtype=torch.int32, device="cuda")
    dinv = torch.empty(max(n, 1), dtype=torch.float32, device="cuda")
    order = torch.empty(max(n, 1), dtype=torch.int32, device="cuda")
    B.check(B.retexo_plan_export(g.plan, deg.data_ptr(), dinv.data_ptr(), order.data_ptr(), _stream_ptr()),
            "retexo_plan_export")
    torch.cuda.synchronize()
    return deg[:n].cpu().numpy(), dinv[:n].cpu().numpy(), order[:n].cpu().numpy()


def transform(H: torch.Tensor, d_in: int, W: torch.Tensor, b: Optional[torch.Tensor], relu: bool,
              out: Optional[torch.Tensor] = None, ld_out: Optional[int] = None) -> torch.Tensor:
    n = H.shape[0]
    d_out = W.shape[1]
    if out is None:
        out = torch.empty((n, ld_out or pad_ld(d_out)), dtype=torch.float32, device="cuda")
    st = B.retexo_transform(n, d_in, d_out, H.data_ptr(), H.stride(0), W.data_ptr(),
                            b.data_ptr() if b is not None else 0, B.F_RELU if relu else 0,
                            out.data_ptr(), out.stride(0), _stream_ptr())
    B.check(st, "retexo_transform")
    return out


def aggregate(g: DeviceGraph, mode: str, Z: torch.Tensor, F: int, *, heads: int = 1,
              a_src: Optional[torch.Tensor] = None, a_dst: Optional[torch.Tensor] = None,
              slope: float = 0.2, concat: bool = False, out: Optional[torch.Tensor] = None,
              ld_out: Optional[int] = None, workspace: Optional[torch.Tensor] = None,
              save: bool = False) -> torch.Tensor:
    """``save``: edge softmax in save mode; pass ``workspace`` (sized for it) and keep it for the backward."""
    ow = 2 * F if concat else F
    if out is None:
        out = torch.empty((g.n_nodes, ld_out or pad_ld(ow)), dtype=torch.float32, device="cuda")
    flags = (B.F_SELF_CONCAT if concat else 0) | (B.F_SAVE if save else 0)
    need = B.retexo_workspace_bytes(g.plan, F, B.MODES[mode], heads, flags)
    if need < 0:
        raise B.RetexoError(need, "retexo_workspace_bytes")
    if workspace is None:
        workspace = ws_tensor(need)
    st = B.retexo_aggregate(g.plan, B.MODES[mode], F, heads, Z.data_ptr(), Z.stride(0),
                            a_src.data_ptr() if a_src is not None else 0,
                            a_dst.data_ptr() if a_dst is not None else 0, slope, flags,
                            out.data_ptr(), out.stride(0), workspace.data_ptr(), workspace.numel(),
                            _stream_ptr())
    B.check(st, "retexo_aggregate")
    return out


def store_rows(X: torch.Tensor, F: int, fmt: str, ld: Optional[int] = None) -> torch.Tensor:
    """float32 table -> int16 tensor of bf16 / fp16 patterns, row pitch ``ld`` elements (default: F rounded up to 64)."""
    n = int(X.shape[0])
    ld = ld or (F + 63) // 64 * 64
    out = torch.zeros((n, ld), dtype=torch.int16, device="cuda")
    B.check(B.retexo_store_rows(B.STORAGE[fmt], n, F, X.data_ptr(), X.stride(0), out.data_ptr(), out.stride(0),
                                _stream_ptr()), "retexo_store_rows")
    return out


def aggregate_stored(g: DeviceGraph, mode: str, Z16: torch.Tensor, F: int, fmt: str, *, heads: int = 1,
                     a_src: Optional[torch.Tensor] = None, a_dst: Optional[torch.Tensor] = None,
                     slope: float = 0.2, concat: bool = False, out: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    ow = 2 * F if concat else F
    if out is None:
        out = torch.empty((g.n_nodes, pad_ld(ow)), dtype=torch.float32, device="cuda")
    flags = B.F_SELF_CONCAT if concat else 0
    need = B.retexo_workspace_bytes(g.plan, F, B.MODES[mode], heads, flags)
    if need < 0:
        raise B.RetexoError(need, "retexo_workspace_bytes")
    if workspace is None:
        workspace = ws_tensor(need)
    st = B.retexo_aggregate_stored(g.plan, B.MODES[mode], B.STORAGE[fmt], F, heads, Z16.data_ptr(), Z16.stride(0),
                                   a_src.data_ptr() if a_src is not None else 0,
                                   a_dst.data_ptr() if a_dst is not None else 0, slope, flags,
                                   out.data_ptr(), out.stride(0), workspace.data_ptr(), workspace.numel(),
                                   _stream_ptr())
    B.check(st, "retexo_aggregate_stored")
    return out


def aggregate_backward(g: DeviceGraph, mode: str, F: int, G: torch.Tensor, *, Z: Optional[torch.Tensor] = None,
                       heads: int = 1, a_src: Optional[torch.Tensor] = None, a_dst: Optional[torch.Tensor] = None,
                       slope: float = 0.2, concat: bool = False, dZ: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None, saved: Optional[torch.Tensor] = None):
    """-> (dZ, da_src, da_dst) device tensors (da_* None unless mode is gat_softmax).
    ``saved``: the workspace of a forward pass in save mode (one gather pass instead of two)."""
    if dZ is None:
        dZ = torch.empty((g.n_nodes, pad_ld(F)), dtype=torch.float32, device="cuda")
    need = B.retexo_aggregate_backward_workspace_bytes(g.plan, B.MODES[mode], F, heads)
    if need < 0:
        raise B.RetexoError(need, "retexo_aggregate_backward_workspace_bytes")
    if workspace is None:
        workspace = ws_tensor(need)
    das = dad = None
    if mode == "gat_softmax":
        das = torch.empty((heads, F // heads), dtype=torch.float32, device="cuda")
        dad = torch.empty_like(das)
    p = lambda t: t.data_ptr() if t is not None else 0
    if saved is not None:
        st = B.retexo_aggregate_backward_saved(g.plan, B.MODES[mode], F, heads, p(Z), Z.stride(0), p(a_src), p(a_dst),
                                               slope, B.F_SELF_CONCAT if concat else 0, G.data_ptr(), G.stride(0),
                                               saved.data_ptr(), saved.numel(),
                                               dZ.data_ptr(), dZ.stride(0), p(das), p(dad),
                                               workspace.data_ptr(), workspace.numel(), _stream_ptr())
        B.check(st, "retexo_aggregate_backward_saved")
        return dZ, das, dad
    st = B.retexo_aggregate_backward(g.plan, B.MODES[mode], F, heads, p(Z), Z.stride(0) if Z is not None else 0,
                                     p(a_src), p(a_dst), slope, B.F_SELF_CONCAT if concat else 0,
                                     G.data_ptr(), G.stride(0), dZ.data_ptr(), dZ.stride(0), p(das), p(dad),
                                     workspace.data_ptr(), workspace.numel(), _stream_ptr())
    B.check(st, "retexo_aggregate_backward")
    return dZ, das, dad


def round_(g: DeviceGraph, st: Stage, H: torch.Tensor, W, b, a_src, a_dst, out: torch.Tensor,
           workspace: torch.Tensor, slope: float = 0.2) -> None:
    flags = (B.F_RELU if st.relu else 0) | (B.F_SELF_CONCAT if st.concat else 0)
    rc = B.retexo_round(g.plan, B.MODES[st.mode], st.d_in, st.d_out, st.heads, H.data_ptr(), H.stride(0),
                        W.data_ptr() if W is not None else 0, b.data_ptr() if b is not None else 0,
                        a_src.data_ptr() if a_src is not None else 0,
                        a_dst.data_ptr() if a_dst is not None else 0, slope, flags,
                        out.data_ptr(), out.stride(0), workspace.data_ptr(), workspace.numel(),
                        _stream_ptr())
    B.check(rc, "retexo_round")


def transform_backward(H: torch.Tensor, d_in: int, dZ: torch.Tensor, d_out: int,
                       workspace: Optional[torch.Tensor] = None):
    """-> (gW [d_in, d_out], gb [d_out]) of Z = H W + b given dZ = dL/dZ."""
    n = int(H.shape[0])
    need = B.retexo_transform_backward_workspace_bytes(n, d_in, d_out)
    if need < 0:
        raise B.RetexoError(need, "retexo_transform_backward_workspace_bytes")
    if workspace is None:
        workspace = ws_tensor(need)
    gW = torch.empty((d_in, d_out), dtype=torch.float32, device="cuda")
    gb = torch.empty(d_out, dtype=torch.float32, device="cuda")
    B.check(B.retexo_transform_backward(n, d_in, d_out, H.data_ptr(), H.stride(0), dZ.data_ptr(), dZ.stride(0),
                                        gW.data_ptr(), gb.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                        _stream_ptr()), "retexo_transform_backward")
    return gW, gb


def layer_grad(X: torch.Tensor, d_in: int, labels: torch.Tensor, W1, b1, Wc=None, bc=None,
               workspace: Optional[torch.Tensor] = None, gX: Optional[torch.Tensor] = None, dropout=None):
    """Loss and gradients of one locally trained layer -> (loss [1], gW1, gb1, gWc, gbc) device tensors;
    with ``gX`` given, dL/dX is written into it as well.  ``dropout`` = (p_drop, seed, draw) trains with
    dropout on the hidden units."""
    n = int(labels.numel())
    h = 0 if Wc is None else int(W1.shape[1])
    c = int(W1.shape[1]) if Wc is None else int(Wc.shape[1])
    need = B.retexo_train_workspace_bytes(n, d_in, h, c)
    if need < 0:
        raise B.RetexoError(need, "retexo_train_workspace_bytes")
    if workspace is None:
        workspace = ws_tensor(need)
    gW1, gb1 = torch.empty_like(W1), torch.empty_like(b1)
    gWc = torch.empty_like(Wc) if Wc is not None else None
    gbc = torch.empty_like(bc) if Wc is not None else None
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    p = lambda t: t.data_ptr() if t is not None else 0
    if dropout is not None:
        p_drop, seed, draw = dropout
        st = B.retexo_layer_grad_dropout(n, d_in, h, c, X.data_ptr(), X.stride(0), labels.data_ptr(), p(W1), p(b1),
                                         p(Wc), p(bc), p(gW1), p(gb1), p(gWc), p(gbc), loss.data_ptr(), p(gX),
                                         gX.stride(0) if gX is not None else 0, float(p_drop), int(seed), int(draw),
                                         workspace.data_ptr(), workspace.numel(), _stream_ptr())
    elif gX is None:
        st = B.retexo_layer_grad(n, d_in, h, c, X.data_ptr(), X.stride(0), labels.data_ptr(), p(W1), p(b1), p(Wc),
                                 p(bc), p(gW1), p(gb1), p(gWc), p(gbc), loss.data_ptr(), workspace.data_ptr(),
                                 workspace.numel(), _stream_ptr())
    else:
        st = B.retexo_layer_grad_x(n, d_in, h, c, X.data_ptr(), X.stride(0), labels.data_ptr(), p(W1), p(b1), p(Wc),
                                   p(bc), p(gW1), p(gb1), p(gWc), p(gbc), loss.data_ptr(), gX.data_ptr(),
                                   gX.stride(0), workspace.data_ptr(), workspace.numel(), _stream_ptr())
    B.check(st, "retexo_layer_grad")
    return loss, gW1, gb1, gWc, gbc


class Pipeline:
    """All device buffers of one workload, allocated once; ``run`` replays the
    whole hot path: CSR construction, plan, then every stage in order."""

    def __init__(self, wl: Workload, src: np.ndarray, dst: np.ndarray, feats: np.ndarray,
                 params: Sequence[StageParams]):
        self.wl = wl
        self.n = wl.n_nodes
        self.src = dev(src.astype(np.int32))
        self.dst = dev(dst.astype(np.int32))
        self.H0 = dev(feats)
        n_pairs = int(self.src.numel())
        self.csr_ws = ws_tensor(B.retexo_csr_workspace_bytes(n_pairs, self.n, wl.self_loops))
        cap = 2 * n_pairs + (self.n if wl.self_loops else 0)
        self.row_ptr = torch.empty(self.n + 1, dtype=torch.int64, device="cuda")
        self.col_idx = torch.empty(max(cap, 1), dtype=torch.int32, device="cuda")
        self.params = []
        for p in params:
            self.params.append(tuple(None if a is None else dev(a) for a in (p.W, p.b, p.a_src, p.a_dst)))
        self.outs: List[torch.Tensor] = []
        for st in wl.stages:
            self.outs.append(torch.empty((self.n, pad_ld(st.out_width)), dtype=torch.float32, device="cuda"))
        self.graph: Optional[DeviceGraph] = None
        self.round_ws: Optional[torch.Tensor] = None
        self.plan_ws: Optional[torch.Tensor] = None

    def build_graph(self) -> DeviceGraph:
        if self.graph is not None:
            self.graph.destroy()
        g = csr_from_coo(self.src, self.dst, self.n, self.wl.self_loops, self.csr_ws,
                         self.row_ptr, self.col_idx)
        # the plan lives in a buffer of the pipeline: a step allocates nothing
        need = B.retexo_plan_workspace_bytes(self.n, g.nnz, 0)
        if self.plan_ws is None or self.plan_ws.numel() < need:
            self.plan_ws = ws_tensor(need)
        self.graph = make_plan(g, workspace=self.plan_ws)
        if self.round_ws is None:
            need = 0
            for st in self.wl.stages:
                if st.kind == "round":
                    flags = B.F_SELF_CONCAT if st.concat else 0
                    need = max(need, B.retexo_workspace_bytes(self.graph.plan, st.d_out, B.MODES[st.mode],
                                                              st.heads, flags))
            self.round_ws = ws_tensor(need)
        return self.graph

    def run_stage(self, i: int) -> torch.Tensor:
        st = self.wl.stages[i]
        H = self.H0 if i == 0 else self.outs[i - 1]
        W, b, a_src, a_dst = self.params[i]
        if st.kind == "transform":
            transform(H, st.d_in, W, b, st.relu, out=self.outs[i])
        elif st.kind == "head_mean":
            B.check(B.retexo_head_mean(self.n, st.heads, st.d_out, H.data_ptr(), H.stride(0),
                                       self.outs[i].data_ptr(), self.outs[i].stride(0), _stream_ptr()),
                    "retexo_head_mean")
        else:
            round_(self.graph, st, H, W, b, a_src, a_dst, self.outs[i], self.round_ws)
        return self.outs[i]

    def run(self, events=None) -> List[torch.Tensor]:
        """One pass of the whole path.  ``events``: optional list that receives
        (label, start_event, end_event) per step for timing."""
        def mark():
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            return e
        t0 = mark() if events is not None else None
        self.build_graph()
        if events is not None:
            t1 = mark()
            events.append(("csr+plan", t0, t1))
        for i, st in enumerate(self.wl.stages):
            s = mark() if events is not None else None
            self.run_stage(i)
            if events is not None:
                events.append(("%s%d" % (st.kind, i), s, mark()))
        return self.outs

    def close(self) -> None:
        if self.graph is not None:
            self.graph.destroy()
            self.graph = None
