"""Python face of the CPU oracle (test infrastructure, not product code).

Compiles ``retexo_oracle.c`` with gcc on first use and exposes its functions
on numpy arrays.  Only tests, the smoke check and the benchmark's
``cpu_baseline`` leg import this package; the GPU library never does, and this
package never touches the GPU library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "retexo_oracle.c")
_LIB = os.path.join(_HERE, "libretexo_oracle.so")

MODES = {"mean": 0, "sum": 1, "gcn_sym": 2, "gat_softmax": 3, "max": 4}


def build(force: bool = False) -> str:
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        i64, i32p, i64p = C.c_int64, C.POINTER(C.c_int32), C.POINTER(C.c_int64)
        f32p, f64p = C.POINTER(C.c_float), C.POINTER(C.c_double)
        u8p = C.POINTER(C.c_uint8)
        lib.oracle_threads.restype = C.c_int
        lib.oracle_csr_from_coo.restype = i64
        lib.oracle_csr_from_coo.argtypes = [i64, i32p, i32p, i64, C.c_int, i64p, i32p]
        lib.oracle_degree.restype = None
        lib.oracle_degree.argtypes = [i64, i64p, i32p, f32p]
        lib.oracle_transform.restype = None
        lib.oracle_transform.argtypes = [i64, i64p, i64, i64, f32p, i64, f32p, f32p, C.c_int, f64p]
        lib.oracle_aggregate.restype = None
        lib.oracle_aggregate.argtypes = [C.c_int, i64, i64p, i64p, i32p, f32p, i64, C.c_int,
                                         f32p, i64, f32p, f32p, C.c_double, C.c_int, f64p]
        lib.oracle_aggregate_abs.restype = None
        lib.oracle_aggregate_abs.argtypes = lib.oracle_aggregate.argtypes
        lib.oracle_gat_alpha.restype = None
        lib.oracle_gat_alpha.argtypes = [i64, C.c_int, i64p, i32p, i64, C.c_int, f32p, i64,
                                         f32p, f32p, C.c_double, f64p]
        lib.oracle_aggregate_backward.restype = C.c_int
        lib.oracle_aggregate_backward.argtypes = [C.c_int, i64, i64, i64p, i64p, i32p, f32p, i64, C.c_int,
                                                  f32p, i64, f32p, f32p, C.c_double, f32p, i64, C.c_int,
                                                  f64p, f64p, f64p]
        lib.oracle_aggregate_backward_slack.restype = C.c_int
        lib.oracle_aggregate_backward_slack.argtypes = lib.oracle_aggregate_backward.argtypes + [C.c_double, f64p]
        lib.oracle_layer_grad.restype = C.c_double
        lib.oracle_layer_grad.argtypes = [i64, i64, i64, i64, f32p, i64, i32p, f32p, f32p, f32p, f32p,
                                          f64p, f64p, f64p, f64p, f64p, u8p, C.c_double]
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_philox4x32_10.argtypes = [C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
        lib.oracle_dropout_keep.restype = None
        lib.oracle_dropout_keep.argtypes = [i64, i64, C.c_float, C.c_uint64, C.c_uint64, u8p]
        lib.oracle_transform_backward.restype = None
        lib.oracle_transform_backward.argtypes = [i64, i64, i64, f32p, i64, f32p, i64, f64p, f64p]
        lib.oracle_layer_loss.restype = C.c_double
        lib.oracle_layer_loss.argtypes = [i64, i64, i64, i64, f32p, i64, i32p, f64p, f64p, f64p, f64p, u8p, C.c_double]
        _lib = lib
    return _lib


def _p(a: Optional[np.ndarray], ctype):
    if a is None:
        return None
    return a.ctypes.data_as(C.POINTER(ctype))


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def threads() -> int:
    return int(_load().oracle_threads())


def csr_from_coo(src, dst, n_nodes: int, add_self_loops: bool):
    """-> (row_ptr int64[N+1], col_idx int32[nnz])"""
    src, dst = _c(src, np.int32), _c(dst, np.int32)
    assert src.shape == dst.shape and src.ndim == 1
    row_ptr = np.empty(n_nodes + 1, np.int64)
    col = np.empty(2 * src.size + n_nodes + 1, np.int32)
    nnz = _load().oracle_csr_from_coo(src.size, _p(src, C.c_int32), _p(dst, C.c_int32),
                                      n_nodes, int(add_self_loops),
                                      _p(row_ptr, C.c_int64), _p(col, C.c_int32))
    if nnz < 0:
        raise ValueError("oracle_csr_from_coo failed with %d" % nnz)
    return row_ptr, col[:nnz].copy()


def degree(row_ptr):
    """-> (deg int32[N], dinv float32[N])"""
    row_ptr = _c(row_ptr, np.int64)
    n = row_ptr.size - 1
    deg = np.empty(n, np.int32)
    dinv = np.empty(n, np.float32)
    _load().oracle_degree(n, _p(row_ptr, C.c_int64), _p(deg, C.c_int32), _p(dinv, C.c_float))
    return deg, dinv


def _matrix(a):
    a = np.asarray(a)
    assert a.dtype == np.float32 and a.ndim == 2 and a.strides[1] == 4 and a.strides[0] % 4 == 0
    return a, a.strides[0] // 4


def transform(H, d_in: int, W, b=None, relu: bool = False, rows=None) -> np.ndarray:
    """Z = act(H[:, :d_in] W + b) in float64, for all rows or for ``rows``."""
    H, ldh = _matrix(H)
    W = _c(W, np.float32)
    assert W.shape[0] == d_in and d_in <= H.shape[1]
    d_out = W.shape[1]
    b = None if b is None else _c(b, np.float32)
    rows = None if rows is None else _c(rows, np.int64)
    n = H.shape[0] if rows is None else rows.size
    Z = np.empty((n, d_out), np.float64)
    _load().oracle_transform(n, _p(rows, C.c_int64), d_in, d_out, _p(H, C.c_float), ldh,
                             _p(W, C.c_float), _p(b, C.c_float), int(relu), _p(Z, C.c_double))
    return Z


def aggregate(mode: str, row_ptr, col_idx, Z, F: int, *, heads: int = 1, a_src=None, a_dst=None,
              slope: float = 0.2, self_concat: bool = False, rows=None) -> np.ndarray:
    """Aggregate Z[:, :F] over the CSR, float64 output [n, F or 2F]."""
    Z, ldz = _matrix(Z)
    row_ptr, col_idx = _c(row_ptr, np.int64), _c(col_idx, np.int32)
    n_nodes = row_ptr.size - 1
    assert Z.shape[0] >= n_nodes and F <= Z.shape[1]
    dinv = None
    if mode == "gcn_sym":
        _, dinv = degree(row_ptr)
    if mode == "gat_softmax":
        assert F % heads == 0
        a_src, a_dst = _c(a_src, np.float32), _c(a_dst, np.float32)
        assert a_src.size == F and a_dst.size == F
    rows = None if rows is None else _c(rows, np.int64)
    n = n_nodes if rows is None else rows.size
    out = np.empty((n, 2 * F if self_concat else F), np.float64)
    _load().oracle_aggregate(MODES[mode], n, _p(rows, C.c_int64), _p(row_ptr, C.c_int64),
                             _p(col_idx, C.c_int32), _p(dinv, C.c_float), F, heads,
                             _p(Z, C.c_float), ldz, _p(a_src, C.c_float), _p(a_dst, C.c_float),
                             float(slope), int(self_concat), _p(out, C.c_double))
    return out


def aggregate_abs(mode: str, row_ptr, col_idx, Z, F: int, *, heads: int = 1, a_src=None, a_dst=None,
                  slope: float = 0.2, self_concat: bool = False, rows=None) -> np.ndarray:
    """Size of the terms behind every element of ``aggregate``: sum_u |c_vu z_uj| (same shape)."""
    Z, ldz = _matrix(Z)
    row_ptr, col_idx = _c(row_ptr, np.int64), _c(col_idx, np.int32)
    n_nodes = row_ptr.size - 1
    assert Z.shape[0] >= n_nodes and F <= Z.shape[1]
    dinv = None
    if mode == "gcn_sym":
        _, dinv = degree(row_ptr)
    if mode == "gat_softmax":
        assert F % heads == 0
        a_src, a_dst = _c(a_src, np.float32), _c(a_dst, np.float32)
        assert a_src.size == F and a_dst.size == F
    rows = None if rows is None else _c(rows, np.int64)
    n = n_nodes if rows is None else rows.size
    out = np.empty((n, 2 * F if self_concat else F), np.float64)
    _load().oracle_aggregate_abs(MODES[mode], n, _p(rows, C.c_int64), _p(row_ptr, C.c_int64),
                                 _p(col_idx, C.c_int32), _p(dinv, C.c_float), F, heads,
                                 _p(Z, C.c_float), ldz, _p(a_src, C.c_float), _p(a_dst, C.c_float),
                                 float(slope), int(self_concat), _p(out, C.c_double))
    return out


def aggregate_backward(mode: str, row_ptr, col_idx, Z, F: int, G, *, heads: int = 1, a_src=None, a_dst=None,
                       slope: float = 0.2, self_concat: bool = False, rows=None, kink_rel=None):
    """Gradient of ``aggregate`` with respect to its inputs, given G = dL/d(out) ([N, F or 2F] float32).
    -> dZ float64 [n, F] for linear modes; (dZ, da_src, da_dst) for gat (da_* None when ``rows`` is given).
    With ``kink_rel`` given, one more item is returned: slack float64 [n, F], how far each element of dZ can
    move when the entries whose score lies within kink_rel (relative to the size of its terms) of the
    LeakyReLU kink take the derivative of the other side (see oracle_aggregate_backward_slack)."""
    Z, ldz = _matrix(Z)
    G, ldg = _matrix(G)
    row_ptr, col_idx = _c(row_ptr, np.int64), _c(col_idx, np.int32)
    n_nodes = row_ptr.size - 1
    assert Z.shape[0] >= n_nodes and G.shape[0] >= n_nodes and F <= Z.shape[1]
    assert G.shape[1] >= (2 * F if self_concat else F)
    dinv = None
    if mode == "gcn_sym":
        _, dinv = degree(row_ptr)
    gat = mode == "gat_softmax"
    da_s = da_d = None
    if gat:
        assert F % heads == 0
        a_src, a_dst = _c(a_src, np.float32), _c(a_dst, np.float32)
        assert a_src.size == F and a_dst.size == F
        if rows is None:
            da_s, da_d = np.empty(F, np.float64), np.empty(F, np.float64)
    rows = None if rows is None else _c(rows, np.int64)
    n = n_nodes if rows is None else rows.size
    dZ = np.empty((n, F), np.float64)
    args = (MODES[mode], n_nodes, n, _p(rows, C.c_int64), _p(row_ptr, C.c_int64),
            _p(col_idx, C.c_int32), _p(dinv, C.c_float), F, heads,
            _p(Z, C.c_float), ldz, _p(a_src, C.c_float), _p(a_dst, C.c_float),
            float(slope), _p(G, C.c_float), ldg, int(self_concat),
            _p(dZ, C.c_double), _p(da_s, C.c_double), _p(da_d, C.c_double))
    slack = None
    if kink_rel is None:
        rc = _load().oracle_aggregate_backward(*args)
    else:
        slack = np.empty((n, F), np.float64)
        rc = _load().oracle_aggregate_backward_slack(*args, float(kink_rel), _p(slack, C.c_double))
    if rc != 0:
        raise ValueError("mode %r has no backward" % mode)
    res = (dZ,)
    if gat:
        res = (dZ, (None if da_s is None else da_s.reshape(heads, F // heads)),
               (None if da_d is None else da_d.reshape(heads, F // heads)))
    if slack is not None:
        return res + (slack,)
    return res if gat else dZ


def gat_alpha(v: int, h: int, row_ptr, col_idx, Z, F: int, heads: int, a_src, a_dst,
              slope: float = 0.2) -> np.ndarray:
    Z, ldz = _matrix(Z)
    row_ptr, col_idx = _c(row_ptr, np.int64), _c(col_idx, np.int32)
    a_src, a_dst = _c(a_src, np.float32), _c(a_dst, np.float32)
    deg = int(row_ptr[v + 1] - row_ptr[v])
    alpha = np.empty(deg, np.float64)
    _load().oracle_gat_alpha(v, h, _p(row_ptr, C.c_int64), _p(col_idx, C.c_int32), F, heads,
                             _p(Z, C.c_float), ldz, _p(a_src, C.c_float), _p(a_dst, C.c_float),
                             float(slope), _p(alpha, C.c_double))
    return alpha


def round_(mode: str, row_ptr, col_idx, H, d_in: int, W, b, *, relu: bool = False, heads: int = 1,
           a_src=None, a_dst=None, slope: float = 0.2, self_concat: bool = False,
           rows=None) -> np.ndarray:
    """One lazy-message-passing round: Z = act(H W + b) (W None: Z = H), stored
    as float32 the way the real pipeline stores it, then aggregated.

    With ``rows`` given only those output rows are produced, and the transform
    is evaluated only where the aggregation will look (the rows themselves and
    their neighbours); every other row of the intermediate is NaN so that a
    stray read shows up.
    """
    row_ptr, col_idx = _c(row_ptr, np.int64), _c(col_idx, np.int32)
    n_nodes = row_ptr.size - 1
    if W is None:
        Z32, F = H, d_in
    else:
        F = np.asarray(W).shape[1]
        if rows is None:
            Z32 = transform(H, d_in, W, b, relu).astype(np.float32)
        else:
            rows = _c(rows, np.int64)
            need = [rows]
            for v in rows:
                need.append(col_idx[row_ptr[v]:row_ptr[v + 1]].astype(np.int64))
            need = np.unique(np.concatenate(need))
            Z32 = np.full((n_nodes, F), np.nan, np.float32)
            Z32[need] = transform(H, d_in, W, b, relu, rows=need).astype(np.float32)
    return aggregate(mode, row_ptr, col_idx, Z32, F, heads=heads, a_src=a_src, a_dst=a_dst,
                     slope=slope, self_concat=self_concat, rows=rows)


def head_mean(X, heads: int, n_classes: int) -> np.ndarray:
    """Average of the ``heads`` column blocks of X[:, :heads * n_classes], float64 [n, n_classes]:
    out[v, c] = (1 / heads) * sum_h X[v, h * n_classes + c].  The last attention round of a classifier
    keeps one block of class scores per head and averages them (the standard form of the attention
    network the paper's evaluation set-up names; the paper itself does not print it)."""
    X = np.asarray(X)
    assert X.shape[1] >= heads * n_classes
    out = np.zeros((X.shape[0], n_classes), np.float64)
    for h in range(heads):
        out += X[:, h * n_classes:(h + 1) * n_classes].astype(np.float64)
    return out / float(heads)


def philox4x32_10(counter, key):
    """One block of the counter-based generator behind the dropout mask: four 32-bit words."""
    c = (C.c_uint32 * 4)(*[int(x) for x in counter])
    k = (C.c_uint32 * 2)(*[int(x) for x in key])
    out = (C.c_uint32 * 4)()
    _load().oracle_philox4x32_10(c, k, out)
    return [int(x) for x in out]


def dropout_keep(n: int, h: int, p_drop: float, seed: int, draw: int) -> np.ndarray:
    """-> uint8 [n, h]: 1 where unit j of node v survives dropout number ``draw`` of stream ``seed``."""
    keep = np.empty((n, h), np.uint8)
    _load().oracle_dropout_keep(n, h, np.float32(p_drop), seed, draw, _p(keep, C.c_uint8))
    return keep


def _dropout_args(dropout, n: int, h: int):
    """dropout = None or (p_drop, seed, draw) -> (mask array or None, scale)"""
    if dropout is None:
        return None, 1.0
    assert h > 0, "dropout acts on the hidden units"
    p_drop, seed, draw = dropout
    p32 = np.float32(p_drop)
    assert 0.0 <= p32 < 1.0
    return dropout_keep(n, h, p32, seed, draw), 1.0 / (1.0 - float(p32))


def layer_grad(X, d_in: int, labels, W1, b1, Wc=None, bc=None, input_grad: bool = False, dropout=None):
    """Loss and parameter gradients of one locally trained layer (see oracle_layer_grad).
    Wc None: the layer is the final classifier (logits = X W1 + b1).
    dropout: None, or (p_drop, seed, draw) for dropout on the hidden units.
    -> (loss, gW1, gb1, gWc or None, gbc or None), float64; with ``input_grad`` a sixth item,
    dL/dX [n, d_in]."""
    X, ldx = _matrix(X)
    labels = _c(labels, np.int32)
    W1, b1 = _c(W1, np.float32), _c(b1, np.float32)
    n = labels.size
    assert X.shape[0] >= n and W1.shape[0] == d_in
    if Wc is None:
        H, Cc = 0, W1.shape[1]
        Wc_ = bc_ = None
        gWc = gbc = None
    else:
        Wc_, bc_ = _c(Wc, np.float32), _c(bc, np.float32)
        H, Cc = W1.shape[1], Wc_.shape[1]
        assert Wc_.shape[0] == H
        gWc = np.empty((H, Cc), np.float64)
        gbc = np.empty(Cc, np.float64)
    gW1 = np.empty(W1.shape, np.float64)
    gb1 = np.empty(W1.shape[1], np.float64)
    gX = np.empty((n, d_in), np.float64) if input_grad else None
    keep, scale = _dropout_args(dropout, n, H)
    loss = _load().oracle_layer_grad(n, d_in, H, Cc, _p(X, C.c_float), ldx, _p(labels, C.c_int32),
                                     _p(W1, C.c_float), _p(b1, C.c_float), _p(Wc_, C.c_float),
                                     _p(bc_, C.c_float), _p(gW1, C.c_double), _p(gb1, C.c_double),
                                     _p(gWc, C.c_double), _p(gbc, C.c_double), _p(gX, C.c_double),
                                     _p(keep, C.c_uint8), scale)
    if input_grad:
        return float(loss), gW1, gb1, gWc, gbc, gX
    return float(loss), gW1, gb1, gWc, gbc


def transform_backward(H, d_in: int, dZ, d_out: int):
    """-> (gW [d_in, d_out], gb [d_out]) float64: gradients of Z = H W + b given dZ = dL/dZ."""
    H, ldh = _matrix(H)
    dZ, lddz = _matrix(dZ)
    n = H.shape[0]
    assert dZ.shape[0] == n and d_in <= H.shape[1] and d_out <= dZ.shape[1]
    gW, gb = np.empty((d_in, d_out), np.float64), np.empty(d_out, np.float64)
    _load().oracle_transform_backward(n, d_in, d_out, _p(H, C.c_float), ldh, _p(dZ, C.c_float), lddz,
                                      _p(gW, C.c_double), _p(gb, C.c_double))
    return gW, gb


def layer_loss(X, d_in: int, labels, W1, b1, Wc=None, bc=None, dropout=None) -> float:
    """The loss alone, with float64 parameters (for numerical differencing in tests)."""
    X, ldx = _matrix(X)
    labels = _c(labels, np.int32)
    W1, b1 = _c(W1, np.float64), _c(b1, np.float64)
    if Wc is None:
        H, Cc, Wc_, bc_ = 0, W1.shape[1], None, None
    else:
        Wc_, bc_ = _c(Wc, np.float64), _c(bc, np.float64)
        H, Cc = W1.shape[1], Wc_.shape[1]
    keep, scale = _dropout_args(dropout, labels.size, H)
    return float(_load().oracle_layer_loss(labels.size, d_in, H, Cc, _p(X, C.c_float), ldx,
                                           _p(labels, C.c_int32), _p(W1, C.c_double), _p(b1, C.c_double),
                                           _p(Wc_, C.c_double), _p(bc_, C.c_double),
                                           _p(keep, C.c_uint8), scale))
