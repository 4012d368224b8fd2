"""ctypes binding of libretexo.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
``include/retexo.h`` and takes raw device addresses (ints, e.g.
``tensor.data_ptr()``) and sizes.  Nothing is computed here, and there is no
fallback: if the library is missing, ``load()`` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libretexo.so")

MEAN, SUM, GCN_SYM, GAT_SOFTMAX, MAX = 0, 1, 2, 3, 4
MODES = {"mean": MEAN, "sum": SUM, "gcn_sym": GCN_SYM, "gat_softmax": GAT_SOFTMAX, "max": MAX}
F_RELU, F_SELF_CONCAT, F_VALIDATE, F_SPLIT_ROWS, F_SAVE = 1, 2, 4, 8, 16

OK = 0
E_NULL, E_SIZE, E_LD, E_MODE, E_FLAGS, E_HEADS = -1, -2, -3, -4, -5, -6
E_CSR, E_WORKSPACE, E_ALIAS, E_HIP, E_CAPACITY = -7, -8, -9, -10, -11

EXPORTS = (
    "retexo_status_string", "retexo_csr_workspace_bytes", "retexo_csr_from_coo",
    "retexo_plan_create", "retexo_plan_workspace_bytes", "retexo_plan_create_in", "retexo_plan_destroy", "retexo_plan_num_nodes", "retexo_plan_nnz",
    "retexo_plan_max_degree", "retexo_plan_deg", "retexo_plan_dinv", "retexo_plan_export",
    "retexo_plan_export_split",
    "retexo_workspace_bytes",
    "retexo_transform", "retexo_aggregate", "retexo_aggregate_noalloc", "retexo_round", "retexo_set_option",
    "retexo_aggregate_backward_workspace_bytes", "retexo_aggregate_backward", "retexo_aggregate_backward_saved",
    "retexo_partition_workspace_bytes", "retexo_partition_share", "retexo_halo_pack", "retexo_halo_unpack",
    "retexo_plan_set_degrees", "retexo_data_volumes", "retexo_gamma",
    "retexo_store_rows", "retexo_aggregate_stored", "retexo_head_mean",
    "retexo_train_workspace_bytes", "retexo_layer_grad", "retexo_sgd_update",
    "retexo_layer_grad_x", "retexo_layer_grad_dropout", "retexo_transform_backward_workspace_bytes", "retexo_transform_backward",
)

_lib = None


class RetexoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %d (%s)" % (where, status, status_string(status)))


def load():
    """Load libretexo.so (built by ``paper_2302_13053_amd.build.build()``)."""
    global _lib
    if _lib is not None:
        return _lib
    # torch owns the device memory and streams handed to the library; importing it
    # first also makes both sides share one HIP runtime (same soname)
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libretexo.so is not built: run `python -m paper_2302_13053_amd.build` "
                           "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    i64, i32, vp, u32, f32 = C.c_int64, C.c_int, C.c_void_p, C.c_uint, C.c_float
    lib.retexo_status_string.restype = C.c_char_p
    lib.retexo_status_string.argtypes = [i32]
    lib.retexo_csr_workspace_bytes.restype = i64
    lib.retexo_csr_workspace_bytes.argtypes = [i64, i64, i32]
    lib.retexo_csr_from_coo.restype = i32
    lib.retexo_csr_from_coo.argtypes = [i64, vp, vp, i64, i32, vp, vp, i64, C.POINTER(i64), vp, i64, vp]
    lib.retexo_plan_create.restype = i32
    lib.retexo_plan_create.argtypes = [C.POINTER(vp), i64, vp, vp, u32, vp]
    lib.retexo_plan_workspace_bytes.restype = i64
    lib.retexo_plan_workspace_bytes.argtypes = [i64, i64, u32]
    lib.retexo_plan_create_in.restype = i32
    lib.retexo_plan_create_in.argtypes = [C.POINTER(vp), i64, i64, vp, vp, u32, vp, i64, vp]
    lib.retexo_plan_destroy.restype = i32
    lib.retexo_plan_destroy.argtypes = [vp]
    lib.retexo_plan_num_nodes.restype = i64
    lib.retexo_plan_num_nodes.argtypes = [vp]
    lib.retexo_plan_nnz.restype = i64
    lib.retexo_plan_nnz.argtypes = [vp]
    lib.retexo_plan_max_degree.restype = C.c_int32
    lib.retexo_plan_max_degree.argtypes = [vp]
    lib.retexo_plan_deg.restype = vp
    lib.retexo_plan_deg.argtypes = [vp]
    lib.retexo_plan_dinv.restype = vp
    lib.retexo_plan_dinv.argtypes = [vp]
    lib.retexo_plan_export.restype = i32
    lib.retexo_plan_export.argtypes = [vp, vp, vp, vp, vp]
    lib.retexo_plan_export_split.restype = i64
    lib.retexo_plan_export_split.argtypes = [vp, vp, vp]
    lib.retexo_workspace_bytes.restype = i64
    lib.retexo_workspace_bytes.argtypes = [vp, i64, i32, i32, u32]
    lib.retexo_transform.restype = i32
    lib.retexo_transform.argtypes = [i64, i64, i64, vp, i64, vp, vp, u32, vp, i64, vp]
    lib.retexo_aggregate.restype = i32
    lib.retexo_aggregate.argtypes = [vp, i32, i64, i32, vp, i64, vp, vp, f32, u32, vp, i64, vp, i64, vp]
    lib.retexo_aggregate_noalloc.restype = i32
    lib.retexo_aggregate_noalloc.argtypes = [vp, i32, i64, i32, vp, i64, vp, vp, f32, u32, vp, i64, vp]
    lib.retexo_aggregate_backward_workspace_bytes.restype = i64
    lib.retexo_aggregate_backward_workspace_bytes.argtypes = [vp, i32, i64, i32]
    lib.retexo_aggregate_backward.restype = i32
    lib.retexo_aggregate_backward.argtypes = [vp, i32, i64, i32, vp, i64, vp, vp, f32, u32, vp, i64,
                                              vp, i64, vp, vp, vp, i64, vp]
    lib.retexo_aggregate_backward_saved.restype = i32
    lib.retexo_aggregate_backward_saved.argtypes = [vp, i32, i64, i32, vp, i64, vp, vp, f32, u32, vp, i64,
                                                    vp, i64, vp, i64, vp, vp, vp, i64, vp]
    lib.retexo_head_mean.restype = i32
    lib.retexo_head_mean.argtypes = [i64, i32, i64, vp, i64, vp, i64, vp]
    lib.retexo_store_rows.restype = i32
    lib.retexo_store_rows.argtypes = [i32, i64, i64, vp, i64, vp, i64, vp]
    lib.retexo_aggregate_stored.restype = i32
    lib.retexo_aggregate_stored.argtypes = [vp, i32, i32, i64, i32, vp, i64, vp, vp, f32, u32, vp, i64, vp, i64, vp]
    lib.retexo_partition_workspace_bytes.restype = i64
    lib.retexo_partition_workspace_bytes.argtypes = [i64, i32, i64]
    lib.retexo_partition_share.restype = i32
    lib.retexo_partition_share.argtypes = [i64, vp, vp, vp, i32, i32, i64, i64, i64, vp, vp, vp, vp, vp, vp,
                                           C.POINTER(i64), C.POINTER(i64), C.POINTER(i64), vp, i64, vp]
    lib.retexo_halo_pack.restype = i32
    lib.retexo_halo_pack.argtypes = [i64, vp, i64, i64, vp, i64, vp, i64, vp]
    lib.retexo_halo_unpack.restype = i32
    lib.retexo_halo_unpack.argtypes = [i64, vp, i64, i64, vp, i64, vp, i64, vp]
    lib.retexo_plan_set_degrees.restype = i32
    lib.retexo_plan_set_degrees.argtypes = [vp, vp, vp]
    lib.retexo_data_volumes.restype = i32
    lib.retexo_data_volumes.argtypes = [C.c_double] * 7 + [C.POINTER(C.c_double)]
    lib.retexo_gamma.restype = C.c_double
    lib.retexo_gamma.argtypes = [C.c_double] * 6
    lib.retexo_round.restype = i32
    lib.retexo_round.argtypes = [vp, i32, i64, i64, i32, vp, i64, vp, vp, vp, vp, f32, u32, vp, i64,
                                 vp, i64, vp]
    lib.retexo_train_workspace_bytes.restype = i64
    lib.retexo_train_workspace_bytes.argtypes = [i64, i64, i64, i64]
    lib.retexo_layer_grad.restype = i32
    lib.retexo_layer_grad.argtypes = [i64, i64, i64, i64, vp, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                      vp, i64, vp]
    lib.retexo_layer_grad_x.restype = i32
    lib.retexo_layer_grad_x.argtypes = [i64, i64, i64, i64, vp, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                        vp, i64, vp, i64, vp]
    lib.retexo_layer_grad_dropout.restype = i32
    lib.retexo_layer_grad_dropout.argtypes = [i64, i64, i64, i64, vp, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                              vp, i64, C.c_float, C.c_uint64, C.c_uint64, vp, i64, vp]
    lib.retexo_transform_backward_workspace_bytes.restype = i64
    lib.retexo_transform_backward_workspace_bytes.argtypes = [i64, i64, i64]
    lib.retexo_transform_backward.restype = i32
    lib.retexo_transform_backward.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, vp, vp, i64, vp]
    lib.retexo_sgd_update.restype = i32
    lib.retexo_sgd_update.argtypes = [i64, vp, vp, f32, vp]
    lib.retexo_set_option.restype = i32
    lib.retexo_set_option.argtypes = [C.c_char_p, i64]
    _lib = lib
    return lib


def _vp(addr: Optional[int]):
    return C.c_void_p(addr) if addr else None


def retexo_status_string(status: int) -> str:
    return load().retexo_status_string(int(status)).decode()


status_string = retexo_status_string


def retexo_csr_workspace_bytes(n_pairs: int, n_nodes: int, add_self_loops: bool) -> int:
    return int(load().retexo_csr_workspace_bytes(n_pairs, n_nodes, int(add_self_loops)))


def retexo_csr_from_coo(n_pairs, d_src, d_dst, n_nodes, add_self_loops, d_row_ptr, d_col_idx,
                        col_capacity, d_workspace, workspace_bytes, stream=0):
    """-> (status, nnz)"""
    nnz = C.c_int64(-1)
    st = load().retexo_csr_from_coo(n_pairs, _vp(d_src), _vp(d_dst), n_nodes, int(add_self_loops),
                                    _vp(d_row_ptr), _vp(d_col_idx), col_capacity, C.byref(nnz),
                                    _vp(d_workspace), workspace_bytes, _vp(stream))
    return int(st), int(nnz.value)


def retexo_plan_create(n_nodes, d_row_ptr, d_col_idx, flags=0, stream=0):
    """-> (status, plan handle or None)"""
    h = C.c_void_p()
    st = load().retexo_plan_create(C.byref(h), n_nodes, _vp(d_row_ptr), _vp(d_col_idx), flags, _vp(stream))
    return int(st), (h.value if st == 0 else None)


def retexo_plan_workspace_bytes(n_nodes, nnz, flags=0) -> int:
    return int(load().retexo_plan_workspace_bytes(n_nodes, nnz, flags))


def retexo_plan_create_in(n_nodes, nnz, d_row_ptr, d_col_idx, flags, d_workspace, workspace_bytes, stream=0):
    """-> (status, plan handle or None); the plan's device arrays live in the caller's workspace"""
    h = C.c_void_p()
    st = load().retexo_plan_create_in(C.byref(h), n_nodes, nnz, _vp(d_row_ptr), _vp(d_col_idx), flags,
                                      _vp(d_workspace), workspace_bytes, _vp(stream))
    return int(st), (h.value if st == 0 else None)


def retexo_plan_destroy(plan) -> int:
    return int(load().retexo_plan_destroy(_vp(plan)))


def retexo_plan_num_nodes(plan) -> int:
    return int(load().retexo_plan_num_nodes(_vp(plan)))


def retexo_plan_nnz(plan) -> int:
    return int(load().retexo_plan_nnz(_vp(plan)))


def retexo_plan_max_degree(plan) -> int:
    return int(load().retexo_plan_max_degree(_vp(plan)))


def retexo_plan_deg(plan) -> int:
    return int(load().retexo_plan_deg(_vp(plan)) or 0)


def retexo_plan_dinv(plan) -> int:
    return int(load().retexo_plan_dinv(_vp(plan)) or 0)


def retexo_plan_export(plan, d_deg, d_dinv, d_order, stream=0) -> int:
    return int(load().retexo_plan_export(_vp(plan), _vp(d_deg), _vp(d_dinv), _vp(d_order), _vp(stream)))


SPLIT_PARTS = 16


def retexo_plan_export_split(plan, d_pos, stream=0) -> int:
    return int(load().retexo_plan_export_split(_vp(plan), _vp(d_pos), _vp(stream)))


def retexo_workspace_bytes(plan, d_out, mode, heads=1, flags=0) -> int:
    return int(load().retexo_workspace_bytes(_vp(plan), d_out, mode, heads, flags))


def retexo_transform(n, d_in, d_out, d_H, ldh, d_W, d_b, flags, d_Z, ldz, stream=0) -> int:
    return int(load().retexo_transform(n, d_in, d_out, _vp(d_H), ldh, _vp(d_W), _vp(d_b), flags,
                                       _vp(d_Z), ldz, _vp(stream)))


def retexo_aggregate(plan, mode, F, heads, d_Z, ldz, d_attn_src, d_attn_dst, negative_slope, flags,
                     d_out, ldo, d_workspace, workspace_bytes, stream=0) -> int:
    return int(load().retexo_aggregate(_vp(plan), mode, F, heads, _vp(d_Z), ldz, _vp(d_attn_src),
                                       _vp(d_attn_dst), negative_slope, flags, _vp(d_out), ldo,
                                       _vp(d_workspace), workspace_bytes, _vp(stream)))


NOALLOC_SCRATCH_BYTES = 33554432


def retexo_aggregate_noalloc(plan, mode, F, heads, d_Z, ldz, d_attn_src, d_attn_dst, negative_slope, flags,
                             d_out, ldo, stream=0) -> int:
    return int(load().retexo_aggregate_noalloc(_vp(plan), mode, F, heads, _vp(d_Z), ldz, _vp(d_attn_src),
                                               _vp(d_attn_dst), negative_slope, flags, _vp(d_out), ldo,
                                               _vp(stream)))


def retexo_aggregate_backward_workspace_bytes(plan, mode, F, heads) -> int:
    return int(load().retexo_aggregate_backward_workspace_bytes(_vp(plan), mode, F, heads))


def retexo_aggregate_backward(plan, mode, F, heads, d_Z, ldz, d_attn_src, d_attn_dst, negative_slope, flags,
                              d_G, ldg, d_dZ, lddz, d_dattn_src, d_dattn_dst, d_workspace, workspace_bytes,
                              stream=0) -> int:
    return int(load().retexo_aggregate_backward(_vp(plan), mode, F, heads, _vp(d_Z), ldz, _vp(d_attn_src),
                                                _vp(d_attn_dst), negative_slope, flags, _vp(d_G), ldg,
                                                _vp(d_dZ), lddz, _vp(d_dattn_src), _vp(d_dattn_dst),
                                                _vp(d_workspace), workspace_bytes, _vp(stream)))


def retexo_aggregate_backward_saved(plan, mode, F, heads, d_Z, ldz, d_attn_src, d_attn_dst, negative_slope, flags,
                                    d_G, ldg, d_saved, saved_bytes, d_dZ, lddz, d_dattn_src,
                                    d_dattn_dst, d_workspace, workspace_bytes, stream=0) -> int:
    return int(load().retexo_aggregate_backward_saved(_vp(plan), mode, F, heads, _vp(d_Z), ldz, _vp(d_attn_src),
                                                      _vp(d_attn_dst), negative_slope, flags, _vp(d_G), ldg,
                                                      _vp(d_saved), saved_bytes, _vp(d_dZ), lddz,
                                                      _vp(d_dattn_src), _vp(d_dattn_dst), _vp(d_workspace),
                                                      workspace_bytes, _vp(stream)))


def retexo_head_mean(n, heads, C_, d_in, ldi, d_out, ldo, stream=0) -> int:
    return int(load().retexo_head_mean(n, heads, C_, _vp(d_in), ldi, _vp(d_out), ldo, _vp(stream)))


STORAGE = {"bf16": 1, "fp16": 2}


def retexo_store_rows(storage, n, F, d_src, lds, d_dst, ldd, stream=0) -> int:
    return int(load().retexo_store_rows(storage, n, F, _vp(d_src), lds, _vp(d_dst), ldd, _vp(stream)))


def retexo_aggregate_stored(plan, mode, storage, F, heads, d_Z, ldz, d_attn_src, d_attn_dst, negative_slope, flags,
                            d_out, ldo, d_workspace, workspace_bytes, stream=0) -> int:
    return int(load().retexo_aggregate_stored(_vp(plan), mode, storage, F, heads, _vp(d_Z), ldz, _vp(d_attn_src),
                                              _vp(d_attn_dst), negative_slope, flags, _vp(d_out), ldo,
                                              _vp(d_workspace), workspace_bytes, _vp(stream)))


def retexo_partition_workspace_bytes(n_nodes, n_parts, send_capacity) -> int:
    return int(load().retexo_partition_workspace_bytes(n_nodes, n_parts, send_capacity))


def retexo_partition_share(n_nodes, d_row_ptr, d_col_idx, d_part, n_parts, part, local_capacity, col_capacity,
                           send_capacity, d_local_ids, d_local_row_ptr, d_local_col_idx, d_global_deg,
                           d_send_ids, d_recv_ids, d_workspace, workspace_bytes, stream=0):
    """-> (status, [n_inner, n_halo, nnz_local, n_send], send_offsets, recv_offsets) with host lists"""
    sizes = (C.c_int64 * 4)(-1, -1, -1, -1)
    so = (C.c_int64 * (n_parts + 1))()
    ro = (C.c_int64 * (n_parts + 1))()
    st = load().retexo_partition_share(n_nodes, _vp(d_row_ptr), _vp(d_col_idx), _vp(d_part), n_parts, part,
                                       local_capacity, col_capacity, send_capacity, _vp(d_local_ids),
                                       _vp(d_local_row_ptr), _vp(d_local_col_idx), _vp(d_global_deg),
                                       _vp(d_send_ids), _vp(d_recv_ids), sizes, so, ro,
                                       _vp(d_workspace), workspace_bytes, _vp(stream))
    return int(st), list(sizes), list(so), list(ro)


def retexo_halo_pack(n, d_ids, table_rows, F, d_H, ldh, d_buf, ldb, stream=0) -> int:
    return int(load().retexo_halo_pack(n, _vp(d_ids), table_rows, F, _vp(d_H), ldh, _vp(d_buf), ldb, _vp(stream)))


def retexo_halo_unpack(n, d_ids, table_rows, F, d_buf, ldb, d_H, ldh, stream=0) -> int:
    return int(load().retexo_halo_unpack(n, _vp(d_ids), table_rows, F, _vp(d_buf), ldb, _vp(d_H), ldh, _vp(stream)))


def retexo_plan_set_degrees(plan, d_deg, stream=0) -> int:
    return int(load().retexo_plan_set_degrees(_vp(plan), _vp(d_deg), _vp(stream)))


def retexo_data_volumes(n, B, R, H0, sum_H, sum_C, M):
    """-> (status, [standard_lt, lazy_lt, standard_reduce, lazy_reduce])"""
    out = (C.c_double * 4)()
    st = load().retexo_data_volumes(n, B, R, H0, sum_H, sum_C, M, out)
    return int(st), list(out)


def retexo_gamma(B, R, H0, sum_H, sum_C, M) -> float:
    return float(load().retexo_gamma(B, R, H0, sum_H, sum_C, M))


def retexo_round(plan, mode, d_in, d_out, heads, d_H, ldh, d_W, d_b, d_attn_src, d_attn_dst,
                 negative_slope, flags, d_out_ptr, ldo, d_workspace, workspace_bytes, stream=0) -> int:
    return int(load().retexo_round(_vp(plan), mode, d_in, d_out, heads, _vp(d_H), ldh, _vp(d_W),
                                   _vp(d_b), _vp(d_attn_src), _vp(d_attn_dst), negative_slope, flags,
                                   _vp(d_out_ptr), ldo, _vp(d_workspace), workspace_bytes, _vp(stream)))


def retexo_train_workspace_bytes(n, d_in, h, c) -> int:
    return int(load().retexo_train_workspace_bytes(n, d_in, h, c))


def retexo_layer_grad(n, d_in, h, c, d_X, ldx, d_labels, d_W1, d_b1, d_Wc, d_bc, d_gW1, d_gb1, d_gWc,
                      d_gbc, d_loss, d_workspace, workspace_bytes, stream=0) -> int:
    return int(load().retexo_layer_grad(n, d_in, h, c, _vp(d_X), ldx, _vp(d_labels), _vp(d_W1), _vp(d_b1),
                                        _vp(d_Wc), _vp(d_bc), _vp(d_gW1), _vp(d_gb1), _vp(d_gWc),
                                        _vp(d_gbc), _vp(d_loss), _vp(d_workspace), workspace_bytes,
                                        _vp(stream)))


def retexo_layer_grad_x(n, d_in, h, c, d_X, ldx, d_labels, d_W1, d_b1, d_Wc, d_bc, d_gW1, d_gb1, d_gWc, d_gbc,
                        d_loss, d_gX, ldgx, d_workspace, workspace_bytes, stream=0) -> int:
    return int(load().retexo_layer_grad_x(n, d_in, h, c, _vp(d_X), ldx, _vp(d_labels), _vp(d_W1), _vp(d_b1),
                                          _vp(d_Wc), _vp(d_bc), _vp(d_gW1), _vp(d_gb1), _vp(d_gWc), _vp(d_gbc),
                                          _vp(d_loss), _vp(d_gX), ldgx, _vp(d_workspace), workspace_bytes,
                                          _vp(stream)))


def retexo_layer_grad_dropout(n, d_in, h, c, d_X, ldx, d_labels, d_W1, d_b1, d_Wc, d_bc, d_gW1, d_gb1, d_gWc,
                              d_gbc, d_loss, d_gX, ldgx, p_drop, seed, draw, d_workspace, workspace_bytes,
                              stream=0) -> int:
    return int(load().retexo_layer_grad_dropout(n, d_in, h, c, _vp(d_X), ldx, _vp(d_labels), _vp(d_W1), _vp(d_b1),
                                                _vp(d_Wc), _vp(d_bc), _vp(d_gW1), _vp(d_gb1), _vp(d_gWc),
                                                _vp(d_gbc), _vp(d_loss), _vp(d_gX), ldgx, p_drop, seed, draw,
                                                _vp(d_workspace), workspace_bytes, _vp(stream)))


def retexo_transform_backward_workspace_bytes(n, d_in, d_out) -> int:
    return int(load().retexo_transform_backward_workspace_bytes(n, d_in, d_out))


def retexo_transform_backward(n, d_in, d_out, d_H, ldh, d_dZ, lddz, d_gW, d_gb, d_workspace, workspace_bytes,
                              stream=0) -> int:
    return int(load().retexo_transform_backward(n, d_in, d_out, _vp(d_H), ldh, _vp(d_dZ), lddz, _vp(d_gW),
                                                _vp(d_gb), _vp(d_workspace), workspace_bytes, _vp(stream)))


def retexo_sgd_update(n, d_param, d_grad, lr, stream=0) -> int:
    return int(load().retexo_sgd_update(n, _vp(d_param), _vp(d_grad), lr, _vp(stream)))


def retexo_set_option(name: str, value: int) -> int:
    return int(load().retexo_set_option(name.encode(), int(value)))


def check(status: int, where: str) -> None:
    if status != OK:
        raise RetexoError(status, where)
