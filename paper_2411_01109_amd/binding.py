"""ctypes binding of libhgnn.so: the same entry points as include/hgnn.h, taking
torch CUDA tensors.  Argument marshalling only -- every step of the path runs in
the library's HIP kernels; torch supplies device memory and the stream.  There is
no CPU fallback: a missing library or a failing call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhgnn.so")

HGNN_OK, HGNN_EINVAL, HGNN_EUNSUPPORTED, HGNN_ENOMEM, HGNN_EHIP = range(5)
HGNN_SUM, HGNN_MEAN = 0, 1
HGNN_SDDMM_DOT, HGNN_SDDMM_GAT_SCORE = 0, 1

EXPORTS = (
    "hgnn_status_str", "hgnn_last_error", "hgnn_csr_validate", "hgnn_transpose", "hgnn_coo_to_csr", "hgnn_plan_create",
    "hgnn_plan_num_segments", "hgnn_plan_num_split_rows", "hgnn_plan_seg_edges", "hgnn_plan_col_blocks", "hgnn_plan_col_blocks_fine",
    "hgnn_plan_cache_bytes",
    "hgnn_plan_block_export", "hgnn_plan_export",
    "hgnn_plan_destroy", "hgnn_spmm", "hgnn_spmm_discretized", "hgnn_spmm_discretized_fused", "hgnn_sddmm", "hgnn_edge_softmax",
    "hgnn_edge_softmax_bwd", "hgnn_edge_rowsum", "hgnn_spmm_discretized_variant", "hgnn_plan_add_groups",
    "hgnn_plan_num_groups", "hgnn_plan_group_edges", "hgnn_plan_groups_export", "hgnn_plan_set_vector_halves",
    "hgnn_plan_vector_halves", "hgnn_spmm_workspace", "hgnn_plan_add_slices", "hgnn_plan_num_slices", "hgnn_edge_colsum", "hgnn_spmm_static", "hgnn_spmm_static_limit", "hgnn_gat_forward_fused", "hgnn_gat_alpha", "hgnn_gat_backward_fused",
    "hgnn_edge_to_transposed", "hgnn_scale_rows", "hgnn_linear", "hgnn_linear_wgrad", "hgnn_linear_wgrad_workspace",
    "hgnn_gat_feature_grad", "hgnn_gat_feature_grad_workspace", "hgnn_gat_forward_fused_save",
    "hgnn_gat_backward_fused_saved",
)

HGNN_EDGE_SEGMENTS, HGNN_EDGE_SEGMENTS_ATOMIC, HGNN_VERTEX_GROUPS, HGNN_VERTEX_GROUPS_HALF2 = 0, 1, 2, 3


class HgnnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(message)
        self.status = status


class _FusionStruct(ctypes.Structure):
    _fields_ = [("col_scale", ctypes.c_void_p), ("self", ctypes.c_void_p), ("ld_self", ctypes.c_int64),
                ("self_coef", ctypes.c_float), ("agg_coef", ctypes.c_float), ("scaled_x", ctypes.c_void_p),
                ("ld_scaled", ctypes.c_int64)]


class _CsrStruct(ctypes.Structure):
    _fields_ = [("nrows", ctypes.c_int32), ("ncols", ctypes.c_int32), ("nnz", ctypes.c_int64),
                ("rowptr", ctypes.c_void_p), ("col", ctypes.c_void_p), ("row", ctypes.c_void_p),
                ("eid", ctypes.c_void_p)]


_lib = None


def load() -> ctypes.CDLL:
    """Load libhgnn.so; raises when it has not been built (no fallback of any kind)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    csr = ctypes.POINTER(_CsrStruct)
    lib.hgnn_status_str.restype = ctypes.c_char_p
    lib.hgnn_status_str.argtypes = [ctypes.c_int]
    lib.hgnn_last_error.restype = ctypes.c_char_p
    lib.hgnn_last_error.argtypes = []
    lib.hgnn_csr_validate.argtypes = [csr, vp]
    lib.hgnn_transpose.argtypes = [csr, vp, vp, vp, vp]
    lib.hgnn_coo_to_csr.argtypes = [i32, i32, i64, vp, vp, vp, vp, vp, vp]
    lib.hgnn_plan_create.argtypes = [csr, i32, i32, i32, i32, ctypes.POINTER(vp), vp]
    lib.hgnn_plan_num_segments.restype = i64
    lib.hgnn_plan_num_segments.argtypes = [vp]
    lib.hgnn_plan_num_split_rows.restype = i32
    lib.hgnn_plan_num_split_rows.argtypes = [vp]
    lib.hgnn_plan_seg_edges.restype = i32
    lib.hgnn_plan_seg_edges.argtypes = [vp]
    lib.hgnn_plan_export.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.hgnn_plan_col_blocks.restype = i32
    lib.hgnn_plan_col_blocks.argtypes = [vp]
    lib.hgnn_plan_col_blocks_fine.restype = i32
    lib.hgnn_plan_col_blocks_fine.argtypes = [vp]
    lib.hgnn_plan_cache_bytes.restype = None
    lib.hgnn_plan_cache_bytes.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.hgnn_plan_block_export.argtypes = [vp, i32, ctypes.POINTER(i64), vp, vp, vp, vp, vp]
    lib.hgnn_plan_destroy.restype = None
    lib.hgnn_plan_destroy.argtypes = [vp]
    lib.hgnn_spmm_workspace.restype = ctypes.c_size_t
    lib.hgnn_spmm_workspace.argtypes = [i32, i32, i64, i32]
    lib.hgnn_spmm.argtypes = [csr, vp, i32, vp, i64, vp, i64, i32, ctypes.c_int, vp, vp, ctypes.c_size_t, vp]
    lib.hgnn_spmm_static_limit.restype = ctypes.c_size_t
    lib.hgnn_spmm_static_limit.argtypes = []
    lib.hgnn_spmm_static.argtypes = [csr, vp, i32, vp, i64, vp, i64, i32, ctypes.c_int, vp, vp]
    lib.hgnn_spmm_discretized.argtypes = [vp, csr, vp, i32, vp, i64, vp, i64, i32, ctypes.c_int, vp, vp]
    lib.hgnn_spmm_discretized_fused.argtypes = [vp, csr, vp, i32, vp, i64, vp, i64, i32, ctypes.c_int, vp,
                                                ctypes.POINTER(_FusionStruct), vp]
    lib.hgnn_sddmm.argtypes = [csr, vp, ctypes.c_int, i32, i32, vp, i64, vp, i64, vp, vp, f32, vp, vp]
    lib.hgnn_edge_softmax.argtypes = [csr, vp, i32, vp, vp, vp]
    lib.hgnn_edge_softmax_bwd.argtypes = [csr, vp, i32, vp, vp, vp, f32, vp, vp]
    lib.hgnn_edge_rowsum.argtypes = [csr, vp, i32, vp, vp, vp]
    lib.hgnn_edge_colsum.argtypes = [csr, vp, i32, vp, vp, vp]
    lib.hgnn_plan_add_slices.argtypes = [vp, csr, i32, vp]
    lib.hgnn_plan_num_slices.restype = i32
    lib.hgnn_plan_num_slices.argtypes = [vp]
    lib.hgnn_spmm_discretized_variant.argtypes = [vp, csr, vp, i32, vp, i64, vp, i64, i32, ctypes.c_int, vp, ctypes.c_int, vp]
    lib.hgnn_plan_add_groups.argtypes = [vp, csr, i32, vp]
    lib.hgnn_plan_num_groups.restype = i64
    lib.hgnn_plan_num_groups.argtypes = [vp]
    lib.hgnn_plan_group_edges.restype = i32
    lib.hgnn_plan_group_edges.argtypes = [vp]
    lib.hgnn_plan_groups_export.argtypes = [vp, csr, vp, vp]
    lib.hgnn_plan_set_vector_halves.argtypes = [vp, i32]
    lib.hgnn_gat_forward_fused.argtypes = [csr, vp, i32, i32, vp, i64, vp, i64, vp, vp, f32, vp, i64, vp, vp]
    lib.hgnn_edge_to_transposed.argtypes = [csr, i32, vp, vp, vp]
    lib.hgnn_scale_rows.argtypes = [i64, i32, vp, i64, vp, vp, i64, vp]
    lib.hgnn_gat_alpha.argtypes = [csr, vp, i32, i32, vp, i64, vp, i64, vp, vp, f32, vp, vp, vp]
    lib.hgnn_gat_backward_fused.argtypes = [csr, vp, csr, vp, i32, i32, vp, i64, vp, i64, vp, vp, f32, vp, i64, vp, vp, i64,
                                            vp, i64, vp, vp, vp]
    lib.hgnn_plan_vector_halves.restype = i32
    lib.hgnn_plan_vector_halves.argtypes = [vp]
    lib.hgnn_gat_forward_fused_save.argtypes = [csr, vp, i32, i32, vp, i64, vp, i64, vp, vp, f32, vp, i64, vp, vp, i64, vp, vp]
    lib.hgnn_gat_backward_fused_saved.argtypes = [csr, vp, csr, vp, i32, i32, vp, i64, vp, i64, vp, vp, f32, vp, i64, vp, vp, i64,
                                                  vp, vp, i64, vp, i64, vp, vp, vp]
    lib.hgnn_linear.argtypes = [i64, i32, i32, vp, i64, vp, i64, i32, vp, i64, vp]
    lib.hgnn_linear_wgrad_workspace.argtypes = [i32, i32]
    lib.hgnn_linear_wgrad_workspace.restype = ctypes.c_size_t
    lib.hgnn_linear_wgrad.argtypes = [i64, i32, i32, vp, i64, vp, i64, vp, i64, vp, ctypes.c_size_t, vp]
    lib.hgnn_gat_feature_grad_workspace.argtypes = [i32, i32]
    lib.hgnn_gat_feature_grad_workspace.restype = ctypes.c_size_t
    lib.hgnn_gat_feature_grad.argtypes = [i64, i32, i32, vp, i64, vp, vp, vp, vp, vp, i64, vp, i64, vp, vp, vp,
                                          ctypes.c_size_t, vp]
    for name in EXPORTS:
        getattr(lib, name)  # every declared entry point must be exported
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != HGNN_OK:
        lib = load()
        detail = lib.hgnn_last_error().decode()
        raise HgnnError(status, f"{lib.hgnn_status_str(status).decode()}: {detail}")


def _ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError("hgnn expects CUDA (HIP) tensors")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ld(t: torch.Tensor) -> int:
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("vertex-level tensors must be 2-D with unit stride along features")
    return t.stride(0)


class Csr:
    """Device CSR graph (hgnn_csr): int32 tensors, kept alive by this object."""

    def __init__(self, rowptr: torch.Tensor, col: torch.Tensor, ncols: Optional[int] = None,
                 row: Optional[torch.Tensor] = None, eid: Optional[torch.Tensor] = None):
        for t in (rowptr, col, row, eid):
            if t is not None and (t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous()):
                raise TypeError("graph arrays must be contiguous int32 CUDA tensors")
        self.rowptr, self.col, self.row, self.eid = rowptr, col, row, eid
        self.nrows = rowptr.numel() - 1
        self.ncols = self.nrows if ncols is None else ncols
        self.nnz = col.numel()
        self.struct = _CsrStruct(self.nrows, self.ncols, self.nnz, rowptr.data_ptr(), col.data_ptr(),
                                 None if row is None else row.data_ptr(), None if eid is None else eid.data_ptr())

    @property
    def ref(self):
        return ctypes.byref(self.struct)


class Plan:
    """Owner of an hgnn_plan handle."""

    def __init__(self, handle: int, graph: Csr):
        self.handle = handle
        self.graph = graph

    def __del__(self):
        h, self.handle = getattr(self, "handle", None), None
        if h and _lib is not None:
            _lib.hgnn_plan_destroy(h)


def hgnn_csr_validate(g: Csr, stream=None) -> None:
    _check(load().hgnn_csr_validate(g.ref, _stream(stream)))


def hgnn_transpose(g: Csr, stream=None) -> Csr:
    """CSR of A^T carrying eid into A's edge tensors."""
    dev = g.rowptr.device
    rowptr_T = torch.empty(g.ncols + 1, dtype=torch.int32, device=dev)
    col_T = torch.empty(g.nnz, dtype=torch.int32, device=dev)
    eid_T = torch.empty(g.nnz, dtype=torch.int32, device=dev)
    _check(load().hgnn_transpose(g.ref, rowptr_T.data_ptr(), col_T.data_ptr(), eid_T.data_ptr(), _stream(stream)))
    return Csr(rowptr_T, col_T, ncols=g.nrows, eid=eid_T)


def hgnn_coo_to_csr(row: torch.Tensor, col: torch.Tensor, nrows: int, ncols: int, want_eid: bool = True, stream=None):
    """-> (Csr without an edge-id map, eid or None): CSR of a COO edge list; eid[k] = list position of CSR non-zero k."""
    if row.numel() != col.numel():
        raise ValueError("row and col must have the same length")
    dev = row.device
    nnz = row.numel()
    rowptr = torch.empty(nrows + 1, dtype=torch.int32, device=dev)
    col_out = torch.empty(nnz, dtype=torch.int32, device=dev)
    eid = torch.empty(nnz, dtype=torch.int32, device=dev) if want_eid else None
    _check(load().hgnn_coo_to_csr(nrows, ncols, nnz, _ptr(row, torch.int32), _ptr(col, torch.int32), rowptr.data_ptr(),
                                  col_out.data_ptr(), None if eid is None else eid.data_ptr(), _stream(stream)))
    return Csr(rowptr, col_out, ncols=ncols), eid


def hgnn_plan_create(g: Csr, seg_edges: int = 256, max_F: int = 128, max_H: int = 8, col_blocks: int = 1,
                     stream=None) -> Plan:
    """col_blocks: 1 = no column blocking, 0 = automatic, n >= 2 = n column blocks."""
    out = ctypes.c_void_p()
    _check(load().hgnn_plan_create(g.ref, seg_edges, max_F, max_H, col_blocks, ctypes.byref(out), _stream(stream)))
    return Plan(out.value, g)


def hgnn_plan_col_blocks(p: Plan) -> int:
    return load().hgnn_plan_col_blocks(p.handle)


def hgnn_plan_col_blocks_fine(p: Plan) -> int:
    return load().hgnn_plan_col_blocks_fine(p.handle)


def hgnn_plan_cache_bytes(p: Plan):
    """-> (L2 bytes, last-level cache bytes) as the plan read them from the device."""
    l2, llc = ctypes.c_int64(0), ctypes.c_int64(0)
    load().hgnn_plan_cache_bytes(p.handle, ctypes.byref(l2), ctypes.byref(llc))
    return l2.value, llc.value


def hgnn_plan_block_export(p: Plan, b: int):
    """-> dict of host int32 numpy arrays of column block b (rowptr, col, eid, seg_row_lo, seg_row_hi)."""
    import numpy as np
    lib = load()
    n = ctypes.c_int64(0)
    _check(lib.hgnn_plan_block_export(p.handle, b, ctypes.byref(n), None, None, None, None, None))
    S = hgnn_plan_seg_edges(p)
    nseg = (n.value + S - 1) // S
    arrs = {"rowptr": np.empty(p.graph.nrows + 1, np.int32), "col": np.empty(n.value, np.int32),
            "eid": np.empty(n.value, np.int32), "seg_row_lo": np.empty(nseg, np.int32),
            "seg_row_hi": np.empty(nseg, np.int32)}
    _check(lib.hgnn_plan_block_export(p.handle, b, ctypes.byref(n), *[a.ctypes.data for a in arrs.values()]))
    return arrs


def hgnn_plan_num_segments(p: Plan) -> int:
    return load().hgnn_plan_num_segments(p.handle)


def hgnn_plan_num_split_rows(p: Plan) -> int:
    return load().hgnn_plan_num_split_rows(p.handle)


def hgnn_plan_seg_edges(p: Plan) -> int:
    return load().hgnn_plan_seg_edges(p.handle)


def hgnn_plan_export(p: Plan):
    """-> dict of host int32 numpy arrays (seg_row_lo, seg_row_hi, split_row, split_seg_lo, split_seg_hi)."""
    import numpy as np
    nseg, ns = hgnn_plan_num_segments(p), hgnn_plan_num_split_rows(p)
    arrs = {"seg_row_lo": np.empty(nseg, np.int32), "seg_row_hi": np.empty(nseg, np.int32),
            "split_row": np.empty(ns, np.int32), "split_seg_lo": np.empty(ns, np.int32),
            "split_seg_hi": np.empty(ns, np.int32)}
    _check(load().hgnn_plan_export(p.handle, *[a.ctypes.data for a in arrs.values()]))
    return arrs


def hgnn_plan_destroy(p: Plan) -> None:
    h, p.handle = p.handle, None
    if h:
        load().hgnn_plan_destroy(h)


def hgnn_spmm_workspace(nrows: int, ncols: int, nnz: int, F: int) -> int:
    """Bytes of device workspace hgnn_spmm wants for such a graph: the long rows' scratch (0: none can be that long)
    plus, where it walks the columns in passes, the partial rows; ncols = 0 gives the long rows' part alone."""
    return load().hgnn_spmm_workspace(nrows, ncols, nnz, F)


def hgnn_spmm(g: Csr, edge_val: Optional[torch.Tensor], H: int, X: torch.Tensor, Y: torch.Tensor,
              op: int = HGNN_SUM, row_scale: Optional[torch.Tensor] = None, F: Optional[int] = None,
              workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """workspace: device tensor of at least hgnn_spmm_workspace(...) bytes, or None (long rows then take one wave each)."""
    F = X.shape[1] if F is None else F
    _check(load().hgnn_spmm(g.ref, _ptr(edge_val, torch.float16), H, _ptr(X, torch.float16), _ld(X),
                            _ptr(Y, torch.float16), _ld(Y), F, op, _ptr(row_scale, torch.float32),
                            None if workspace is None else workspace.data_ptr(),
                            0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream)))


def hgnn_spmm_static_limit() -> int:
    return load().hgnn_spmm_static_limit()


def hgnn_spmm_static(g: Csr, edge_val: Optional[torch.Tensor], H: int, X: torch.Tensor, Y: torch.Tensor,
                     op: int = HGNN_SUM, row_scale: Optional[torch.Tensor] = None, F: Optional[int] = None, stream=None) -> None:
    """hgnn_spmm with the library's static scratch array instead of a workspace: allocates nothing."""
    F = X.shape[1] if F is None else F
    _check(load().hgnn_spmm_static(g.ref, _ptr(edge_val, torch.float16), H, _ptr(X, torch.float16), _ld(X),
                                   _ptr(Y, torch.float16), _ld(Y), F, op, _ptr(row_scale, torch.float32), _stream(stream)))


def hgnn_spmm_discretized(p: Plan, g: Csr, edge_val: Optional[torch.Tensor], H: int, X: torch.Tensor, Y: torch.Tensor,
                          op: int = HGNN_SUM, row_scale: Optional[torch.Tensor] = None, F: Optional[int] = None,
                          stream=None) -> None:
    F = X.shape[1] if F is None else F
    _check(load().hgnn_spmm_discretized(p.handle, g.ref, _ptr(edge_val, torch.float16), H, _ptr(X, torch.float16),
                                        _ld(X), _ptr(Y, torch.float16), _ld(Y), F, op,
                                        _ptr(row_scale, torch.float32), _stream(stream)))


def hgnn_spmm_discretized_fused(p: Plan, g: Csr, edge_val: Optional[torch.Tensor], H: int, X: torch.Tensor,
                                Y: torch.Tensor, op: int = HGNN_SUM, row_scale: Optional[torch.Tensor] = None,
                                col_scale: Optional[torch.Tensor] = None, self_feat: Optional[torch.Tensor] = None,
                                self_coef: float = 0.0, agg_coef: float = 1.0, F: Optional[int] = None,
                                scaled_x: Optional[torch.Tensor] = None, stream=None) -> None:
    F = X.shape[1] if F is None else F
    fz = _FusionStruct(_ptr(col_scale, torch.float32), _ptr(self_feat, torch.float16),
                       0 if self_feat is None else _ld(self_feat), self_coef, agg_coef, _ptr(scaled_x, torch.float16),
                       0 if scaled_x is None else _ld(scaled_x))
    _check(load().hgnn_spmm_discretized_fused(p.handle, g.ref, _ptr(edge_val, torch.float16), H, _ptr(X, torch.float16),
                                              _ld(X), _ptr(Y, torch.float16), _ld(Y), F, op,
                                              _ptr(row_scale, torch.float32), ctypes.byref(fz), _stream(stream)))


def hgnn_spmm_discretized_variant(p: Plan, g: Csr, edge_val: Optional[torch.Tensor], H: int, X: torch.Tensor,
                                  Y: torch.Tensor, variant: int, op: int = HGNN_SUM,
                                  row_scale: Optional[torch.Tensor] = None, F: Optional[int] = None, stream=None) -> None:
    F = X.shape[1] if F is None else F
    _check(load().hgnn_spmm_discretized_variant(p.handle, g.ref, _ptr(edge_val, torch.float16), H,
                                                _ptr(X, torch.float16), _ld(X), _ptr(Y, torch.float16), _ld(Y), F, op,
                                                _ptr(row_scale, torch.float32), variant, _stream(stream)))


def hgnn_plan_add_groups(p: Plan, g: Csr, group_edges: int, stream=None) -> None:
    _check(load().hgnn_plan_add_groups(p.handle, g.ref, group_edges, _stream(stream)))


def hgnn_plan_num_groups(p: Plan) -> int:
    return load().hgnn_plan_num_groups(p.handle)


def hgnn_plan_group_edges(p: Plan) -> int:
    return load().hgnn_plan_group_edges(p.handle)


def hgnn_plan_groups_export(p: Plan, g: Csr):
    """-> (group_row, group_first) host int32 numpy arrays."""
    import numpy as np
    n = hgnn_plan_num_groups(p)
    row, first = np.empty(max(n, 1), np.int32), np.empty(max(n, 1), np.int32)
    _check(load().hgnn_plan_groups_export(p.handle, g.ref, row.ctypes.data, first.ctypes.data))
    return row[:n], first[:n]


def hgnn_gat_forward_fused(g: Csr, p: Plan, H: int, D: int, U: torch.Tensor, Vt: torch.Tensor, a_l: torch.Tensor,
                           a_r: torch.Tensor, out: torch.Tensor, lse: Optional[torch.Tensor] = None,
                           neg_slope: float = 0.2, stream=None) -> None:
    _check(load().hgnn_gat_forward_fused(g.ref, p.handle, H, D, _ptr(U, torch.float16), _ld(U), _ptr(Vt, torch.float16),
                                         _ld(Vt), _ptr(a_l, torch.float16), _ptr(a_r, torch.float16), neg_slope,
                                         _ptr(out, torch.float16), _ld(out), _ptr(lse, torch.float32), _stream(stream)))


def hgnn_gat_backward_fused(g: Csr, p: Plan, gt: Csr, pt: Plan, H: int, D: int, U: torch.Tensor, Vt: torch.Tensor,
                            a_l: torch.Tensor, a_r: torch.Tensor, out: torch.Tensor, lse: torch.Tensor,
                            dOut: torch.Tensor, dV: torch.Tensor, d_el: torch.Tensor, d_er: torch.Tensor,
                            neg_slope: float = 0.2, stream=None) -> None:
    _check(load().hgnn_gat_backward_fused(g.ref, p.handle, gt.ref, pt.handle, H, D, _ptr(U, torch.float16), _ld(U),
                                          _ptr(Vt, torch.float16), _ld(Vt), _ptr(a_l, torch.float16),
                                          _ptr(a_r, torch.float16), neg_slope, _ptr(out, torch.float16), _ld(out),
                                          _ptr(lse, torch.float32), _ptr(dOut, torch.float16), _ld(dOut),
                                          _ptr(dV, torch.float16), _ld(dV), _ptr(d_el, torch.float16),
                                          _ptr(d_er, torch.float16), _stream(stream)))


def hgnn_gat_forward_fused_save(g: Csr, p: Plan, H: int, D: int, U: torch.Tensor, Vt: torch.Tensor, a_l: torch.Tensor,
                                a_r: torch.Tensor, out: torch.Tensor, lse: torch.Tensor, out_masked: torch.Tensor,
                                csum: torch.Tensor, neg_slope: float = 0.2, stream=None) -> None:
    _check(load().hgnn_gat_forward_fused_save(g.ref, p.handle, H, D, _ptr(U, torch.float16), _ld(U), _ptr(Vt, torch.float16),
                                              _ld(Vt), _ptr(a_l, torch.float16), _ptr(a_r, torch.float16), neg_slope,
                                              _ptr(out, torch.float16), _ld(out), _ptr(lse, torch.float32),
                                              _ptr(out_masked, torch.float16), _ld(out_masked), _ptr(csum, torch.float32),
                                              _stream(stream)))


def hgnn_gat_backward_fused_saved(g: Csr, p: Plan, gt: Csr, pt: Plan, H: int, D: int, U: torch.Tensor, Vt: torch.Tensor,
                                  a_l: torch.Tensor, a_r: torch.Tensor, out: torch.Tensor, lse: torch.Tensor,
                                  out_masked: torch.Tensor, csum: torch.Tensor, dOut: torch.Tensor, dV: torch.Tensor,
                                  d_el: torch.Tensor, d_er: torch.Tensor, neg_slope: float = 0.2, stream=None) -> None:
    _check(load().hgnn_gat_backward_fused_saved(g.ref, p.handle, gt.ref, pt.handle, H, D, _ptr(U, torch.float16), _ld(U),
                                                _ptr(Vt, torch.float16), _ld(Vt), _ptr(a_l, torch.float16),
                                                _ptr(a_r, torch.float16), neg_slope, _ptr(out, torch.float16), _ld(out),
                                                _ptr(lse, torch.float32), _ptr(out_masked, torch.float16), _ld(out_masked),
                                                _ptr(csum, torch.float32), _ptr(dOut, torch.float16), _ld(dOut),
                                                _ptr(dV, torch.float16), _ld(dV), _ptr(d_el, torch.float16),
                                                _ptr(d_er, torch.float16), _stream(stream)))


def hgnn_scale_rows(X: torch.Tensor, scale: torch.Tensor, out: torch.Tensor, F: Optional[int] = None, stream=None) -> None:
    F = X.shape[1] if F is None else F
    _check(load().hgnn_scale_rows(X.shape[0], F, _ptr(X, torch.float16), _ld(X), _ptr(scale, torch.float32),
                                  _ptr(out, torch.float16), _ld(out), _stream(stream)))


def hgnn_linear(X: torch.Tensor, W: torch.Tensor, Y: torch.Tensor, trans_w: bool = False, K: Optional[int] = None,
                F: Optional[int] = None, stream=None) -> None:
    """Y = X.W (W is [K][F]) or X.W^T (trans_w, W is [F][K])."""
    K = X.shape[1] if K is None else K
    F = (W.shape[0] if trans_w else W.shape[1]) if F is None else F
    _check(load().hgnn_linear(X.shape[0], K, F, _ptr(X, torch.float16), _ld(X), _ptr(W, torch.float16), _ld(W),
                              1 if trans_w else 0, _ptr(Y, torch.float16), _ld(Y), _stream(stream)))


def hgnn_linear_wgrad_workspace(K: int, F: int) -> int:
    return load().hgnn_linear_wgrad_workspace(K, F)


def hgnn_linear_wgrad(X: torch.Tensor, dY: torch.Tensor, dW: torch.Tensor, workspace: torch.Tensor, K: Optional[int] = None,
                      F: Optional[int] = None, stream=None) -> None:
    """dW (fp32 [K][F]) = X^T.dY; workspace is a device byte/float tensor of hgnn_linear_wgrad_workspace(K, F) bytes."""
    K = X.shape[1] if K is None else K
    F = dY.shape[1] if F is None else F
    _check(load().hgnn_linear_wgrad(X.shape[0], K, F, _ptr(X, torch.float16), _ld(X), _ptr(dY, torch.float16), _ld(dY),
                                    _ptr(dW, torch.float32), _ld(dW), workspace.data_ptr(),
                                    workspace.numel() * workspace.element_size(), _stream(stream)))


def hgnn_gat_feature_grad_workspace(H: int, D: int) -> int:
    return load().hgnn_gat_feature_grad_workspace(H, D)


def hgnn_gat_feature_grad(H: int, D: int, dV: torch.Tensor, d_el: torch.Tensor, d_er: torch.Tensor, a_l: torch.Tensor,
                          a_r: torch.Tensor, hfeat: torch.Tensor, dh: torch.Tensor, da_l: torch.Tensor, da_r: torch.Tensor,
                          workspace: torch.Tensor, stream=None) -> None:
    _check(load().hgnn_gat_feature_grad(dV.shape[0], H, D, _ptr(dV, torch.float16), _ld(dV), _ptr(d_el, torch.float16),
                                        _ptr(d_er, torch.float16), _ptr(a_l, torch.float16), _ptr(a_r, torch.float16),
                                        _ptr(hfeat, torch.float16), _ld(hfeat), _ptr(dh, torch.float16), _ld(dh),
                                        _ptr(da_l, torch.float32), _ptr(da_r, torch.float32), workspace.data_ptr(),
                                        workspace.numel() * workspace.element_size(), _stream(stream)))


def hgnn_edge_to_transposed(gt: Csr, H: int, t: torch.Tensor, t_T: torch.Tensor, stream=None) -> None:
    _check(load().hgnn_edge_to_transposed(gt.ref, H, _ptr(t, torch.float16), _ptr(t_T, torch.float16), _stream(stream)))


def hgnn_gat_alpha(g: Csr, p: Plan, H: int, D: int, U: torch.Tensor, Vt: torch.Tensor, a_l: torch.Tensor,
                   a_r: torch.Tensor, lse: torch.Tensor, alpha: torch.Tensor, neg_slope: float = 0.2, stream=None) -> None:
    _check(load().hgnn_gat_alpha(g.ref, p.handle, H, D, _ptr(U, torch.float16), _ld(U), _ptr(Vt, torch.float16), _ld(Vt),
                                 _ptr(a_l, torch.float16), _ptr(a_r, torch.float16), neg_slope, _ptr(lse, torch.float32),
                                 _ptr(alpha, torch.float16), _stream(stream)))


def hgnn_plan_set_vector_halves(p: Plan, halves: int) -> None:
    _check(load().hgnn_plan_set_vector_halves(p.handle, halves))


def hgnn_plan_vector_halves(p: Plan) -> int:
    return load().hgnn_plan_vector_halves(p.handle)


def hgnn_sddmm(g: Csr, p: Optional[Plan], op: int, H: int, D: int, U: torch.Tensor, Vt: torch.Tensor,
               out: torch.Tensor, a_l: Optional[torch.Tensor] = None, a_r: Optional[torch.Tensor] = None,
               neg_slope: float = 0.2, stream=None) -> None:
    _check(load().hgnn_sddmm(g.ref, None if p is None else p.handle, op, H, D, _ptr(U, torch.float16), _ld(U),
                             _ptr(Vt, torch.float16), _ld(Vt), _ptr(a_l, torch.float16), _ptr(a_r, torch.float16),
                             neg_slope, _ptr(out, torch.float16), _stream(stream)))


def hgnn_edge_softmax(g: Csr, p: Optional[Plan], H: int, e: torch.Tensor, alpha: torch.Tensor, stream=None) -> None:
    _check(load().hgnn_edge_softmax(g.ref, None if p is None else p.handle, H, _ptr(e, torch.float16),
                                    _ptr(alpha, torch.float16), _stream(stream)))


def hgnn_edge_softmax_bwd(g: Csr, p: Optional[Plan], H: int, alpha: torch.Tensor, dalpha: torch.Tensor,
                          de: torch.Tensor, e: Optional[torch.Tensor] = None, neg_slope: float = 0.2, stream=None) -> None:
    _check(load().hgnn_edge_softmax_bwd(g.ref, None if p is None else p.handle, H, _ptr(alpha, torch.float16),
                                        _ptr(dalpha, torch.float16), _ptr(e, torch.float16), neg_slope,
                                        _ptr(de, torch.float16), _stream(stream)))


def hgnn_edge_rowsum(g: Csr, p: Optional[Plan], H: int, t: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    _check(load().hgnn_edge_rowsum(g.ref, None if p is None else p.handle, H, _ptr(t, torch.float16),
                                   _ptr(out, torch.float16), _stream(stream)))


def hgnn_edge_colsum(g: Csr, p: Plan, H: int, t: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    """out[j] = sum of t over the non-zeros of column j (needs column slices in the plan)."""
    _check(load().hgnn_edge_colsum(g.ref, p.handle, H, _ptr(t, torch.float16), _ptr(out, torch.float16), _stream(stream)))


def hgnn_plan_add_slices(p: Plan, g: Csr, slice_cols: int = 0, stream=None) -> None:
    _check(load().hgnn_plan_add_slices(p.handle, g.ref, slice_cols, _stream(stream)))


def hgnn_plan_num_slices(p: Plan) -> int:
    return load().hgnn_plan_num_slices(p.handle)
