"""ctypes front end of the CPU oracle (oracle.c): plain single-threaded fp64
definitions of SpMM, transposed SpMM, SDDMM, GAT score, edge softmax (Eq. 1 of
the paper) and its backward, plus the integer segment plan.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg; never by the product path, and it imports nothing
from the GPU package.  fp16 arrays are numpy float16; results are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_SRC = os.path.join(_HERE, "oracle.c")
_lib = None

SUM, MEAN = 0, 1


def build(force: bool = True) -> str:
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-shared", "-fPIC", "-o", _LIB_PATH, _SRC, "-lm"])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        build(force=True)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
    lib.orc_half_to_double.restype = dbl
    lib.orc_half_to_double.argtypes = [ctypes.c_uint16]
    lib.orc_double_to_half.restype = ctypes.c_uint16
    lib.orc_double_to_half.argtypes = [dbl]
    lib.orc_decode.restype = None
    lib.orc_decode.argtypes = [vp, vp, i64]
    lib.orc_spmm.restype = None
    lib.orc_spmm.argtypes = [i32, vp, vp, vp, vp, i32, vp, i64, i32, i32, vp, vp, vp, i64, dbl, dbl, vp, i32, vp, vp]
    lib.orc_spmm_T_scatter.restype = None
    lib.orc_spmm_T_scatter.argtypes = [i32, i32, vp, vp, vp, i32, vp, i64, i32, vp]
    lib.orc_transpose.restype = None
    lib.orc_transpose.argtypes = [i32, i32, vp, vp, vp, vp, vp]
    lib.orc_coo_to_csr.restype = None
    lib.orc_coo_to_csr.argtypes = [i64, i32, vp, vp, vp, vp, vp]
    lib.orc_sddmm_dot.restype = None
    lib.orc_sddmm_dot.argtypes = [i32, vp, vp, vp, i32, i32, vp, i64, vp, i64, vp]
    lib.orc_gat_score.restype = None
    lib.orc_gat_score.argtypes = [i32, vp, vp, i32, i32, vp, i64, vp, vp, dbl, vp]
    lib.orc_gat_forward.restype = None
    lib.orc_gat_forward.argtypes = [i32, vp, vp, i32, i32, vp, i64, vp, i64, vp, vp, dbl, vp, vp, vp, vp, vp]
    lib.orc_gat_backward.restype = None
    lib.orc_gat_backward.argtypes = [i32, i32, vp, vp, i32, i32, vp, i64, vp, i64, vp, vp, dbl, vp, i64, vp, vp, vp]
    lib.orc_edge_softmax.restype = None
    lib.orc_edge_softmax.argtypes = [i32, vp, i32, vp, vp]
    lib.orc_edge_softmax_bwd.restype = None
    lib.orc_edge_softmax_bwd.argtypes = [i32, vp, i32, vp, vp, vp, dbl, vp]
    lib.orc_edge_rowsum.restype = None
    lib.orc_edge_rowsum.argtypes = [i32, vp, i32, vp, vp]
    lib.orc_edge_colsum.restype = None
    lib.orc_edge_colsum.argtypes = [i32, i32, vp, vp, i32, vp, vp]
    lib.orc_edge_gather.restype = None
    lib.orc_edge_gather.argtypes = [i64, vp, i32, vp, vp]
    lib.orc_linear.restype = None
    lib.orc_linear.argtypes = [i64, i32, i32, vp, i64, vp, i64, i32, vp, vp]
    lib.orc_linear_wgrad.restype = None
    lib.orc_linear_wgrad.argtypes = [i64, i32, i32, vp, i64, vp, i64, vp, vp]
    lib.orc_gat_feature_grad.restype = None
    lib.orc_gat_feature_grad.argtypes = [i32, i32, i32, vp, i64, vp, vp, vp, vp, vp, i64, vp, vp, vp, vp, vp]
    lib.orc_segment_plan.restype = i32
    lib.orc_segment_plan.argtypes = [i32, vp, i32, vp, vp, vp, vp, vp]
    lib.orc_spmm_naive_fp16.restype = None
    lib.orc_spmm_naive_fp16.argtypes = [i32, vp, vp, vp, i64, i32, i32, i32, vp, i32, vp]
    lib.orc_spmm_discretized.restype = None
    lib.orc_spmm_discretized.argtypes = [i32, vp, vp, vp, vp, i32, vp, i64, i32, i32, vp, i32, i32, vp, i32, vp, vp]
    lib.orc_neighbor_groups.restype = i64
    lib.orc_neighbor_groups.argtypes = [i32, vp, i32, vp, vp]
    _lib = lib
    return lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _f16(a):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16, a.dtype
    return a


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def half_to_double(bits: int) -> float:
    return _load().orc_half_to_double(bits)


def double_to_half(v: float) -> int:
    return _load().orc_double_to_half(v)


def decode(x: np.ndarray) -> np.ndarray:
    x = _f16(x)
    out = np.empty(x.shape, dtype=np.float64)
    _load().orc_decode(_ptr(x), _ptr(out), x.size)
    return out


def spmm(rowptr, col, X, w=None, H: int = 1, reduce: int = SUM, row_scale=None, eid=None, rows=None,
         want_sabs: bool = False, col_scale=None, self_feat=None, self_coef: float = 0.0, agg_coef: float = 1.0):
    """Y = self_coef*self + agg_coef * s . (A_w diag(col_scale) X); rows=None gives all rows, else the listed ones."""
    rowptr, col, eid, rows = _i32(rowptr), _i32(col), _i32(eid), _i32(rows)
    X, w, row_scale, col_scale, self_feat = _f16(X), _f16(w), _f64(row_scale), _f64(col_scale), _f16(self_feat)
    V, F = rowptr.size - 1, X.shape[1]
    n = V if rows is None else rows.size
    out = np.empty((n, F), dtype=np.float64)
    sabs = np.empty((n, F), dtype=np.float64) if want_sabs else None
    _load().orc_spmm(V, _ptr(rowptr), _ptr(col), _ptr(eid), _ptr(w), H, _ptr(X), X.strides[0] // 2, F, reduce,
                     _ptr(row_scale), _ptr(col_scale), _ptr(self_feat),
                     0 if self_feat is None else self_feat.strides[0] // 2, self_coef, agg_coef,
                     _ptr(rows), 0 if rows is None else rows.size, _ptr(out), _ptr(sabs))
    return (out, sabs) if want_sabs else out


def spmm_T_scatter(rowptr, col, dY, ncols: int, w=None, H: int = 1):
    rowptr, col, dY, w = _i32(rowptr), _i32(col), _f16(dY), _f16(w)
    V, F = rowptr.size - 1, dY.shape[1]
    out = np.empty((ncols, F), dtype=np.float64)
    _load().orc_spmm_T_scatter(V, ncols, _ptr(rowptr), _ptr(col), _ptr(w), H, _ptr(dY), dY.strides[0] // 2, F, _ptr(out))
    return out


def transpose(rowptr, col, ncols: int):
    rowptr, col = _i32(rowptr), _i32(col)
    V, E = rowptr.size - 1, col.size
    rowptr_T = np.empty(ncols + 1, dtype=np.int32)
    col_T = np.empty(E, dtype=np.int32)
    eid_T = np.empty(E, dtype=np.int32)
    _load().orc_transpose(V, ncols, _ptr(rowptr), _ptr(col), _ptr(rowptr_T), _ptr(col_T), _ptr(eid_T))
    return rowptr_T, col_T, eid_T


def coo_to_csr(row, col, nrows: int):
    """-> (rowptr [nrows+1], col [E], eid [E]): CSR of a COO edge list, columns ascending inside a row, duplicate
    edges in list order; eid = list index of every CSR non-zero."""
    row, col = _i32(row), _i32(col)
    E = row.size
    rowptr = np.empty(nrows + 1, dtype=np.int32)
    col_out = np.empty(E, dtype=np.int32)
    eid = np.empty(E, dtype=np.int32)
    _load().orc_coo_to_csr(E, nrows, _ptr(row), _ptr(col), _ptr(rowptr), _ptr(col_out), _ptr(eid))
    return rowptr, col_out, eid


def sddmm_dot(rowptr, col, U, Vt, H: int = 1, eid=None):
    rowptr, col, eid, U, Vt = _i32(rowptr), _i32(col), _i32(eid), _f16(U), _f16(Vt)
    V, F = rowptr.size - 1, U.shape[1]
    out = np.empty((col.size, H), dtype=np.float64)
    _load().orc_sddmm_dot(V, _ptr(rowptr), _ptr(col), _ptr(eid), H, F // H, _ptr(U), U.strides[0] // 2, _ptr(Vt),
                          Vt.strides[0] // 2, _ptr(out))
    return out


def gat_score(rowptr, col, feat, a_l, a_r, H: int, slope: float = 0.2):
    rowptr, col, feat, a_l, a_r = _i32(rowptr), _i32(col), _f16(feat), _f16(a_l), _f16(a_r)
    V, F = rowptr.size - 1, feat.shape[1]
    out = np.empty((col.size, H), dtype=np.float64)
    _load().orc_gat_score(V, _ptr(rowptr), _ptr(col), H, F // H, _ptr(feat), feat.strides[0] // 2, _ptr(a_l), _ptr(a_r),
                          slope, _ptr(out))
    return out


def gat_forward(rowptr, col, U, Vt, a_l, a_r, H: int, slope: float = 0.2, want_saved: bool = False):
    """-> (out [V][F], lse [V][H], sabs [V][F]) of one GAT aggregation, nothing rounded in between; with want_saved
    also (out_masked [V][F], csum [V][H]), the sums weighted by the LeakyReLU derivative that a backward pass can use."""
    rowptr, col, U, Vt, a_l, a_r = _i32(rowptr), _i32(col), _f16(U), _f16(Vt), _f16(a_l), _f16(a_r)
    V, F = rowptr.size - 1, U.shape[1]
    out = np.empty((V, F), dtype=np.float64)
    sabs = np.empty((V, F), dtype=np.float64)
    lse = np.empty((V, H), dtype=np.float64)
    outm = np.empty((V, F), dtype=np.float64) if want_saved else None
    csum = np.empty((V, H), dtype=np.float64) if want_saved else None
    _load().orc_gat_forward(V, _ptr(rowptr), _ptr(col), H, F // H, _ptr(U), U.strides[0] // 2, _ptr(Vt),
                            Vt.strides[0] // 2, _ptr(a_l), _ptr(a_r), slope, _ptr(out), _ptr(lse), _ptr(sabs), _ptr(outm),
                            _ptr(csum))
    return (out, lse, sabs, outm, csum) if want_saved else (out, lse, sabs)


def gat_backward(rowptr, col, U, Vt, a_l, a_r, dOut, H: int, slope: float = 0.2):
    """-> (dV [ncols][F], d_el [V][H], d_er [ncols][H]) of L = sum <dOut, out> for one GAT aggregation."""
    rowptr, col, U, Vt, a_l, a_r, dOut = _i32(rowptr), _i32(col), _f16(U), _f16(Vt), _f16(a_l), _f16(a_r), _f16(dOut)
    V, F, ncols = rowptr.size - 1, U.shape[1], Vt.shape[0]
    dV = np.empty((ncols, F), dtype=np.float64)
    d_el = np.empty((V, H), dtype=np.float64)
    d_er = np.empty((ncols, H), dtype=np.float64)
    _load().orc_gat_backward(V, ncols, _ptr(rowptr), _ptr(col), H, F // H, _ptr(U), U.strides[0] // 2, _ptr(Vt),
                             Vt.strides[0] // 2, _ptr(a_l), _ptr(a_r), slope, _ptr(dOut), dOut.strides[0] // 2, _ptr(dV),
                             _ptr(d_el), _ptr(d_er))
    return dV, d_el, d_er


def edge_softmax(rowptr, e):
    rowptr, e = _i32(rowptr), _f64(e)
    alpha = np.zeros_like(e)
    _load().orc_edge_softmax(rowptr.size - 1, _ptr(rowptr), e.shape[1], _ptr(e), _ptr(alpha))
    return alpha


def edge_softmax_bwd(rowptr, alpha, dalpha, e=None, slope: float = 0.2):
    rowptr, alpha, dalpha, e = _i32(rowptr), _f64(alpha), _f64(dalpha), _f64(e)
    de = np.zeros_like(alpha)
    _load().orc_edge_softmax_bwd(rowptr.size - 1, _ptr(rowptr), alpha.shape[1], _ptr(alpha), _ptr(dalpha), _ptr(e), slope,
                                 _ptr(de))
    return de


def edge_rowsum(rowptr, t):
    rowptr, t = _i32(rowptr), _f64(t)
    out = np.empty((rowptr.size - 1, t.shape[1]), dtype=np.float64)
    _load().orc_edge_rowsum(rowptr.size - 1, _ptr(rowptr), t.shape[1], _ptr(t), _ptr(out))
    return out


def edge_colsum(rowptr, col, t, ncols: int):
    rowptr, col, t = _i32(rowptr), _i32(col), _f64(t)
    out = np.empty((ncols, t.shape[1]), dtype=np.float64)
    _load().orc_edge_colsum(rowptr.size - 1, ncols, _ptr(rowptr), _ptr(col), t.shape[1], _ptr(t), _ptr(out))
    return out


def edge_gather(eid, t):
    """t (fp16 [nnz][H]) in the edge order of the transposed graph."""
    eid, t = _i32(eid), _f16(t)
    out = np.empty_like(t)
    _load().orc_edge_gather(eid.size, _ptr(eid), t.shape[1], _ptr(t), _ptr(out))
    return out


def linear(X, W, trans: bool = False, want_sabs: bool = False):
    """Y = X.W (W is [K][F]) or X.W^T (trans, W is [F][K]); fp16 in, fp64 out."""
    X, W = _f16(X), _f16(W)
    n, K = X.shape
    F = W.shape[0] if trans else W.shape[1]
    assert (W.shape[1] if trans else W.shape[0]) == K
    out = np.empty((n, F), dtype=np.float64)
    sabs = np.empty((n, F), dtype=np.float64)
    _load().orc_linear(n, K, F, _ptr(X), X.shape[1], _ptr(W), W.shape[1], 1 if trans else 0, _ptr(out), _ptr(sabs))
    return (out, sabs) if want_sabs else out


def linear_wgrad(X, dY, want_sabs: bool = False):
    """dW = X^T.dY ([K][F]); fp16 in, fp64 out."""
    X, dY = _f16(X), _f16(dY)
    n, K = X.shape
    F = dY.shape[1]
    assert dY.shape[0] == n
    out = np.empty((K, F), dtype=np.float64)
    sabs = np.empty((K, F), dtype=np.float64)
    _load().orc_linear_wgrad(n, K, F, _ptr(X), K, _ptr(dY), F, _ptr(out), _ptr(sabs))
    return (out, sabs) if want_sabs else out


def gat_feature_grad(dV, d_el, d_er, a_l, a_r, hfeat, H: int):
    """-> dh [V][F], da_l [F], da_r [F], and the term magnitudes of da_l, da_r (all fp64) from fp16 inputs."""
    dV, d_el, d_er, hfeat = _f16(dV), _f16(d_el), _f16(d_er), _f16(hfeat)
    a_l, a_r = _f16(np.asarray(a_l).reshape(-1)), _f16(np.asarray(a_r).reshape(-1))
    V, F = dV.shape
    D = F // H
    dh = np.empty((V, F), dtype=np.float64)
    da_l, da_r, sl, sr = (np.empty(F, dtype=np.float64) for _ in range(4))
    _load().orc_gat_feature_grad(V, H, D, _ptr(dV), F, _ptr(d_el), _ptr(d_er), _ptr(a_l), _ptr(a_r), _ptr(hfeat), F,
                                 _ptr(dh), _ptr(da_l), _ptr(da_r), _ptr(sl), _ptr(sr))
    return dh, da_l, da_r, sl, sr


def segment_plan(rowptr, S: int):
    """-> dict(seg_row_lo, seg_row_hi, split_row, split_seg_lo, split_seg_hi)."""
    rowptr = _i32(rowptr)
    V, E = rowptr.size - 1, int(rowptr[-1])
    nseg = (E + S - 1) // S
    lo = np.empty(nseg, dtype=np.int32)
    hi = np.empty(nseg, dtype=np.int32)
    cap = max(min(nseg, V), 1)
    sr = np.empty(cap, dtype=np.int32)
    sa = np.empty(cap, dtype=np.int32)
    sb = np.empty(cap, dtype=np.int32)
    n = _load().orc_segment_plan(V, _ptr(rowptr), S, _ptr(lo), _ptr(hi), _ptr(sr), _ptr(sa), _ptr(sb))
    return {"seg_row_lo": lo, "seg_row_hi": hi, "split_row": sr[:n].copy(), "split_seg_lo": sa[:n].copy(),
            "split_seg_hi": sb[:n].copy()}


def neighbor_groups(rowptr, ng: int):
    """-> (grp_row, grp_first): the neighbour groups of at most ng non-zeros, in row order."""
    rowptr = _i32(rowptr)
    V = rowptr.size - 1
    lib = _load()
    n = lib.orc_neighbor_groups(V, _ptr(rowptr), ng, None, None)
    row = np.empty(max(n, 1), dtype=np.int32)
    first = np.empty(max(n, 1), dtype=np.int32)
    lib.orc_neighbor_groups(V, _ptr(rowptr), ng, _ptr(row), _ptr(first))
    return row[:n].copy(), first[:n].copy()


def spmm_naive_fp16(rowptr, col, X, reduce: int = SUM, rows=None, wide_sum: bool = False):
    rowptr, col, rows, X = _i32(rowptr), _i32(col), _i32(rows), _f16(X)
    V, F = rowptr.size - 1, X.shape[1]
    n = V if rows is None else rows.size
    out = np.empty((n, F), dtype=np.uint16)
    _load().orc_spmm_naive_fp16(V, _ptr(rowptr), _ptr(col), _ptr(X), X.strides[0] // 2, F, reduce, 1 if wide_sum else 0,
                                _ptr(rows), 0 if rows is None else rows.size, _ptr(out))
    return out.view(np.float16)


def spmm_discretized(rowptr, col, X, S: int, w=None, H: int = 1, reduce: int = SUM, row_scale=None, eid=None, rows=None,
                     by_row: bool = False):
    """(sum of fp16-rounded scaled partials per row, max |partial| before rounding).  by_row: the batches are
    the row's own neighbour groups of S (vertex-parallel form) instead of the storage-order segments."""
    rowptr, col, eid, rows = _i32(rowptr), _i32(col), _i32(eid), _i32(rows)
    X, w, row_scale = _f16(X), _f16(w), _f64(row_scale)
    V, F = rowptr.size - 1, X.shape[1]
    n = V if rows is None else rows.size
    out = np.empty((n, F), dtype=np.float64)
    mp = ctypes.c_double(0.0)
    _load().orc_spmm_discretized(V, _ptr(rowptr), _ptr(col), _ptr(eid), _ptr(w), H, _ptr(X), X.strides[0] // 2, F, reduce,
                                 _ptr(row_scale), S, 1 if by_row else 0, _ptr(rows), 0 if rows is None else rows.size,
                                 _ptr(out), ctypes.byref(mp))
    return out, mp.value
