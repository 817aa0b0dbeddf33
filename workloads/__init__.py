"""Seeded synthetic inputs shaped like the paper's workloads (Table 1 graphs,
hidden width 64, kernel widths 32/64) for the fp16 SpMM / SDDMM / edge-softmax
path.  Input manufacture only: nothing here computes what the kernels or the
oracle compute, so both sides may consume these arrays.

Conventions: CSR with int32 ``rowptr`` (offset array) and ``col`` (paper
section 2.1.1); row i = destination vertex, column j = neighbour; duplicates are
kept; fp16 tensors are numpy ``float16`` arrays, vertex-level ``[V, F]`` row
major and edge-level ``[E, H]`` edge major.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libworkloads.so")
_SRC = os.path.join(_HERE, "gen.c")
_lib = None

BASE_SEED = 0x48474E4E


def build(force: bool = True) -> str:
    """Compile gen.c into libworkloads.so (host code, gcc)."""
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, _SRC, "-lm"]
        )
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        build(force=True)
    lib = ctypes.CDLL(_LIB_PATH)
    i32p = ctypes.POINTER(ctypes.c_int32)
    u16p = ctypes.POINTER(ctypes.c_uint16)
    f64p = ctypes.POINTER(ctypes.c_double)
    i64, i32, u64, dbl = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_double
    lib.wl_rnd_u64.restype = u64
    lib.wl_rnd_u64.argtypes = [u64, u64]
    lib.wl_fill_normal_f16.argtypes = [u16p, i64, u64, dbl, dbl]
    lib.wl_fill_uniform_f16.argtypes = [u16p, i64, u64, dbl, dbl]
    lib.wl_double_to_f16.argtypes = [f64p, u16p, i64]
    lib.wl_edges_uniform.argtypes = [i32p, i32p, i64, i32, u64]
    lib.wl_edges_rmat.argtypes = [i32p, i32p, i64, i32, dbl, dbl, dbl, i32, u64]
    lib.wl_permutation.argtypes = [i32p, i32, u64]
    lib.wl_relabel.argtypes = [i32p, i64, i32p]
    lib.wl_coo_to_csr.restype = ctypes.c_int
    lib.wl_coo_to_csr.argtypes = [i32p, i32p, i64, i32, i32, i32p, i32p]
    lib.wl_lognormal_degrees.restype = ctypes.c_int
    lib.wl_lognormal_degrees.argtypes = [i32p, i32, i64, dbl, dbl, i32, u64]
    lib.wl_fill_cols_uniform_sorted.argtypes = [i32p, i32p, i32, i32, u64]
    lib.wl_symnorm_f16.restype = ctypes.c_int
    lib.wl_symnorm_f16.argtypes = [i32p, i32p, i32, i32, u16p]
    for name in ("wl_fill_normal_f16", "wl_fill_uniform_f16", "wl_double_to_f16", "wl_edges_uniform",
                 "wl_edges_rmat", "wl_permutation", "wl_relabel", "wl_fill_cols_uniform_sorted"):
        getattr(lib, name).restype = None
    _lib = lib
    return lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def seed_for(config: int, stream: int) -> int:
    return BASE_SEED + 1000 * config + stream


# --------------------------------------------------------------------------- tensors
def normal_f16(shape, seed: int, mean: float = 0.0, sd: float = 1.0) -> np.ndarray:
    out = np.empty(shape, dtype=np.uint16)
    _load().wl_fill_normal_f16(_p(out, ctypes.c_uint16), out.size, seed, mean, sd)
    return out.view(np.float16)


def uniform_f16(shape, seed: int, lo: float, hi: float) -> np.ndarray:
    out = np.empty(shape, dtype=np.uint16)
    _load().wl_fill_uniform_f16(_p(out, ctypes.c_uint16), out.size, seed, lo, hi)
    return out.view(np.float16)


def to_f16(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint16)
    _load().wl_double_to_f16(_p(x, ctypes.c_double), _p(out, ctypes.c_uint16), x.size)
    return out.view(np.float16)


# --------------------------------------------------------------------------- graphs
def coo_to_csr(row: np.ndarray, col: np.ndarray, nrows: int, ncols: int):
    row = np.ascontiguousarray(row, dtype=np.int32)
    col = np.ascontiguousarray(col, dtype=np.int32)
    n = row.size
    rowptr = np.empty(nrows + 1, dtype=np.int32)
    col_out = np.empty(n, dtype=np.int32)
    rc = _load().wl_coo_to_csr(_p(row, ctypes.c_int32), _p(col, ctypes.c_int32), n, nrows, ncols,
                               _p(rowptr, ctypes.c_int32), _p(col_out, ctypes.c_int32))
    if rc:
        raise MemoryError("wl_coo_to_csr failed")
    return rowptr, col_out


def _with_self_loops(row, col, V):
    loops = np.arange(V, dtype=np.int32)
    return np.concatenate([row, loops]), np.concatenate([col, loops])


def uniform_graph(V: int, n_edges: int, seed: int, self_loops: bool = True):
    """n_edges directed (i,j) with uniform endpoints, then one (i,i) per vertex."""
    row = np.empty(n_edges, dtype=np.int32)
    col = np.empty(n_edges, dtype=np.int32)
    _load().wl_edges_uniform(_p(row, ctypes.c_int32), _p(col, ctypes.c_int32), n_edges, V, seed)
    if self_loops:
        row, col = _with_self_loops(row, col, V)
    return coo_to_csr(row, col, V, V)


def rmat_graph(scale: int, n_edges: int, seed: int, V: Optional[int] = None, self_loops: bool = False,
               relabel: bool = True, a: float = 0.57, b: float = 0.19, c: float = 0.19):
    """R-MAT draws (duplicates kept); endpoints >= V are redrawn; seeded vertex
    relabel so hubs are not all at low ids; optional self-loop per vertex."""
    V = (1 << scale) if V is None else V
    row = np.empty(n_edges, dtype=np.int32)
    col = np.empty(n_edges, dtype=np.int32)
    lib = _load()
    lib.wl_edges_rmat(_p(row, ctypes.c_int32), _p(col, ctypes.c_int32), n_edges, scale, a, b, c, V, seed)
    if relabel:
        perm = np.empty(V, dtype=np.int32)
        lib.wl_permutation(_p(perm, ctypes.c_int32), V, seed ^ 0x5EED5EED)
        lib.wl_relabel(_p(row, ctypes.c_int32), n_edges, _p(perm, ctypes.c_int32))
        lib.wl_relabel(_p(col, ctypes.c_int32), n_edges, _p(perm, ctypes.c_int32))
    if self_loops:
        row, col = _with_self_loops(row, col, V)
    return coo_to_csr(row, col, V, V)


def lognormal_graph(V: int, n_edges: int, seed: int, mean_degree: Optional[float] = None, sigma: float = 1.0):
    """Row degrees log-normal (mu = ln(mean) - sigma^2/2) rescaled to n_edges and
    clipped to [1, V]; columns uniform with replacement, ascending inside a row."""
    mean_degree = n_edges / V if mean_degree is None else mean_degree
    deg = np.empty(V, dtype=np.int32)
    lib = _load()
    rc = lib.wl_lognormal_degrees(_p(deg, ctypes.c_int32), V, n_edges, float(np.log(mean_degree) - 0.5 * sigma * sigma),
                                  sigma, V, seed)
    if rc:
        raise RuntimeError("wl_lognormal_degrees failed (%d)" % rc)
    rowptr = np.zeros(V + 1, dtype=np.int64)
    np.cumsum(deg, out=rowptr[1:])
    rowptr = rowptr.astype(np.int32)
    col = np.empty(n_edges, dtype=np.int32)
    lib.wl_fill_cols_uniform_sorted(_p(rowptr, ctypes.c_int32), _p(col, ctypes.c_int32), V, V, seed ^ 0xC01C01)
    return rowptr, col


def symnorm_f16(rowptr: np.ndarray, col: np.ndarray, ncols: int) -> np.ndarray:
    w = np.empty(col.size, dtype=np.uint16)
    rc = _load().wl_symnorm_f16(_p(rowptr, ctypes.c_int32), _p(col, ctypes.c_int32), rowptr.size - 1, ncols,
                                _p(w, ctypes.c_uint16))
    if rc:
        raise MemoryError("wl_symnorm_f16 failed")
    return w.view(np.float16)


# --------------------------------------------------------------------------- the five configurations
@dataclass
class Workload:
    name: str
    V: int
    rowptr: np.ndarray
    col: np.ndarray
    F: int
    H: int = 1
    tensors: Dict[str, np.ndarray] = field(default_factory=dict)

    @property
    def E(self) -> int:
        return int(self.col.size)


def gcn_tiny(V: int = 4096, n_rand: int = 32768, F: int = 64, cfg: int = 1) -> Workload:
    """Config 1: uniform-random edges plus self-loops, sym-norm fp16 edge values,
    X and dY ~ N(0,1)."""
    rowptr, col = uniform_graph(V, n_rand, seed_for(cfg, 0))
    t = {"w": symnorm_f16(rowptr, col, V), "X": normal_f16((V, F), seed_for(cfg, 1)),
         "dY": normal_f16((V, F), seed_for(cfg, 2))}
    return Workload("c1_gcn_tiny", V, rowptr, col, F, 1, t)


def gin_overflow(scale: int = 17, avg_degree: int = 16, F: int = 128, positive: bool = False, cfg: int = 2) -> Workload:
    """Config 2: R-MAT, unweighted, X ~ uniform[-8,8]; positive=True gives the
    all-positive variant uniform[0,8] whose hub sums leave the fp16 range."""
    V = 1 << scale
    rowptr, col = rmat_graph(scale, V * avg_degree, seed_for(cfg, 0))
    lo = 0.0 if positive else -8.0
    t = {"X": uniform_f16((V, F), seed_for(cfg, 1), lo, 8.0), "dY": uniform_f16((V, F), seed_for(cfg, 2), lo, 8.0)}
    return Workload("c2b_gin_overflow_pos" if positive else "c2_gin_overflow", V, rowptr, col, F, 1, t)


def gat_rmat(scale: int = 18, avg_degree: int = 20, H: int = 4, D: int = 16, cfg: int = 3) -> Workload:
    """Config 3: R-MAT plus self-loops; h ~ N(0,1), a_l, a_r ~ N(0, sd 0.1), dOut ~ N(0,1)."""
    V = 1 << scale
    rowptr, col = rmat_graph(scale, V * avg_degree, seed_for(cfg, 0), self_loops=True)
    F = H * D
    t = {"h": normal_f16((V, F), seed_for(cfg, 1)), "a_l": normal_f16((H, D), seed_for(cfg, 2), 0.0, 0.1),
         "a_r": normal_f16((H, D), seed_for(cfg, 3), 0.0, 0.1), "dOut": normal_f16((V, F), seed_for(cfg, 4))}
    return Workload("c3_gat_rmat", V, rowptr, col, F, H, t)


def gcn_large(V: int = 2_400_000, n_edges: int = 62_000_000, F: int = 128, scale: int = 22, cfg: int = 4) -> Workload:
    """Config 4: power-law R-MAT restricted to V vertices, sym-norm fp16 edge values."""
    rowptr, col = rmat_graph(scale, n_edges, seed_for(cfg, 0), V=V)
    t = {"w": symnorm_f16(rowptr, col, V), "X": normal_f16((V, F), seed_for(cfg, 1)),
         "dY": normal_f16((V, F), seed_for(cfg, 2))}
    return Workload("c4_gcn_large", V, rowptr, col, F, 1, t)


def dense_degree(V: int = 233_000, n_edges: int = 114_000_000, F: int = 64, cfg: int = 5) -> Workload:
    """Config 5: log-normal degrees (sigma 1, mean ~490); GAT with one head of 64
    and GIN sum aggregation."""
    rowptr, col = lognormal_graph(V, n_edges, seed_for(cfg, 0))
    t = {"X": normal_f16((V, F), seed_for(cfg, 1)), "a_l": normal_f16((1, F), seed_for(cfg, 2), 0.0, 0.1),
         "a_r": normal_f16((1, F), seed_for(cfg, 3), 0.0, 0.1), "dY": normal_f16((V, F), seed_for(cfg, 4))}
    return Workload("c5_dense_degree", V, rowptr, col, F, 1, t)
