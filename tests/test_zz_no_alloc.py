"""hgnn_spmm_static, the entry point that allocates nothing (its scratch is a static device array), against hgnn_spmm
with a caller-owned workspace: same kernels, same summation order, so the outputs must agree bit for bit; and against
the fp64 oracle.  Two calls in a row share the array, the second on a smaller input: what the first left behind must
not leak into the second."""
import numpy as np
import pytest
import torch

import oracle
from parity import compare, down, f16, rand_graph, up

pytestmark = pytest.mark.gpu


def run_pair(hgnn, dev, V, avg, hubs, F, has_w, reduce, seed):
    rowptr, col = rand_graph(V, V, avg, seed, hubs=hubs, empties=(0, V - 1))
    r = np.random.default_rng(seed)
    Xh = f16(r.standard_normal((V, F)))
    w = f16(r.standard_normal((col.size, 1))) if has_w else None
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    X, wd = up(Xh, dev), None if w is None else up(w, dev)
    need = hgnn.hgnn_spmm_workspace(V, 0, col.size, F)
    assert 0 < need <= hgnn.hgnn_spmm_static_limit()
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    Y_ws = torch.full((V, F), 3.0, dtype=torch.float16, device=dev)
    Y_st = torch.full((V, F), 5.0, dtype=torch.float16, device=dev)
    hgnn.hgnn_spmm(g, wd, 1, X, Y_ws, op=reduce, workspace=ws)
    hgnn.hgnn_spmm_static(g, wd, 1, X, Y_st, op=reduce)
    a, b = down(Y_ws), down(Y_st)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16)), "static scratch and workspace forms differ"
    ref, sabs = oracle.spmm(rowptr, col, Xh, w=w, reduce=reduce, want_sabs=True)
    return compare(f"hgnn_spmm_static V={V} F={F}", b, ref, sabs)


def test_static_scratch_two_calls_in_a_row(hgnn, dev):
    print("static scratch: first call (large), second call (smaller)", flush=True)
    s1 = run_pair(hgnn, dev, 6000, 12, ((7, 20000), (3000, 5000), (5999, 1500), (10, 700)), 128, True, hgnn.HGNN_SUM, 1)
    s2 = run_pair(hgnn, dev, 900, 6, ((5, 3000), (400, 600)), 64, False, hgnn.HGNN_MEAN, 2)
    s3 = run_pair(hgnn, dev, 2500, 20, ((1, 9000),), 40, True, hgnn.HGNN_MEAN, 3)
    print(s1, s2, s3, flush=True)


def test_static_scratch_rejects_what_does_not_fit(hgnn, dev):
    """A graph whose worst-case scratch exceeds the array is refused on the host, before any launch."""
    limit = hgnn.hgnn_spmm_static_limit()
    assert limit == 32 << 20
    V, E, F = 1000, 40_000_000, 128
    assert hgnn.hgnn_spmm_workspace(V, 0, E, F) > limit
    # the arrays are never touched: the size check comes first (rowptr / col only need to be non-null device tensors)
    rowptr = torch.zeros(V + 1, dtype=torch.int32, device=dev)
    col = torch.zeros(16, dtype=torch.int32, device=dev)
    g = hgnn.Csr(rowptr, col)
    g.struct.nnz = E
    X = torch.zeros((V, F), dtype=torch.float16, device=dev)
    with pytest.raises(hgnn.HgnnError) as ei:
        hgnn.hgnn_spmm_static(g, None, 1, X, torch.empty_like(X))
    assert ei.value.status == hgnn.HGNN_EUNSUPPORTED and "static" in str(ei.value)
    # a graph with no row long enough needs no scratch at all and runs
    rowptr2, col2 = rand_graph(50, 50, 3, 9)
    g2 = hgnn.Csr(up(rowptr2, dev), up(col2, dev))
    Xh = f16(np.random.default_rng(0).standard_normal((50, 16)))
    Y = torch.empty((50, 16), dtype=torch.float16, device=dev)
    hgnn.hgnn_spmm_static(g2, None, 1, up(Xh, dev), Y)
    compare("static, tiny graph", down(Y), *oracle.spmm(rowptr2, col2, Xh, want_sabs=True))
