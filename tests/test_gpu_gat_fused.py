"""GPU parity of the single-pass GAT aggregation (score + edge softmax + weighted sum in one kernel
sequence) against the CPU fp64 oracle's unrounded chain."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from parity import compare, down, f16, rand_graph, sample_rows, up

pytestmark = pytest.mark.gpu


def check_lse(name, got, ref, deg):
    nz = deg > 0
    err = np.abs(got[nz].astype(np.float64) - ref[nz])
    assert np.all(err <= 2e-3 + 1e-3 * np.abs(ref[nz])), f"{name}: lse off by {err.max():.3e}"
    assert np.all(got[~nz] == 0)


CASES = [  # (H, D, S, col_blocks, scale of the attention vectors)
    (1, 64, 256, 1, 0.1), (4, 16, 256, 1, 0.1), (8, 8, 128, 1, 0.3), (2, 32, 64, 1, 0.1), (1, 8, 7, 1, 0.5),
    (1, 128, 256, 1, 0.1), (1, 64, 256, 3, 0.1), (4, 16, 100, 4, 0.2), (1, 64, 256, 1, 3.0), (2, 64, 512, 1, 0.1),
]


@pytest.mark.parametrize("H,D,S,nb,ascale", CASES)
def test_gat_forward_fused_shapes(hgnn, dev, H, D, S, nb, ascale):
    print(f"gat fused H={H} D={D} S={S} nb={nb} ascale={ascale}", flush=True)
    V = 1100
    F = H * D
    rowptr, col = rand_graph(V, V, 12, H * 100 + D + S, hubs=((5, 5000), (700, 777), (1099, 300)), empties=(0, 6, 1098))
    r = np.random.default_rng(H * 7 + D)
    X = f16(r.standard_normal((V, F)))
    a_l, a_r = f16(ascale * r.standard_normal(F)), f16(ascale * r.standard_normal(F))
    ref, ref_lse, sabs = oracle.gat_forward(rowptr, col, X, X, a_l, a_r, H, slope=0.2)
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    p = hgnn.hgnn_plan_create(g, S, F, H, col_blocks=nb)
    assert hgnn.hgnn_plan_col_blocks(p) == nb
    Xd = up(X, dev)
    out = torch.full((V, F), 7.0, dtype=torch.float16, device=dev)
    lse = torch.full((V, H), 7.0, dtype=torch.float32, device=dev)
    hgnn.hgnn_gat_forward_fused(g, p, H, D, Xd, Xd, up(a_l, dev), up(a_r, dev), out, lse)
    got = down(out)
    compare("gat fused", got, ref, sabs)
    deg = np.diff(rowptr)
    check_lse("gat fused", down(lse), ref_lse, deg)
    # deterministic; lse optional
    out2 = torch.full((V, F), -3.0, dtype=torch.float16, device=dev)
    hgnn.hgnn_gat_forward_fused(g, p, H, D, Xd, Xd, up(a_l, dev), up(a_r, dev), out2, None)
    assert np.array_equal(down(out2).view(np.uint16), got.view(np.uint16))
    # alpha rebuilt from lse = the edge softmax of the scores
    alpha = torch.full((col.size, H), 7.0, dtype=torch.float16, device=dev)
    hgnn.hgnn_gat_alpha(g, p, H, D, Xd, Xd, up(a_l, dev), up(a_r, dev), lse, alpha)
    aref = oracle.edge_softmax(rowptr, oracle.gat_score(rowptr, col, X, a_l, a_r, H, slope=0.2))
    compare("alpha from lse", down(alpha), aref, None, rel_l2=5e-3, rel_elem=2e-2)
    hgnn.hgnn_plan_destroy(p)


def test_gat_forward_fused_separate_row_and_column_tables(hgnn, dev):
    V, ncols, H, D = 500, 700, 2, 16
    F = H * D
    rowptr, col = rand_graph(V, ncols, 8, 3, hubs=((9, 900),), empties=(2,))
    r = np.random.default_rng(1)
    U, Vt = f16(r.standard_normal((V, F))), f16(r.standard_normal((ncols, F)))
    a_l, a_r = f16(0.2 * r.standard_normal(F)), f16(0.2 * r.standard_normal(F))
    ref, ref_lse, sabs = oracle.gat_forward(rowptr, col, U, Vt, a_l, a_r, H)
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    p = hgnn.hgnn_plan_create(g, 128, F, H)
    out = torch.empty((V, F), dtype=torch.float16, device=dev)
    lse = torch.empty((V, H), dtype=torch.float32, device=dev)
    hgnn.hgnn_gat_forward_fused(g, p, H, D, up(U, dev), up(Vt, dev), up(a_l, dev), up(a_r, dev), out, lse)
    compare("gat fused, two tables", down(out), ref, sabs)
    check_lse("gat fused, two tables", down(lse), ref_lse, np.diff(rowptr))
    hgnn.hgnn_plan_destroy(p)


def test_gat_forward_fused_large_scores_stay_finite(hgnn, dev):
    """Scores of several hundred: Eq. 1's shift by the maximum, carried through every merge."""
    V, H, D = 600, 1, 16
    rowptr, col = rand_graph(V, V, 10, 8, hubs=((3, 2000),))
    r = np.random.default_rng(2)
    X = f16(np.abs(r.standard_normal((V, D))) * 8)
    a_l, a_r = f16(np.full(D, 4.0)), f16(np.full(D, 4.0))
    ref, ref_lse, sabs = oracle.gat_forward(rowptr, col, X, X, a_l, a_r, H)
    assert ref_lse.max() > 500
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    p = hgnn.hgnn_plan_create(g, 64, D, H)
    out = torch.empty((V, D), dtype=torch.float16, device=dev)
    lse = torch.empty((V, H), dtype=torch.float32, device=dev)
    hgnn.hgnn_gat_forward_fused(g, p, H, D, up(X, dev), up(X, dev), up(a_l, dev), up(a_r, dev), out, lse)
    got = down(out)
    assert np.all(np.isfinite(got)) and np.all(np.isfinite(down(lse)))
    # el, er are fp32 sums of fp16 products of magnitude ~500: scores carry ~1e-4 absolute error, weights ~1e-4 relative
    compare("gat fused, large scores", got, ref, sabs)
    hgnn.hgnn_plan_destroy(p)


def test_gat_forward_fused_argument_errors(hgnn, dev):
    rowptr, col = rand_graph(50, 50, 4, 2)
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    p = hgnn.hgnn_plan_create(g, 64, 64, 1)
    X = torch.ones((50, 64), dtype=torch.float16, device=dev)
    a = torch.ones(64, dtype=torch.float16, device=dev)
    out = torch.empty_like(X)
    with pytest.raises(hgnn.HgnnError) as ei:  # more heads than the plan allows
        hgnn.hgnn_gat_forward_fused(g, p, 2, 32, X, X, a, a, out)
    assert ei.value.status == hgnn.HGNN_EINVAL
    X12 = torch.ones((50, 16), dtype=torch.float16, device=dev)
    with pytest.raises(hgnn.HgnnError) as ei:  # D = 12 is not 8 * 2^k
        hgnn.hgnn_gat_forward_fused(g, p, 1, 12, X12[:, :12], X12[:, :12], a, a, out[:, :16])
    assert ei.value.status == hgnn.HGNN_EUNSUPPORTED
    hgnn.hgnn_plan_destroy(p)


@pytest.mark.parametrize("maker,nb", [(wl.gat_rmat, 1), (wl.dense_degree, 0)])
def test_gat_forward_fused_full_configs(hgnn, dev, maker, nb):
    """Configs 3 and 5 at full size in the launch configuration of the benchmark, on sampled rows."""
    w = maker()
    print(f"gat fused full config {w.name}", flush=True)
    feat = w.tensors["h"] if "h" in w.tensors else w.tensors["X"]
    H, D = w.H, w.F // w.H
    g = hgnn.Csr(up(w.rowptr, dev), up(w.col, dev))
    p = hgnn.hgnn_plan_create(g, 256, w.F, H, col_blocks=nb)
    Xd = up(feat, dev)
    out = torch.empty((w.V, w.F), dtype=torch.float16, device=dev)
    lse = torch.empty((w.V, H), dtype=torch.float32, device=dev)
    hgnn.hgnn_gat_forward_fused(g, p, H, D, Xd, Xd, up(w.tensors["a_l"], dev), up(w.tensors["a_r"], dev), out, lse)
    got, got_lse = down(out), down(lse)
    assert np.all(np.isfinite(got))
    rows = sample_rows(w.rowptr, 300, 5)
    # the oracle on the sampled rows only: a sub-graph with those rows and all columns
    sub_ptr = np.concatenate([[0], np.cumsum(np.diff(w.rowptr)[rows])]).astype(np.int32)
    sub_col = np.concatenate([w.col[w.rowptr[r]:w.rowptr[r + 1]] for r in rows]).astype(np.int32)
    ref, ref_lse, sabs = oracle.gat_forward(sub_ptr, sub_col, feat[rows], feat, w.tensors["a_l"], w.tensors["a_r"], H)
    compare(f"{w.name} gat fused", got[rows], ref, sabs)
    check_lse(f"{w.name} gat fused", got_lse[rows], ref_lse, np.diff(sub_ptr))
    hgnn.hgnn_plan_destroy(p)


# ------------------------------------------------------------------ fused backward
def gat_backward_check(hgnn, dev, rowptr, col, ncols, U, Vt, a_l, a_r, dOut, H, S, nb, name, rows=None, cols=None):
    """Forward + backward through the C ABI; compares dV, d_el, d_er with the oracle (on sampled rows/columns when given)."""
    V = rowptr.size - 1
    F = U.shape[1]
    D = F // H
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    gt = hgnn.hgnn_transpose(g)
    p = hgnn.hgnn_plan_create(g, S, F, H, col_blocks=nb)
    pt = hgnn.hgnn_plan_create(gt, S, F, H, col_blocks=nb)
    Ud, Vd, ald, ard, dOd = up(U, dev), up(Vt, dev), up(a_l, dev), up(a_r, dev), up(dOut, dev)
    out = torch.empty((V, F), dtype=torch.float16, device=dev)
    lse = torch.empty((V, H), dtype=torch.float32, device=dev)
    hgnn.hgnn_gat_forward_fused(g, p, H, D, Ud, Vd, ald, ard, out, lse)
    dV = torch.full((ncols, F), 7.0, dtype=torch.float16, device=dev)
    d_el = torch.full((V, H), 7.0, dtype=torch.float16, device=dev)
    d_er = torch.full((ncols, H), 7.0, dtype=torch.float16, device=dev)
    hgnn.hgnn_gat_backward_fused(g, p, gt, pt, H, D, Ud, Vd, ald, ard, out, lse, dOd, dV, d_el, d_er)
    got = (down(dV), down(d_el), down(d_er))
    # deterministic
    dV2, d_el2, d_er2 = torch.empty_like(dV), torch.empty_like(d_el), torch.empty_like(d_er)
    hgnn.hgnn_gat_backward_fused(g, p, gt, pt, H, D, Ud, Vd, ald, ard, out, lse, dOd, dV2, d_el2, d_er2)
    for a, b in zip(got, (down(dV2), down(d_el2), down(d_er2))):
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    hgnn.hgnn_plan_destroy(p)
    hgnn.hgnn_plan_destroy(pt)
    return got


def bwd_reference(rowptr, col, ncols, U, Vt, a_l, a_r, dOut, H, slope=0.2):
    """Oracle values plus magnitudes (sum of |terms|) for the tolerance rule."""
    V, F = U.shape
    D = F // H
    dV, d_el, d_er = oracle.gat_backward(rowptr, col, U, Vt, a_l, a_r, dOut, H, slope=slope)
    row = np.repeat(np.arange(V), np.diff(rowptr))
    el = (U.astype(np.float64).reshape(V, H, D) * a_l.astype(np.float64).reshape(H, D)).sum(-1)
    er = (Vt.astype(np.float64).reshape(ncols, H, D) * a_r.astype(np.float64).reshape(H, D)).sum(-1)
    raw = el[row] + er[col]
    e = np.where(raw > 0, raw, slope * raw)
    alpha = oracle.edge_softmax(rowptr, e)
    dO, V64 = dOut.astype(np.float64), Vt.astype(np.float64)
    dalpha_abs = (np.abs(dO[row]) * np.abs(V64[col])).reshape(-1, H, D).sum(-1)
    t_abs = oracle.edge_rowsum(rowptr, alpha * dalpha_abs)
    ds_abs = alpha * (dalpha_abs + t_abs[row])
    dV_abs = np.zeros((ncols, F))
    np.add.at(dV_abs, col, np.repeat(alpha, D, axis=1) * np.abs(dO[row]))
    return (dV, dV_abs), (d_el, oracle.edge_rowsum(rowptr, ds_abs)), (d_er, oracle.edge_colsum(rowptr, col, ds_abs, ncols))


BWD_CASES = [(1, 64, 256, 1), (4, 16, 256, 1), (8, 8, 128, 1), (2, 32, 64, 1), (1, 8, 7, 1), (1, 128, 256, 1),
             (1, 64, 256, 3), (4, 16, 100, 4), (1, 256, 128, 2)]  # one head of 128 or more: weights staged per segment


@pytest.mark.parametrize("H,D,S,nb", BWD_CASES)
def test_gat_backward_fused_shapes(hgnn, dev, H, D, S, nb):
    print(f"gat fused backward H={H} D={D} S={S} nb={nb}", flush=True)
    V, ncols = 900, 1000
    F = H * D
    rowptr, col = rand_graph(V, ncols, 12, H * 100 + D + S, hubs=((5, 4000), (700, 777), (899, 300)), empties=(0, 6, 898))
    r = np.random.default_rng(H * 7 + D)
    U, Vt, dOut = f16(r.standard_normal((V, F))), f16(r.standard_normal((ncols, F))), f16(r.standard_normal((V, F)))
    a_l, a_r = f16(0.2 * r.standard_normal(F)), f16(0.2 * r.standard_normal(F))
    (dV, dV_abs), (d_el, el_abs), (d_er, er_abs) = bwd_reference(rowptr, col, ncols, U, Vt, a_l, a_r, dOut, H)
    g_dV, g_el, g_er = gat_backward_check(hgnn, dev, rowptr, col, ncols, U, Vt, a_l, a_r, dOut, H, S, nb, "bwd")
    compare("dV", g_dV, dV, dV_abs)
    compare("d_el", g_el, d_el, el_abs, rel_l2=2e-2)  # cancelling sums: the L2 norm of the result is far below that of its terms
    compare("d_er", g_er, d_er, er_abs, rel_l2=2e-2)


@pytest.mark.parametrize("maker,nb", [(wl.gat_rmat, 1), (wl.dense_degree, 0)])
def test_gat_backward_fused_full_configs(hgnn, dev, maker, nb):
    """Configs 3 and 5 at full size; the oracle runs on the sub-graphs of sampled rows and of sampled columns."""
    w = maker()
    print(f"gat fused backward full config {w.name}", flush=True)
    feat = w.tensors["h"] if "h" in w.tensors else w.tensors["X"]
    dOut = w.tensors["dOut"] if "dOut" in w.tensors else w.tensors["dY"]
    H = w.H
    a_l, a_r = w.tensors["a_l"], w.tensors["a_r"]
    g_dV, g_el, g_er = gat_backward_check(hgnn, dev, w.rowptr, w.col, w.V, feat, feat, a_l, a_r, dOut, H, 256, nb, w.name)
    assert np.all(np.isfinite(g_dV)) and np.all(np.isfinite(g_el)) and np.all(np.isfinite(g_er))
    # d_el on sampled rows: a sub-graph with those rows and all columns
    rows = sample_rows(w.rowptr, 200, 5)
    sub_ptr = np.concatenate([[0], np.cumsum(np.diff(w.rowptr)[rows])]).astype(np.int32)
    sub_col = np.concatenate([w.col[w.rowptr[r]:w.rowptr[r + 1]] for r in rows]).astype(np.int32)
    (_, _), (d_el, el_abs), (_, _) = bwd_reference(sub_ptr, sub_col, w.V, feat[rows], feat, a_l, a_r, dOut[rows], H)
    compare(f"{w.name} d_el", g_el[rows], d_el, el_abs, rel_l2=2e-2)
    # dV and d_er on sampled columns: every row that has one of them as neighbour is needed in full (softmax),
    # so the columns are drawn among the neighbours of a few rows and only those rows' contribution is... not enough:
    # take the full rows of all in-neighbours of the sampled columns instead
    rng_ = np.random.default_rng(3)
    cols = np.unique(rng_.integers(0, w.V, size=12)).astype(np.int64)
    row_of = np.repeat(np.arange(w.V), np.diff(w.rowptr))
    need = np.unique(row_of[np.isin(w.col, cols)])
    if need.size > 40000:  # keep the oracle's work bounded on the dense-degree graph
        cols = cols[:3]
        need = np.unique(row_of[np.isin(w.col, cols)])
    sub_ptr = np.concatenate([[0], np.cumsum(np.diff(w.rowptr)[need])]).astype(np.int32)
    sub_col = np.concatenate([w.col[w.rowptr[r]:w.rowptr[r + 1]] for r in need]).astype(np.int32)
    (dV, dV_abs), (_, _), (d_er, er_abs) = bwd_reference(sub_ptr, sub_col, w.V, feat[need], feat, a_l, a_r, dOut[need], H)
    compare(f"{w.name} dV", g_dV[cols], dV[cols], dV_abs[cols])
    compare(f"{w.name} d_er", g_er[cols], d_er[cols], er_abs[cols], rel_l2=2e-2)


# ------------------------------------------------------------------ forward that saves for the backward
SAVE_CASES = [(1, 64, 256, 1), (4, 16, 256, 1), (8, 8, 128, 1), (2, 32, 64, 1), (1, 8, 7, 1), (1, 128, 256, 1), (1, 64, 256, 3),
              (4, 16, 100, 4), (3, 8, 33, 2), (8, 64, 256, 1), (1, 256, 128, 2)]


@pytest.mark.parametrize("H,D,S,nb", SAVE_CASES)
def test_gat_forward_save_and_backward_saved(hgnn, dev, H, D, S, nb):
    """The saving forward leaves out_masked / csum; the backward that takes them skips its pass over g.  Everything
    against the oracle; the tensors both variants produce (out, lse, dV, d_er) must not depend on the variant."""
    print(f"gat save H={H} D={D} S={S} nb={nb}", flush=True)
    V = 1000
    F = H * D
    rowptr, col = rand_graph(V, V, 12, H * 100 + D + S, hubs=((5, 4500), (700, 777), (999, 300)), empties=(0, 6, 998))
    r = np.random.default_rng(H * 11 + D)
    X, dOut = f16(r.standard_normal((V, F))), f16(r.standard_normal((V, F)))
    a_l, a_r = f16(0.3 * r.standard_normal(F)), f16(0.3 * r.standard_normal(F))
    oref, lref, oabs, mref, cref = oracle.gat_forward(rowptr, col, X, X, a_l, a_r, H, slope=0.2, want_saved=True)
    (dV, dV_abs), (d_el, el_abs), (d_er, er_abs) = bwd_reference(rowptr, col, V, X, X, a_l, a_r, dOut, H)
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    gt = hgnn.hgnn_transpose(g)
    p = hgnn.hgnn_plan_create(g, S, F, H, col_blocks=nb)
    pt = hgnn.hgnn_plan_create(gt, S, F, H, col_blocks=nb)
    Xd, ald, ard, dOd = up(X, dev), up(a_l, dev), up(a_r, dev), up(dOut, dev)
    half = lambda *s: torch.full(s, 7.0, dtype=torch.float16, device=dev)
    f32 = lambda *s: torch.full(s, 7.0, dtype=torch.float32, device=dev)
    out, outm_buf, lse, csum = half(V, F), half(V, F + 8), f32(V, H), f32(V, H)
    outm = outm_buf[:, :F]
    hgnn.hgnn_gat_forward_fused_save(g, p, H, D, Xd, Xd, ald, ard, out, lse, outm, csum)
    compare("out", down(out), oref, oabs)
    check_lse("save", down(lse), lref, np.diff(rowptr))
    compare("out_masked", down(outm_buf)[:, :F], mref, oabs)
    assert np.all(down(outm_buf)[:, F:] == 7.0)
    assert np.abs(down(csum).astype(np.float64) - cref).max() <= 2e-3
    # the plain forward gives the same out and lse
    out0, lse0 = half(V, F), f32(V, H)
    hgnn.hgnn_gat_forward_fused(g, p, H, D, Xd, Xd, ald, ard, out0, lse0)
    assert np.array_equal(down(out0).view(np.uint16), down(out).view(np.uint16))
    assert np.array_equal(down(lse0), down(lse))
    # backward with the saved tensors
    dVs, d_els, d_ers = half(V, F), half(V, H), half(V, H)
    hgnn.hgnn_gat_backward_fused_saved(g, p, gt, pt, H, D, Xd, Xd, ald, ard, out, lse, outm, csum, dOd, dVs, d_els, d_ers)
    compare("dV", down(dVs), dV, dV_abs)
    compare("d_el saved", down(d_els), d_el, el_abs, rel_l2=2e-2)
    compare("d_er", down(d_ers), d_er, er_abs, rel_l2=2e-2)
    dV0, d_el0, d_er0 = half(V, F), half(V, H), half(V, H)
    hgnn.hgnn_gat_backward_fused(g, p, gt, pt, H, D, Xd, Xd, ald, ard, out, lse, dOd, dV0, d_el0, d_er0)
    assert np.array_equal(down(dV0).view(np.uint16), down(dVs).view(np.uint16))
    assert np.array_equal(down(d_er0).view(np.uint16), down(d_ers).view(np.uint16))
    hgnn.hgnn_plan_destroy(p)
    hgnn.hgnn_plan_destroy(pt)


def test_gat_save_argument_errors(hgnn, dev):
    V, H, D = 50, 1, 8
    rowptr, col = rand_graph(V, V, 4, 3)
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    p = hgnn.hgnn_plan_create(g, 64, 8, 1)
    X = torch.zeros((V, 8), dtype=torch.float16, device=dev)
    a = torch.zeros(8, dtype=torch.float16, device=dev)
    lse = torch.zeros((V, 1), dtype=torch.float32, device=dev)
    with pytest.raises(hgnn.HgnnError) as e:
        hgnn.hgnn_gat_forward_fused_save(g, p, H, D, X, X, a, a, X.clone(), lse, X.clone(), lse.clone(), neg_slope=-0.1)
    assert e.value.status == hgnn.HGNN_EINVAL and "slope" in str(e.value)
    hgnn.hgnn_plan_destroy(p)


@pytest.mark.parametrize("maker,nb", [(wl.gat_rmat, 1), (wl.dense_degree, 0)])
def test_gat_save_and_saved_backward_full_configs(hgnn, dev, maker, nb):
    """Configs 3 and 5 at full size through the saving forward and the one-pass backward: out_masked, csum and d_el on
    sampled rows against the oracle (on the sub-graph of those rows); out / lse / dV / d_er must be the bits of the
    plain forward and the two-pass backward."""
    w = maker()
    print(f"gat save full config {w.name}", flush=True)
    feat = w.tensors["h"] if "h" in w.tensors else w.tensors["X"]
    dOut = w.tensors["dOut"] if "dOut" in w.tensors else w.tensors["dY"]
    H, V = w.H, w.V
    F = feat.shape[1]
    D = F // H
    a_l, a_r = w.tensors["a_l"].reshape(-1), w.tensors["a_r"].reshape(-1)
    g = hgnn.Csr(up(w.rowptr, dev), up(w.col, dev))
    gt = hgnn.hgnn_transpose(g)
    p = hgnn.hgnn_plan_create(g, 256, F, H, col_blocks=nb)
    pt = hgnn.hgnn_plan_create(gt, 256, F, H, col_blocks=nb)
    Xd, ald, ard, dOd = up(feat, dev), up(a_l, dev), up(a_r, dev), up(dOut, dev)
    half = lambda *s: torch.empty(s, dtype=torch.float16, device=dev)
    f32 = lambda *s: torch.empty(s, dtype=torch.float32, device=dev)
    out, outm, lse, csum = half(V, F), half(V, F), f32(V, H), f32(V, H)
    hgnn.hgnn_gat_forward_fused_save(g, p, H, D, Xd, Xd, ald, ard, out, lse, outm, csum)
    out0, lse0 = half(V, F), f32(V, H)
    hgnn.hgnn_gat_forward_fused(g, p, H, D, Xd, Xd, ald, ard, out0, lse0)
    assert np.array_equal(down(out0).view(np.uint16), down(out).view(np.uint16)) and np.array_equal(down(lse0), down(lse))
    dVs, d_els, d_ers = half(V, F), half(V, H), half(V, H)
    hgnn.hgnn_gat_backward_fused_saved(g, p, gt, pt, H, D, Xd, Xd, ald, ard, out, lse, outm, csum, dOd, dVs, d_els, d_ers)
    dV0, d_el0, d_er0 = half(V, F), half(V, H), half(V, H)
    hgnn.hgnn_gat_backward_fused(g, p, gt, pt, H, D, Xd, Xd, ald, ard, out, lse, dOd, dV0, d_el0, d_er0)
    assert np.array_equal(down(dV0).view(np.uint16), down(dVs).view(np.uint16))
    assert np.array_equal(down(d_er0).view(np.uint16), down(d_ers).view(np.uint16))
    rows = sample_rows(w.rowptr, 200, 9)
    sub_ptr = np.concatenate([[0], np.cumsum(np.diff(w.rowptr)[rows])]).astype(np.int32)
    sub_col = np.concatenate([w.col[w.rowptr[r]:w.rowptr[r + 1]] for r in rows]).astype(np.int32)
    oref, _, oabs, mref, cref = oracle.gat_forward(sub_ptr, sub_col, feat[rows], feat, a_l, a_r, H, want_saved=True)
    compare(f"{w.name} out_masked", down(outm)[rows], mref, oabs)
    assert np.abs(down(csum)[rows].astype(np.float64) - cref).max() <= 2e-3
    (_, _), (d_el, el_abs), (_, _) = bwd_reference(sub_ptr, sub_col, V, feat[rows], feat, a_l, a_r, dOut[rows], H)
    compare(f"{w.name} d_el saved", down(d_els)[rows], d_el, el_abs, rel_l2=2e-2)
    compare(f"{w.name} d_el two-pass", down(d_el0)[rows], d_el, el_abs, rel_l2=2e-2)
    hgnn.hgnn_plan_destroy(p)
    hgnn.hgnn_plan_destroy(pt)
