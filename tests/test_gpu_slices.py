"""The column-slice kernels: the factorised GAT score (and alpha rebuilt from the row log-sum-exp) with a slice's
per-column term in LDS, and the column sums of an edge tensor accumulated exactly in LDS.  Compared with the fp64 oracle
on graphs whose columns span one to many slices, with hubs, empty rows and rows longer than a wave's 64 lanes per piece."""
import numpy as np
import pytest
import torch

import oracle
from parity import compare, down, f16, rand_graph, up

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("V,ncols,avg,W,D", [(700, 900, 12, 64, 16), (3000, 2500, 40, 256, 64), (1500, 40000, 60, 0, 32),
                                             (257, 100, 3, 128, 8), (5000, 5000, 5, 1024, 128)])
def test_score_alpha_and_column_sums_over_slices(hgnn, dev, V, ncols, avg, W, D):
    print(f"slices V={V} ncols={ncols} avg={avg} W={W} D={D}", flush=True)
    hubs = ((3, min(6000, 4 * ncols)), (V // 2, 300), (V - 1, 65))
    rowptr, col = rand_graph(V, ncols, avg, V + W, hubs=hubs, empties=(0, 7, V - 2))
    E = col.size
    r = np.random.default_rng(V + D)
    n = max(V, ncols)
    feat = f16(r.standard_normal((n, D)))
    a_l, a_r = f16(0.3 * r.standard_normal(D)), f16(0.3 * r.standard_normal(D))
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    p = hgnn.hgnn_plan_create(g, 256, D, 1, col_blocks=1)
    assert hgnn.hgnn_plan_num_slices(p) == 0
    e_plain = torch.empty((E, 1), dtype=torch.float16, device=dev)
    U, Vt = up(feat[:V], dev), up(feat[:ncols], dev)
    hgnn.hgnn_sddmm(g, p, hgnn.HGNN_SDDMM_GAT_SCORE, 1, D, U, Vt, e_plain, up(a_l, dev), up(a_r, dev), 0.2)
    hgnn.hgnn_plan_add_slices(p, g, W)
    width = W if W else 16384
    assert hgnn.hgnn_plan_num_slices(p) == (ncols + width - 1) // width
    e_sl = torch.full((E, 1), 9.0, dtype=torch.float16, device=dev)
    hgnn.hgnn_sddmm(g, p, hgnn.HGNN_SDDMM_GAT_SCORE, 1, D, U, Vt, e_sl, up(a_l, dev), up(a_r, dev), 0.2)
    # the oracle's score takes one table for both sides: rows and columns index the same padded table
    e_ref = oracle.gat_score(np.concatenate([rowptr, np.full(n - V, rowptr[-1], np.int32)]), col, feat, a_l.reshape(1, D),
                             a_r.reshape(1, D), 1)
    row = np.repeat(np.arange(V), np.diff(rowptr))
    mag = (np.abs(feat[row].astype(np.float64)) @ np.abs(a_l.astype(np.float64)) +
           np.abs(feat[col].astype(np.float64)) @ np.abs(a_r.astype(np.float64)))[:, None]
    compare("score over slices", down(e_sl), e_ref, mag)
    # same arithmetic as the segment kernel: el + er in fp32, one rounding
    assert np.array_equal(down(e_sl).view(np.uint16), down(e_plain).view(np.uint16))
    # alpha rebuilt from the row log-sum-exp (taken from the oracle's unrounded scores)
    e64 = e_ref[:, 0]
    lse = np.zeros(V)
    for i in range(V):
        if rowptr[i + 1] > rowptr[i]:
            seg = e64[rowptr[i]:rowptr[i + 1]]
            lse[i] = seg.max() + np.log(np.exp(seg - seg.max()).sum())
    a_ref = np.exp(e64 - lse[row])[:, None]
    np.testing.assert_allclose(a_ref, oracle.edge_softmax(rowptr, e_ref), rtol=1e-9, atol=1e-12)
    alpha = torch.full((E, 1), 9.0, dtype=torch.float16, device=dev)
    hgnn.hgnn_gat_alpha(g, p, 1, D, U, Vt, up(a_l, dev), up(a_r, dev), up(lse.astype(np.float32).reshape(V, 1), dev), alpha)
    # exp(s - lse) in fp32: the exponent carries the fp32 rounding of s and of lse (2^-23 of their magnitude)
    compare("alpha from lse over slices", down(alpha), a_ref, a_ref * (1.0 + 2.0 ** -10 * (mag + np.abs(lse[row])[:, None])) + 2.0 ** -14)
    # column sums of an edge tensor, exact accumulation
    t = f16(r.standard_normal((E, 1)) * r.choice([1e-4, 1.0, 50.0], size=(E, 1)))
    t64 = t.astype(np.float64)
    cs = torch.full((ncols, 1), 5.0, dtype=torch.float16, device=dev)
    hgnn.hgnn_edge_colsum(g, p, 1, up(t, dev), cs)
    got = down(cs).copy()
    ref = oracle.edge_colsum(rowptr, col, t64, ncols)
    compare("column sums over slices", got, ref, oracle.edge_colsum(rowptr, col, np.abs(t64), ncols))
    # the sum is exact, so the only error is the output rounding: half an ulp of the result (one more fp32 rounding on the way)
    fin = np.abs(ref) < 65000
    assert np.all(np.abs(got.astype(np.float64) - ref)[fin] <= np.abs(ref[fin]) * 2.0 ** -11 * (1 + 2.0 ** -10) + 2.0 ** -25)
    # order-independent: a second call gives the same bits
    cs.fill_(1.0)
    hgnn.hgnn_edge_colsum(g, p, 1, up(t, dev), cs)
    assert np.array_equal(down(cs).view(np.uint16), got.view(np.uint16))
    # agrees with the row sums over the transposed graph (the other way to the same numbers)
    gt = hgnn.hgnn_transpose(g)
    cs2 = torch.empty((ncols, 1), dtype=torch.float16, device=dev)
    hgnn.hgnn_edge_rowsum(gt, None, 1, up(t, dev), cs2)
    compare("row sums over the transposed graph", down(cs2), ref, oracle.edge_colsum(rowptr, col, np.abs(t64), ncols))
    hgnn.hgnn_plan_destroy(p)


def test_column_sums_special_values_and_errors(hgnn, dev):
    V, ncols = 400, 300
    rowptr, col = rand_graph(V, ncols, 8, 5, hubs=((2, 900),), empties=(0,))
    E = col.size
    r = np.random.default_rng(5)
    t = f16(r.standard_normal((E, 1)))
    # subnormals, the largest finite value, signed zeros, infinities and a nan in chosen columns
    k_sub, k_max, k_inf, k_nan, k_pm = 3, 50, 200, 777, 1200
    t[k_sub, 0] = np.float16(2.0 ** -24)
    t[k_max, 0] = np.float16(65504.0)
    t[k_inf, 0] = np.float16(np.inf)
    t[k_nan, 0] = np.float16(np.nan)
    t[k_pm, 0] = np.float16(-0.0)
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    p = hgnn.hgnn_plan_create(g, 256, 8, 1, col_blocks=1)
    out = torch.empty((ncols, 1), dtype=torch.float16, device=dev)
    with pytest.raises(hgnn.HgnnError) as ei:
        hgnn.hgnn_edge_colsum(g, p, 1, up(t, dev), out)
    assert ei.value.status == hgnn.HGNN_EINVAL and "slices" in str(ei.value)
    hgnn.hgnn_plan_add_slices(p, g, 64)
    with pytest.raises(hgnn.HgnnError) as ei:
        hgnn.hgnn_edge_colsum(g, p, 2, up(t, dev), out)
    assert ei.value.status == hgnn.HGNN_EUNSUPPORTED
    with pytest.raises(hgnn.HgnnError):
        hgnn.hgnn_plan_add_slices(p, g, 63)
    for rep in range(2):  # the side array of non-finite inputs is cleared by the call that used it
        tt = t.copy()
        if rep == 1:
            tt[k_inf, 0] = np.float16(1.0)
            tt[k_nan, 0] = np.float16(1.0)
        hgnn.hgnn_edge_colsum(g, p, 1, up(tt, dev), out)
        got16 = down(out).copy()
        got = got16.astype(np.float64)
        t64 = tt.astype(np.float64)
        ref = oracle.edge_colsum(rowptr, col, t64, ncols)
        assert np.array_equal(np.isnan(got), np.isnan(ref)), rep
        if rep == 0:
            assert np.isnan(ref).sum() == 1 and np.isinf(ref).sum() == 1
        # infinite sums must come out infinite with the right sign, everything else within the output rounding
        compare(f"column sums, special values, call {rep}", got16, ref, oracle.edge_colsum(rowptr, col, np.abs(np.nan_to_num(t64, nan=0.0, posinf=0.0, neginf=0.0)), ncols))
        ok = np.isfinite(ref) & (np.abs(ref) < 65000)
        assert np.all(np.abs(got - ref)[ok] <= np.abs(ref[ok]) * 2.0 ** -11 * (1 + 2.0 ** -10) + 2.0 ** -25), rep
    hgnn.hgnn_plan_destroy(p)


def test_slices_are_added_automatically_for_long_rows(hgnn, dev):
    """hgnn_plan_create(col_blocks = 0) adds the slices where a row's piece of a slice averages 16 non-zeros or more."""
    rowptr, col = rand_graph(600, 20000, 40, 1)   # two slices, rows of 40: pieces of 20
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=20000)
    p = hgnn.hgnn_plan_create(g, 256, 64, 1, col_blocks=0)
    assert hgnn.hgnn_plan_num_slices(p) == 2
    rowptr2, col2 = rand_graph(600, 40000, 20, 2)  # three slices, rows of 20: too short
    g2 = hgnn.Csr(up(rowptr2, dev), up(col2, dev), ncols=40000)
    p2 = hgnn.hgnn_plan_create(g2, 256, 64, 1, col_blocks=0)
    assert hgnn.hgnn_plan_num_slices(p2) == 0
    p3 = hgnn.hgnn_plan_create(g, 256, 64, 1, col_blocks=1)  # nothing automatic asked for
    assert hgnn.hgnn_plan_num_slices(p3) == 0
    for q in (p, p2, p3):
        hgnn.hgnn_plan_destroy(q)


def test_slices_degenerate_graphs(hgnn, dev):
    """No non-zeros, a single row, fewer columns than the narrowest slice, slice widths that do not divide the columns."""
    D = 8
    r = np.random.default_rng(11)
    cases = [("no non-zeros", np.zeros(6, np.int32), np.zeros(0, np.int32), 5, 70, 64),
             ("one row", np.array([0, 40], np.int32), np.sort(r.integers(0, 300, 40)).astype(np.int32), 1, 300, 100),
             ("few columns", *rand_graph(50, 9, 4, 3), 50, 9, 64),
             ("193 columns in slices of 65", *rand_graph(300, 193, 30, 4, hubs=((7, 500),)), 300, 193, 65)]
    for name, rowptr, col, V, ncols, W in cases:
        print("degenerate:", name, flush=True)
        E = col.size
        g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
        p = hgnn.hgnn_plan_create(g, 64, D, 1, col_blocks=1)
        hgnn.hgnn_plan_add_slices(p, g, W)
        t = f16(r.standard_normal((E, 1)))
        out = torch.full((ncols, 1), 3.0, dtype=torch.float16, device=dev)
        hgnn.hgnn_edge_colsum(g, p, 1, up(t, dev) if E else None, out)
        ref = oracle.edge_colsum(rowptr, col, t.astype(np.float64), ncols)
        compare(f"column sums, {name}", down(out), ref, oracle.edge_colsum(rowptr, col, np.abs(t.astype(np.float64)), ncols))
        if E:
            n = max(V, ncols)
            feat = f16(r.standard_normal((n, D)))
            a_l, a_r = f16(0.3 * r.standard_normal(D)), f16(0.3 * r.standard_normal(D))
            e = torch.full((E, 1), 9.0, dtype=torch.float16, device=dev)
            hgnn.hgnn_sddmm(g, p, hgnn.HGNN_SDDMM_GAT_SCORE, 1, D, up(feat[:V], dev), up(feat[:ncols], dev), e, up(a_l, dev), up(a_r, dev), 0.2)
            e_ref = oracle.gat_score(np.concatenate([rowptr, np.full(n - V, rowptr[-1], np.int32)]), col, feat, a_l.reshape(1, D),
                                     a_r.reshape(1, D), 1)
            compare(f"score, {name}", down(e), e_ref, np.abs(e_ref) + 0.5)
        hgnn.hgnn_plan_destroy(p)
