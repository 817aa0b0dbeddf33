"""Seeded random configurations through the main entry points: shapes, segment sizes, column blocks, head counts,
degree mixes and reductions are drawn together, so that combinations no hand-written case lists are exercised.
Every draw is valid input; every result is compared with the CPU fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
import functools

import parity
from parity import down, f16, rand_graph, spmm_plain, up
from test_gpu_gat_fused import bwd_reference, check_lse, gat_backward_check

pytestmark = pytest.mark.gpu

# drawn shapes include graphs of one or two vertices whose results cancel to (nearly) nothing: the sweep alone may take
# the cancelling branch of the norm rule, and every time it does the call is recorded and printed
compare = functools.partial(parity.compare, allow_cancel=True)


def draw(seed):
    r = np.random.default_rng(1000 + seed)
    V = int(r.choice([1, 2, 37, 300, 1111, 2500]))
    avg = float(r.choice([0.3, 2.0, 8.0, 30.0]))
    hubs = tuple((int(r.integers(0, V)), int(r.integers(300, 6000))) for _ in range(int(r.integers(0, 3)))) if V >= 37 else ()
    empties = tuple(int(x) for x in r.integers(0, V, size=int(r.integers(0, 4)))) if V >= 37 else ()
    H, D = [(1, 8), (1, 16), (1, 64), (1, 128), (2, 32), (4, 16), (8, 8), (3, 8), (2, 64), (8, 64), (1, 256)][int(r.integers(0, 11))]
    S = int(r.choice([1, 5, 64, 100, 128, 256, 512]))
    nb = int(r.choice([1, 1, 2, 3, 5])) if V >= 300 else 1
    return dict(V=V, avg=avg, hubs=hubs, empties=empties, H=H, D=D, S=S, nb=nb, reduce=int(r.integers(0, 2)),
                has_w=bool(r.integers(0, 2)), ng=int(r.choice([16, 64, 256])), seed=seed)


@pytest.mark.parametrize("seed", range(128))
def test_random_configuration(hgnn, dev, seed):
    c = draw(seed)
    print(f"sweep {c}", flush=True)
    V, H, D, S, nb = c["V"], c["H"], c["D"], c["S"], c["nb"]
    F = H * D
    rowptr, col = rand_graph(V, V, c["avg"], 77 + seed, hubs=c["hubs"], empties=c["empties"])
    E = col.size
    r = np.random.default_rng(seed)
    X = f16(r.standard_normal((V, F)))
    w = f16(r.standard_normal((E, H))) if c["has_w"] else None
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    p = hgnn.hgnn_plan_create(g, S, F, H, col_blocks=nb)
    Xd = up(X, dev)
    wd = None if w is None else up(w, dev)
    # ---- SpMM: plain, discretized (with the drawn blocks), vertex groups
    ref, sabs = oracle.spmm(rowptr, col, X, w=w, H=H, reduce=c["reduce"], want_sabs=True)
    Y = torch.full((V, F), 7.0, dtype=torch.float16, device=dev)
    spmm_plain(hgnn, g, wd, H, Xd, Y, op=c["reduce"])
    compare("plain", down(Y), ref, sabs)
    Y.fill_(7.0)
    hgnn.hgnn_spmm_discretized(p, g, wd, H, Xd, Y, op=c["reduce"])
    compare("discretized", down(Y), ref, sabs)
    hgnn.hgnn_plan_add_groups(p, g, c["ng"])
    Y.fill_(7.0)
    hgnn.hgnn_spmm_discretized_variant(p, g, wd, H, Xd, Y, hgnn.HGNN_VERTEX_GROUPS, op=c["reduce"])
    compare("vertex groups", down(Y), ref, sabs)
    # ---- SDDMM dot and GAT score, edge softmax of the device's own scores
    a_l, a_r = f16(0.3 * r.standard_normal(F)), f16(0.3 * r.standard_normal(F))
    ald, ard = up(a_l, dev), up(a_r, dev)
    dOut = f16(r.standard_normal((V, F)))
    dOd = up(dOut, dev)
    if E > 0:
        e = torch.full((E, H), 7.0, dtype=torch.float16, device=dev)
        hgnn.hgnn_sddmm(g, p, hgnn.HGNN_SDDMM_DOT, H, D, dOd, Xd, e)
        dref = oracle.sddmm_dot(rowptr, col, dOut, X, H=H)
        row = np.repeat(np.arange(V), np.diff(rowptr))
        dabs = (np.abs(dOut.astype(np.float64)[row]) * np.abs(X.astype(np.float64)[col])).reshape(E, H, D).sum(-1)
        compare("sddmm dot", down(e), dref, dabs)
        hgnn.hgnn_sddmm(g, p, hgnn.HGNN_SDDMM_GAT_SCORE, H, D, Xd, Xd, e, ald, ard, 0.2)
        sref = oracle.gat_score(rowptr, col, X, a_l, a_r, H, slope=0.2)
        got_e = down(e)
        assert np.abs(got_e.astype(np.float64) - sref).max() <= 2e-3 * max(1.0, np.abs(sref).max())
        alpha = torch.full((E, H), 7.0, dtype=torch.float16, device=dev)
        hgnn.hgnn_edge_softmax(g, p, H, e, alpha)
        aref = oracle.edge_softmax(rowptr, got_e.astype(np.float64))
        assert np.abs(down(alpha).astype(np.float64) - aref).max() <= 2e-3
    # ---- fused GAT forward and backward
    oref, lref, oabs = oracle.gat_forward(rowptr, col, X, X, a_l, a_r, H, slope=0.2)
    out = torch.full((V, F), 7.0, dtype=torch.float16, device=dev)
    lse = torch.full((V, H), 7.0, dtype=torch.float32, device=dev)
    hgnn.hgnn_gat_forward_fused(g, p, H, D, Xd, Xd, ald, ard, out, lse)
    compare("gat fused", down(out), oref, oabs)
    check_lse("gat fused", down(lse), lref, np.diff(rowptr))
    hgnn.hgnn_plan_destroy(p)
    (dV, dV_abs), (d_el, el_abs), (d_er, er_abs) = bwd_reference(rowptr, col, V, X, X, a_l, a_r, dOut, H)
    g_dV, g_el, g_er = gat_backward_check(hgnn, dev, rowptr, col, V, X, X, a_l, a_r, dOut, H, S, nb, "sweep")
    # dV of a column is staged in up to nb * (ceil(deg / S) + 1) fp16 pieces; with alpha ~ 1 / (hub degree) the pieces
    # fall below fp16's normal range, where every stored piece is quantised to 2^-24 absolute: one such step per piece
    pieces = nb * (np.ceil(np.bincount(col, minlength=V) / S) + 1)
    compare("dV", g_dV, dV, dV_abs + pieces[:, None] * 2.0 ** -13)
    compare("d_el", g_el, d_el, el_abs, rel_l2=2e-2)
    compare("d_er", g_er, d_er, er_abs, rel_l2=2e-2)


@pytest.mark.parametrize("seed", range(48))
def test_random_plan_and_transpose_bit_exact(hgnn, dev, seed):
    """Integer work on drawn graphs: segment plan (with and without column blocks the top-level arrays are the
    same), transpose with its edge-id map, and the plan of the transpose, each against the oracle bit for bit."""
    c = draw(500 + seed)
    print(f"plan sweep {c}", flush=True)
    V, S, nb = c["V"], c["S"], c["nb"]
    ncols = V + int(np.random.default_rng(seed).integers(0, 40))
    rowptr, col = rand_graph(V, ncols, c["avg"], 900 + seed, hubs=c["hubs"], empties=c["empties"])
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    hgnn.hgnn_csr_validate(g)
    p = hgnn.hgnn_plan_create(g, S, 64, 1, col_blocks=nb)
    got, ref = hgnn.hgnn_plan_export(p), oracle.segment_plan(rowptr, S)
    for k in ref:
        assert np.array_equal(got[k], ref[k]), k
    hgnn.hgnn_plan_destroy(p)
    gt = hgnn.hgnn_transpose(g)
    rT, cT, eT = oracle.transpose(rowptr, col, ncols)
    assert np.array_equal(down(gt.rowptr), rT) and np.array_equal(down(gt.col), cT) and np.array_equal(down(gt.eid), eT)
    pt = hgnn.hgnn_plan_create(gt, S, 64, 1)
    gotT, refT = hgnn.hgnn_plan_export(pt), oracle.segment_plan(rT, S)
    for k in refT:
        assert np.array_equal(gotT[k], refT[k]), k
    hgnn.hgnn_plan_destroy(pt)


@pytest.mark.parametrize("seed", range(24))
def test_random_coo_to_csr_bit_exact(hgnn, dev, seed):
    """A drawn graph's edges in shuffled list order, with the duplicates the generator makes: rowptr, columns and
    the list positions against the oracle bit for bit; the result passes the library's own validation and carries
    an edge tensor given in list order to the right non-zeros."""
    c = draw(700 + seed)
    print(f"coo sweep {c}", flush=True)
    V = c["V"]
    ncols = V + seed % 5
    rowptr, col = rand_graph(V, ncols, c["avg"], 1200 + seed, hubs=c["hubs"], empties=c["empties"])
    E = col.size
    r = np.random.default_rng(seed)
    perm = r.permutation(E)
    row_l, col_l = np.repeat(np.arange(V, dtype=np.int32), np.diff(rowptr))[perm], col[perm]
    ref_rp, ref_col, ref_eid = oracle.coo_to_csr(row_l, col_l, V)
    g, eid = hgnn.hgnn_coo_to_csr(up(row_l, dev), up(col_l, dev), V, ncols)
    assert np.array_equal(down(g.rowptr), ref_rp) and np.array_equal(down(g.col), ref_col)
    assert np.array_equal(down(eid), ref_eid)
    assert np.array_equal(ref_rp, rowptr) and np.array_equal(ref_col, col)  # the graph the list came from
    hgnn.hgnn_csr_validate(g)
    g2, none = hgnn.hgnn_coo_to_csr(up(row_l, dev), up(col_l, dev), V, ncols, want_eid=False)
    assert none is None and np.array_equal(down(g2.col), ref_col)
    if E > 0:  # values given per list entry reach their non-zero through the map
        w_l = f16(r.standard_normal((E, 1)))
        X = f16(r.standard_normal((ncols, 16)))
        ref, sabs = oracle.spmm(rowptr, col, X, w=w_l, eid=ref_eid, want_sabs=True)
        Y = torch.empty((V, 16), dtype=torch.float16, device=dev)
        spmm_plain(hgnn, hgnn.Csr(g.rowptr, g.col, ncols=ncols, eid=eid), up(w_l, dev), 1, up(X, dev), Y)
        compare("values in list order", down(Y), ref, sabs)
        bad = row_l.copy()
        bad[E // 2] = V  # one row id out of range
        with pytest.raises(hgnn.HgnnError):
            hgnn.hgnn_coo_to_csr(up(bad, dev), up(col_l, dev), V, ncols)


def test_coo_to_csr_full_size_round_trip(hgnn, dev):
    """Config 4's 62 M edges as a shuffled list: the library must give the graph back (the columns of the
    generator's CSR are ascending inside a row, so the result is unique up to the order of duplicate edges, which
    the edge-id map must resolve in list order)."""
    import workloads as wl
    w = wl.gcn_large()
    print(f"coo full size {w.name}: E = {w.col.size}", flush=True)
    E, V = w.col.size, w.V
    perm = torch.randperm(E, device=dev, generator=torch.Generator(device=dev).manual_seed(3))
    row = torch.repeat_interleave(torch.arange(V, dtype=torch.int32, device=dev),
                                  torch.from_numpy(np.diff(w.rowptr)).to(dev))
    col = up(w.col, dev)
    g, eid = hgnn.hgnn_coo_to_csr(row[perm].contiguous(), col[perm].contiguous(), V, V)
    assert torch.equal(g.rowptr, up(w.rowptr, dev)) and torch.equal(g.col, col)
    # eid[k] is a list position holding the same (row, col) pair, every position once, duplicates in list order
    back = perm[eid.long()]  # position in the original CSR of the list entry chosen for CSR slot k
    assert torch.equal(col[back], col) and torch.equal(row[back], row)
    assert torch.equal(torch.sort(eid).values, torch.arange(E, dtype=torch.int32, device=dev))
    same = (row[1:] == row[:-1]) & (col[1:] == col[:-1])
    assert bool(torch.all(eid[1:][same] > eid[:-1][same]))
    hgnn.hgnn_csr_validate(g)


def test_coo_to_csr_degenerate_lists(hgnn, dev):
    empty = torch.empty(0, dtype=torch.int32, device=dev)
    g, eid = hgnn.hgnn_coo_to_csr(empty, empty, 5, 3)
    assert down(g.rowptr).tolist() == [0] * 6 and g.nnz == 0 and eid.numel() == 0
    g, eid = hgnn.hgnn_coo_to_csr(empty, empty, 0, 0)
    assert down(g.rowptr).tolist() == [0]
    # one pair repeated: the list order is the only order there is
    row = torch.full((1000,), 2, dtype=torch.int32, device=dev)
    col = torch.full((1000,), 1, dtype=torch.int32, device=dev)
    g, eid = hgnn.hgnn_coo_to_csr(row, col, 4, 2)
    assert down(g.rowptr).tolist() == [0, 0, 0, 1000, 1000] and np.all(down(g.col) == 1)
    assert np.array_equal(down(eid), np.arange(1000, dtype=np.int32))
    # the largest ids of a graph whose sizes are not powers of two, and a negative id
    row = torch.tensor([4, 0, 4], dtype=torch.int32, device=dev)
    col = torch.tensor([6, 6, 0], dtype=torch.int32, device=dev)
    g, eid = hgnn.hgnn_coo_to_csr(row, col, 5, 7)
    assert down(g.rowptr).tolist() == [0, 1, 1, 1, 1, 3] and down(g.col).tolist() == [6, 0, 6] and down(eid).tolist() == [1, 2, 0]
    with pytest.raises(hgnn.HgnnError):
        hgnn.hgnn_coo_to_csr(row, torch.tensor([6, -1, 0], dtype=torch.int32, device=dev), 5, 7)
    with pytest.raises(hgnn.HgnnError):
        hgnn.hgnn_coo_to_csr(row, torch.tensor([7, 6, 0], dtype=torch.int32, device=dev), 5, 7)
