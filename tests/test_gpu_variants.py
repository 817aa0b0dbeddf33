"""GPU parity of the comparison variants of the discretized SpMM (vertex-parallel neighbour groups,
atomic conflict writes) against the CPU fp64 oracle, and of the neighbour-group lists, bit exact."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from parity import compare, down, f16, rand_graph, sample_rows, spmm_plain, up

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("ng", [1, 7, 32, 64, 256, 1024])
def test_neighbor_groups_bit_exact(hgnn, dev, ng):
    print(f"groups ng={ng}", flush=True)
    rowptr, col = rand_graph(3000, 3000, 9, 1, hubs=((17, 5000), (2999, 700), (40, ng), (41, ng + 1)),
                             empties=(0, 18, 2998))
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    p = hgnn.hgnn_plan_create(g, 256, 64, 1)
    assert hgnn.hgnn_plan_num_groups(p) == 0 and hgnn.hgnn_plan_group_edges(p) == 0
    hgnn.hgnn_plan_add_groups(p, g, ng)
    ref_row, ref_first = oracle.neighbor_groups(rowptr, ng)
    row, first = hgnn.hgnn_plan_groups_export(p, g)
    assert hgnn.hgnn_plan_num_groups(p) == ref_row.size and hgnn.hgnn_plan_group_edges(p) == ng
    assert np.array_equal(row, ref_row) and np.array_equal(first, ref_first)
    # rebuilding with another size replaces the lists
    hgnn.hgnn_plan_add_groups(p, g, 2 * ng if ng < 1024 else 3)
    ref_row, ref_first = oracle.neighbor_groups(rowptr, 2 * ng if ng < 1024 else 3)
    row, first = hgnn.hgnn_plan_groups_export(p, g)
    assert np.array_equal(row, ref_row) and np.array_equal(first, ref_first)
    hgnn.hgnn_plan_destroy(p)


def test_neighbor_groups_of_an_empty_graph(hgnn, dev):
    rowptr = np.zeros(11, dtype=np.int32)
    g = hgnn.Csr(up(rowptr, dev), torch.empty(0, dtype=torch.int32, device=dev))
    p = hgnn.hgnn_plan_create(g, 256, 64, 1)
    hgnn.hgnn_plan_add_groups(p, g, 64)
    assert hgnn.hgnn_plan_num_groups(p) == 0
    X = torch.ones((10, 64), dtype=torch.float16, device=dev)
    Y = torch.full((10, 64), 5.0, dtype=torch.float16, device=dev)
    hgnn.hgnn_spmm_discretized_variant(p, g, None, 1, X, Y, hgnn.HGNN_VERTEX_GROUPS)
    assert np.all(down(Y) == 0)
    hgnn.hgnn_plan_destroy(p)


VSHAPES = [  # (F, H, has_w, reduce, ng, pad)
    (64, 1, True, 0, 64, 0), (64, 1, False, 1, 256, 0), (128, 1, True, 1, 256, 8), (32, 1, True, 0, 32, 0),
    (16, 1, False, 0, 512, 0), (8, 1, True, 0, 7, 0), (256, 1, False, 0, 64, 0), (512, 1, True, 1, 1024, 0),
    (64, 4, True, 0, 64, 0), (128, 8, True, 1, 100, 0), (48, 1, True, 0, 64, 0), (64, 1, True, 0, 1, 0),
]


@pytest.mark.parametrize("F,H,has_w,reduce,ng,pad", VSHAPES)
def test_vertex_groups_shapes(hgnn, dev, F, H, has_w, reduce, ng, pad):
    print(f"vgroups F={F} H={H} w={has_w} reduce={reduce} ng={ng} pad={pad}", flush=True)
    V, ncols = 1237, 997
    rowptr, col = rand_graph(V, ncols, 11, F + ng, hubs=((5, 5000), (700, 777), (1236, 300)), empties=(0, 6, 1235))
    E = col.size
    r = np.random.default_rng(F * 7 + H)
    Xh = f16(r.standard_normal((ncols, F + pad)))
    w = f16(r.standard_normal((E, H))) if has_w else None
    rs = r.uniform(0.5, 2.0, V).astype(np.float32)
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    Xd = up(Xh, dev)[:, :F]
    ref, sabs = oracle.spmm(rowptr, col, Xh[:, :F], w=w, H=H, reduce=reduce, row_scale=rs.astype(np.float64),
                            want_sabs=True)
    p = hgnn.hgnn_plan_create(g, 256, max(F, 8), H)
    hgnn.hgnn_plan_add_groups(p, g, ng)
    Yfull = torch.full((V, F + pad), 7.0, dtype=torch.float16, device=dev)
    Y = Yfull[:, :F]
    bits = []
    # edge values at a 4-byte aligned base (pair fetch) and at an odd element offset (element fetch)
    for shift in ((0, 1) if has_w else (0,)):
        wd = None
        if has_w:
            buf = torch.zeros(E * H + 1, dtype=torch.float16, device=dev)
            buf[shift:shift + E * H] = up(w, dev).reshape(-1)
            wd = buf[shift:shift + E * H].view(E, H)
        Y.fill_(7.0)
        hgnn.hgnn_spmm_discretized_variant(p, g, wd, H, Xd, Y, hgnn.HGNN_VERTEX_GROUPS, op=reduce, row_scale=up(rs, dev))
        got = down(Y)
        compare(f"vertex groups shift={shift}", got, ref, sabs)
        bits.append(got.view(np.uint16).copy())
    Y.fill_(-3.0)
    hgnn.hgnn_spmm_discretized_variant(p, g, wd, H, Xd, Y, hgnn.HGNN_VERTEX_GROUPS, op=reduce, row_scale=up(rs, dev))
    assert all(np.array_equal(down(Y).view(np.uint16), b) for b in bits)  # deterministic, whatever the fetch path
    if pad:
        assert np.all(down(Yfull)[:, F:] == 7.0)
    hgnn.hgnn_plan_destroy(p)


@pytest.mark.parametrize("F,H,has_w,reduce,ng", [(64, 1, True, 0, 64), (64, 1, False, 1, 256), (128, 1, True, 0, 128),
                                                 (32, 4, True, 1, 64), (16, 1, False, 0, 32), (256, 1, True, 0, 512)])
def test_vertex_groups_half2_arithmetic(hgnn, dev, F, H, has_w, reduce, ng):
    """The paper's packed-fp16 products and sums (section 4.2) inside a lane's share of a neighbour group.  The result
    carries fp16 accumulation error: one rounding per term at the magnitude of the lane's running sum, so the floor of
    the elementwise rule grows by the number of edges a lane adds up (its chunk), and the rel-L2 band is 2e-2."""
    print(f"vgroups half2 F={F} H={H} w={has_w} reduce={reduce} ng={ng}", flush=True)
    V, ncols = 1100, 900
    rowptr, col = rand_graph(V, ncols, 11, F + ng, hubs=((5, 5000), (700, 777)), empties=(0, 6, 1099))
    E = col.size
    r = np.random.default_rng(F * 3 + H)
    Xh = f16(r.standard_normal((ncols, F)))
    w = f16(r.standard_normal((E, H))) if has_w else None
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    ref, sabs = oracle.spmm(rowptr, col, Xh, w=w, H=H, reduce=reduce, want_sabs=True)
    p = hgnn.hgnn_plan_create(g, 256, max(F, 8), H)
    hgnn.hgnn_plan_add_groups(p, g, ng)
    Y = torch.full((V, F), 7.0, dtype=torch.float16, device=dev)
    wd = None if w is None else up(w, dev)
    hgnn.hgnn_spmm_discretized_variant(p, g, wd, H, up(Xh, dev), Y, hgnn.HGNN_VERTEX_GROUPS_HALF2, op=reduce)
    got = down(Y)
    lanes_per_row = 1
    while lanes_per_row < (F + 7) // 8:
        lanes_per_row *= 2
    chunk = 4 * -(-ng // (4 * (64 // lanes_per_row)))  # edges one lane adds up
    compare("vertex groups half2", got, ref, sabs * (1 + chunk), rel_l2=2e-2)
    # and it is not simply the fp32 kernel: some outputs differ in their last bits
    Y2 = torch.empty_like(Y)
    hgnn.hgnn_spmm_discretized_variant(p, g, wd, H, up(Xh, dev), Y2, hgnn.HGNN_VERTEX_GROUPS, op=reduce)
    assert not np.array_equal(down(Y2).view(np.uint16), got.view(np.uint16))
    compare("vertex groups fp32", down(Y2), ref, sabs)
    # deterministic
    Y3 = torch.empty_like(Y)
    hgnn.hgnn_spmm_discretized_variant(p, g, wd, H, up(Xh, dev), Y3, hgnn.HGNN_VERTEX_GROUPS_HALF2, op=reduce)
    assert np.array_equal(down(Y3).view(np.uint16), got.view(np.uint16))
    hgnn.hgnn_plan_destroy(p)


@pytest.mark.parametrize("F,H,has_w,reduce,S", [(64, 1, True, 0, 256), (128, 1, False, 1, 128), (64, 4, True, 1, 64),
                                                (32, 1, True, 0, 7)])
def test_atomic_variant_shapes(hgnn, dev, F, H, has_w, reduce, S):
    print(f"atomic F={F} H={H} w={has_w} reduce={reduce} S={S}", flush=True)
    V, ncols = 1237, 997
    rowptr, col = rand_graph(V, ncols, 11, F + S, hubs=((5, 5000), (700, 777), (1236, 300)), empties=(0, 6, 1235))
    r = np.random.default_rng(F * 7 + H)
    Xh = f16(r.standard_normal((ncols, F)))
    w = f16(r.standard_normal((col.size, H))) if has_w else None
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    wd = None if w is None else up(w, dev)
    ref, sabs = oracle.spmm(rowptr, col, Xh, w=w, H=H, reduce=reduce, want_sabs=True)
    p = hgnn.hgnn_plan_create(g, S, F, H)
    Y = torch.full((V, F), 7.0, dtype=torch.float16, device=dev)
    hgnn.hgnn_spmm_discretized_variant(p, g, wd, H, up(Xh, dev), Y, hgnn.HGNN_EDGE_SEGMENTS_ATOMIC, op=reduce)
    got = down(Y)
    # every addition into a split row rounds to fp16 at the magnitude of the running sum: allow one such
    # rounding per piece on top of the usual rule
    pieces = np.maximum((rowptr[1:] - 1) // S - rowptr[:-1] // S, 0)[:, None]
    compare("atomic", got, ref, sabs * (1 + pieces))
    # rows inside one segment never meet an atomic: bit-identical to the staged design
    Y2 = torch.empty_like(Y)
    hgnn.hgnn_spmm_discretized_variant(p, g, wd, H, up(Xh, dev), Y2, hgnn.HGNN_EDGE_SEGMENTS, op=reduce)
    whole = (pieces[:, 0] == 0)
    assert np.array_equal(got[whole].view(np.uint16), down(Y2)[whole].view(np.uint16))
    hgnn.hgnn_plan_destroy(p)


def test_vertex_groups_on_the_transposed_graph_with_edge_ids(hgnn, dev):
    V, ncols, F, H = 900, 1100, 64, 2
    rowptr, col = rand_graph(V, ncols, 14, 3, hubs=((9, 1500),), empties=(2,))
    r = np.random.default_rng(5)
    w = f16(r.standard_normal((col.size, H)))
    dY = f16(r.standard_normal((V, F)))
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    gt = hgnn.hgnn_transpose(g)
    rT, cT, eT = down(gt.rowptr), down(gt.col), down(gt.eid)
    ref, sabs = oracle.spmm(rT, cT, dY, w=w, H=H, eid=eT, want_sabs=True)
    pt = hgnn.hgnn_plan_create(gt, 256, F, H)
    hgnn.hgnn_plan_add_groups(pt, gt, 64)
    dX = torch.empty((ncols, F), dtype=torch.float16, device=dev)
    hgnn.hgnn_spmm_discretized_variant(pt, gt, up(w, dev), H, up(dY, dev), dX, hgnn.HGNN_VERTEX_GROUPS)
    compare("vgroups transposed", down(dX), ref, sabs)
    hgnn.hgnn_plan_destroy(pt)


def test_vertex_groups_do_not_overflow_where_naive_fp16_does(hgnn, dev):
    """Config 2b (all-positive features, hubs > 10^4): per-group scaling keeps every stored partial in range."""
    w = wl.gin_overflow(positive=True)
    g = hgnn.Csr(up(w.rowptr, dev), up(w.col, dev))
    p = hgnn.hgnn_plan_create(g, 256, w.F, 1)
    hgnn.hgnn_plan_add_groups(p, g, 64)
    X = up(w.tensors["X"], dev)
    Y = torch.empty((w.V, w.F), dtype=torch.float16, device=dev)
    hgnn.hgnn_spmm_discretized_variant(p, g, None, 1, X, Y, hgnn.HGNN_VERTEX_GROUPS, op=hgnn.HGNN_MEAN)
    got = down(Y)
    assert np.all(np.isfinite(got))
    rows = sample_rows(w.rowptr, 400, 11)
    ref, sabs = oracle.spmm(w.rowptr, w.col, w.tensors["X"], reduce=oracle.MEAN, rows=rows, want_sabs=True)
    compare("c2b vertex groups mean", got[rows], ref, sabs)
    _, maxpart = oracle.spmm_discretized(w.rowptr, w.col, w.tensors["X"], 64, reduce=oracle.MEAN, rows=rows, by_row=True)
    assert maxpart <= 8.0
    hgnn.hgnn_plan_destroy(p)


def test_variant_argument_errors(hgnn, dev):
    rowptr, col = rand_graph(50, 50, 4, 2)
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    p = hgnn.hgnn_plan_create(g, 64, 64, 1)
    X = torch.ones((50, 64), dtype=torch.float16, device=dev)
    Y = torch.empty_like(X)
    with pytest.raises(hgnn.HgnnError) as ei:
        hgnn.hgnn_spmm_discretized_variant(p, g, None, 1, X, Y, hgnn.HGNN_VERTEX_GROUPS)
    assert ei.value.status == hgnn.HGNN_EINVAL and "neighbour groups" in str(ei.value)
    with pytest.raises(hgnn.HgnnError) as ei:
        hgnn.hgnn_spmm_discretized_variant(p, g, None, 1, X, Y, 9)
    assert ei.value.status == hgnn.HGNN_EINVAL
    for bad in (0, 1025):
        with pytest.raises(hgnn.HgnnError) as ei:
            hgnn.hgnn_plan_add_groups(p, g, bad)
        assert ei.value.status == hgnn.HGNN_EINVAL
    hgnn.hgnn_plan_destroy(p)


# ------------------------------------------------------------------ feature lengths that are not multiples of 8
@pytest.mark.parametrize("F", [2, 6, 8, 14, 42, 48, 130])
def test_padded_feature_lengths(hgnn, dev, F):
    """Class counts such as 7, 41, 47 (Table 1) padded to the next even number: rows keep a pitch that is a
    multiple of 8 halves, the padding columns hold NaN on input and must come back untouched on output."""
    print(f"padded F={F}", flush=True)
    V, ncols = 700, 640
    pitch = (F + 7) // 8 * 8 + 8
    rowptr, col = rand_graph(V, ncols, 9, F, hubs=((5, 3000), (300, 400)), empties=(0, 6, 699))
    E = col.size
    r = np.random.default_rng(F)
    Xh = np.full((ncols, pitch), np.nan, dtype=np.float16)
    Xh[:, :F] = f16(r.standard_normal((ncols, F)))
    Uh = np.full((V, pitch), np.nan, dtype=np.float16)
    Uh[:, :F] = f16(r.standard_normal((V, F)))
    w = f16(r.standard_normal((E, 1)))
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    Xd, Ud, wd = up(Xh, dev), up(Uh, dev), up(w, dev)
    ref, sabs = oracle.spmm(rowptr, col, Xh[:, :F], w=w, reduce=oracle.MEAN, want_sabs=True)
    Yfull = torch.full((V, pitch), 7.0, dtype=torch.float16, device=dev)
    Y = Yfull[:, :F]

    def check(name):
        got = down(Yfull)
        compare(name, got[:, :F], ref, sabs)
        assert np.all(got[:, F:] == 7.0), f"{name}: padding columns written"
        Yfull.fill_(7.0)

    spmm_plain(hgnn, g, wd, 1, Xd[:, :F], Y, op=hgnn.HGNN_MEAN)
    check("plain")
    for nb in (1, 3):
        p = hgnn.hgnn_plan_create(g, 64, pitch, 1, col_blocks=nb)
        hgnn.hgnn_spmm_discretized(p, g, wd, 1, Xd[:, :F], Y, op=hgnn.HGNN_MEAN)
        check(f"discretized nb={nb}")
        if nb == 1:
            hgnn.hgnn_spmm_discretized_variant(p, g, wd, 1, Xd[:, :F], Y, hgnn.HGNN_EDGE_SEGMENTS_ATOMIC, op=hgnn.HGNN_MEAN)
            pieces = np.maximum((rowptr[1:] - 1) // 64 - rowptr[:-1] // 64, 0)[:, None]
            got = down(Yfull)
            compare("atomic", got[:, :F], ref, sabs * (1 + pieces))
            assert np.all(got[:, F:] == 7.0)
            Yfull.fill_(7.0)
            hgnn.hgnn_plan_add_groups(p, g, 64)
            hgnn.hgnn_spmm_discretized_variant(p, g, wd, 1, Xd[:, :F], Y, hgnn.HGNN_VERTEX_GROUPS, op=hgnn.HGNN_MEAN)
            check("vertex groups")
        # GIN epilogue with the self term read from a padded table
        gin_ref, gin_sabs = oracle.spmm(rowptr, col, Xh[:ncols, :F], w=w, reduce=oracle.MEAN, self_feat=Uh[:, :F],
                                        self_coef=1.25, agg_coef=0.1, want_sabs=True)
        hgnn.hgnn_spmm_discretized_fused(p, g, wd, 1, Xd[:, :F], Y, op=hgnn.HGNN_MEAN, self_feat=Ud[:, :F], self_coef=1.25,
                                         agg_coef=0.1)
        got = down(Yfull)
        compare(f"gin epilogue nb={nb}", got[:, :F], gin_ref, gin_sabs)
        assert np.all(got[:, F:] == 7.0)
        Yfull.fill_(7.0)
        # SDDMM dot, one head of length F
        e = torch.full((E, 1), 3.0, dtype=torch.float16, device=dev)
        hgnn.hgnn_sddmm(g, p, hgnn.HGNN_SDDMM_DOT, 1, F, Ud[:, :F], Xd[:, :F], e)
        row = np.repeat(np.arange(V), np.diff(rowptr))
        dref = oracle.sddmm_dot(rowptr, col, Uh[:, :F], Xh[:, :F], H=1)
        dabs = np.einsum("ef,ef->e", np.abs(Uh[row, :F].astype(np.float64)), np.abs(Xh[col, :F].astype(np.float64)))[:, None]
        compare(f"sddmm dot nb={nb}", down(e), dref, dabs)
        hgnn.hgnn_plan_destroy(p)


# ------------------------------------------------------------------ vector-width study: 2, 4, 8 halves per lane
@pytest.mark.parametrize("F,H", [(16, 1), (32, 1), (64, 1), (128, 1), (64, 4), (128, 8), (256, 2)])
def test_vector_width_variants(hgnn, dev, F, H):
    print(f"width F={F} H={H}", flush=True)
    V, ncols = 900, 800
    rowptr, col = rand_graph(V, ncols, 10, F + H, hubs=((5, 2500), (300, 300)), empties=(0, 899))
    E = col.size
    r = np.random.default_rng(F + H)
    Xh, Uh = f16(r.standard_normal((ncols, F))), f16(r.standard_normal((V, F)))
    w = f16(r.standard_normal((E, H)))
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    Xd, Ud, wd = up(Xh, dev), up(Uh, dev), up(w, dev)
    ref, sabs = oracle.spmm(rowptr, col, Xh, w=w, H=H, want_sabs=True)
    dref = oracle.sddmm_dot(rowptr, col, Uh, Xh, H=H)
    row = np.repeat(np.arange(V), np.diff(rowptr))
    D = F // H
    dabs = (np.abs(Uh[row].astype(np.float64)) * np.abs(Xh[col].astype(np.float64))).reshape(E, H, D).sum(-1)
    p = hgnn.hgnn_plan_create(g, 256, F, H, col_blocks=1)
    hgnn.hgnn_plan_add_groups(p, g, 64)
    Y = torch.empty((V, F), dtype=torch.float16, device=dev)
    e = torch.empty((E, H), dtype=torch.float16, device=dev)
    for vw in (2, 4, 8):
        hgnn.hgnn_plan_set_vector_halves(p, vw)
        assert hgnn.hgnn_plan_vector_halves(p) == vw
        fits = F <= 64 * vw and D % vw == 0
        if not fits:
            with pytest.raises(hgnn.HgnnError) as ei:
                hgnn.hgnn_spmm_discretized_variant(p, g, wd, H, Xd, Y, hgnn.HGNN_VERTEX_GROUPS)
            assert ei.value.status == hgnn.HGNN_EUNSUPPORTED
            continue
        Y.fill_(7.0)
        hgnn.hgnn_spmm_discretized_variant(p, g, wd, H, Xd, Y, hgnn.HGNN_VERTEX_GROUPS)
        compare(f"vertex groups, {vw} halves per lane", down(Y), ref, sabs)
        e.fill_(7.0)
        hgnn.hgnn_sddmm(g, p, hgnn.HGNN_SDDMM_DOT, H, D, Ud, Xd, e)
        compare(f"sddmm dot, {vw} halves per lane", down(e), dref, dabs)
    with pytest.raises(hgnn.HgnnError):
        hgnn.hgnn_plan_set_vector_halves(p, 3)
    # the width belongs to the plan: a second plan of the same graph keeps the default
    p2 = hgnn.hgnn_plan_create(g, 256, F, H, col_blocks=1)
    assert hgnn.hgnn_plan_vector_halves(p2) == 8 and hgnn.hgnn_plan_vector_halves(p) == 8
    hgnn.hgnn_plan_destroy(p2)
    hgnn.hgnn_plan_destroy(p)


# ------------------------------------------------------------------ feature tables of 4 GiB and more (64-bit row addresses)
def test_feature_table_beyond_4gib(hgnn, dev):
    """Below 4 GiB the kernels address neighbour rows with 32-bit byte offsets from a scalar base; this table is
    larger, so every segment kernel takes its 64-bit path.  Only the referenced rows are filled; the oracle
    works on the compacted table."""
    ncols, pitch, F, H = (1 << 21) + 64, 1024, 64, 1  # 2^21 rows of 2 KiB
    V = 600
    r = np.random.default_rng(12)
    rowptr, col_small = rand_graph(V, 5000, 10, 7, hubs=((3, 1500),), empties=(1,))
    pick = np.sort(r.choice(ncols, size=5000, replace=False)).astype(np.int64)
    pick[-1] = ncols - 1  # the very last row of the table is referenced
    col = pick[col_small].astype(np.int32)  # ascending inside a row is preserved (pick is increasing)
    Xs = f16(r.standard_normal((5000, F)))
    w = f16(r.standard_normal((col.size, 1)))
    ref, sabs = oracle.spmm(rowptr, col_small, Xs, w=w, reduce=oracle.MEAN, want_sabs=True)
    Xbig = torch.zeros((ncols, pitch), dtype=torch.float16, device=dev)
    assert Xbig.numel() * 2 >= (1 << 32)
    Xbig[torch.from_numpy(pick).to(dev), :F] = up(Xs, dev)
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    p = hgnn.hgnn_plan_create(g, 256, F, H)
    Y = torch.empty((V, F), dtype=torch.float16, device=dev)
    X = Xbig[:, :F]
    spmm_plain(hgnn, g, up(w, dev), 1, X, Y, op=hgnn.HGNN_MEAN)
    compare("plain, 64-bit rows", down(Y), ref, sabs)
    hgnn.hgnn_spmm_discretized(p, g, up(w, dev), 1, X, Y, op=hgnn.HGNN_MEAN)
    compare("discretized, 64-bit rows", down(Y), ref, sabs)
    hgnn.hgnn_plan_add_groups(p, g, 64)
    hgnn.hgnn_spmm_discretized_variant(p, g, up(w, dev), 1, X, Y, hgnn.HGNN_VERTEX_GROUPS, op=hgnn.HGNN_MEAN)
    compare("vertex groups, 64-bit rows", down(Y), ref, sabs)
    # fused GAT with the big table on the column side: one head (staged scores) and four (scores formed in the
    # main loop); the backward's forward-graph pass gathers rows of the big table too
    U = f16(r.standard_normal((V, F)))
    a_l, a_r = f16(0.2 * r.standard_normal(F)), f16(0.2 * r.standard_normal(F))
    dOut = f16(r.standard_normal((V, F)))
    gt = hgnn.hgnn_transpose(g)
    pick_d = torch.from_numpy(pick).to(dev)
    for Hg in (1, 4):
        pg = hgnn.hgnn_plan_create(g, 256, F, Hg)
        pt = hgnn.hgnn_plan_create(gt, 256, F, Hg)
        gref, gl, gabs = oracle.gat_forward(rowptr, col_small, U, Xs, a_l, a_r, Hg)
        lse = torch.empty((V, Hg), dtype=torch.float32, device=dev)
        hgnn.hgnn_gat_forward_fused(g, pg, Hg, F // Hg, up(U, dev), X, up(a_l, dev), up(a_r, dev), Y, lse)
        compare(f"gat fused, 64-bit rows, H={Hg}", down(Y), gref, gabs)
        dV = torch.zeros((ncols, F), dtype=torch.float16, device=dev)
        d_el = torch.empty((V, Hg), dtype=torch.float16, device=dev)
        d_er = torch.empty((ncols, Hg), dtype=torch.float16, device=dev)
        hgnn.hgnn_gat_backward_fused(g, pg, gt, pt, Hg, F // Hg, up(U, dev), X, up(a_l, dev), up(a_r, dev), Y, lse,
                                     up(dOut, dev), dV, d_el, d_er)
        bV, b_el, b_er = oracle.gat_backward(rowptr, col_small, U, Xs, a_l, a_r, dOut, Hg)
        scale = np.abs(bV).max()
        assert np.max(np.abs(down(dV[pick_d]).astype(np.float64) - bV)) <= 2e-2 * scale
        assert np.max(np.abs(down(d_er[pick_d]).astype(np.float64) - b_er)) <= 2e-2 * max(np.abs(b_er).max(), 1e-3)
        assert np.max(np.abs(down(d_el).astype(np.float64) - b_el)) <= 2e-2 * max(np.abs(b_el).max(), 1e-3)
        hgnn.hgnn_plan_destroy(pt)
        hgnn.hgnn_plan_destroy(pg)
    # SDDMM dot against the big table
    e = torch.empty((col.size, 1), dtype=torch.float16, device=dev)
    hgnn.hgnn_sddmm(g, p, hgnn.HGNN_SDDMM_DOT, 1, F, up(U, dev), X, e)
    dref = oracle.sddmm_dot(rowptr, col_small, U, Xs, H=1)
    row = np.repeat(np.arange(V), np.diff(rowptr))
    dabs = (np.abs(U[row].astype(np.float64)) * np.abs(Xs[col_small].astype(np.float64))).sum(-1, keepdims=True)
    compare("sddmm dot, 64-bit rows", down(e), dref, dabs)
    hgnn.hgnn_plan_destroy(p)
    del Xbig
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ static edge values in transposed order
@pytest.mark.parametrize("H", [1, 4])
def test_edge_to_transposed_and_backward_without_edge_ids(hgnn, dev, H):
    V, ncols, F = 800, 900, 64
    rowptr, col = rand_graph(V, ncols, 11, 4 + H, hubs=((7, 3000),), empties=(3,))
    r = np.random.default_rng(H)
    w = f16(r.standard_normal((col.size, H)))
    dY = f16(r.standard_normal((V, F)))
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    gt = hgnn.hgnn_transpose(g)
    eT = down(gt.eid)
    wT = torch.empty((col.size, H), dtype=torch.float16, device=dev)
    hgnn.hgnn_edge_to_transposed(gt, H, up(w, dev), wT)
    assert np.array_equal(down(wT).view(np.uint16), oracle.edge_gather(eT, w).view(np.uint16))  # a permutation: bit exact
    # the backward SpMM on the transposed graph without its edge-id map, reading wT as a stream
    gt_plain = hgnn.Csr(gt.rowptr, gt.col, ncols=V)
    pt = hgnn.hgnn_plan_create(gt, 256, F, H)
    a = torch.empty((ncols, F), dtype=torch.float16, device=dev)
    b = torch.empty_like(a)
    hgnn.hgnn_spmm_discretized(pt, gt, up(w, dev), H, up(dY, dev), a)
    hgnn.hgnn_spmm_discretized(pt, gt_plain, wT, H, up(dY, dev), b)
    assert np.array_equal(down(a).view(np.uint16), down(b).view(np.uint16))  # same edges in the same order
    ref, sabs = oracle.spmm(down(gt.rowptr), down(gt.col), dY, w=w, H=H, eid=eT, want_sabs=True)
    compare("backward with pre-permuted values", down(b), ref, sabs)
    with pytest.raises(hgnn.HgnnError):
        hgnn.hgnn_edge_to_transposed(g, H, up(w, dev), wT)  # no edge-id map
    hgnn.hgnn_plan_destroy(pt)


def test_scale_rows_then_unweighted_spmm_is_the_column_norm(hgnn, dev):
    """Eq. 2 with the column-side norm applied to the table first: the same as col_scale in the fused call, up to
    one fp16 rounding of every scaled feature."""
    V, ncols, F = 500, 600, 64
    rowptr, col = rand_graph(V, ncols, 10, 5, hubs=((4, 2000),), empties=(9,))
    r = np.random.default_rng(3)
    X = f16(r.standard_normal((ncols, F)))
    cs = r.uniform(0.05, 1.0, ncols).astype(np.float32)
    rs = r.uniform(0.05, 1.0, V).astype(np.float32)
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    p = hgnn.hgnn_plan_create(g, 256, F, 1)
    Xs = torch.empty((ncols, F), dtype=torch.float16, device=dev)
    hgnn.hgnn_scale_rows(up(X, dev), up(cs, dev), Xs)
    want = (cs[:, None] * X.astype(np.float32)).astype(np.float16)  # fp32 product, then one RNE rounding to fp16
    assert np.array_equal(down(Xs).view(np.uint16), want.view(np.uint16))
    Y = torch.empty((V, F), dtype=torch.float16, device=dev)
    hgnn.hgnn_spmm_discretized(p, g, None, 1, Xs, Y, row_scale=up(rs, dev))
    ref, sabs = oracle.spmm(rowptr, col, X, row_scale=rs.astype(np.float64), col_scale=cs.astype(np.float64), want_sabs=True)
    compare("pre-scaled column norm", down(Y), ref, 2 * sabs)  # the extra rounding of the scaled table
    hgnn.hgnn_plan_destroy(p)


# ------------------------------------------------------------------ per-head edge values: vector and element-wise staging
@pytest.mark.parametrize("H", [2, 4, 8])
@pytest.mark.parametrize("shift", [0, 1])
def test_edge_values_with_heads_aligned_or_not(hgnn, dev, H, shift):
    """The segment kernel reads the H values of an edge as one 4-, 8- or 16-byte vector when the tensor's base
    allows it and one by one otherwise (shift = 1: the tensor starts one half past an aligned address).  Forward
    (values in edge order), transposed (through the edge-id map) and column-blocked (through per-row offsets)."""
    print(f"edge values H={H} shift={shift}", flush=True)
    V, ncols, F = 700, 650, 64
    rowptr, col = rand_graph(V, ncols, 14, 90 + H, hubs=((3, 2500), (600, 400)), empties=(0, 9))
    E = col.size
    r = np.random.default_rng(100 + H)
    Xh, dYh = f16(r.standard_normal((ncols, F))), f16(r.standard_normal((V, F)))
    w = f16(r.standard_normal((E, H)))
    buf = torch.zeros(E * H + 8, dtype=torch.float16, device=dev)
    wd = buf[shift:shift + E * H].view(E, H)
    wd.copy_(up(w, dev))
    assert (wd.data_ptr() % 16 == 0) == (shift == 0)
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    gt = hgnn.hgnn_transpose(g)
    ref, sabs = oracle.spmm(rowptr, col, Xh, w=w, H=H, want_sabs=True)
    refb, sabsb = oracle.spmm(down(gt.rowptr), down(gt.col), dYh, w=w, H=H, eid=down(gt.eid), want_sabs=True)
    for nb in (1, 3):
        p = hgnn.hgnn_plan_create(g, 256, F, H, col_blocks=nb)
        pt = hgnn.hgnn_plan_create(gt, 256, F, H, col_blocks=nb)
        Y = torch.empty((V, F), dtype=torch.float16, device=dev)
        hgnn.hgnn_spmm_discretized(p, g, wd, H, up(Xh, dev), Y)
        compare(f"forward, {nb} block(s)", down(Y), ref, sabs)
        dX = torch.empty((ncols, F), dtype=torch.float16, device=dev)
        hgnn.hgnn_spmm_discretized(pt, gt, wd, H, up(dYh, dev), dX)
        compare(f"transposed, {nb} block(s)", down(dX), refb, sabsb)
        hgnn.hgnn_plan_destroy(p)
        hgnn.hgnn_plan_destroy(pt)


# ------------------------------------------------------------------ plan-free SpMM at its row-length thresholds
@pytest.mark.parametrize("avg", [3, 40, 200])
def test_plain_spmm_rows_at_the_group_wave_and_hub_thresholds(hgnn, dev, avg):
    """hgnn_spmm hands a row to a lane group (up to 32 non-zeros), to the whole wave, or to the chunked hub kernels
    (above 8 times the mean row length, the threshold held within 256..1024): rows whose lengths sit on and next to
    every one of those borders, and on the 512-edge chunk border, in graphs of three densities."""
    V, ncols, F = 900, 1300, 64
    lengths = [31, 32, 33, 255, 256, 257, 8 * avg - 1, 8 * avg, 8 * avg + 1, 511, 512, 513, 1023, 1024, 1025, 1536, 1537]
    hubs = tuple((20 + 7 * i, n) for i, n in enumerate(lengths))
    rowptr, col = rand_graph(V, ncols, avg, 300 + avg, hubs=hubs, empties=(0, 1, 899))
    r = np.random.default_rng(avg)
    X = f16(r.standard_normal((ncols, F)))
    w = f16(r.standard_normal((col.size, 1)))
    g = hgnn.Csr(up(rowptr, dev), up(col, dev), ncols=ncols)
    for reduce in (0, 1):
        for ww in (None, w):
            ref, sabs = oracle.spmm(rowptr, col, X, w=ww, reduce=reduce, want_sabs=True)
            Y = torch.full((V, F), 5.0, dtype=torch.float16, device=dev)
            spmm_plain(hgnn, g, None if ww is None else up(ww, dev), 1, up(X, dev), Y, op=reduce)
            compare(f"plain, avg {avg}, reduce {reduce}, w {ww is not None}", down(Y), ref, sabs)


# ------------------------------------------------------------------ edge-row kernels at their tier borders
@pytest.mark.parametrize("H,avg", [(1, 3), (4, 3), (4, 60), (8, 12)])
def test_edge_softmax_and_row_sums_at_the_tier_borders(hgnn, dev, H, avg):
    """Rows on and next to every border between the tiers of the edge-row kernels: what a lane team keeps in
    registers (8 * 2 * team / H edges for teams of 4 to 64 lanes), the plan's 32- and 2048-edge thresholds, and a
    row that starts at an odd offset into a 16-byte vector."""
    V = 700
    lengths = [1, 2, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513,
               1023, 1024, 1025, 2047, 2048, 2049, 4097]
    hubs = tuple((10 + 13 * i, n) for i, n in enumerate(lengths))
    rowptr, col = rand_graph(V, V, avg, 500 + H + avg, hubs=hubs, empties=(0, 3, 699))
    E = col.size
    r = np.random.default_rng(H + avg)
    e16, da16 = f16(3 * r.standard_normal((E, H))), f16(r.standard_normal((E, H)))
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    p = hgnn.hgnn_plan_create(g, 256, 64, 8)
    rows = np.repeat(np.arange(V), np.diff(rowptr))
    ref_a = oracle.edge_softmax(rowptr, e16.astype(np.float64))
    for plan in (p, None):
        alpha = torch.full((E, H), -1.0, dtype=torch.float16, device=dev)
        hgnn.hgnn_edge_softmax(g, plan, H, up(e16, dev), alpha)
        compare("alpha", down(alpha), ref_a, np.maximum(ref_a, 2.0 ** -14), rel_elem=2e-2)
        a16 = down(alpha)
        de = torch.empty((E, H), dtype=torch.float16, device=dev)
        hgnn.hgnn_edge_softmax_bwd(g, plan, H, alpha, up(da16, dev), de, e=up(e16, dev))
        ref_de = oracle.edge_softmax_bwd(rowptr, a16.astype(np.float64), da16.astype(np.float64), e=e16.astype(np.float64))
        t_abs = np.zeros((V, H))
        np.add.at(t_abs, rows, np.abs(a16.astype(np.float64) * da16.astype(np.float64)))
        compare("de", down(de), ref_de, a16.astype(np.float64) * (np.abs(da16.astype(np.float64)) + t_abs[rows]) + 2.0 ** -14)
        out = torch.empty((V, H), dtype=torch.float16, device=dev)
        hgnn.hgnn_edge_rowsum(g, plan, H, up(da16, dev), out)
        ref_s, abs_s = np.zeros((V, H)), np.zeros((V, H))
        np.add.at(ref_s, rows, da16.astype(np.float64))
        np.add.at(abs_s, rows, np.abs(da16.astype(np.float64)))
        compare("row sums", down(out), ref_s, abs_s)
    hgnn.hgnn_plan_destroy(p)
    if H > 1:  # a plan made for fewer heads has no room for the long rows' partial results: they go to the wave tier
        p1 = hgnn.hgnn_plan_create(g, 256, 64, 1)
        alpha = torch.full((E, H), -1.0, dtype=torch.float16, device=dev)
        hgnn.hgnn_edge_softmax(g, p1, H, up(e16, dev), alpha)
        compare("alpha, plan for one head", down(alpha), ref_a, np.maximum(ref_a, 2.0 ** -14), rel_elem=2e-2)
        hgnn.hgnn_plan_destroy(p1)
