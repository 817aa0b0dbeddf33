"""Pins for the CPU oracle: every oracle function is checked against something
other than itself -- a hand-worked example (tests/golden), dense brute force,
closed forms, invariants, library routines on special cases, finite differences.
CPU only."""
import numpy as np
import pytest
import scipy.special

import oracle

rng = np.random.default_rng(20241101)


def small_graph(V, ncols, density, seed, dup=True, empty_rows=(), full_rows=()):
    """Random CSR with duplicates, some empty rows and some full rows (numpy only)."""
    r = np.random.default_rng(seed)
    rows, cols = [], []
    for i in range(V):
        if i in empty_rows:
            continue
        if i in full_rows:
            c = np.arange(ncols)
        else:
            n = r.integers(1, max(2, int(density * ncols)) + 1)
            c = r.integers(0, ncols, size=n)
            if dup and n > 2:
                c[1] = c[0]  # force a duplicate edge
        c = np.sort(c)
        rows += [i] * len(c)
        cols += list(c)
    rowptr = np.zeros(V + 1, dtype=np.int32)
    np.add.at(rowptr, np.array(rows, dtype=np.int64) + 1, 1)
    rowptr = np.cumsum(rowptr).astype(np.int32)
    return rowptr, np.array(cols, dtype=np.int32), np.array(rows, dtype=np.int32)


def dense_from(rowptr, col, row, ncols, w=None):
    A = np.zeros((rowptr.size - 1, ncols))
    np.add.at(A, (row, col), 1.0 if w is None else w)
    return A


# ------------------------------------------------------------------ fp16 codec
def test_codec_exhaustive_decode_matches_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = oracle.decode(bits.view(np.float16))
    nan = np.isnan(ref)
    assert np.array_equal(nan, np.isnan(got))
    assert np.array_equal(ref[~nan], got[~nan])
    assert np.array_equal(np.signbit(ref[~nan]), np.signbit(got[~nan]))


def test_codec_round_trip_and_range():
    for b in range(65536):
        v = oracle.half_to_double(b)
        if v != v:
            continue
        assert oracle.double_to_half(v) == b, hex(b)
    # section 2.2: largest finite (2 - 2^-10) * 2^15, least normal 2^-14
    assert oracle.half_to_double(0x7BFF) == (2 - 2.0 ** -10) * 2.0 ** 15 == 65504.0
    assert oracle.half_to_double(0x0400) == 2.0 ** -14
    assert oracle.double_to_half(65519.99) == 0x7BFF and oracle.double_to_half(65520.0) == 0x7C00
    assert oracle.double_to_half(-1e9) == 0xFC00


def test_codec_rounds_to_nearest_even():
    one = 0x3C00
    assert oracle.double_to_half(1 + 2.0 ** -11) == one          # tie -> even (down)
    assert oracle.double_to_half(1 + 3 * 2.0 ** -11) == one + 2  # tie -> even (up)
    assert oracle.double_to_half(1 + 2.0 ** -11 + 2.0 ** -30) == one + 1
    assert oracle.double_to_half(2.0 ** -25) == 0 and oracle.double_to_half(2.0 ** -25 * 1.0001) == 1
    x = rng.standard_normal(200000) * np.exp(rng.uniform(-20, 12, 200000))
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    got = np.array([oracle.double_to_half(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(ref, got)


# ------------------------------------------------------------------ hand-worked example
def g5(golden5):
    rowptr = np.array(golden5["rowptr"], dtype=np.int32)
    col = np.array(golden5["col"], dtype=np.int32)
    X = np.array(golden5["X"]).reshape(5, 2).astype(np.float16)
    return rowptr, col, X


def test_five_vertex_spmm(golden5):
    rowptr, col, X = g5(golden5)
    assert np.array_equal(oracle.spmm(rowptr, col, X), np.array(golden5["Y_sum"]).reshape(5, 2))
    np.testing.assert_allclose(oracle.spmm(rowptr, col, X, reduce=oracle.MEAN),
                               np.array(golden5["Y_mean"]).reshape(5, 2), rtol=1e-15)
    w = np.array(golden5["w"], dtype=np.float16).reshape(-1, 1)
    assert np.array_equal(oracle.spmm(rowptr, col, X, w=w), np.array(golden5["Y_w"]).reshape(5, 2))
    # subset of rows
    assert np.array_equal(oracle.spmm(rowptr, col, X, rows=[3, 0]), np.array([[21, 24], [13, 16]]))


def test_five_vertex_transpose_and_backward(golden5):
    rowptr, col, _ = g5(golden5)
    dY = np.array(golden5["dY"]).reshape(5, 2).astype(np.float16)
    dX = np.array(golden5["dX"]).reshape(5, 2)
    assert np.array_equal(oracle.spmm_T_scatter(rowptr, col, dY, 5), dX)
    rT, cT, eT = oracle.transpose(rowptr, col, 5)
    assert list(rT) == [0, 2, 5, 8, 11, 14]
    assert list(cT) == [0, 1, 0, 1, 2, 1, 2, 3, 2, 3, 4, 0, 3, 4]
    assert list(eT) == [0, 3, 1, 4, 6, 5, 7, 9, 8, 10, 12, 2, 11, 13]
    assert np.array_equal(oracle.spmm(rT, cT, dY), dX)
    assert not np.array_equal(oracle.spmm(rowptr, col, dY), dX)  # the example is asymmetric


def test_five_vertex_sddmm_softmax_gat(golden5):
    rowptr, col, X = g5(golden5)
    dY = np.array(golden5["dY"]).reshape(5, 2).astype(np.float16)
    assert np.array_equal(oracle.sddmm_dot(rowptr, col, dY, X)[:, 0], np.array(golden5["sddmm"]))
    e = np.log(np.array(golden5["exp_e"])).reshape(-1, 1)
    alpha = oracle.edge_softmax(rowptr, e)
    np.testing.assert_allclose(alpha[:, 0], golden5["alpha"], rtol=1e-14)
    # alpha as edge weights: values chosen exactly representable where possible; compare loosely
    # after fp16 rounding of alpha, tightly with the fp64 alpha applied by hand
    Y = np.zeros((5, 2))
    row = np.repeat(np.arange(5), np.diff(rowptr))
    np.add.at(Y, row, alpha * X.astype(np.float64)[col])
    np.testing.assert_allclose(Y, np.array(golden5["Y_alpha"]).reshape(5, 2), rtol=1e-14)
    Yo = oracle.spmm(rowptr, col, X, w=alpha.astype(np.float16))
    np.testing.assert_allclose(Yo, np.array(golden5["Y_alpha"]).reshape(5, 2), rtol=1e-3)


def test_five_vertex_plan(golden5):
    rowptr, _, _ = g5(golden5)
    p = oracle.segment_plan(rowptr, int(golden5["plan_S"][0]))
    for k in ("seg_row_lo", "seg_row_hi", "split_row", "split_seg_lo", "split_seg_hi"):
        assert list(p[k]) == [int(v) for v in golden5[k]], k


# ------------------------------------------------------------------ SpMM against dense brute force
@pytest.mark.parametrize("H", [1, 2, 4])
@pytest.mark.parametrize("reduce", [oracle.SUM, oracle.MEAN])
def test_spmm_dense_bruteforce(H, reduce):
    V, ncols, F = 37, 29, 8
    rowptr, col, row = small_graph(V, ncols, 0.4, 7 + H, empty_rows=(0, 5, 36), full_rows=(3,))
    E = col.size
    X = rng.standard_normal((ncols, F)).astype(np.float16)
    w = rng.standard_normal((E, H)).astype(np.float16)
    rs = rng.uniform(0.5, 2.0, V)
    D = F // H
    ref = np.zeros((V, F))
    for h in range(H):  # dense A_h @ X_h per head
        A = dense_from(rowptr, col, row, ncols, w[:, h].astype(np.float64))
        ref[:, h * D:(h + 1) * D] = A @ X[:, h * D:(h + 1) * D].astype(np.float64)
    deg = np.diff(rowptr)
    if reduce == oracle.MEAN:
        ref /= np.maximum(deg, 1)[:, None]
    ref *= rs[:, None]
    got, sabs = oracle.spmm(rowptr, col, X, w=w, H=H, reduce=reduce, row_scale=rs, want_sabs=True)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)
    assert np.all(got[deg == 0] == 0.0)
    assert np.all(sabs + 1e-12 >= np.abs(got))
    # unweighted and a non-contiguous (padded) X
    Xp = np.zeros((ncols, F + 8), dtype=np.float16)
    Xp[:, :F] = X
    A1 = dense_from(rowptr, col, row, ncols)
    np.testing.assert_allclose(oracle.spmm(rowptr, col, Xp[:, :F]), A1 @ X.astype(np.float64), rtol=1e-12, atol=1e-12)


def test_spmm_all_ones_gives_degree():
    rowptr, col, _ = small_graph(50, 50, 0.3, 11, empty_rows=(4, 9))
    X = np.ones((50, 4), dtype=np.float16)
    deg = np.diff(rowptr).astype(np.float64)
    assert np.array_equal(oracle.spmm(rowptr, col, X), np.repeat(deg[:, None], 4, 1))
    m = oracle.spmm(rowptr, col, X, reduce=oracle.MEAN)
    assert np.array_equal(m[deg > 0], np.ones((int((deg > 0).sum()), 4)))
    assert np.all(m[deg == 0] == 0)


@pytest.mark.parametrize("H", [1, 4])
def test_spmm_adjoint_identity_and_transpose(H):
    """<A_w X, dY> = <X, A_w^T dY> pins the transposed graph and its edge-id map."""
    V, ncols, F = 41, 33, 8
    rowptr, col, row = small_graph(V, ncols, 0.3, 5, empty_rows=(2,))
    E = col.size
    X = rng.standard_normal((ncols, F)).astype(np.float16)
    dY = rng.standard_normal((V, F)).astype(np.float16)
    w = rng.standard_normal((E, H)).astype(np.float16)
    Y = oracle.spmm(rowptr, col, X, w=w, H=H)
    rT, cT, eT = oracle.transpose(rowptr, col, ncols)
    dX_g = oracle.spmm(rT, cT, dY, w=w, H=H, eid=eT)
    dX_s = oracle.spmm_T_scatter(rowptr, col, dY, ncols, w=w, H=H)
    np.testing.assert_allclose(dX_g, dX_s, rtol=1e-12, atol=1e-12)
    lhs = np.sum(Y * dY.astype(np.float64))
    rhs = np.sum(X.astype(np.float64) * dX_g)
    assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(lhs))
    # structure of the transpose: a permutation, grouped by column, positions ascending inside
    assert sorted(eT) == list(range(E))
    assert np.array_equal(col[eT], np.repeat(np.arange(ncols), np.diff(rT)))
    assert np.array_equal(row[eT], cT)
    for j in range(ncols):
        seg = eT[rT[j]:rT[j + 1]]
        assert np.all(np.diff(seg) > 0)


# ------------------------------------------------------------------ SDDMM
@pytest.mark.parametrize("H", [1, 2])
def test_sddmm_bruteforce_and_duality(H):
    V, ncols, F = 23, 31, 8
    D = F // H
    rowptr, col, row = small_graph(V, ncols, 0.3, 3)
    U = rng.standard_normal((V, F)).astype(np.float16)
    Vt = rng.standard_normal((ncols, F)).astype(np.float16)
    out = oracle.sddmm_dot(rowptr, col, U, Vt, H=H)
    for h in range(H):
        full = U[:, h * D:(h + 1) * D].astype(np.float64) @ Vt[:, h * D:(h + 1) * D].astype(np.float64).T
        np.testing.assert_allclose(out[:, h], full[row, col], rtol=1e-12, atol=1e-12)
    ones = np.ones((max(V, ncols), F), dtype=np.float16)
    assert np.all(oracle.sddmm_dot(rowptr, col, ones[:V], ones[:ncols], H=H) == D)
    # duality: sum_k dW_k w_k = <dY, A_w X>
    w = rng.standard_normal((col.size, H)).astype(np.float16)
    lhs = np.sum(out * w.astype(np.float64))
    rhs = np.sum(U.astype(np.float64) * oracle.spmm(rowptr, col, Vt, w=w, H=H))
    assert abs(lhs - rhs) < 1e-9 * max(1.0, abs(lhs))
    # edge-id indirection: results land in slot eid[k]
    perm = rng.permutation(col.size).astype(np.int32)
    out_p = oracle.sddmm_dot(rowptr, col, U, Vt, H=H, eid=perm)
    assert np.array_equal(out_p[perm], out)


# ------------------------------------------------------------------ GAT score
def test_gat_score_special_cases_and_factorisation():
    V, H, D = 19, 2, 4
    F = H * D
    rowptr, col, row = small_graph(V, V, 0.3, 9)
    h = rng.standard_normal((V, F)).astype(np.float16)
    al = (0.1 * rng.standard_normal((H, D))).astype(np.float16)
    ar = (0.1 * rng.standard_normal((H, D))).astype(np.float16)
    z = np.zeros((H, D), dtype=np.float16)
    assert np.all(oracle.gat_score(rowptr, col, h, z, z, H) == 0)
    # independent evaluation: per-vertex projections, then add and LeakyReLU
    h64 = h.astype(np.float64).reshape(V, H, D)
    el = np.einsum("vhd,hd->vh", h64, al.astype(np.float64))
    er = np.einsum("vhd,hd->vh", h64, ar.astype(np.float64))
    s = el[row] + er[col]
    ref = np.where(s > 0, s, 0.2 * s)
    np.testing.assert_allclose(oracle.gat_score(rowptr, col, h, al, ar, H), ref, rtol=1e-12, atol=1e-15)
    hp, ap = np.abs(h), np.abs(al)
    sp = oracle.gat_score(rowptr, col, hp, ap, ap, H)  # positive only: LeakyReLU is the identity
    hp64 = hp.astype(np.float64).reshape(V, H, D)
    e1 = np.einsum("vhd,hd->vh", hp64, ap.astype(np.float64))
    np.testing.assert_allclose(sp, e1[row] + e1[col], rtol=1e-12)
    sn = oracle.gat_score(rowptr, col, hp, -ap, -ap, H)  # negative only: times the slope
    np.testing.assert_allclose(sn, -0.2 * (e1[row] + e1[col]), rtol=1e-12)
    np.testing.assert_allclose(oracle.gat_score(rowptr, col, hp, -ap, -ap, H, slope=0.5), -0.5 * (e1[row] + e1[col]),
                               rtol=1e-12)


# ------------------------------------------------------------------ edge softmax (Eq. 1)
def test_edge_softmax_invariants_and_library():
    V, H = 30, 3
    rowptr, col, row = small_graph(V, 40, 0.5, 21, empty_rows=(7,))
    E = col.size
    e = rng.standard_normal((E, H)) * 3
    a = oracle.edge_softmax(rowptr, e)
    assert np.all(a >= 0) and np.all(a <= 1)
    sums = np.zeros((V, H))
    np.add.at(sums, row, a)
    deg = np.diff(rowptr)
    np.testing.assert_allclose(sums[deg > 0], 1.0, rtol=1e-12)
    for i in range(V):  # library softmax row by row
        if deg[i]:
            np.testing.assert_allclose(a[rowptr[i]:rowptr[i + 1]],
                                       scipy.special.softmax(e[rowptr[i]:rowptr[i + 1]], axis=0), rtol=1e-12)
    shift = rng.standard_normal((V, H)) * 50
    np.testing.assert_allclose(oracle.edge_softmax(rowptr, e + shift[row]), a, rtol=1e-9)
    eq = oracle.edge_softmax(rowptr, np.full((E, H), 1.7))
    np.testing.assert_allclose(eq, (1.0 / deg[row])[:, None].repeat(H, 1), rtol=1e-14)
    # numerically safe on huge scores (the max is subtracted first)
    big = oracle.edge_softmax(rowptr, e + 60000.0)
    np.testing.assert_allclose(big, a, rtol=1e-9)
    # degree one
    rp1 = np.arange(6, dtype=np.int32)
    assert np.all(oracle.edge_softmax(rp1, rng.standard_normal((5, 2))) == 1.0)


def test_zero_attention_gat_equals_mean_spmm():
    """With a_l = a_r = 0 all scores are equal, alpha = 1/deg, and the GAT output is the mean SpMM."""
    V, H, D = 26, 2, 4
    rowptr, col, _ = small_graph(V, V, 0.3, 2)
    h = rng.standard_normal((V, H * D)).astype(np.float16)
    z = np.zeros((H, D), dtype=np.float16)
    alpha = oracle.edge_softmax(rowptr, oracle.gat_score(rowptr, col, h, z, z, H))
    deg = np.diff(rowptr)
    row = np.repeat(np.arange(V), deg)
    np.testing.assert_allclose(alpha, (1.0 / deg[row])[:, None].repeat(H, 1))
    # alpha is not fp16-exact in general, so apply it by hand in fp64 and compare with MEAN
    out = np.zeros((V, H * D))
    np.add.at(out, row, np.repeat(alpha, D, axis=1) * h.astype(np.float64)[col])
    np.testing.assert_allclose(out, oracle.spmm(rowptr, col, h, reduce=oracle.MEAN), rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ backward formulas by finite differences
def test_softmax_backward_finite_differences():
    V, H = 9, 2
    rowptr, col, row = small_graph(V, 12, 0.5, 33)
    E = col.size
    e = rng.standard_normal((E, H))
    dalpha = rng.standard_normal((E, H))
    a = oracle.edge_softmax(rowptr, e)
    de = oracle.edge_softmax_bwd(rowptr, a, dalpha)
    loss = lambda ee: np.sum(oracle.edge_softmax(rowptr, ee) * dalpha)
    eps = 1e-6
    num = np.zeros_like(e)
    for k in range(E):
        for h in range(H):
            ep, em = e.copy(), e.copy()
            ep[k, h] += eps
            em[k, h] -= eps
            num[k, h] = (loss(ep) - loss(em)) / (2 * eps)
    np.testing.assert_allclose(de, num, rtol=1e-6, atol=1e-8)
    rs = np.zeros((V, H))
    np.add.at(rs, row, de)
    np.testing.assert_allclose(rs, 0, atol=1e-12)  # softmax gradients sum to zero per row


def test_score_backward_finite_differences():
    """d loss / d el and d er through LeakyReLU and Eq. 1: row sums and column sums of ds."""
    V, H = 8, 2
    rowptr, col, row = small_graph(V, V, 0.5, 44)
    E = col.size
    el = rng.standard_normal((V, H))
    er = rng.standard_normal((V, H))
    dalpha = rng.standard_normal((E, H))

    def fwd(el_, er_):
        s = el_[row] + er_[col]
        e_ = np.where(s > 0, s, 0.2 * s)
        return e_, oracle.edge_softmax(rowptr, e_)

    e, a = fwd(el, er)
    ds = oracle.edge_softmax_bwd(rowptr, a, dalpha, e=e, slope=0.2)
    d_el = oracle.edge_rowsum(rowptr, ds)
    d_er = oracle.edge_colsum(rowptr, col, ds, V)
    eps = 1e-6
    for (arr, grad, which) in ((el, d_el, 0), (er, d_er, 1)):
        num = np.zeros_like(arr)
        for v in range(V):
            for h in range(H):
                p, m = arr.copy(), arr.copy()
                p[v, h] += eps
                m[v, h] -= eps
                lp = np.sum((fwd(p, er) if which == 0 else fwd(el, p))[1] * dalpha)
                lm = np.sum((fwd(m, er) if which == 0 else fwd(el, m))[1] * dalpha)
                num[v, h] = (lp - lm) / (2 * eps)
        np.testing.assert_allclose(grad, num, rtol=1e-5, atol=1e-7)
    # column sums agree with row sums over the transposed graph read through the edge-id map
    rT, cT, eT = oracle.transpose(rowptr, col, V)
    np.testing.assert_allclose(oracle.edge_rowsum(rT, ds[eT]), d_er, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ segment plan
def brute_plan(rowptr, S):
    V, E = rowptr.size - 1, int(rowptr[-1])
    row_of = np.empty(E, dtype=np.int64)
    for i in range(V):
        row_of[rowptr[i]:rowptr[i + 1]] = i
    nseg = (E + S - 1) // S
    lo = [int(row_of[k * S:(k + 1) * S].min()) for k in range(nseg)]
    hi = [int(row_of[k * S:(k + 1) * S].max()) for k in range(nseg)]
    seg_of = np.arange(E) // S
    split = []
    for i in range(V):
        segs = set(seg_of[rowptr[i]:rowptr[i + 1]])
        if len(segs) > 1:
            split.append((i, min(segs), max(segs)))
    return lo, hi, split


@pytest.mark.parametrize("S", [1, 2, 7, 64, 128, 256, 512])
def test_plan_bruteforce(S):
    deg = rng.integers(0, 40, size=300)
    deg[10] = 1500  # a hub spanning many segments
    deg[11] = 0
    deg[299] = 0   # trailing empty row
    deg[0] = 0     # leading empty row
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    p = oracle.segment_plan(rowptr, S)
    lo, hi, split = brute_plan(rowptr, S)
    assert list(p["seg_row_lo"]) == lo and list(p["seg_row_hi"]) == hi
    assert [(int(a), int(b), int(c)) for a, b, c in zip(p["split_row"], p["split_seg_lo"], p["split_seg_hi"])] == split
    # rule 2: rows never decrease from one segment to the next
    assert np.all(np.diff(p["seg_row_lo"]) >= 0) and np.all(p["seg_row_hi"] >= p["seg_row_lo"])
    if S == 1:
        assert np.array_equal(p["seg_row_lo"], p["seg_row_hi"])
        assert np.array_equal(p["split_row"], np.nonzero(deg >= 2)[0])  # one edge per segment: any row of 2+ edges is split


def test_plan_degenerate():
    rowptr = np.array([0, 3, 3, 10], dtype=np.int32)
    for S in (10, 11, 1000):
        p = oracle.segment_plan(rowptr, S)
        assert list(p["seg_row_lo"]) == [0] and list(p["seg_row_hi"]) == [2] and p["split_row"].size == 0
    p = oracle.segment_plan(np.zeros(5, dtype=np.int32), 8)  # no edges at all
    assert p["seg_row_lo"].size == 0 and p["split_row"].size == 0


# ------------------------------------------------------------------ discretized reduction scaling
def test_discretized_equals_plain_when_partials_are_exact():
    """Small-integer data: every partial is an integer below 2048, hence exact in fp16,
    so batching the reduction changes nothing."""
    deg = rng.integers(0, 30, size=60)
    deg[7] = 400
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    E = int(rowptr[-1])
    col = rng.integers(0, 60, size=E).astype(np.int32)
    X = rng.integers(-3, 4, size=(60, 4)).astype(np.float16)
    plain = oracle.spmm(rowptr, col, X)
    for S in (4, 16, 64):
        disc, mp = oracle.spmm_discretized(rowptr, col, X, S)
        assert np.array_equal(disc, plain)
        assert mp <= S * 3


def test_discretized_bounds_partials_where_naive_fp16_overflows():
    """Section 5.2.2: a hub with all-positive features leaves the fp16 range under
    post-reduction scaling, while per-batch scaling keeps every stored partial small."""
    deg = np.array([5, 20000, 3], dtype=np.int64)
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    col = rng.integers(0, 64, size=int(rowptr[-1])).astype(np.int32)
    X = rng.uniform(4, 8, size=(64, 2)).astype(np.float16)
    exact = oracle.spmm(rowptr, col, X, reduce=oracle.MEAN)
    naive = oracle.spmm_naive_fp16(rowptr, col, X, reduce=oracle.MEAN, wide_sum=True).astype(np.float64)
    assert np.all(np.isinf(naive[1])) and np.all(np.isfinite(naive[[0, 2]]))
    # a running sum kept in fp16 stalls once its spacing exceeds the addends: finite but far off
    stalled = oracle.spmm_naive_fp16(rowptr, col, X, reduce=oracle.MEAN).astype(np.float64)
    assert np.all(np.abs(stalled[1] - exact[1]) > 0.5 * np.abs(exact[1]))
    disc, mp = oracle.spmm_discretized(rowptr, col, X, 256, reduce=oracle.MEAN)
    assert mp <= 256 * 8 / 20000 + 8  # scaled partials: hub pieces are tiny, small rows at most max|x|
    np.testing.assert_allclose(disc, exact, rtol=2e-3)
    # SUM on the hub does not fit fp16 at all; its partials still do (<= S * max|x|)
    _, mp_sum = oracle.spmm_discretized(rowptr, col, X, 256, reduce=oracle.SUM)
    assert mp_sum <= 256 * 8 and oracle.spmm(rowptr, col, X)[1].min() > 65504
    # naive fp16 on small-integer data is exact (pins the emulation itself)
    Xi = rng.integers(0, 3, size=(64, 2)).astype(np.float16)
    assert np.array_equal(oracle.spmm_naive_fp16(rowptr[:2], col, Xi).astype(np.float64), oracle.spmm(rowptr[:2], col, Xi))


# ------------------------------------------------------------------ one GAT aggregation, unrounded chain
def test_gat_forward_dense_bruteforce():
    """Sections 2.1.1 / 3.1.2 and Eq. 1 with dense matrices: scores on a V x ncols grid, softmax over the
    neighbours with multiplicity (A counts duplicate edges), then P @ Vt."""
    V, ncols, H, D = 23, 19, 2, 4
    F = H * D
    rowptr, col, row = small_graph(V, ncols, 0.4, 5, empty_rows=(3,), full_rows=(7,))
    A = dense_from(rowptr, col, row, ncols)
    U = rng.standard_normal((V, F)).astype(np.float16)
    Vt = rng.standard_normal((ncols, F)).astype(np.float16)
    a_l = (0.5 * rng.standard_normal(F)).astype(np.float16)
    a_r = (0.5 * rng.standard_normal(F)).astype(np.float16)
    out, lse, sabs = oracle.gat_forward(rowptr, col, U, Vt, a_l, a_r, H, slope=0.2)
    U64, V64, al, ar = (x.astype(np.float64) for x in (U, Vt, a_l, a_r))
    for h in range(H):
        sl = slice(h * D, (h + 1) * D)
        S = (U64[:, sl] @ al[sl])[:, None] + (V64[:, sl] @ ar[sl])[None, :]
        S = np.where(S > 0, S, 0.2 * S)
        W = A * np.exp(S)  # multiplicity times exp(score); small scores, no shift needed
        Z = W.sum(1)
        P = W / np.where(Z > 0, Z, 1.0)[:, None]
        np.testing.assert_allclose(out[:, sl], P @ V64[:, sl], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(sabs[:, sl], P @ np.abs(V64[:, sl]), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(lse[Z > 0, h], np.log(Z[Z > 0]), rtol=1e-12, atol=1e-13)
    assert np.all(out[3] == 0) and np.all(lse[3] == 0)


def test_gat_forward_special_cases():
    V, ncols, H, D = 40, 40, 4, 2
    F = H * D
    rowptr, col, row = small_graph(V, ncols, 0.2, 9, empty_rows=(0,))
    X = rng.standard_normal((V, F)).astype(np.float16)
    zero = np.zeros(F, dtype=np.float16)
    # zero attention vectors: every score is 0, alpha = 1/deg, the result is the mean aggregation
    out, lse, _ = oracle.gat_forward(rowptr, col, X, X, zero, zero, H)
    np.testing.assert_allclose(out, oracle.spmm(rowptr, col, X, reduce=oracle.MEAN), rtol=1e-12, atol=1e-14)
    deg = np.diff(rowptr)
    np.testing.assert_allclose(lse[deg > 0], np.log(deg[deg > 0])[:, None].repeat(H, 1), rtol=1e-12)
    # the row-side term is constant over a row and cancels in Eq. 1: a_l does not change the weights where
    # LeakyReLU is linear (all scores of one sign); with slope 1 it never does
    a_l = rng.standard_normal(F).astype(np.float16)
    a_r = rng.standard_normal(F).astype(np.float16)
    o1, l1, _ = oracle.gat_forward(rowptr, col, X, X, a_l, a_r, H, slope=1.0)
    o0, l0, _ = oracle.gat_forward(rowptr, col, X, X, zero, a_r, H, slope=1.0)
    np.testing.assert_allclose(o1, o0, rtol=1e-10, atol=1e-12)
    el = (X.astype(np.float64).reshape(V, H, D) * a_l.astype(np.float64).reshape(H, D)).sum(-1)
    np.testing.assert_allclose((l1 - l0)[deg > 0], el[deg > 0], rtol=1e-10, atol=1e-12)
    # it is the composition of the three separately pinned definitions (score, Eq. 1, weighted sum)
    e = oracle.gat_score(rowptr, col, X, a_l, a_r, H, slope=0.2)
    alpha = oracle.edge_softmax(rowptr, e)
    o2, l2, _ = oracle.gat_forward(rowptr, col, X, X, a_l, a_r, H, slope=0.2)
    ref = np.zeros((V, F))
    X64 = X.astype(np.float64)
    for k in range(col.size):
        ref[row[k]] += np.repeat(alpha[k], D) * X64[col[k]]
    np.testing.assert_allclose(o2, ref, rtol=1e-11, atol=1e-13)
    # huge scores do not overflow (the shift by the row maximum of Eq. 1)
    big = np.full(F, 60.0, dtype=np.float16)
    o3, l3, _ = oracle.gat_forward(rowptr, col, np.abs(X) * 50, np.abs(X) * 50, big, big, H)
    assert np.all(np.isfinite(o3)) and np.all(np.isfinite(l3)) and l3.max() > 1000


def test_gat_backward_matches_finite_differences_of_the_forward():
    """L = sum <dOut, out>.  U enters the forward only through el = a_l.U, so dL/dU = d_el * a_l; Vt enters
    through er = a_r.Vt and through the aggregated values, so dL/dVt = d_er * a_r + dV; dL/da_r = sum_j d_er_j Vt_j."""
    V, ncols, H, D = 9, 8, 2, 4
    F = H * D
    rowptr, col, row = small_graph(V, ncols, 0.5, 21, empty_rows=(2,))
    # values on a coarse binary grid so that fp16 storage of the perturbed inputs is exact
    q = lambda x: (np.round(x * 64) / 64).astype(np.float16)
    U, Vt, dOut = q(rng.standard_normal((V, F))), q(rng.standard_normal((ncols, F))), q(rng.standard_normal((V, F)))
    a_l, a_r = q(0.5 * rng.standard_normal(F)), q(0.5 * rng.standard_normal(F))
    dV, d_el, d_er = oracle.gat_backward(rowptr, col, U, Vt, a_l, a_r, dOut, H, slope=0.25)

    def loss(U_, Vt_, a_r_):
        out, _, _ = oracle.gat_forward(rowptr, col, U_, Vt_, a_l, a_r_, H, slope=0.25)
        return float((out * dOut.astype(np.float64)).sum())

    eps = 2.0 ** -8  # exactly representable next to the grid values
    al, ar = a_l.astype(np.float64).reshape(H, D), a_r.astype(np.float64).reshape(H, D)
    for (i, f) in [(0, 0), (3, 5), (8, 7), (5, 2)]:
        Up, Um = U.copy(), U.copy()
        Up[i, f] += np.float16(eps)
        Um[i, f] -= np.float16(eps)
        fd = (loss(Up, Vt, a_r) - loss(Um, Vt, a_r)) / (2 * eps)
        assert abs(fd - d_el[i, f // D] * al[f // D, f % D]) < 2e-3, (i, f)
    for (j, f) in [(0, 0), (4, 6), (7, 3), (2, 1)]:
        Vp, Vm = Vt.copy(), Vt.copy()
        Vp[j, f] += np.float16(eps)
        Vm[j, f] -= np.float16(eps)
        fd = (loss(U, Vp, a_r) - loss(U, Vm, a_r)) / (2 * eps)
        assert abs(fd - (d_er[j, f // D] * ar[f // D, f % D] + dV[j, f])) < 2e-3, (j, f)
    for f in (0, 3, 6):
        ap, am = a_r.copy(), a_r.copy()
        ap[f] += np.float16(eps)
        am[f] -= np.float16(eps)
        fd = (loss(U, Vt, ap) - loss(U, Vt, am)) / (2 * eps)
        want = (d_er[:, f // D] * Vt.astype(np.float64)[:, f]).sum()
        assert abs(fd - want) < 2e-3, f


def test_gat_backward_special_cases_and_composition():
    V, ncols, H, D = 30, 26, 2, 4
    F = H * D
    rowptr, col, row = small_graph(V, ncols, 0.3, 4, empty_rows=(1,))
    U, Vt = rng.standard_normal((V, F)).astype(np.float16), rng.standard_normal((ncols, F)).astype(np.float16)
    dOut = rng.standard_normal((V, F)).astype(np.float16)
    a_l, a_r = (0.4 * rng.standard_normal(F)).astype(np.float16), (0.4 * rng.standard_normal(F)).astype(np.float16)
    dV, d_el, d_er = oracle.gat_backward(rowptr, col, U, Vt, a_l, a_r, dOut, H)
    # the composition of the separately pinned pieces: alpha, SDDMM dot, softmax backward with mask, sums, SpMM on A^T
    el = (U.astype(np.float64).reshape(V, H, D) * a_l.astype(np.float64).reshape(H, D)).sum(-1)
    er = (Vt.astype(np.float64).reshape(ncols, H, D) * a_r.astype(np.float64).reshape(H, D)).sum(-1)
    raw = el[row] + er[col]
    e = np.where(raw > 0, raw, 0.2 * raw)
    alpha = oracle.edge_softmax(rowptr, e)
    dalpha = oracle.sddmm_dot(rowptr, col, dOut, Vt, H=H)
    ds = oracle.edge_softmax_bwd(rowptr, alpha, dalpha, e=e, slope=0.2)
    np.testing.assert_allclose(d_el, oracle.edge_rowsum(rowptr, ds), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(d_er, oracle.edge_colsum(rowptr, col, ds, ncols), rtol=1e-10, atol=1e-12)
    ref = np.zeros((ncols, F))
    for k in range(col.size):
        ref[col[k]] += np.repeat(alpha[k], D) * dOut.astype(np.float64)[row[k]]
    np.testing.assert_allclose(dV, ref, rtol=1e-10, atol=1e-12)
    # slope 1 (no mask): the score gradients of a row sum to zero (softmax weights sum to one)
    _, d_el1, _ = oracle.gat_backward(rowptr, col, U, Vt, a_l, a_r, dOut, H, slope=1.0)
    assert np.max(np.abs(d_el1)) < 1e-12


def test_gat_saved_tensors_give_the_row_side_gradient():
    """out_masked and csum against their definition on a dense graph, and the identity that makes them useful:
    d_el[i,h] = <dOut[i,h], out_masked[i,h]> - <dOut[i,h], out[i,h]> * csum[i,h], with d_el from the separately
    pinned backward."""
    V, ncols, H, D = 21, 17, 2, 4
    F = H * D
    rowptr, col, row = small_graph(V, ncols, 0.4, 8, empty_rows=(3,))
    U, Vt = rng.standard_normal((V, F)).astype(np.float16), rng.standard_normal((ncols, F)).astype(np.float16)
    dOut = rng.standard_normal((V, F)).astype(np.float16)
    a_l, a_r = (0.6 * rng.standard_normal(F)).astype(np.float16), (0.6 * rng.standard_normal(F)).astype(np.float16)
    slope = 0.3
    out, lse, _, outm, csum = oracle.gat_forward(rowptr, col, U, Vt, a_l, a_r, H, slope=slope, want_saved=True)
    # definition, edge by edge in python
    el = (U.astype(np.float64).reshape(V, H, D) * a_l.astype(np.float64).reshape(H, D)).sum(-1)
    er = (Vt.astype(np.float64).reshape(ncols, H, D) * a_r.astype(np.float64).reshape(H, D)).sum(-1)
    raw = el[row] + er[col]
    alpha = oracle.edge_softmax(rowptr, np.where(raw > 0, raw, slope * raw))
    mu = np.where(raw > 0, 1.0, slope)
    assert (raw > 0).any() and (raw <= 0).any()  # both branches of the mask occur
    want_m, want_c = np.zeros((V, F)), np.zeros((V, H))
    for k in range(col.size):
        want_m[row[k]] += np.repeat(alpha[k] * mu[k], D) * Vt.astype(np.float64)[col[k]]
        want_c[row[k]] += alpha[k] * mu[k]
    np.testing.assert_allclose(outm, want_m, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(csum, want_c, rtol=1e-12, atol=1e-13)
    assert np.all(csum[3] == 0) and np.all(outm[3] == 0)  # the empty row
    # slope 1: the mask is all ones, so the masked sums are the plain ones
    o1, _, _, om1, c1 = oracle.gat_forward(rowptr, col, U, Vt, a_l, a_r, H, slope=1.0, want_saved=True)
    np.testing.assert_allclose(om1, o1, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(c1[np.diff(rowptr) > 0], 1.0, rtol=1e-13)
    # the identity with the backward's d_el
    _, d_el, _ = oracle.gat_backward(rowptr, col, U, Vt, a_l, a_r, dOut, H, slope=slope)
    dO = dOut.astype(np.float64).reshape(V, H, D)
    t = (dO * out.reshape(V, H, D)).sum(-1)
    got = (dO * outm.reshape(V, H, D)).sum(-1) - t * csum
    np.testing.assert_allclose(got, d_el, rtol=1e-10, atol=1e-12)
    assert np.abs(d_el).max() > 1e-2


def test_coo_to_csr_hand_example_library_sort_and_round_trip():
    """Section 2.1.1's two formats: a seven-edge list worked out by hand (a duplicate edge, an empty row), the
    same order from numpy's lexicographic sort with the list index as the last key, the dense matrix of both
    forms, and CSR -> shuffled COO -> CSR giving the CSR back."""
    row = np.array([2, 0, 2, 1, 0, 2, 2], dtype=np.int32)
    col = np.array([1, 3, 0, 1, 3, 1, 4], dtype=np.int32)
    rowptr, c, eid = oracle.coo_to_csr(row, col, 4)
    assert rowptr.tolist() == [0, 2, 3, 7, 7]      # rows 0..3 hold 2, 1, 4, 0 edges
    assert c.tolist() == [3, 3, 1, 0, 1, 1, 4]     # ascending inside a row
    assert eid.tolist() == [1, 4, 3, 2, 0, 5, 6]   # the two (0,3) and the two (2,1) edges keep their list order
    r = np.random.default_rng(77)
    for V, ncols, E in ((1, 1, 5), (9, 4, 60), (50, 70, 400), (30, 30, 0)):
        row = r.integers(0, V, size=E).astype(np.int32)
        col = r.integers(0, ncols, size=E).astype(np.int32)
        rowptr, c, eid = oracle.coo_to_csr(row, col, V)
        order = np.lexsort((np.arange(E), col, row))
        assert np.array_equal(eid, order.astype(np.int32))
        assert np.array_equal(c, col[order]) and np.array_equal(np.diff(rowptr), np.bincount(row, minlength=V))
        A = np.zeros((V, ncols))
        np.add.at(A, (row, col), 1.0)
        assert np.array_equal(dense_from(rowptr, c, np.repeat(np.arange(V), np.diff(rowptr)), ncols), A)
    rowptr, col, row = small_graph(23, 19, 0.3, 5, empty_rows=(0, 7), dup=True)
    perm = r.permutation(col.size)
    rp2, c2, e2 = oracle.coo_to_csr(row[perm], col[perm], 23)
    assert np.array_equal(rp2, rowptr) and np.array_equal(c2, col)
    assert np.array_equal(np.sort(e2), np.arange(col.size)) and np.array_equal(row[perm][e2], row)


def test_edge_gather_is_the_transposed_order():
    """The k-th non-zero of the transpose carries the value of non-zero eid[k]: with the pre-permuted values and no
    edge-id map the transposed SpMM gives the same result as with the map, and the dense transpose agrees."""
    V, ncols = 17, 13
    rowptr, col, row = small_graph(V, ncols, 0.4, 31, empty_rows=(5,))
    w = rng.standard_normal((col.size, 2)).astype(np.float16)
    rT, cT, eT = oracle.transpose(rowptr, col, ncols)
    wT = oracle.edge_gather(eT, w)
    assert np.array_equal(wT.view(np.uint16), w[eT].view(np.uint16))
    X = rng.standard_normal((V, 4)).astype(np.float16)
    a = oracle.spmm(rT, cT, X, w=w, H=2, eid=eT)
    b = oracle.spmm(rT, cT, X, w=wT, H=2)
    assert np.array_equal(a, b)
    for h in range(2):
        A = dense_from(rowptr, col, row, ncols, w=w[:, h].astype(np.float64))
        np.testing.assert_allclose(b[:, 2 * h:2 * h + 2], A.T @ X.astype(np.float64)[:, 2 * h:2 * h + 2], rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ dense side of a layer
def test_linear_against_matmul_and_special_cases():
    """Section 3.1.3 (Eq. 2): the linear layer is a plain matrix product; numpy's fp64 matmul is the library form."""
    n, K, F = 23, 12, 10
    X = rng.standard_normal((n, K)).astype(np.float16)
    W = rng.standard_normal((K, F)).astype(np.float16)
    Xd, Wd = X.astype(np.float64), W.astype(np.float64)
    Y, sabs = oracle.linear(X, W, want_sabs=True)
    np.testing.assert_allclose(Y, Xd @ Wd, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(sabs, np.abs(Xd) @ np.abs(Wd), rtol=1e-13, atol=1e-13)
    # the transposed form reads the same weight the other way round
    np.testing.assert_allclose(oracle.linear(X, np.ascontiguousarray(W.T), trans=True), Y, rtol=0, atol=0)
    G = rng.standard_normal((n, F)).astype(np.float16)
    np.testing.assert_allclose(oracle.linear(G, W, trans=True), G.astype(np.float64) @ Wd.T, rtol=1e-13, atol=1e-13)
    # identity weight copies the input; a one-hot input row picks one row of W (not a column)
    assert np.array_equal(oracle.linear(X, np.eye(K, dtype=np.float16)), Xd)
    onehot = np.zeros((K, K), dtype=np.float16)
    onehot[np.arange(K), np.arange(K)[::-1]] = 1
    assert np.array_equal(oracle.linear(onehot, W), Wd[::-1])
    # non-square, asymmetric closed form: X = column index pattern, W = outer product
    u, v = np.arange(1, K + 1, dtype=np.float64), np.arange(1, F + 1, dtype=np.float64)
    Y2 = oracle.linear(np.ones((3, K), dtype=np.float16), np.outer(u, v).astype(np.float16))
    np.testing.assert_allclose(Y2, np.tile(u.sum() * v, (3, 1)), rtol=1e-13)


def test_linear_adjoints():
    """<X W, G> = <X, G W^T> = <W, X^T G>: ties the forward product, the transposed product and the weight gradient."""
    n, K, F = 31, 7, 5
    X = rng.standard_normal((n, K)).astype(np.float16)
    W = rng.standard_normal((K, F)).astype(np.float16)
    G = rng.standard_normal((n, F)).astype(np.float16)
    a = float((oracle.linear(X, W) * G.astype(np.float64)).sum())
    b = float((X.astype(np.float64) * oracle.linear(G, W, trans=True)).sum())
    dW, sabs = oracle.linear_wgrad(X, G, want_sabs=True)
    c = float((W.astype(np.float64) * dW).sum())
    assert abs(a - b) < 1e-10 and abs(a - c) < 1e-10
    np.testing.assert_allclose(dW, X.astype(np.float64).T @ G.astype(np.float64), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(sabs, np.abs(X.astype(np.float64)).T @ np.abs(G.astype(np.float64)), rtol=1e-13, atol=1e-13)
    # a single row: the weight gradient is the outer product x g^T (k indexes rows, f columns)
    np.testing.assert_array_equal(oracle.linear_wgrad(X[:1], G[:1]), np.outer(X[0].astype(np.float64), G[0].astype(np.float64)))


def test_gat_layer_gradients_match_finite_differences():
    """A whole layer, h = X W then the aggregation on (h, h): L = sum <dOut, out>.  Its gradients, chained as
    gat_backward -> gat_feature_grad -> linear (transposed) / linear_wgrad, against central differences of the
    forward chain.  All values sit on binary grids so that every perturbed h is exact in fp16; the chained
    gradients pass through fp16 (as on the device), hence the 5e-3 band."""
    V, H, D, K = 9, 2, 4, 4
    F = H * D
    rowptr, col, row = small_graph(V, V, 0.5, 77, empty_rows=(4,))
    own = np.random.default_rng(11)  # a draw whose scores keep clear of the LeakyReLU kink (checked below)
    grid = lambda shape: (own.integers(-4, 5, size=shape) / 4.0).astype(np.float16)
    X, W, dOut = grid((V, K)), grid((K, F)), grid((V, F))
    a_l, a_r = grid(F), grid(F)
    slope = 0.25
    h0 = oracle.linear(X, W).reshape(V, H, D)
    score = (h0 * a_l.astype(np.float64).reshape(H, D)).sum(-1)[row] + (h0 * a_r.astype(np.float64).reshape(H, D)).sum(-1)[col]
    assert np.abs(score).min() >= 0.2  # a bump of 2^-6 moves a score by at most 2^-6 * 2 * D: no sign changes

    def forward(X_, W_, al_, ar_):
        h64 = oracle.linear(X_, W_)
        h = h64.astype(np.float16)
        assert np.array_equal(h.astype(np.float64), h64)  # exact: nothing is lost between the two stages
        out, _, _ = oracle.gat_forward(rowptr, col, h, h, al_, ar_, H, slope=slope)
        return h, float((out * dOut.astype(np.float64)).sum())

    h, _ = forward(X, W, a_l, a_r)
    dV, d_el, d_er = oracle.gat_backward(rowptr, col, h, h, a_l, a_r, dOut, H, slope=slope)
    dh, da_l, da_r, _, _ = oracle.gat_feature_grad(dV.astype(np.float16), d_el.astype(np.float16), d_er.astype(np.float16),
                                                   a_l, a_r, h, H)
    # the un-rounded definition of the feature gradient, term by term
    want = dV + np.repeat(d_el, D, axis=1) * a_l.astype(np.float64) + np.repeat(d_er, D, axis=1) * a_r.astype(np.float64)
    assert np.max(np.abs(dh - want)) < 5e-3
    dX = oracle.linear(dh.astype(np.float16), W, trans=True)
    dW = oracle.linear_wgrad(X, dh.astype(np.float16))
    eps = 2.0 ** -6

    def central(make):
        return (forward(*make(+eps))[1] - forward(*make(-eps))[1]) / (2 * eps)

    def bump(a, idx, d):
        b = a.copy()
        b[idx] += np.float16(d)
        return b

    for idx in [(0, 0), (3, 2), (8, 3), (4, 1)]:
        fd = central(lambda d: (bump(X, idx, d), W, a_l, a_r))
        assert abs(fd - dX[idx]) < 5e-3, (idx, fd, dX[idx])
    for idx in [(0, 0), (1, 5), (3, 7), (2, 2)]:
        fd = central(lambda d: (X, bump(W, idx, d), a_l, a_r))
        assert abs(fd - dW[idx]) < 5e-3, (idx, fd, dW[idx])
    for f in (0, 3, 6):
        fd = central(lambda d: (X, W, bump(a_l, f, d), a_r))
        assert abs(fd - da_l[f]) < 5e-3, (f, fd, da_l[f])
        fd = central(lambda d: (X, W, a_l, bump(a_r, f, d)))
        assert abs(fd - da_r[f]) < 5e-3, (f, fd, da_r[f])
    # the gradients are not trivially small: the bands above mean something
    assert np.abs(dX).max() > 0.2 and np.abs(dW).max() > 0.2 and np.abs(da_l).max() > 0.05 and np.abs(da_r).max() > 0.05


# ------------------------------------------------------------------ neighbour groups (vertex-parallel variant)
@pytest.mark.parametrize("ng", [1, 4, 32, 64])
def test_neighbor_groups_bruteforce(ng):
    """Section 5.4: groups of at most ng neighbours that never cross a row."""
    deg = rng.integers(0, 90, size=200)
    deg[3] = 1000
    deg[4] = 0
    deg[5] = ng
    deg[6] = ng + 1
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    row, first = oracle.neighbor_groups(rowptr, ng)
    # definition, in python: walk every row in steps of ng
    want = [(i, k) for i in range(len(deg)) for k in range(int(rowptr[i]), int(rowptr[i + 1]), ng)]
    assert list(zip(row.tolist(), first.tolist())) == want
    # invariants: closed-form count; the groups tile [0, E) in order; no group leaves its row
    assert row.size == int(np.sum((deg + ng - 1) // ng))
    end = np.minimum(first + ng, rowptr[row + 1])
    assert np.array_equal(first[1:], end[:-1]) and first[0] == 0 and end[-1] == rowptr[-1]
    assert np.all(first >= rowptr[row]) and np.all(end <= rowptr[row + 1]) and np.all(end - first <= ng)
    assert not np.any(row == 4)


def test_neighbor_groups_degenerate():
    row, first = oracle.neighbor_groups(np.zeros(4, dtype=np.int32), 64)
    assert row.size == 0 and first.size == 0
    # the misalignment example of section 5.4: a first vertex with 11 neighbours makes the next
    # vertex's groups start at an odd position
    row, first = oracle.neighbor_groups(np.array([0, 11, 80], dtype=np.int32), 32)
    assert row.tolist() == [0, 1, 1, 1] and first.tolist() == [0, 11, 43, 75]


def test_discretized_by_row_batches():
    """Per-row batching: exact data gives the plain result; the largest partial is bounded by the
    group size; with S at least the longest row there is one batch per row, i.e. one rounding."""
    deg = rng.integers(0, 30, size=60)
    deg[7] = 400
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    E = int(rowptr[-1])
    col = rng.integers(0, 60, size=E).astype(np.int32)
    X = rng.integers(-3, 4, size=(60, 4)).astype(np.float16)
    plain = oracle.spmm(rowptr, col, X)
    for S in (4, 16, 64):
        disc, mp = oracle.spmm_discretized(rowptr, col, X, S, by_row=True)
        assert np.array_equal(disc, plain) and mp <= S * 3
    Xr = rng.standard_normal((60, 4)).astype(np.float16)
    one, _ = oracle.spmm_discretized(rowptr, col, Xr, 400, reduce=oracle.MEAN, by_row=True)
    ref = oracle.spmm(rowptr, col, Xr, reduce=oracle.MEAN)
    assert np.array_equal(one, ref.astype(np.float16).astype(np.float64))
    # the two batchings differ only in where a row is cut: a row that starts on a segment
    # boundary is cut at the same places
    rp = np.array([0, 64, 64 + 150], dtype=np.int32)
    c2 = rng.integers(0, 60, size=int(rp[-1])).astype(np.int32)
    a, _ = oracle.spmm_discretized(rp, c2, Xr, 64, by_row=False)
    b, _ = oracle.spmm_discretized(rp, c2, Xr, 64, by_row=True)
    assert np.array_equal(a, b)


# ------------------------------------------------------------------ fused norms and the GIN epilogue
def test_gcn_both_norm_dense_bruteforce():
    """Eq. 2: D^-1/2 A D^-1/2 X with row degrees on the left and column degrees on the right."""
    V, F = 31, 4
    rowptr, col, row = small_graph(V, V, 0.3, 17, empty_rows=(4,))
    A = dense_from(rowptr, col, row, V)
    dr = np.maximum(A.sum(1), 1.0)
    dc = np.maximum(A.sum(0), 1.0)
    X = rng.standard_normal((V, F)).astype(np.float16)
    ref = np.diag(dr ** -0.5) @ A @ np.diag(dc ** -0.5) @ X.astype(np.float64)
    got = oracle.spmm(rowptr, col, X, row_scale=dr ** -0.5, col_scale=dc ** -0.5)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)
    # the same through per-edge values 1/sqrt(deg_i deg_j), up to their fp16 rounding
    wsym = (1.0 / np.sqrt(dr[row] * dc[col])).astype(np.float16).reshape(-1, 1)
    np.testing.assert_allclose(oracle.spmm(rowptr, col, X, w=wsym), ref, rtol=2e-3, atol=1e-3)
    # left norm only = column scale only
    np.testing.assert_allclose(oracle.spmm(rowptr, col, X, col_scale=1.0 / dc), A @ np.diag(1.0 / dc) @ X.astype(np.float64),
                               rtol=1e-12, atol=1e-13)


def test_gin_aggregation_dense_bruteforce():
    """Eq. 3: (1+eps) x_u + sum x_v, and the half-precision form (1+eps) x_u + lambda * mean x_v."""
    V, F, eps, lam = 29, 6, 0.25, 0.1
    rowptr, col, row = small_graph(V, V, 0.4, 23, empty_rows=(0, 11))
    A = dense_from(rowptr, col, row, V)
    X = rng.standard_normal((V, F)).astype(np.float16)
    X64 = X.astype(np.float64)
    got = oracle.spmm(rowptr, col, X, self_feat=X, self_coef=1 + eps, agg_coef=1.0)
    np.testing.assert_allclose(got, (1 + eps) * X64 + A @ X64, rtol=1e-12, atol=1e-13)
    deg = np.maximum(A.sum(1), 1.0)
    got2, sabs = oracle.spmm(rowptr, col, X, reduce=oracle.MEAN, self_feat=X, self_coef=1 + eps, agg_coef=lam, want_sabs=True)
    np.testing.assert_allclose(got2, (1 + eps) * X64 + lam * (A @ X64) / deg[:, None], rtol=1e-12, atol=1e-13)
    assert np.array_equal(got2[[0, 11]], (1 + eps) * X64[[0, 11]])  # empty rows keep the self term alone
    assert np.all(sabs + 1e-12 >= np.abs(got2))
    # weighted, multi-head, row subset, all options at once against a dense evaluation per head
    H = 2
    w = rng.standard_normal((col.size, H)).astype(np.float16)
    cs, rs = rng.uniform(0.5, 1.5, V), rng.uniform(0.5, 1.5, V)
    ref = np.zeros((V, F))
    for h in range(H):
        Ah = dense_from(rowptr, col, row, V, w[:, h].astype(np.float64))
        ref[:, h * 3:(h + 1) * 3] = Ah @ (cs[:, None] * X64[:, h * 3:(h + 1) * 3])
    ref = 0.5 * X64 + 2.0 * rs[:, None] * ref
    rows = np.array([5, 0, 28], dtype=np.int32)
    got3 = oracle.spmm(rowptr, col, X, w=w, H=H, row_scale=rs, col_scale=cs, self_feat=X, self_coef=0.5, agg_coef=2.0, rows=rows)
    np.testing.assert_allclose(got3, ref[rows], rtol=1e-12, atol=1e-12)
