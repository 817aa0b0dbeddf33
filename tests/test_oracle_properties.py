"""Property tests of the CPU oracle on random small graphs (hypothesis): each property is a fact of the mathematics
that holds for every input, checked against numpy on dense matrices or against an invariant.  CPU only."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle

SETTINGS = dict(max_examples=40, deadline=None)


@st.composite
def graphs(draw, max_v=12, max_c=12):
    V = draw(st.integers(1, max_v))
    ncols = draw(st.integers(1, max_c))
    deg = draw(st.lists(st.integers(0, 2 * ncols), min_size=V, max_size=V))
    seed = draw(st.integers(0, 2 ** 31 - 1))
    r = np.random.default_rng(seed)
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    col = np.concatenate([np.sort(r.integers(0, ncols, size=d)) for d in deg] + [np.zeros(0, dtype=np.int64)]).astype(np.int32)
    row = np.repeat(np.arange(V), deg).astype(np.int32)
    return V, ncols, rowptr, col, row, r


def dense(V, ncols, row, col, w=None):
    A = np.zeros((V, ncols))
    np.add.at(A, (row, col), 1.0 if w is None else w)
    return A


@settings(**SETTINGS)
@given(graphs(), st.integers(1, 3), st.booleans())
def test_spmm_is_the_dense_product(gr, H, mean):
    V, ncols, rowptr, col, row, r = gr
    D = 2
    F = H * D
    X = r.standard_normal((ncols, F)).astype(np.float16)
    w = r.standard_normal((col.size, H)).astype(np.float16)
    got = oracle.spmm(rowptr, col, X, w=w, H=H, reduce=oracle.MEAN if mean else oracle.SUM)
    deg = np.maximum(np.diff(rowptr), 1)
    for h in range(H):
        A = dense(V, ncols, row, col, w[:, h].astype(np.float64))
        want = A @ X.astype(np.float64)[:, h * D:(h + 1) * D]
        if mean:
            want = want / deg[:, None]
        np.testing.assert_allclose(got[:, h * D:(h + 1) * D], want, rtol=1e-12, atol=1e-12)


@settings(**SETTINGS)
@given(graphs())
def test_transpose_twice_is_the_identity_and_eid_is_a_permutation(gr):
    V, ncols, rowptr, col, row, r = gr
    rT, cT, eT = oracle.transpose(rowptr, col, ncols)
    assert sorted(eT.tolist()) == list(range(col.size))
    assert np.array_equal(cT, row[eT]) and np.array_equal(np.repeat(np.arange(ncols), np.diff(rT)), col[eT])
    r2, c2, e2 = oracle.transpose(rT, cT, V)
    assert np.array_equal(r2, rowptr)
    # duplicates keep their order, so the double transpose restores the column list and the composed map is the identity
    assert np.array_equal(c2, col) and np.array_equal(eT[e2], np.arange(col.size))
    # adjoint: <A x, y> = <x, A^T y>
    x, y = r.standard_normal((ncols, 2)).astype(np.float16), r.standard_normal((V, 2)).astype(np.float16)
    a = (oracle.spmm(rowptr, col, x) * y.astype(np.float64)).sum()
    b = (oracle.spmm(rT, cT, y) * x.astype(np.float64)).sum()
    assert abs(a - b) <= 1e-10 * (1 + abs(a))


@settings(**SETTINGS)
@given(graphs(), st.integers(1, 3))
def test_edge_softmax_rows_sum_to_one_and_shift_invariance(gr, H):
    V, ncols, rowptr, col, row, r = gr
    e = r.standard_normal((col.size, H)) * 5
    a = oracle.edge_softmax(rowptr, e)
    sums = oracle.edge_rowsum(rowptr, a)
    nz = np.diff(rowptr) > 0
    np.testing.assert_allclose(sums[nz], 1.0, rtol=1e-12)
    assert np.all(a >= 0) and np.all(a <= 1 + 1e-15)
    shift = r.standard_normal((V, H)) * 50
    np.testing.assert_allclose(oracle.edge_softmax(rowptr, e + shift[row]), a, rtol=1e-9, atol=1e-15)
    # backward: the gradient of a row sums to zero (the weights of a row sum to one)
    d = oracle.edge_softmax_bwd(rowptr, a, r.standard_normal((col.size, H)))
    np.testing.assert_allclose(oracle.edge_rowsum(rowptr, d)[nz], 0.0, atol=1e-12)


@settings(**SETTINGS)
@given(graphs(), st.integers(1, 2))
def test_sddmm_samples_the_dense_product(gr, H):
    V, ncols, rowptr, col, row, r = gr
    D = 3
    U = r.standard_normal((V, H * D)).astype(np.float16)
    Vt = r.standard_normal((ncols, H * D)).astype(np.float16)
    got = oracle.sddmm_dot(rowptr, col, U, Vt, H=H)
    for h in range(H):
        P = U.astype(np.float64)[:, h * D:(h + 1) * D] @ Vt.astype(np.float64)[:, h * D:(h + 1) * D].T
        np.testing.assert_allclose(got[:, h], P[row, col], rtol=1e-12, atol=1e-12)


@settings(**SETTINGS)
@given(graphs(max_v=30), st.integers(1, 9))
def test_segment_plan_tiles_the_edges(gr, S):
    V, ncols, rowptr, col, row, r = gr
    E = col.size
    p = oracle.segment_plan(rowptr, S)
    nseg = (E + S - 1) // S
    assert p["seg_row_lo"].size == nseg
    for k in range(nseg):
        e0, e1 = k * S, min(E, (k + 1) * S) - 1
        assert p["seg_row_lo"][k] == row[e0] and p["seg_row_hi"][k] == row[e1]
    want = [i for i in range(V) if rowptr[i + 1] > rowptr[i] and rowptr[i] // S != (rowptr[i + 1] - 1) // S]
    assert p["split_row"].tolist() == want
    assert np.array_equal(p["split_seg_lo"], rowptr[want] // S) if want else p["split_seg_lo"].size == 0
    # discretized SpMM (fp16 staging) stays within one rounding per piece of the exact result
    X = r.standard_normal((ncols, 2)).astype(np.float16)
    exact, sabs = oracle.spmm(rowptr, col, X, want_sabs=True)
    disc, _ = oracle.spmm_discretized(rowptr, col, X, S)
    pieces = np.ceil(np.diff(rowptr) / S) + 1
    assert np.all(np.abs(disc.astype(np.float64) - exact) <= (pieces[:, None] + 1) * 2.0 ** -11 * (sabs + 1e-30) + 2.0 ** -24)


@settings(**SETTINGS)
@given(graphs())
def test_coo_list_in_any_order_gives_the_same_csr_and_two_transposes_do_too(gr):
    V, ncols, rowptr, col, row, r = gr
    perm = r.permutation(col.size)
    rp, c, eid = oracle.coo_to_csr(row[perm], col[perm], V)
    assert np.array_equal(rp, rowptr) and np.array_equal(c, col)
    assert sorted(eid.tolist()) == list(range(col.size))
    assert np.array_equal(row[perm][eid], row) and np.array_equal(col[perm][eid], col)
    # equal (row, col) pairs keep their list order
    same = (row[1:] == row[:-1]) & (col[1:] == col[:-1])
    assert np.all(eid[1:][same] > eid[:-1][same])
    # the same sort done another way: rows of the list in list order (an unsorted "CSR"), transposed twice
    order = np.argsort(row[perm], kind="stable")
    rT, cT, eT = oracle.transpose(rp, col[perm][order].astype(np.int32), ncols)
    r2, c2, e2 = oracle.transpose(rT, cT, V)
    assert np.array_equal(r2, rowptr) and np.array_equal(c2, col)
    assert np.array_equal(order[eT[e2]].astype(np.int32), eid)
