"""The two largest configurations at full size, in the launch configuration the benchmark times
(segments of 256 edges).  Three layers of checks:
  * against the fp64 oracle on sampled rows it computes one by one (tens of thousands of random rows plus the
    longest hubs; the oracle is single-threaded per call, several calls on disjoint row sets run in host threads);
  * every row of every output against a float32 product formed by scipy's sparse library on the host (a second,
    library-made reference: not the oracle, it only widens the coverage to all rows);
  * the device paths against each other over every row (plain, discretized, column-blocked, vertex groups) at the
    bound two fp16 results of one exact value can differ by.
Integer work (plan arrays, the transposed graph) is compared bit for bit with the oracle at full size."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import scipy.sparse as sp
import torch

import oracle
import workloads as wl
from parity import compare, down, sample_rows, spmm_plain, up
from test_gpu_parity import gat_layer_check

pytestmark = pytest.mark.gpu

U16 = 2.0 ** -11  # fp16 unit roundoff


def oracle_rows(fn, rows, threads=8):
    """fn(rows_chunk) -> (values, magnitudes) for disjoint chunks of `rows` in host threads (the oracle's C calls release
    the interpreter lock; each call is itself single-threaded), concatenated in order."""
    chunks = [c for c in np.array_split(rows, threads) if c.size]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        parts = list(ex.map(fn, chunks))
    return np.concatenate([p[0] for p in parts]), np.concatenate([p[1] for p in parts])


def host_products(rowptr, col, vals, X, ncols):
    """float32 (A_w X, |A_w| |X|) over every row, by scipy's CSR product."""
    V = rowptr.size - 1
    data = np.ones(col.size, np.float32) if vals is None else vals.astype(np.float32).reshape(-1)
    A = sp.csr_matrix((data, col, rowptr), shape=(V, ncols))
    Xf = X.astype(np.float32)
    P = A @ Xf
    A.data = np.abs(A.data)
    S = A @ np.abs(Xf)
    return P, S


def all_rows_agree(name, a16, b16, P, S, scale=None):
    """Two fp16 results of the same exact row sums: each is within one rounding of the result plus one rounding at the
    magnitude of the terms, so they differ by at most twice that."""
    a, b = a16.astype(np.float32), b16.astype(np.float32)
    Pm, Sm = (np.abs(P), S) if scale is None else (np.abs(P) * scale[:, None], S * scale[:, None])
    tol = 2 * U16 * Pm + 2 * U16 * Sm * (1 + 2.0 ** -8) + 2.0 ** -23
    bad = np.abs(a - b) > tol
    assert not bad.any(), f"{name}: {int(bad.sum())} entries differ beyond two roundings (worst {np.abs(a - b)[bad].max():.3e})"
    return float(np.abs(a - b).max())


def test_config4_large_gcn(hgnn, dev):
    w = wl.gcn_large()
    print(f"c4 generated: V={w.V} E={w.E} max deg={np.diff(w.rowptr).max()}", flush=True)
    g = hgnn.Csr(up(w.rowptr, dev), up(w.col, dev))
    gt = hgnn.hgnn_transpose(g)
    p = hgnn.hgnn_plan_create(g, 256, 128, 1)
    pt = hgnn.hgnn_plan_create(gt, 256, 128, 1)
    print(f"c4 plans: nseg={hgnn.hgnn_plan_num_segments(p)} split={hgnn.hgnn_plan_num_split_rows(p)}", flush=True)
    # the plan at full size, bit exact
    ref_plan = oracle.segment_plan(w.rowptr, 256)
    got_plan = hgnn.hgnn_plan_export(p)
    for k in ref_plan:
        assert np.array_equal(got_plan[k], ref_plan[k]), k
    # the transposed graph and its edge-id map at full size, bit exact against the oracle's counting sort
    rT, cT, eT = down(gt.rowptr), down(gt.col), down(gt.eid)
    o_rT, o_cT, o_eT = oracle.transpose(w.rowptr, w.col, w.V)
    assert np.array_equal(rT, o_rT) and np.array_equal(cT, o_cT) and np.array_equal(eT, o_eT)
    del o_rT, o_cT, o_eT
    print("c4 transpose: bit exact", flush=True)
    ew = w.tensors["w"].reshape(-1, 1)
    Xh, dYh = w.tensors["X"], w.tensors["dY"]
    X, dY, ewd = up(Xh, dev), up(dYh, dev), up(ew, dev)
    rows = sample_rows(w.rowptr, 60000, 41)
    rows_t = sample_rows(rT, 60000, 42)
    ref_f, abs_f = oracle_rows(lambda r: oracle.spmm(w.rowptr, w.col, Xh, w=ew, rows=r, want_sabs=True), rows)
    ref_b, abs_b = oracle_rows(lambda r: oracle.spmm(rT, cT, dYh, w=ew, eid=eT, rows=r, want_sabs=True), rows_t)
    print(f"c4 oracle: {rows.size} + {rows_t.size} rows", flush=True)
    Y = torch.empty_like(X)
    for tag, G, P_, A, rws, ref, sab, host in (
            ("fwd", g, p, X, rows, ref_f, abs_f, lambda: host_products(w.rowptr, w.col, ew, Xh, w.V)),
            ("bwd", gt, pt, dY, rows_t, ref_b, abs_b, lambda: host_products(rT, cT, ew.reshape(-1)[eT], dYh, w.V))):
        Ph, Sh = host()
        outs = {}
        for name, fn in (("plain", lambda: spmm_plain(hgnn, G, ewd, 1, A, Y)),
                         ("disc", lambda: hgnn.hgnn_spmm_discretized(P_, G, ewd, 1, A, Y))):
            fn()
            full = down(Y).copy()
            deg = np.diff(down(G.rowptr))
            assert np.all(full[deg == 0] == 0)
            s = compare(f"c4 {tag} {name}", full[rws], ref, sab)
            s_all = compare(f"c4 {tag} {name}, every row against the host product", full, Ph.astype(np.float64), Sh.astype(np.float64))
            assert not s["cancelled"] and not s_all["cancelled"]
            print(f"c4 {tag} {name}: oracle rows {s}; all rows {s_all}", flush=True)
            outs[name] = full
        d = all_rows_agree(f"c4 {tag} plain vs disc", outs["plain"], outs["disc"], Ph, Sh)
        print(f"c4 {tag}: plain vs discretized over every row, max |diff| {d:.3e}", flush=True)
        del Ph, Sh, outs


def test_config5_dense_degree_gin_and_gat(hgnn, dev):
    w = wl.dense_degree()
    print(f"c5 generated: V={w.V} E={w.E} max deg={np.diff(w.rowptr).max()}", flush=True)
    g = hgnn.Csr(up(w.rowptr, dev), up(w.col, dev))
    gt = hgnn.hgnn_transpose(g)
    rT, cT, eT = down(gt.rowptr), down(gt.col), down(gt.eid)
    o_rT, o_cT, o_eT = oracle.transpose(w.rowptr, w.col, w.V)
    assert np.array_equal(rT, o_rT) and np.array_equal(cT, o_cT) and np.array_equal(eT, o_eT)
    del o_rT, o_cT, o_eT, eT
    print("c5 transpose: bit exact", flush=True)
    p = hgnn.hgnn_plan_create(g, 256, 64, 1)
    pt = hgnn.hgnn_plan_create(gt, 256, 64, 1)
    # column-blocked plans chosen automatically for this table size (about 30 MB, rows of ~490 edges)
    pb = hgnn.hgnn_plan_create(g, 256, 64, 1, col_blocks=0)
    ptb = hgnn.hgnn_plan_create(gt, 256, 64, 1, col_blocks=0)
    assert hgnn.hgnn_plan_col_blocks(pb) == 4 and hgnn.hgnn_plan_col_blocks(ptb) == 4
    assert hgnn.hgnn_plan_col_blocks_fine(pb) == 8 and hgnn.hgnn_plan_col_blocks_fine(ptb) == 8
    assert hgnn.hgnn_plan_num_slices(pb) == 15 and hgnn.hgnn_plan_num_slices(p) == 0  # 233 000 columns in slices of <= 16 384
    hgnn.hgnn_plan_add_groups(p, g, 256)
    Xh, dYh = w.tensors["X"], w.tensors["dY"]
    X, dY = up(Xh, dev), up(dYh, dev)
    rows = sample_rows(w.rowptr, 30000, 51)
    rows_t = sample_rows(rT, 30000, 52)
    Y = torch.empty_like(X)
    hosts = {"fwd": host_products(w.rowptr, w.col, None, Xh, w.V), "bwd": host_products(rT, cT, None, dYh, w.V)}
    inv_deg = {"fwd": 1.0 / np.maximum(np.diff(w.rowptr), 1).astype(np.float32),
               "bwd": 1.0 / np.maximum(np.diff(rT), 1).astype(np.float32)}
    for red in (oracle.SUM, oracle.MEAN):
        ref_f, abs_f = oracle_rows(lambda r: oracle.spmm(w.rowptr, w.col, Xh, reduce=red, rows=r, want_sabs=True), rows)
        ref_b, abs_b = oracle_rows(lambda r: oracle.spmm(rT, cT, dYh, reduce=red, rows=r, want_sabs=True), rows_t)
        for tag, G, P_, PB, A, rws, ref, sab in (("fwd", g, p, pb, X, rows, ref_f, abs_f),
                                                 ("bwd", gt, pt, ptb, dY, rows_t, ref_b, abs_b)):
            Ph, Sh = hosts[tag]
            scale = inv_deg[tag] if red == oracle.MEAN else None
            Pr = Ph if scale is None else Ph * scale[:, None]
            Sr = Sh if scale is None else Sh * scale[:, None]
            calls = [("plain", lambda: spmm_plain(hgnn, G, None, 1, A, Y, op=red)),
                     ("disc", lambda: hgnn.hgnn_spmm_discretized(P_, G, None, 1, A, Y, op=red)),
                     ("blocked", lambda: hgnn.hgnn_spmm_discretized(PB, G, None, 1, A, Y, op=red))]
            if tag == "fwd":
                calls.append(("vertex groups", lambda: hgnn.hgnn_spmm_discretized_variant(P_, G, None, 1, A, Y, hgnn.HGNN_VERTEX_GROUPS, op=red)))
            outs = {}
            for name, fn in calls:
                fn()
                full = down(Y).copy()
                s = compare(f"c5 gin {tag} {name} red={red}", full[rws], ref, sab)
                s_all = compare(f"c5 gin {tag} {name} red={red}, every row against the host product", full, Pr.astype(np.float64),
                                Sr.astype(np.float64))
                assert not s["cancelled"] and not s_all["cancelled"]
                print(f"c5 gin {tag} {name} red={red}: oracle rows {s}; all rows {s_all}", flush=True)
                outs[name] = full
            for name in outs:
                if name != "plain":
                    d = all_rows_agree(f"c5 {tag} red={red} plain vs {name}", outs["plain"], outs[name], Ph, Sh, scale)
                    print(f"c5 {tag} red={red}: plain vs {name} over every row, max |diff| {d:.3e}", flush=True)
            del outs, Pr, Sr
    del Y, p, pt, pb, ptb, gt, g, hosts
    torch.cuda.empty_cache()
    gat_layer_check(hgnn, dev, w, 1, 64, rows_fwd=sample_rows(w.rowptr, 1200, 53), tag="c5 gat")
    # the same layer with column-blocked plans (what the benchmark times on this configuration)
    gat_layer_check(hgnn, dev, w, 1, 64, rows_fwd=sample_rows(w.rowptr, 1200, 54), tag="c5 gat blocked", col_blocks=0)
