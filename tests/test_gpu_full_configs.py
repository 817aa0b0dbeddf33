"""The two largest configurations at full size, in the launch configuration the benchmark times
(segments of 256 edges): outputs are compared on sampled rows the oracle computes one by one
(random rows plus the longest hubs), since a full fp64 pass takes tens of seconds per call."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from parity import compare, down, sample_rows, up
from test_gpu_parity import gat_layer_check

pytestmark = pytest.mark.gpu


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
    ew = w.tensors["w"].reshape(-1, 1)
    X, dY, ewd = up(w.tensors["X"], dev), up(w.tensors["dY"], dev), up(ew, dev)
    rows = sample_rows(w.rowptr, 6000, 41)
    ref_f, abs_f = oracle.spmm(w.rowptr, w.col, w.tensors["X"], w=ew, rows=rows, want_sabs=True)
    rT, cT, eT = down(gt.rowptr), down(gt.col), down(gt.eid)
    # transposed graph: structural identities at full size (the bit-exact comparison runs at small sizes)
    assert rT[-1] == w.E and np.array_equal(np.sort(eT[:100000]), np.sort(eT[:100000])) and np.array_equal(w.col[eT], np.repeat(np.arange(w.V, dtype=np.int32), np.diff(rT)))
    rows_t = sample_rows(rT, 6000, 42)
    ref_b, abs_b = oracle.spmm(rT, cT, w.tensors["dY"], w=ew, eid=eT, rows=rows_t, want_sabs=True)
    Y = torch.empty_like(X)
    for name, fn in (("plain", lambda G, P, A, B: hgnn.hgnn_spmm(G, ewd, 1, A, B)),
                     ("disc", lambda G, P, A, B: hgnn.hgnn_spmm_discretized(P, G, ewd, 1, A, B))):
        fn(g, p, X, Y)
        full = down(Y)
        assert np.isfinite(full.astype(np.float32)).all()
        assert np.all(full[np.diff(w.rowptr) == 0] == 0)
        s = compare(f"c4 fwd {name}", full[rows], ref_f, abs_f)
        fn(gt, pt, dY, Y)
        full = down(Y)
        assert np.isfinite(full.astype(np.float32)).all()
        s2 = compare(f"c4 bwd {name}", full[rows_t], ref_b, abs_b)
        print(f"c4 {name}: fwd {s} bwd {s2}", flush=True)


def test_config5_dense_degree_gin_and_gat(hgnn, dev):
    w = wl.dense_degree()
    print(f"c5 generated: V={w.V} E={w.E} max deg={np.diff(w.rowptr).max()}", flush=True)
    g = hgnn.Csr(up(w.rowptr, dev), up(w.col, dev))
    gt = hgnn.hgnn_transpose(g)
    p = hgnn.hgnn_plan_create(g, 256, 64, 1)
    pt = hgnn.hgnn_plan_create(gt, 256, 64, 1)
    X, dY = up(w.tensors["X"], dev), up(w.tensors["dY"], dev)
    rows = sample_rows(w.rowptr, 1500, 51)
    rT, cT = down(gt.rowptr), down(gt.col)
    rows_t = sample_rows(rT, 1500, 52)
    Y = torch.empty_like(X)
    for red in (oracle.SUM, oracle.MEAN):
        ref_f, abs_f = oracle.spmm(w.rowptr, w.col, w.tensors["X"], reduce=red, rows=rows, want_sabs=True)
        ref_b, abs_b = oracle.spmm(rT, cT, w.tensors["dY"], reduce=red, rows=rows_t, want_sabs=True)
        hgnn.hgnn_spmm(g, None, 1, X, Y, op=red)
        s = compare(f"c5 gin plain fwd red={red}", down(Y)[rows], ref_f, abs_f)
        hgnn.hgnn_spmm_discretized(p, g, None, 1, X, Y, op=red)
        full = down(Y)
        assert np.isfinite(full.astype(np.float32)).all()
        s1 = compare(f"c5 gin disc fwd red={red}", full[rows], ref_f, abs_f)
        hgnn.hgnn_spmm_discretized(pt, gt, None, 1, dY, Y, op=red)
        s2 = compare(f"c5 gin disc bwd red={red}", down(Y)[rows_t], ref_b, abs_b)
        hgnn.hgnn_spmm(gt, None, 1, dY, Y, op=red)
        s3 = compare(f"c5 gin plain bwd red={red}", down(Y)[rows_t], ref_b, abs_b)
        # column-blocked plans chosen automatically for this table size (about 30 MB, rows of ~490 edges)
        pb = hgnn.hgnn_plan_create(g, 256, 64, 1, col_blocks=0)
        ptb = hgnn.hgnn_plan_create(gt, 256, 64, 1, col_blocks=0)
        assert hgnn.hgnn_plan_col_blocks(pb) == 4 and hgnn.hgnn_plan_col_blocks(ptb) == 4
        hgnn.hgnn_spmm_discretized(pb, g, None, 1, X, Y, op=red)
        s4 = compare(f"c5 gin blocked fwd red={red}", down(Y)[rows], ref_f, abs_f)
        hgnn.hgnn_spmm_discretized(ptb, gt, None, 1, dY, Y, op=red)
        s5 = compare(f"c5 gin blocked bwd red={red}", down(Y)[rows_t], ref_b, abs_b)
        del pb, ptb
        print(f"c5 gin red={red}: {s} {s1} {s2} {s3} blocked {s4} {s5}", flush=True)
    del Y, p, pt, gt, g
    torch.cuda.empty_cache()
    gat_layer_check(hgnn, dev, w, 1, 64, rows_fwd=sample_rows(w.rowptr, 1200, 53), tag="c5 gat")
    # the same layer with column-blocked plans (what the benchmark times on this configuration)
    gat_layer_check(hgnn, dev, w, 1, 64, rows_fwd=sample_rows(w.rowptr, 1200, 54), tag="c5 gat blocked", col_blocks=0)
