"""The compute entry points that take a plan neither allocate nor synchronize, so a whole layer can be
recorded into a HIP graph and replayed: every replay must give, bit for bit, what the same calls give eagerly."""
import numpy as np
import pytest
import torch

import workloads as wl
from parity import down, f16, rand_graph, up

pytestmark = pytest.mark.gpu


def test_gat_layer_and_spmm_under_graph_replay(hgnn, dev):
    V, H, D = 3000, 4, 16
    F = H * D
    rowptr, col = rand_graph(V, V, 12, 21, hubs=((5, 6000), (2999, 400)), empties=(0, 17))
    r = np.random.default_rng(0)
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    gt = hgnn.hgnn_transpose(g)
    p = hgnn.hgnn_plan_create(g, 256, F, H)
    pt = hgnn.hgnn_plan_create(gt, 256, F, H)
    a_l, a_r = up(f16(0.2 * r.standard_normal(F)), dev), up(f16(0.2 * r.standard_normal(F)), dev)
    E = col.size
    # static buffers of the recorded step
    X = torch.empty((V, F), dtype=torch.float16, device=dev)
    dO = torch.empty((V, F), dtype=torch.float16, device=dev)
    bufs = {k: torch.empty((V, F), dtype=torch.float16, device=dev) for k in ("out", "dV", "agg", "out3")}
    lse = torch.empty((V, H), dtype=torch.float32, device=dev)
    d_el = torch.empty((V, H), dtype=torch.float16, device=dev)
    d_er = torch.empty((V, H), dtype=torch.float16, device=dev)
    e = torch.empty((E, H), dtype=torch.float16, device=dev)
    alpha = torch.empty((E, H), dtype=torch.float16, device=dev)

    def step(o):
        hgnn.hgnn_gat_forward_fused(g, p, H, D, X, X, a_l, a_r, o["out"], lse)
        hgnn.hgnn_gat_backward_fused(g, p, gt, pt, H, D, X, X, a_l, a_r, o["out"], lse, dO, o["dV"], d_el, d_er)
        hgnn.hgnn_spmm_discretized(p, g, None, 1, X, o["agg"], op=hgnn.HGNN_MEAN)
        hgnn.hgnn_sddmm(g, p, hgnn.HGNN_SDDMM_GAT_SCORE, H, D, X, X, e, a_l, a_r, 0.2)
        hgnn.hgnn_edge_softmax(g, p, H, e, alpha)
        hgnn.hgnn_spmm_discretized(p, g, alpha, H, X, o["out3"])

    def fill(seed):
        rr = np.random.default_rng(seed)
        X.copy_(up(f16(rr.standard_normal((V, F))), dev))
        dO.copy_(up(f16(rr.standard_normal((V, F))), dev))

    fill(1)
    step(bufs)  # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(bufs)
    eager = {k: torch.empty_like(v) for k, v in bufs.items()}
    for rep in range(4):
        fill(10 + rep)
        graph.replay()
        torch.cuda.synchronize()
        got = {k: down(v).copy() for k, v in bufs.items()}
        got_s = (down(d_el).copy(), down(d_er).copy(), down(lse).copy())
        # the program's own eager work and synchronisation between replays
        step(eager)
        torch.cuda.synchronize()
        for k in bufs:
            assert np.array_equal(got[k].view(np.uint16), down(eager[k]).view(np.uint16)), (rep, k)
        assert np.array_equal(got_s[0].view(np.uint16), down(d_el).view(np.uint16)), rep
        assert np.array_equal(got_s[1].view(np.uint16), down(d_er).view(np.uint16)), rep
        assert np.array_equal(got_s[2], down(lse)), rep
        assert np.all(np.isfinite(got["out"])) and np.abs(got["out"]).max() > 0
    hgnn.hgnn_plan_destroy(p)
    hgnn.hgnn_plan_destroy(pt)


def test_all_sixteen_ops_of_a_step_under_graph_replay(hgnn, dev):
    """Every op of the benchmark's step on a GAT workload -- plain SpMM forward and backward (with its caller-owned
    workspace), discretized SUM / MEAN, the GIN fusions, score, softmax, weighted SpMM both ways, SDDMM, softmax
    backward, row and column sums -- recorded as one graph; no call allocates or synchronizes."""
    V, H, D = 2500, 1, 64
    F = H * D
    rowptr, col = rand_graph(V, V, 20, 77, hubs=((11, 7000), (2400, 1300)), empties=(0, 5))
    E = col.size
    r = np.random.default_rng(3)
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    gt = hgnn.hgnn_transpose(g)
    p = hgnn.hgnn_plan_create(g, 256, F, H, col_blocks=2)
    pt = hgnn.hgnn_plan_create(gt, 256, F, H, col_blocks=2)
    a_l, a_r = up(f16(0.2 * r.standard_normal(F)), dev), up(f16(0.2 * r.standard_normal(F)), dev)
    X = torch.empty((V, F), dtype=torch.float16, device=dev)
    dY = torch.empty((V, F), dtype=torch.float16, device=dev)
    ws = torch.empty(hgnn.hgnn_spmm_workspace(V, V, E, F), dtype=torch.uint8, device=dev)
    assert ws.numel() > 0
    scaled = torch.empty((V, F), dtype=torch.float16, device=dev)
    lam = up((0.1 / np.maximum(np.diff(rowptr), 1)).astype(np.float32), dev)
    half = lambda *s: torch.empty(s, dtype=torch.float16, device=dev)
    names = ("y0", "y1", "y2", "y3", "y4", "y5", "y6", "y7", "out", "dh")
    edge_names = ("e", "alpha", "dalpha", "ds")

    def make():
        o = {k: half(V, F) for k in names}
        o.update({k: half(E, H) for k in edge_names})
        o.update({"d_el": half(V, H), "d_er": half(V, H)})
        return o

    def step(o):
        hgnn.hgnn_spmm(g, None, 1, X, o["y0"], workspace=ws)
        hgnn.hgnn_spmm(gt, None, 1, dY, o["y1"], workspace=ws)
        hgnn.hgnn_spmm_discretized(p, g, None, 1, X, o["y2"])
        hgnn.hgnn_spmm_discretized(pt, gt, None, 1, dY, o["y3"])
        hgnn.hgnn_spmm_discretized(p, g, None, 1, X, o["y4"], op=hgnn.HGNN_MEAN)
        hgnn.hgnn_spmm_discretized(pt, gt, None, 1, dY, o["y5"], op=hgnn.HGNN_MEAN)
        hgnn.hgnn_spmm_discretized_fused(p, g, None, 1, X, o["y6"], op=hgnn.HGNN_MEAN, self_feat=X, self_coef=1.0, agg_coef=0.1)
        hgnn.hgnn_spmm_discretized_fused(pt, gt, None, 1, dY, o["y7"], col_scale=lam, self_feat=dY, self_coef=1.0, scaled_x=scaled)
        hgnn.hgnn_sddmm(g, p, hgnn.HGNN_SDDMM_GAT_SCORE, H, D, X, X, o["e"], a_l, a_r, 0.2)
        hgnn.hgnn_edge_softmax(g, p, H, o["e"], o["alpha"])
        hgnn.hgnn_spmm_discretized(p, g, o["alpha"], H, X, o["out"])
        hgnn.hgnn_spmm_discretized(pt, gt, o["alpha"], H, dY, o["dh"])
        hgnn.hgnn_sddmm(g, p, hgnn.HGNN_SDDMM_DOT, H, D, dY, X, o["dalpha"])
        hgnn.hgnn_edge_softmax_bwd(g, p, H, o["alpha"], o["dalpha"], o["ds"], e=o["e"], neg_slope=0.2)
        hgnn.hgnn_edge_rowsum(g, p, H, o["ds"], o["d_el"])
        hgnn.hgnn_edge_rowsum(gt, pt, H, o["ds"], o["d_er"])

    def fill(seed):
        rr = np.random.default_rng(seed)
        X.copy_(up(f16(rr.standard_normal((V, F))), dev))
        dY.copy_(up(f16(rr.standard_normal((V, F))), dev))

    bufs, eager = make(), make()
    fill(1)
    step(bufs)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(bufs)
    for rep in range(3):
        fill(40 + rep)
        graph.replay()
        torch.cuda.synchronize()
        got = {k: down(v).copy() for k, v in bufs.items()}
        step(eager)
        torch.cuda.synchronize()
        for k in bufs:
            assert np.array_equal(got[k].view(np.uint16), down(eager[k]).view(np.uint16)), (rep, k)
        assert np.all(np.isfinite(got["y0"].astype(np.float32))) and np.abs(got["dh"].astype(np.float32)).max() > 0
    hgnn.hgnn_plan_destroy(p)
    hgnn.hgnn_plan_destroy(pt)


def test_dense_side_under_graph_replay(hgnn, dev):
    """The dense calls take a caller-owned workspace and allocate nothing either: projection, GAT aggregation and all
    gradients of a layer recorded as one graph."""
    V, K, H, D = 2000, 48, 2, 16
    F = H * D
    rowptr, col = rand_graph(V, V, 10, 31, hubs=((7, 3000),), empties=(1,))
    r = np.random.default_rng(0)
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    gt = hgnn.hgnn_transpose(g)
    p = hgnn.hgnn_plan_create(g, 256, F, H)
    pt = hgnn.hgnn_plan_create(gt, 256, F, H)
    a_l, a_r = up(f16(0.2 * r.standard_normal(F)), dev), up(f16(0.2 * r.standard_normal(F)), dev)
    W = up(f16(r.standard_normal((K, F)) / np.sqrt(K)), dev)
    X = torch.empty((V, K), dtype=torch.float16, device=dev)
    dO = torch.empty((V, F), dtype=torch.float16, device=dev)
    half = lambda *s: torch.empty(s, dtype=torch.float16, device=dev)
    lse = torch.empty((V, H), dtype=torch.float32, device=dev)
    ws = torch.empty(max(hgnn.hgnn_linear_wgrad_workspace(K, F), hgnn.hgnn_gat_feature_grad_workspace(H, D)),
                     dtype=torch.uint8, device=dev)

    def make():
        return {"h": half(V, F), "out": half(V, F), "dV": half(V, F), "d_el": half(V, H), "d_er": half(V, H), "dh": half(V, F),
                "dX": half(V, K), "dW": torch.empty((K, F), dtype=torch.float32, device=dev),
                "da_l": torch.empty(F, dtype=torch.float32, device=dev), "da_r": torch.empty(F, dtype=torch.float32, device=dev)}

    def step(o):
        hgnn.hgnn_linear(X, W, o["h"])
        hgnn.hgnn_gat_forward_fused(g, p, H, D, o["h"], o["h"], a_l, a_r, o["out"], lse)
        hgnn.hgnn_gat_backward_fused(g, p, gt, pt, H, D, o["h"], o["h"], a_l, a_r, o["out"], lse, dO, o["dV"], o["d_el"], o["d_er"])
        hgnn.hgnn_gat_feature_grad(H, D, o["dV"], o["d_el"], o["d_er"], a_l, a_r, o["h"], o["dh"], o["da_l"], o["da_r"], ws)
        hgnn.hgnn_linear(o["dh"], W, o["dX"], trans_w=True)
        hgnn.hgnn_linear_wgrad(X, o["dh"], o["dW"], ws)

    def fill(seed):
        rr = np.random.default_rng(seed)
        X.copy_(up(f16(rr.standard_normal((V, K))), dev))
        dO.copy_(up(f16(rr.standard_normal((V, F))), dev))

    bufs, eager = make(), make()
    fill(1)
    step(bufs)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(bufs)
    for rep in range(3):
        fill(20 + rep)
        graph.replay()
        torch.cuda.synchronize()
        got = {k: down(v).copy() for k, v in bufs.items()}
        step(eager)
        torch.cuda.synchronize()
        for k in bufs:
            assert np.array_equal(got[k].view(np.uint8), down(eager[k]).view(np.uint8)), (rep, k)
        assert np.abs(got["dW"]).max() > 0 and np.all(np.isfinite(got["dW"]))
    hgnn.hgnn_plan_destroy(p)
    hgnn.hgnn_plan_destroy(pt)


def test_long_row_forms_under_graph_replay(hgnn, dev):
    """The forms that the library picks for long rows over a table beyond the L2s -- column passes of the plan-free
    SpMM, automatic column blocks and their finer cut (values behind the edge-id map, SDDMM) -- recorded as one graph."""
    V, F = 52000, 128
    rowptr, col = rand_graph(V, V, 130, 31, hubs=((7, 20000), (900, 3000)), empties=(0, 51999))
    E = col.size
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    gt = hgnn.hgnn_transpose(g)
    p = hgnn.hgnn_plan_create(g, 256, F, 1, col_blocks=0)
    pt = hgnn.hgnn_plan_create(gt, 256, F, 1, col_blocks=0)
    assert hgnn.hgnn_plan_col_blocks(p) >= 2 and hgnn.hgnn_plan_col_blocks_fine(pt) == 2 * hgnn.hgnn_plan_col_blocks(pt)
    need = hgnn.hgnn_spmm_workspace(V, V, E, F)
    assert need > hgnn.hgnn_spmm_workspace(V, 0, E, F)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    X = torch.empty((V, F), dtype=torch.float16, device=dev)
    w = torch.empty((E, 1), dtype=torch.float16, device=dev)
    names = ("plain", "plain_T", "blocked", "mapped", "dot")
    bufs = {k: torch.empty((E, 1) if k == "dot" else (V, F), dtype=torch.float16, device=dev) for k in names}

    def step(o):
        hgnn.hgnn_spmm(g, None, 1, X, o["plain"], op=hgnn.HGNN_MEAN, workspace=ws)
        hgnn.hgnn_spmm(gt, w, 1, X, o["plain_T"], workspace=ws)
        hgnn.hgnn_spmm_discretized(p, g, None, 1, X, o["blocked"])
        hgnn.hgnn_spmm_discretized(pt, gt, w, 1, X, o["mapped"])
        hgnn.hgnn_sddmm(g, p, hgnn.HGNN_SDDMM_DOT, 1, F, X, X, o["dot"])

    def fill(seed):
        rr = np.random.default_rng(seed)
        X.copy_(up(f16(rr.standard_normal((V, F))), dev))
        w.copy_(up(f16(rr.standard_normal((E, 1))), dev))

    fill(1)
    step(bufs)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(bufs)
    eager = {k: torch.empty_like(v) for k, v in bufs.items()}
    for rep in range(3):
        fill(20 + rep)
        graph.replay()
        torch.cuda.synchronize()
        got = {k: down(v).copy() for k, v in bufs.items()}
        step(eager)
        torch.cuda.synchronize()
        for k in names:
            assert np.array_equal(got[k].view(np.uint16), down(eager[k]).view(np.uint16)), (rep, k)
            assert np.all(np.isfinite(got[k])) and np.abs(got[k].astype(np.float32)).max() > 0
    hgnn.hgnn_plan_destroy(p)
    hgnn.hgnn_plan_destroy(pt)
