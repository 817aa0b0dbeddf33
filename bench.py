#!/usr/bin/env python3
"""Benchmark of the fp16 sparse aggregation hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic graph that is already resident in
HBM: plain and discretized SpMM forward and backward (GIN / GCN layer), and a GAT layer forward
(score SDDMM, edge softmax, weighted SpMM) and backward (transposed SpMM, SDDMM dot, softmax and
score backward, row and column sums).  The graph, its transpose and the segment plans are built
once before timing (the graph is static across training iterations).

Prints ONE JSON line.  `value` is the algorithmic (compulsory, infinite-cache) bytes of one step
divided by the step time; `roofline` is the same figure for the dominant kernel alone, measured
with events on the launch stream inside the timed region; `cpu_baseline` is the fp64 oracle
timed on a bounded sample of the same workload on one host core.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c5", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--seg-edges", type=int, default=256)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--detail", action="store_true", help="also print a per-op table to stderr")
    ap.add_argument("--calib-copy", action="store_true",
                    help="first copy a 1 GiB buffer three times (a plain kernel of known traffic, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build measures one GPU only (got --gpus {args.gpus}); "
              "the path is single-GPU, see DESIGN.md for how it would shard", file=sys.stderr)
        return 2
    import numpy as np
    import torch

    import __graft_entry__ as ge
    ge.ensure_built()
    import paper_2411_01109_amd as hgnn
    import workloads as wl

    hgnn.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    makers = {"c1": wl.gcn_tiny, "c2": wl.gin_overflow, "c3": wl.gat_rmat, "c4": wl.gcn_large, "c5": wl.dense_degree}
    t0 = time.time()
    w = makers[args.workload]()
    gen_s = time.time() - t0
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    V, E, F = w.V, w.E, w.F
    feat_np = w.tensors["h"] if "h" in w.tensors else w.tensors["X"]
    grad_np = w.tensors["dOut"] if "dOut" in w.tensors else w.tensors["dY"]
    H = w.H
    D = F // H
    has_gat = "a_l" in w.tensors
    g = hgnn.Csr(up(w.rowptr), up(w.col))
    t0 = time.time()
    gt = hgnn.hgnn_transpose(g)
    plan = hgnn.hgnn_plan_create(g, args.seg_edges, F, H)
    plan_t = hgnn.hgnn_plan_create(gt, args.seg_edges, F, H)
    torch.cuda.synchronize()
    setup_s = time.time() - t0
    X, dY = up(feat_np), up(grad_np)
    ew = up(w.tensors["w"]).reshape(-1, 1) if "w" in w.tensors else None
    Y = torch.empty_like(X)
    half = torch.float16
    if has_gat:
        a_l, a_r = up(w.tensors["a_l"]), up(w.tensors["a_r"])
        e = torch.empty((E, H), dtype=half, device=dev)
        alpha, dalpha, ds = torch.empty_like(e), torch.empty_like(e), torch.empty_like(e)
        out, dh = torch.empty_like(X), torch.empty_like(X)
        d_el = torch.empty((V, H), dtype=half, device=dev)
        d_er = torch.empty((V, H), dtype=half, device=dev)

    # ---- algorithmic (compulsory) bytes per op: every input read once, every output written once
    wbytes = 2 if ew is not None else 0

    def spmm_bytes(weighted_h, transposed):
        return E * (4 + 2 * weighted_h + (4 if (transposed and weighted_h) else 0)) + 4 * (V + 1) + 2 * (2 * V * F)

    ops = []  # (name, kernel family, bytes, fn)
    wH = 1 if ew is not None else 0
    ops.append(("spmm_fwd_plain", "spmm_row", spmm_bytes(wH, False), lambda: hgnn.hgnn_spmm(g, ew, 1, X, Y)))
    ops.append(("spmm_bwd_plain", "spmm_row", spmm_bytes(wH, True), lambda: hgnn.hgnn_spmm(gt, ew, 1, dY, Y)))
    ops.append(("spmm_fwd_disc", "spmm_seg", spmm_bytes(wH, False),
                lambda: hgnn.hgnn_spmm_discretized(plan, g, ew, 1, X, Y)))
    ops.append(("spmm_bwd_disc", "spmm_seg", spmm_bytes(wH, True),
                lambda: hgnn.hgnn_spmm_discretized(plan_t, gt, ew, 1, dY, Y)))
    if args.workload in ("c2", "c5"):  # GIN: mean aggregation as well (discretized reduction scaling)
        ops.append(("spmm_fwd_disc_mean", "spmm_seg", spmm_bytes(0, False),
                    lambda: hgnn.hgnn_spmm_discretized(plan, g, None, 1, X, Y, op=hgnn.HGNN_MEAN)))
        ops.append(("spmm_bwd_disc_mean", "spmm_seg", spmm_bytes(0, True),
                    lambda: hgnn.hgnn_spmm_discretized(plan_t, gt, None, 1, dY, Y, op=hgnn.HGNN_MEAN)))
    if has_gat:
        EH = E * H
        ops.append(("gat_score", "sddmm", E * 4 + 4 * (V + 1) + 2 * V * F + 2 * EH,
                    lambda: hgnn.hgnn_sddmm(g, plan, hgnn.HGNN_SDDMM_GAT_SCORE, H, D, X, X, e, a_l, a_r, 0.2)))
        ops.append(("edge_softmax", "softmax", 4 * EH + 4 * (V + 1), lambda: hgnn.hgnn_edge_softmax(g, plan, H, e, alpha)))
        ops.append(("gat_spmm_fwd", "spmm_seg", spmm_bytes(H, False),
                    lambda: hgnn.hgnn_spmm_discretized(plan, g, alpha, H, X, out)))
        ops.append(("gat_spmm_bwd", "spmm_seg", spmm_bytes(H, True),
                    lambda: hgnn.hgnn_spmm_discretized(plan_t, gt, alpha, H, dY, dh)))
        ops.append(("sddmm_dot", "sddmm", E * 4 + 4 * (V + 1) + 2 * (2 * V * F) + 2 * EH,
                    lambda: hgnn.hgnn_sddmm(g, plan, hgnn.HGNN_SDDMM_DOT, H, D, dY, X, dalpha)))
        ops.append(("edge_softmax_bwd", "softmax", 8 * EH + 4 * (V + 1),
                    lambda: hgnn.hgnn_edge_softmax_bwd(g, plan, H, alpha, dalpha, ds, e=e, neg_slope=0.2)))
        ops.append(("score_bwd_rowsum", "rowsum", 2 * EH + 4 * (V + 1) + 2 * V * H, lambda: hgnn.hgnn_edge_rowsum(g, plan, H, ds, d_el)))
        ops.append(("score_bwd_colsum", "rowsum", 2 * EH + 4 * E + 4 * (V + 1) + 2 * V * H,
                    lambda: hgnn.hgnn_edge_rowsum(gt, plan_t, H, ds, d_er)))
    step_bytes = sum(o[2] for o in ops)

    def step(events=None):
        for i, (_, _, _, fn) in enumerate(ops):
            if events is not None:
                events[i][0].record()
            fn()
            if events is not None:
                events[i][1].record()

    if args.calib_copy:
        src = torch.empty(1 << 29, dtype=half, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in ops]
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(ev[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    op_ms = np.array([[a.elapsed_time(b) for (a, b) in ev[k]] for k in range(args.steps)])  # [steps, ops]
    op_avg = op_ms.mean(axis=0)

    # dominant op = the one with the most time; its roofline uses its own algorithmic bytes
    dom = int(np.argmax(op_avg))
    dom_name, dom_family, dom_bytes, _ = ops[dom]
    dom_gbps = dom_bytes / (op_avg[dom] * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dom_name, "achieved": round(dom_gbps, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(dom_gbps / HBM_PEAK_GBPS, 4), "traffic": None,
                "algorithmic_bytes": int(dom_bytes), "avg_ms": round(float(op_avg[dom]), 4)}

    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    detail = {n: {"ms": round(float(t), 4), "GBps": round(b / (t * 1e-3) / 1e9, 1)} for (n, _, b, _), t in zip(ops, op_avg)}
    layer_ms = {}
    if has_gat:
        layer_ms["gat_fwd_bwd_ms"] = round(float(sum(op_avg[i] for i, o in enumerate(ops) if o[0] in (
            "gat_score", "edge_softmax", "gat_spmm_fwd", "gat_spmm_bwd", "sddmm_dot", "edge_softmax_bwd",
            "score_bwd_rowsum", "score_bwd_colsum"))), 4)
    layer_ms["spmm_fwd_bwd_disc_ms"] = round(float(op_avg[2] + op_avg[3]), 4)
    layer_ms["spmm_fwd_bwd_plain_ms"] = round(float(op_avg[0] + op_avg[1]), 4)

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        # bounded sample: the first rows holding about 1.5 M non-zeros; SpMM forward in fp64 on one core
        target = min(E, 1_500_000)
        nrows_s = int(np.searchsorted(w.rowptr, target, side="left"))
        nrows_s = max(nrows_s, 1)
        rows = np.arange(nrows_s, dtype=np.int32)
        e_s = int(w.rowptr[nrows_s])
        wv = w.tensors["w"].reshape(-1, 1) if "w" in w.tensors else None
        t0 = time.perf_counter()
        oracle.spmm(w.rowptr, w.col, feat_np, w=wv, rows=rows)
        dt = time.perf_counter() - t0
        bytes_s = e_s * (4 + 2 * wH) + 4 * nrows_s + 2 * nrows_s * F + 2 * min(V, e_s) * F
        cpu = {"value": round(bytes_s / dt / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"fp64 SpMM forward on the first {nrows_s} rows ({e_s} non-zeros) of {w.name}, {dt:.2f} s",
               "host_cores_available": os.cpu_count()}

    line = {
        "metric": "fp16 SpMM/SDDMM achieved HBM GB/s (% of peak) + GNN layer fwd+bwd ms",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": w.name, "V": V, "E": E, "F": F, "H": H, "seg_edges": args.seg_edges,
                   "ops_per_step": [o[0] for o in ops]},
        "roofline": roofline, "cpu_baseline": cpu,
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4), "step_algorithmic_bytes": int(step_bytes),
        "layers": layer_ms, "ops": detail,
        "setup": {"generate_s": round(gen_s, 2), "transpose_and_plans_s": round(setup_s, 3)},
    }
    if args.detail:
        for (n, fam, b, _), t in zip(ops, op_avg):
            print(f"{n:22s} {fam:9s} {t:9.4f} ms  {b / 1e6:10.1f} MB  {b / (t * 1e-3) / 1e9:9.1f} GB/s", file=sys.stderr)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
