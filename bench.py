#!/usr/bin/env python3
"""Benchmark of the fp16 sparse aggregation hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic graph that is already resident in
HBM: plain and discretized SpMM forward and backward (GIN / GCN layer), and a GAT layer forward
(score SDDMM, edge softmax, weighted SpMM) and backward (transposed SpMM, SDDMM dot, softmax and
score backward, row and column sums).  The graph, its transpose and the segment plans are built
once before timing (the graph is static across training iterations).

By default the two largest graphs run back to back: config 5 (dense-degree graph, every op of the
path) and config 4 (large sparse GCN, the one whose feature table exceeds every cache).  Prints ONE
JSON line.  Its top-level fields are those of the first workload (config 5); `configs` holds one
object per workload with its ops, layers, roofline and cpu_baseline.  `value` is the algorithmic
(compulsory, infinite-cache) bytes of one step divided by the step time; `roofline` is the same figure
for the dominant kernel alone, measured with events on the launch stream inside the timed region, with
the measured traffic per launch (L2 misses towards the memory side) read from
the data file that the profile summaries are made from; `cpu_baseline` is the fp64 oracle timed on a
bounded, degree-stratified row sample of the same workload on one host core, kernel by kernel.
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
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hgnn_kernel_traffic.json")
WORKLOADS = ("c1", "c2", "c3", "c4", "c5")


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c5,c4",
                    help="comma-separated list out of c1..c5, run one after the other; the first one fills the top-level fields")
    ap.add_argument("--seg-edges", type=int, default=256)
    ap.add_argument("--col-blocks", type=int, default=0, help="column blocks of the SpMM plans: 0 = automatic, 1 = none")
    ap.add_argument("--width-sweep", action="store_true",
                    help="also time SDDMM dot and the vertex-group SpMM at 2, 4 and 8 halves per lane for "
                         "F in {16, 32, 64, 128} on this workload's graph; reported under 'width_sweep'")
    ap.add_argument("--graph", action="store_true",
                    help="also record all ops of the step into one HIP graph and time its replay "
                         "(launch-bound small configs); reported under 'graph'")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-hbm-busy", action="store_true",
                    help="skip the live sampling of the memory controllers' busy percentage per op (sysfs)")
    ap.add_argument("--no-side", action="store_true",
                    help="skip the side measurements (fused GAT passes, dense side, column norm both ways): only the step")
    ap.add_argument("--detail", action="store_true", help="also print a per-op table to stderr")
    ap.add_argument("--variants", action="store_true",
                    help="also time the comparison variants of the discretized SpMM (atomic conflict writes, "
                         "vertex-parallel neighbour groups) beside the path; reported under 'variants', not in the step")
    ap.add_argument("--calib-copy", action="store_true",
                    help="first copy a 1 GiB buffer three times (a plain kernel of known traffic, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    args.workloads = [w.strip() for w in args.workload.split(",") if w.strip()]
    for w in args.workloads:
        if w not in WORKLOADS:
            ap.error(f"unknown workload {w!r}")
    return args


def load_traffic():
    """{workload name: {kernel name: {fetch_bytes, write_bytes, local_memory_read_bytes?, l2_hit_rate?, avg_us, ...}}} as
    written by paper_2411_01109_amd/profile_summary.py from rocprofv3 counter runs; {} when the file is missing."""
    try:
        with open(TRAFFIC_FILE) as fh:
            return json.load(fh)
    except (OSError, ValueError):
        return {}


class HbmBusy:
    """Reads the memory controllers' busy percentage (amdgpu sysfs, mem_busy_percent) while a call is repeated for a
    couple of seconds: the one figure on this machine that tells HBM activity from traffic that the Infinity Cache
    absorbs (no rocprofv3 counter does).  A device-to-device copy of known size calibrates it."""

    def __init__(self, torch, np):
        import glob
        self.torch, self.np = torch, np
        paths = sorted(glob.glob("/sys/class/drm/card*/device/mem_busy_percent"))
        self.path = paths[0] if paths else None

    def _read(self):
        try:
            with open(self.path) as fh:
                return float(fh.read().strip())
        except (OSError, ValueError):
            return None

    def measure(self, fn, seconds=2.3, batch=10):
        """-> (busy % as last read while fn was being repeated for `seconds`, calls per second) or (None, rate).  The
        driver refreshes the figure about once a second, so the loop spans two refreshes and the last reading counts."""
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n = 0
        last = None
        while time.perf_counter() - t0 < seconds:
            for _ in range(batch):
                fn()
            torch.cuda.synchronize()
            n += batch
            if self.path is not None:
                last = self._read()
        dt = time.perf_counter() - t0
        return last, n / dt

    def calibrate(self, dev):
        """Busy % of a plain copy (1 GiB read + 1 GiB written per call) and of a plain read (2 GiB summed)."""
        torch = self.torch
        src = torch.empty(1 << 29, dtype=torch.float16, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        busy, rate = self.measure(lambda: dst.copy_(src))
        out = {"copy_GBps": round(rate * 2 * src.numel() * 2 / 1e9, 1), "copy_busy_percent": busy}
        del dst
        return out


def stratified_rows(np, rowptr, target_edges):
    """A degree-stratified row sample: rows ordered by length, every k-th one taken (with the longest row), k chosen so
    that the sample holds about target_edges non-zeros.  Returns sorted row ids."""
    deg = np.diff(rowptr)
    V, E = deg.size, int(rowptr[-1])
    if target_edges >= E:
        return np.arange(V, dtype=np.int32)
    order = np.argsort(deg, kind="stable")
    k = max(int(round(E / max(target_edges, 1))), 1)
    pick = order[k // 2::k]
    return np.unique(np.concatenate([pick, order[-1:]])).astype(np.int32)


def sub_csr(np, rowptr, col, rows):
    """CSR of the listed rows alone (columns keep their ids) and the positions of its non-zeros in the whole graph."""
    deg = (rowptr[rows + 1] - rowptr[rows]).astype(np.int64)
    rp = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    pos = np.repeat(rowptr[rows].astype(np.int64) - rp[:-1], deg) + np.arange(int(rp[-1]), dtype=np.int64)
    return rp, col[pos], pos


def run_workload(args, wname, torch, np, hgnn, wl, dev, traffic_db, first, busy_probe=None, busy_cal=None):
    makers = {"c1": wl.gcn_tiny, "c2": wl.gin_overflow, "c3": wl.gat_rmat, "c4": wl.gcn_large, "c5": wl.dense_degree}
    t0 = time.time()
    w = makers[wname]()
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
    plan = hgnn.hgnn_plan_create(g, args.seg_edges, F, H, col_blocks=args.col_blocks)
    plan_t = hgnn.hgnn_plan_create(gt, args.seg_edges, F, H, col_blocks=args.col_blocks)
    torch.cuda.synchronize()
    setup_s = time.time() - t0
    X, dY = up(feat_np), up(grad_np)
    ew = up(w.tensors["w"]).reshape(-1, 1) if "w" in w.tensors else None
    Y = torch.empty_like(X)
    half = torch.float16
    ws_bytes = hgnn.hgnn_spmm_workspace(V, V, E, F)
    spmm_ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None
    if has_gat:
        a_l, a_r = up(w.tensors["a_l"]), up(w.tensors["a_r"])
        e = torch.empty((E, H), dtype=half, device=dev)
        alpha, dalpha, ds = torch.empty_like(e), torch.empty_like(e), torch.empty_like(e)
        out, dh = torch.empty_like(X), torch.empty_like(X)
        d_el = torch.empty((V, H), dtype=half, device=dev)
        d_er = torch.empty((V, H), dtype=half, device=dev)

    # ---- bytes per op.  "min": algorithmic / compulsory (every input read once, every output written once,
    # i.e. an infinite cache) -- the figure the roofline fraction uses, it can never exceed the peak.
    # "req": requested bytes of a cache-less machine (one feature row gathered per non-zero).
    def spmm_min(hw, transposed):
        return E * (4 + 2 * hw + (4 if (transposed and hw) else 0)) + 4 * (V + 1) + 2 * (2 * V * F)

    def spmm_req(hw, transposed):
        return E * (4 + 2 * hw + (4 if (transposed and hw) else 0) + 2 * F) + V * (4 + 2 * F)

    Lg = 1
    while Lg < F // 8:
        Lg *= 2
    off32 = "true" if V * X.stride(0) * 2 < (1 << 32) else "false"
    # the weighted segment kernel exists without the code of the edge-id map (last template argument false) for calls
    # whose graph has none, i.e. the forward graph here; every other instantiation carries it
    seg_name = lambda hw, mapped=True: f"hgnn::spmm_seg_kernel<{Lg}, {1 if hw else 0}, {off32}, {'true' if (mapped or not hw) else 'false'}>"
    # the plan-free SpMM walks the columns in passes where its workspace bound says so (room for the partial rows)
    passes = ws_bytes > hgnn.hgnn_spmm_workspace(V, 0, E, F)
    # (otherwise rows and the chunks of long rows share one launch wherever a row of the graph could be long)
    row_kind = "row_pass" if passes else ("row_hub" if ws_bytes else "row")
    row_name = lambda hw: f"hgnn::spmm_{row_kind}_kernel<{Lg}, {'true' if hw else 'false'}>"
    ops = []  # (name, kernel, min bytes, fn, requested bytes)
    wH = 1 if ew is not None else 0
    ops.append(("spmm_fwd_plain", row_name(wH), spmm_min(wH, False), lambda: hgnn.hgnn_spmm(g, ew, 1, X, Y, workspace=spmm_ws), spmm_req(wH, False)))
    ops.append(("spmm_bwd_plain", row_name(wH), spmm_min(wH, True), lambda: hgnn.hgnn_spmm(gt, ew, 1, dY, Y, workspace=spmm_ws), spmm_req(wH, True)))
    ops.append(("spmm_fwd_disc", seg_name(wH, False), spmm_min(wH, False),
                lambda: hgnn.hgnn_spmm_discretized(plan, g, ew, 1, X, Y), spmm_req(wH, False)))
    ops.append(("spmm_bwd_disc", seg_name(wH), spmm_min(wH, True),
                lambda: hgnn.hgnn_spmm_discretized(plan_t, gt, ew, 1, dY, Y), spmm_req(wH, True)))
    if ew is not None:
        # static edge values (GCN norm weights): brought into transposed order once at set-up, so that the backward
        # SpMM reads them as a stream instead of gathering them through the edge-id map
        ew_T = torch.empty_like(ew)
        hgnn.hgnn_edge_to_transposed(gt, 1, ew, ew_T)
        gt_plain = hgnn.Csr(gt.rowptr, gt.col, ncols=V)
    gin = wname in ("c2", "c5")
    if gin:  # GIN: mean aggregation as well (discretized reduction scaling)
        ops.append(("spmm_fwd_disc_mean", seg_name(0), spmm_min(0, False),
                    lambda: hgnn.hgnn_spmm_discretized(plan, g, None, 1, X, Y, op=hgnn.HGNN_MEAN), spmm_req(0, False)))
        ops.append(("spmm_bwd_disc_mean", seg_name(0), spmm_min(0, True),
                    lambda: hgnn.hgnn_spmm_discretized(plan_t, gt, None, 1, dY, Y, op=hgnn.HGNN_MEAN), spmm_req(0, True)))
    # the next-step fusions, measured beside the path: degree norms / GIN epilogue inside the discretized SpMM
    deg_r = torch.clamp(g.rowptr[1:] - g.rowptr[:-1], min=1).to(torch.float32)
    deg_c = torch.clamp(gt.rowptr[1:] - gt.rowptr[:-1], min=1).to(torch.float32)
    # a column-side scale is applied to the table once (scaled_x workspace: one V x F pass, then no per-edge factor)
    # where rows are long enough for that to pay, else fetched per edge inside the kernel
    Xs_buf = torch.empty_like(X)
    use_ws = E / V >= 24
    ws = Xs_buf if use_ws else None
    fused_name = seg_name(0) if use_ws else f"hgnn::spmm_seg_kernel<{Lg}, 2, {off32}, true>"
    cs_min = 4 * V                                        # compulsory: the scale vector, read once
    cs_req = (4 * V + 4 * V * F) if use_ws else 4 * E     # what is asked for: table written and re-read, or a factor per edge
    if gin:  # GIN, half-precision form: (1+eps) x + lambda * mean, forward and backward
        lam_over_deg = (0.1 / deg_r).contiguous()
        b = spmm_min(0, False) + 2 * V * F
        ops.append(("gin_fused_fwd", seg_name(0), b,
                    lambda: hgnn.hgnn_spmm_discretized_fused(plan, g, None, 1, X, Y, op=hgnn.HGNN_MEAN, self_feat=X,
                                                             self_coef=1.0, agg_coef=0.1), spmm_req(0, False) + 2 * V * F))
        ops.append(("gin_fused_bwd", fused_name, b + cs_min,
                    lambda: hgnn.hgnn_spmm_discretized_fused(plan_t, gt, None, 1, dY, Y, col_scale=lam_over_deg,
                                                             self_feat=dY, self_coef=1.0, scaled_x=ws),
                    spmm_req(0, True) + 2 * V * F + cs_req))
    else:  # GCN "both" norm from degree vectors instead of per-edge values
        rs_f, cs_f = deg_r.rsqrt().contiguous(), deg_c.rsqrt().contiguous()
        b = spmm_min(0, False) + 8 * V
        ops.append(("gcn_norm_fused_fwd", fused_name, b + cs_min,
                    lambda: hgnn.hgnn_spmm_discretized_fused(plan, g, None, 1, X, Y, row_scale=rs_f, col_scale=cs_f, scaled_x=ws),
                    spmm_req(0, False) + 8 * V + cs_req))
        ops.append(("gcn_norm_fused_bwd", fused_name, b + cs_min,
                    lambda: hgnn.hgnn_spmm_discretized_fused(plan_t, gt, None, 1, dY, Y, row_scale=cs_f, col_scale=rs_f,
                                                             scaled_x=ws),
                    spmm_req(0, True) + 8 * V + cs_req))
    if has_gat:
        EH = E * H
        b = E * 4 + 4 * (V + 1) + 2 * V * F + 2 * EH
        sliced = H == 1 and hgnn.hgnn_plan_num_slices(plan) > 0  # the plan cut the columns into LDS-sized slices
        ops.append(("gat_score", "hgnn::edge_slice_kernel<false>" if sliced else f"hgnn::edge_score_seg_kernel<{H}>", b,
                    lambda: hgnn.hgnn_sddmm(g, plan, hgnn.HGNN_SDDMM_GAT_SCORE, H, D, X, X, e, a_l, a_r, 0.2), b + 8 * EH))
        b = 4 * EH + 4 * (V + 1)
        ops.append(("edge_softmax", "hgnn::edge_row_team_kernel<0, ..>", b,
                    lambda: hgnn.hgnn_edge_softmax(g, plan, H, e, alpha), b))
        ops.append(("gat_spmm_fwd", seg_name(H, False), spmm_min(H, False),
                    lambda: hgnn.hgnn_spmm_discretized(plan, g, alpha, H, X, out), spmm_req(H, False)))
        ops.append(("gat_spmm_bwd", seg_name(H), spmm_min(H, True),
                    lambda: hgnn.hgnn_spmm_discretized(plan_t, gt, alpha, H, dY, dh), spmm_req(H, True)))
        b = E * 4 + 4 * (V + 1) + 2 * (2 * V * F) + 2 * EH
        ops.append(("sddmm_dot", f"hgnn::sddmm_seg_kernel<{Lg}, 8, false>", b,
                    lambda: hgnn.hgnn_sddmm(g, plan, hgnn.HGNN_SDDMM_DOT, H, D, dY, X, dalpha), b + E * 2 * F))
        b = 8 * EH + 4 * (V + 1)
        ops.append(("edge_softmax_bwd", "hgnn::edge_row_team_kernel<1, ..>", b,
                    lambda: hgnn.hgnn_edge_softmax_bwd(g, plan, H, alpha, dalpha, ds, e=e, neg_slope=0.2), b))
        b = 2 * EH + 4 * (V + 1) + 2 * V * H
        ops.append(("score_bwd_rowsum", "hgnn::edge_row_team_kernel<2, ..>", b,
                    lambda: hgnn.hgnn_edge_rowsum(g, plan, H, ds, d_el), b))
        if sliced:  # column sums over the graph itself, accumulated in LDS slice by slice
            ops.append(("score_bwd_colsum", "hgnn::edge_slice_kernel<true>", b + 4 * E,
                        lambda: hgnn.hgnn_edge_colsum(g, plan, H, ds, d_er), b + 4 * E))
        else:       # row sums over the transposed graph, gathered through its edge-id map
            ops.append(("score_bwd_colsum", "hgnn::edge_row_team_kernel<2, ..>", b + 4 * E,
                        lambda: hgnn.hgnn_edge_rowsum(gt, plan_t, H, ds, d_er), b + 4 * E))
    step_bytes = sum(o[2] for o in ops)

    def step(events=None):
        for i, o in enumerate(ops):
            if events is not None:
                events[i][0].record()
            o[3]()
            if events is not None:
                events[i][1].record()

    if args.calib_copy and first:
        src = torch.empty(1 << 29, dtype=half, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # events are recorded on torch's current stream, which is the stream handed to every hgnn call
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
    op_med, op_min = np.median(op_ms, axis=0), op_ms.min(axis=0)
    del ev

    # cold numbers: every op once more after a 512 MiB scrub buffer has been written, so that nothing of its
    # inputs is left in the 256 MB Infinity Cache or the L2s from the previous iteration (the figure to set
    # beside the measured HBM traffic); a few repetitions, outside the timed step
    scrub = torch.empty(1 << 28, dtype=half, device=dev)
    cold_reps = 3
    op_cold = np.zeros(len(ops))
    for i, o in enumerate(ops):
        ts = []
        for _ in range(cold_reps):
            scrub.fill_(1.0)
            e0_, e1_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0_.record()
            o[3]()
            e1_.record()
            torch.cuda.synchronize()
            ts.append(e0_.elapsed_time(e1_))
        op_cold[i] = float(np.median(ts))
    del scrub

    # HBM activity of the main ops, measured live: each repeated for a good two seconds while the memory controllers'
    # busy percentage is read (a copy of known size read ~60 % at 4.9 TB/s on this machine, i.e. the figure is close
    # to the share of the 8 TB/s peak in use)
    hbm_busy = {}
    if busy_probe is not None and busy_probe.path is not None:
        probed = ("spmm_fwd_plain", "spmm_fwd_disc", "spmm_bwd_disc", "gat_score", "edge_softmax", "gat_spmm_bwd", "sddmm_dot",
                  "edge_softmax_bwd", "score_bwd_colsum")
        for i, o in enumerate(ops):
            if o[0] in probed:
                hbm_busy[o[0]], _ = busy_probe.measure(o[3])

    side_steps = min(args.steps, 20)

    def time_call(fn):
        """mean milliseconds of up to 20 calls of fn after warm-up, HIP events on the launch stream"""
        for _ in range(max(min(args.warmup, 3), 1)):
            fn()
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(side_steps)]
        for a, b in pairs:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        return float(np.mean([a.elapsed_time(b) for a, b in pairs]))

    # dominant kernel = the kernel instantiation with the most time in a step; its launches are averaged
    by_kernel = {}
    for i, o in enumerate(ops):
        by_kernel.setdefault(o[1], []).append(i)
    # an op's time counts for its main kernel up to that kernel's profiled duration (a plain SpMM call on a power-law
    # graph is half row kernel, half hub kernel: the row kernel does not dominate the step because its call is long)
    kdb = traffic_db.get(w.name, {})

    def kernel_time(i):
        rec = kdb.get(ops[i][1])
        return min(op_avg[i], rec["avg_us"] * 1e-3) if rec and rec.get("avg_us") else op_avg[i]

    dom_kernel = max(by_kernel, key=lambda k: sum(kernel_time(i) for i in by_kernel[k]))
    idx = by_kernel[dom_kernel]
    dom_ms = float(np.mean([op_avg[i] for i in idx]))
    dom_bytes = float(np.mean([ops[i][2] for i in idx]))
    dom_req = float(np.mean([ops[i][4] for i in idx]))
    dom_gbps = dom_bytes / (dom_ms * 1e-3) / 1e9
    krec = kdb.get(dom_kernel)
    traffic = None if krec is None else float(krec["fetch_bytes"] + krec["write_bytes"])
    mem_side = None  # bytes between the L2s and the memory side (Infinity Cache + HBM) per launch, from the request counters
    if krec is not None and krec.get("local_memory_read_bytes") is not None:
        mem_side = float(krec["local_memory_read_bytes"] + krec.get("local_memory_write_bytes", 0.0))
    # every call launches its main kernel once (a column-blocked plan walks all its blocks inside one launch); the
    # short follow-up kernels of a call ride along in the time
    per_call = 1
    roofline = {"bound": "hbm", "kernel": dom_kernel, "calls_per_step": len(idx), "kernel_launches_per_call": per_call,
                "achieved": round(dom_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(dom_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "algorithmic_bytes": int(dom_bytes / per_call), "avg_ms": round(dom_ms / per_call, 4),
                "call_ms": round(dom_ms, 4), "call_cold_ms": round(float(np.mean([op_cold[i] for i in idx])), 4),
                "requested_bytes": int(dom_req / per_call),
                "requested_GBps": round(dom_req / (dom_ms * 1e-3) / 1e9, 1),
                "traffic_GBps": None if traffic is None else round(traffic * per_call / (dom_ms * 1e-3) / 1e9, 1),
                "memory_side_bytes": mem_side,
                "memory_side_GBps": None if mem_side is None else round(mem_side * per_call / (dom_ms * 1e-3) / 1e9, 1),
                "memory_side_frac_of_hbm_peak": None if mem_side is None else round(mem_side * per_call / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "l2_hit_rate": None if krec is None else krec.get("l2_hit_rate"),
                "hbm_busy_percent": float(np.mean([hbm_busy[ops[i][0]] for i in idx])) if hbm_busy and all(
                    hbm_busy.get(ops[i][0]) is not None for i in idx) else None,
                "profiled_avg_us": None if krec is None else krec.get("avg_us"),
                "traffic_source": os.path.relpath(TRAFFIC_FILE, ROOT) if krec is not None else None,
                "note": "per launch of the kernel: achieved = compulsory (infinite-cache) bytes / time, HIP events "
                        "around the call divided by its launches; requested_* counts one gathered feature row per "
                        "non-zero and may exceed the peak when caches hit; traffic = L2-miss bytes per launch (FETCH_SIZE + "
                        "WRITE_SIZE, calibrated) and memory_side_bytes = the same flow counted at the L2s' request "
                        "interface to local memory (TCC_EA0_*_DRAM_32B): both include what the Infinity Cache serves, "
                        "no counter of this chip separates it from HBM; from the rocprofv3 runs summarised under profiles/; "
                        "hbm_busy_percent = the memory controllers' busy share sampled live while the op repeats"}

    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    detail = {}
    for i, (o, t) in enumerate(zip(ops, op_avg)):
        d = {"ms": round(float(t), 4), "median_ms": round(float(op_med[i]), 4), "min_ms": round(float(op_min[i]), 4),
             "cold_ms": round(float(op_cold[i]), 4), "min_GBps": round(o[2] / (t * 1e-3) / 1e9, 1),
             "frac_of_hbm_peak": round(o[2] / (t * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
             "req_GBps": round(o[4] / (t * 1e-3) / 1e9, 1), "kernel": o[1]}
        if o[0] in hbm_busy and hbm_busy[o[0]] is not None:
            d["hbm_busy_percent"] = hbm_busy[o[0]]
            if busy_cal and busy_cal.get("copy_busy_percent"):
                d["hbm_GBps_estimate"] = round(hbm_busy[o[0]] * busy_cal["copy_GBps"] / busy_cal["copy_busy_percent"], 1)
        detail[o[0]] = d
    layer_ms = {}
    if has_gat:
        layer_ms["gat_fwd_bwd_ms"] = round(float(sum(op_avg[i] for i, o in enumerate(ops) if o[0] in (
            "gat_score", "edge_softmax", "gat_spmm_fwd", "gat_spmm_bwd", "sddmm_dot", "edge_softmax_bwd",
            "score_bwd_rowsum", "score_bwd_colsum"))), 4)
    layer_ms["spmm_fwd_bwd_disc_ms"] = round(float(op_avg[2] + op_avg[3]), 4)
    layer_ms["spmm_fwd_bwd_plain_ms"] = round(float(op_avg[0] + op_avg[1]), 4)
    if gin:
        layer_ms["gin_fwd_bwd_ms"] = round(float(sum(op_avg[i] for i, o in enumerate(ops) if o[0].startswith("gin_fused"))), 4)
    else:
        layer_ms["gcn_norm_fwd_bwd_ms"] = round(float(sum(op_avg[i] for i, o in enumerate(ops) if o[0].startswith("gcn_norm_fused"))), 4)

    prescaled = graph_info = static_w = fused = dense = variants = width_sweep = None
    if not args.no_side:
        # the column-side scale both ways, whatever the step uses: fetched per edge inside the kernel, and applied to the
        # table first (scaled_x workspace)
        if gin:
            name = "gin_fused_bwd"
            per_edge = lambda: hgnn.hgnn_spmm_discretized_fused(plan_t, gt, None, 1, dY, Y, col_scale=lam_over_deg, self_feat=dY,
                                                                self_coef=1.0)
            on_table = lambda: hgnn.hgnn_spmm_discretized_fused(plan_t, gt, None, 1, dY, Y, col_scale=lam_over_deg, self_feat=dY,
                                                                self_coef=1.0, scaled_x=Xs_buf)
        else:
            name = "gcn_norm_fused_fwd"
            per_edge = lambda: hgnn.hgnn_spmm_discretized_fused(plan, g, None, 1, X, Y, row_scale=rs_f, col_scale=cs_f)
            on_table = lambda: hgnn.hgnn_spmm_discretized_fused(plan, g, None, 1, X, Y, row_scale=rs_f, col_scale=cs_f, scaled_x=Xs_buf)
        prescaled = {"op": name, "step_uses": "scaled_x workspace" if use_ws else "per-edge factor",
                     "per_edge_factor_ms": round(time_call(per_edge), 4), "scaled_table_ms": round(time_call(on_table), 4)}

    if args.graph:
        # no op allocates or synchronizes: record the whole step once, replay it
        step()
        torch.cuda.synchronize()
        cg = torch.cuda.CUDAGraph()
        with torch.cuda.graph(cg):
            step()
        t_graph = time_call(cg.replay)
        t_eager_wall = time_call(step)
        graph_info = {"ops": [o[0] for o in ops], "graph_replay_ms": round(t_graph, 4),
                      "eager_ms": round(t_eager_wall, 4), "sum_of_op_ms": round(float(op_avg.sum()), 4)}

    if ew is not None and not args.no_side:
        t_static = time_call(lambda: hgnn.hgnn_spmm_discretized(plan_t, gt_plain, ew_T, 1, dY, Y))
        static_w = {"spmm_bwd_disc_static_w_ms": round(t_static, 4),
                    "spmm_bwd_disc_ms": round(float(op_avg[3]), 4)}

    if has_gat and not args.no_side:
        # the single-pass GAT aggregation beside the three-call forward path (not part of the step)
        lse = torch.empty((V, H), dtype=torch.float32, device=dev)

        t_f = time_call(lambda: hgnn.hgnn_gat_forward_fused(g, plan, H, D, X, X, a_l, a_r, out, lse))
        t_a = time_call(lambda: hgnn.hgnn_gat_alpha(g, plan, H, D, X, X, a_l, a_r, lse, alpha))
        three = float(sum(op_avg[i] for i, o in enumerate(ops) if o[0] in ("gat_score", "edge_softmax", "gat_spmm_fwd")))
        five = float(sum(op_avg[i] for i, o in enumerate(ops) if o[0] in (
            "gat_spmm_bwd", "sddmm_dot", "edge_softmax_bwd", "score_bwd_rowsum", "score_bwd_colsum")))
        hgnn.hgnn_gat_forward_fused(g, plan, H, D, X, X, a_l, a_r, out, lse)
        t_b = time_call(lambda: hgnn.hgnn_gat_backward_fused(g, plan, gt, plan_t, H, D, X, X, a_l, a_r, out, lse, dY, dh,
                                                            d_el, d_er))
        # training form: the forward also leaves the masked sums, the backward then needs one pass over the edges
        out_m = torch.empty_like(X)
        csum = torch.empty((V, H), dtype=torch.float32, device=dev)
        t_fs = time_call(lambda: hgnn.hgnn_gat_forward_fused_save(g, plan, H, D, X, X, a_l, a_r, out, lse, out_m, csum))
        t_bs = time_call(lambda: hgnn.hgnn_gat_backward_fused_saved(g, plan, gt, plan_t, H, D, X, X, a_l, a_r, out, lse, out_m,
                                                                   csum, dY, dh, d_el, d_er))
        fused = {"gat_forward_fused_ms": round(t_f, 4), "three_call_forward_ms": round(three, 4),
                 "gat_backward_fused_ms": round(t_b, 4), "five_call_backward_ms": round(five, 4),
                 "gat_fwd_bwd_fused_ms": round(t_f + t_b, 4), "alpha_from_lse_ms": round(t_a, 4),
                 "gat_forward_fused_save_ms": round(t_fs, 4), "gat_backward_fused_saved_ms": round(t_bs, 4),
                 "gat_fwd_bwd_fused_saved_ms": round(t_fs + t_bs, 4)}

    if not args.no_side:
        # the dense side of a layer on the matrix cores (hidden -> hidden projection of this workload's width), and for the
        # GAT workloads a whole layer: projection + fused aggregation forward, and every gradient backward
        Wd = (torch.randn((F, F), device=dev, dtype=torch.float32) / (F ** 0.5)).to(half)
        hproj = torch.empty_like(X)
        dW = torch.empty((F, F), dtype=torch.float32, device=dev)
        dws = torch.empty(max(hgnn.hgnn_linear_wgrad_workspace(F, F), hgnn.hgnn_gat_feature_grad_workspace(H, D)),
                          dtype=torch.uint8, device=dev)
        lin_bytes = V * (F + F) * 2 + F * F * 2
        t_lin = time_call(lambda: hgnn.hgnn_linear(X, Wd, hproj))
        t_lint = time_call(lambda: hgnn.hgnn_linear(dY, Wd, hproj, trans_w=True))
        t_wg = time_call(lambda: hgnn.hgnn_linear_wgrad(X, dY, dW, dws))
        dense = {"K": F, "F": F, "linear_ms": round(t_lin, 4), "linear_GBps": round(lin_bytes / (t_lin * 1e-3) / 1e9, 1),
                 "linear_transposed_ms": round(t_lint, 4), "linear_wgrad_ms": round(t_wg, 4),
                 "linear_wgrad_GBps": round((V * 2 * F * 2 + F * F * 4) / (t_wg * 1e-3) / 1e9, 1)}
        if has_gat:
            da_l, da_r = torch.empty(F, dtype=torch.float32, device=dev), torch.empty(F, dtype=torch.float32, device=dev)
            dfeat, dXin = torch.empty_like(X), torch.empty_like(X)

            def layer_fwd():
                hgnn.hgnn_linear(X, Wd, hproj)
                hgnn.hgnn_gat_forward_fused_save(g, plan, H, D, hproj, hproj, a_l, a_r, out, lse, out_m, csum)

            def layer_bwd():
                hgnn.hgnn_gat_backward_fused_saved(g, plan, gt, plan_t, H, D, hproj, hproj, a_l, a_r, out, lse, out_m, csum, dY, dh,
                                                   d_el, d_er)
                hgnn.hgnn_gat_feature_grad(H, D, dh, d_el, d_er, a_l, a_r, hproj, dfeat, da_l, da_r, dws)
                hgnn.hgnn_linear(dfeat, Wd, dXin, trans_w=True)
                hgnn.hgnn_linear_wgrad(X, dfeat, dW, dws)

            t_lf = time_call(layer_fwd)
            t_lb = time_call(layer_bwd)
            t_fg = time_call(lambda: hgnn.hgnn_gat_feature_grad(H, D, dh, d_el, d_er, a_l, a_r, hproj, dfeat, da_l, da_r, dws))
            dense.update({"gat_feature_grad_ms": round(t_fg, 4), "gat_layer_with_projection_fwd_ms": round(t_lf, 4),
                          "gat_layer_with_projection_bwd_ms": round(t_lb, 4),
                          "gat_layer_with_projection_fwd_bwd_ms": round(t_lf + t_lb, 4)})

    if args.variants:
        # the paper's two SpMM micro-benchmarks (atomic vs. non-atomic conflict writes; the vertex-parallel
        # form with neighbour groups), forward SpMM of this workload, all on the whole graph (no column blocks)
        plan1 = hgnn.hgnn_plan_create(g, args.seg_edges, F, H, col_blocks=1)
        cand = [("edge_segments_staged", lambda: hgnn.hgnn_spmm_discretized_variant(plan1, g, ew, 1, X, Y, hgnn.HGNN_EDGE_SEGMENTS)),
                ("edge_segments_atomic", lambda: hgnn.hgnn_spmm_discretized_variant(plan1, g, ew, 1, X, Y, hgnn.HGNN_EDGE_SEGMENTS_ATOMIC))]
        variants = {}

        for name, fn in cand:
            variants[name] = {"ms": round(time_call(fn), 4)}
        for ng in (64, 256):
            hgnn.hgnn_plan_add_groups(plan1, g, ng)
            variants[f"vertex_groups_{ng}"] = {
                "ms": round(time_call(lambda: hgnn.hgnn_spmm_discretized_variant(plan1, g, ew, 1, X, Y, hgnn.HGNN_VERTEX_GROUPS)), 4),
                "groups": hgnn.hgnn_plan_num_groups(plan1)}
        variants["vertex_groups_256_half2_arithmetic"] = {
            "ms": round(time_call(lambda: hgnn.hgnn_spmm_discretized_variant(plan1, g, ew, 1, X, Y, hgnn.HGNN_VERTEX_GROUPS_HALF2)), 4)}
        variants["vertex_rows_no_plan"] = {"ms": round(time_call(lambda: hgnn.hgnn_spmm(g, ew, 1, X, Y, workspace=spmm_ws)), 4)}
        variants["vertex_rows_no_plan_no_workspace"] = {"ms": round(time_call(lambda: hgnn.hgnn_spmm(g, ew, 1, X, Y)), 4)}
        for k in variants:
            variants[k]["req_GBps"] = round(spmm_req(wH, False) / (variants[k]["ms"] * 1e-3) / 1e9, 1)
        hgnn.hgnn_plan_destroy(plan1)

    if args.width_sweep:
        # the half2-against-half8 study of the paper's micro-benchmarks, on this GPU: same kernels, 4 / 8 / 16 bytes per lane
        width_sweep = {}
        plan1 = hgnn.hgnn_plan_create(g, args.seg_edges, 128, 1, col_blocks=1)
        hgnn.hgnn_plan_add_groups(plan1, g, 256)
        gen = torch.Generator(device=dev)
        gen.manual_seed(0x48474E4E)
        e1 = torch.empty((E, 1), dtype=half, device=dev)

        for Fs in (16, 32, 64, 128):
            Xs = torch.randn((V, Fs), generator=gen, device=dev, dtype=torch.float32).to(half)
            Ys = torch.empty_like(Xs)
            for vw in (2, 4, 8):
                hgnn.hgnn_plan_set_vector_halves(plan1, vw)
                width_sweep[f"F{Fs}_halves{vw}"] = {
                    "sddmm_dot_ms": round(time_call(lambda: hgnn.hgnn_sddmm(g, plan1, hgnn.HGNN_SDDMM_DOT, 1, Fs, Xs, Xs, e1)), 4),
                    "spmm_vertex_groups_ms": round(time_call(lambda: hgnn.hgnn_spmm_discretized_variant(
                        plan1, g, None, 1, Xs, Ys, hgnn.HGNN_VERTEX_GROUPS)), 4)}
        hgnn.hgnn_plan_destroy(plan1)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(np, w, gt, feat_np, grad_np, H, D, detail)

    res = {
        "value": round(value, 1), "unit": "GB/s", "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "timed_region_s": round(wall, 3),
        "config": {"workload": w.name, "V": V, "E": E, "F": F, "H": H, "seg_edges": args.seg_edges,
                   "col_blocks": hgnn.hgnn_plan_col_blocks(plan), "col_slices": hgnn.hgnn_plan_num_slices(plan), "cache_bytes_l2_llc": list(hgnn.hgnn_plan_cache_bytes(plan)),
                   "ops_per_step": [o[0] for o in ops]},
        "roofline": roofline, "cpu_baseline": cpu,
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4), "step_algorithmic_bytes": int(step_bytes),
        "layers": layer_ms, "ops": detail, "column_norm": prescaled, "graph": graph_info, "static_edge_values": static_w,
        "gat_fused": fused, "dense": dense, "variants": variants, "width_sweep": width_sweep,
        "setup": {"generate_s": round(gen_s, 2), "transpose_and_plans_s": round(setup_s, 3)},
    }
    if args.detail:
        for o, t in zip(ops, op_avg):
            print(f"{o[0]:20s} {t:9.4f} ms  (cold {op_cold[ops.index(o)]:8.4f})  min {o[2] / 1e6:9.1f} MB {o[2] / (t * 1e-3) / 1e9:8.1f} GB/s   "
                  f"req {o[4] / 1e6:9.1f} MB {o[4] / (t * 1e-3) / 1e9:8.1f} GB/s   {o[1]}", file=sys.stderr)
        for label, obj in (("column norm", prescaled), ("static edge values", static_w), ("gat fused forward", fused)):
            if obj:
                print(label + " " + json.dumps(obj), file=sys.stderr)
        if graph_info:
            print("graph " + json.dumps({k: v for k, v in graph_info.items() if k != "ops"}), file=sys.stderr)
        if width_sweep:
            for k, v in width_sweep.items():
                print(f"width {k:18s} sddmm_dot {v['sddmm_dot_ms']:9.4f} ms   spmm_vertex_groups {v['spmm_vertex_groups_ms']:9.4f} ms",
                      file=sys.stderr)
        if variants:
            for k, v in variants.items():
                print(f"variant {k:24s} {v['ms']:9.4f} ms  req {v['req_GBps']:8.1f} GB/s", file=sys.stderr)
    hgnn.hgnn_plan_destroy(plan)
    hgnn.hgnn_plan_destroy(plan_t)
    return res


def cpu_baseline(np, w, gt, feat_np, grad_np, H, D, detail):
    """The fp64 oracle, one thread, on a degree-stratified row sample of this workload: each of the kernels of the path
    it defines (SpMM forward, SpMM on the transposed graph, SDDMM dot, GAT score, edge softmax forward and backward),
    about two seconds each.  Throughput = compulsory bytes of the sample / seconds, the same accounting as the GPU ops."""
    import oracle
    V, E, F = w.V, w.E, w.F
    wv = w.tensors["w"].reshape(-1, 1) if "w" in w.tensors else None
    wH = 0 if wv is None else 1

    def spmm_bytes(n_rows, n_edges, transposed):
        return n_edges * (4 + 2 * wH + (4 if (transposed and wH) else 0)) + 4 * n_rows + 2 * n_rows * F + 2 * min(V, n_edges) * F

    # a probe sizes the sample: fp64 SpMM over ~0.3 M non-zeros
    rows_p = stratified_rows(np, w.rowptr, 300_000)
    t0 = time.perf_counter()
    oracle.spmm(w.rowptr, w.col, feat_np, w=wv, rows=rows_p)
    dt_p = max(time.perf_counter() - t0, 1e-4)
    e_p = int((w.rowptr[rows_p + 1] - w.rowptr[rows_p]).sum())
    target = int(min(E, max(e_p * 2.0 / dt_p, 50_000)))
    rows = stratified_rows(np, w.rowptr, target)
    rp_s, col_s, pos_s = sub_csr(np, w.rowptr, w.col, rows)
    n_e = int(rp_s[-1])
    kernels = {}

    def timed(name, gpu_op, nbytes, fn):
        t0 = time.perf_counter()
        fn()
        dt = time.perf_counter() - t0
        rec = {"seconds": round(dt, 3), "GBps": round(nbytes / dt / 1e9, 4), "non_zeros": n_e}
        if gpu_op in detail:
            rec["gpu_op"] = gpu_op
            rec["gpu_over_cpu"] = round(detail[gpu_op]["min_GBps"] / max(rec["GBps"], 1e-9), 1)
        kernels[name] = rec
        return dt

    dt_f = timed("spmm_forward", "spmm_fwd_disc", spmm_bytes(rows.size, n_e, False),
                 lambda: oracle.spmm(w.rowptr, w.col, feat_np, w=wv, rows=rows))
    # the transposed graph's arrays come from the device (inputs of a timing run only, nothing is compared)
    rT, cT, eT = gt.rowptr.cpu().numpy(), gt.col.cpu().numpy(), gt.eid.cpu().numpy()
    rows_t = stratified_rows(np, rT, target)
    n_et = int((rT[rows_t + 1] - rT[rows_t]).sum())
    t0 = time.perf_counter()
    oracle.spmm(rT, cT, grad_np, w=wv, eid=eT if wv is not None else None, rows=rows_t)
    dt = time.perf_counter() - t0
    kernels["spmm_transposed"] = {"seconds": round(dt, 3), "GBps": round(spmm_bytes(rows_t.size, n_et, True) / dt / 1e9, 4),
                                  "non_zeros": n_et}
    if "spmm_bwd_disc" in detail:
        kernels["spmm_transposed"]["gpu_op"] = "spmm_bwd_disc"
        kernels["spmm_transposed"]["gpu_over_cpu"] = round(detail["spmm_bwd_disc"]["min_GBps"] / max(kernels["spmm_transposed"]["GBps"], 1e-9), 1)
    del rT, cT, eT
    U_s = np.ascontiguousarray(grad_np[rows])
    nr = rows.size
    timed("sddmm_dot", "sddmm_dot", n_e * 4 + 4 * nr + 2 * nr * F + 2 * min(V, n_e) * F + 2 * n_e * H,
          lambda: oracle.sddmm_dot(rp_s, col_s, U_s, feat_np, H=H))
    a_l = w.tensors["a_l"] if "a_l" in w.tensors else None
    if a_l is None:
        import workloads as wl
        a_l, a_r = wl.normal_f16((H, D), 7, 0.0, 0.1), wl.normal_f16((H, D), 8, 0.0, 0.1)
    else:
        a_r = w.tensors["a_r"]
    # the score oracle takes one feature table for both sides: give it the whole table and a graph whose rows are the
    # sampled ones in place (all other rows empty)
    deg_full = np.zeros(V, dtype=np.int64)
    deg_full[rows] = rp_s[1:] - rp_s[:-1]
    rp_full = np.concatenate([[0], np.cumsum(deg_full)]).astype(np.int32)
    timed("gat_score", "gat_score", n_e * 4 + 4 * nr + 2 * (nr + min(V, n_e)) * F + 2 * n_e * H,
          lambda: oracle.gat_score(rp_full, col_s, feat_np, a_l, a_r, H))
    rng = np.random.default_rng(0x48474E4E)
    e_s = rng.standard_normal((n_e, H))
    alpha_s = [None]

    def sm_fwd():
        alpha_s[0] = oracle.edge_softmax(rp_s, e_s)

    timed("edge_softmax", "edge_softmax", 4 * n_e * H + 4 * nr, sm_fwd)
    da_s = rng.standard_normal((n_e, H))
    timed("edge_softmax_bwd", "edge_softmax_bwd", 8 * n_e * H + 4 * nr,
          lambda: oracle.edge_softmax_bwd(rp_s, alpha_s[0], da_s, e=e_s, slope=0.2))
    total_s = sum(k["seconds"] for k in kernels.values()) + dt_p
    return {"value": kernels["spmm_forward"]["GBps"], "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"fp64 oracle, one thread, on a degree-stratified sample of {w.name}: {rows.size} of {V} rows "
                      f"({n_e} non-zeros, {100.0 * n_e / E:.2f} % of E; every k-th row of the rows ordered by length, plus the "
                      f"longest); value = SpMM forward, the other kernels under 'kernels'; {total_s:.1f} s of CPU work in all",
            "kernels": kernels, "sample_rows": int(rows.size), "sample_non_zeros": n_e,
            "sample_share_of_E": round(n_e / E, 5), "host_cores_available": os.cpu_count()}


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build measures one GPU only (got --gpus {args.gpus}); "
              "the path is single-GPU; sharding by destination-row blocks is a design note only", file=sys.stderr)
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
    traffic_db = load_traffic()
    busy_probe = None if args.no_hbm_busy else HbmBusy(torch, np)
    busy_cal = busy_probe.calibrate(dev) if busy_probe is not None and busy_probe.path is not None else None
    results = {}
    for i, wname in enumerate(args.workloads):
        results[wname] = run_workload(args, wname, torch, np, hgnn, wl, dev, traffic_db, first=(i == 0),
                                      busy_probe=busy_probe, busy_cal=busy_cal)
        torch.cuda.empty_cache()
    head = results[args.workloads[0]]
    line = {"metric": "fp16 SpMM/SDDMM achieved HBM GB/s (% of peak) + GNN layer fwd+bwd ms",
            "value": head["value"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f16", "data": "synthetic"}
    for k in ("config", "roofline", "cpu_baseline", "frac_of_hbm_peak", "step_algorithmic_bytes", "layers", "ops",
              "column_norm", "graph", "static_edge_values", "gat_fused", "dense", "variants", "width_sweep", "setup"):
        line[k] = head[k]
    line["hbm_busy_calibration"] = busy_cal
    line["timed_region_s"] = round(sum(r["timed_region_s"] for r in results.values()), 3)
    line["configs"] = results
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
