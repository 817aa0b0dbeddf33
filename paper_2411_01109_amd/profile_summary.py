"""Turns rocprofv3 CSV output of `bench.py` runs into a short text summary and into the per-kernel traffic
data file that `bench.py` reads for its roofline object.

Expected input, all under one directory (here called D), for a workload tag W (c4, c5, ...), each produced by one
rocprofv3 run of `python3 bench.py --workload W --steps N --warmup 1 --no-cpu-baseline --no-hbm-busy --calib-copy`:

  D/prof_W_trace/W_kernel_stats.csv          --kernel-trace --stats
  D/prof_W_fetch/W_counter_collection.csv    --pmc FETCH_SIZE
  D/prof_W_write/W_counter_collection.csv    --pmc WRITE_SIZE
  D/prof_W_cache/W_counter_collection.csv    --pmc TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum TCC_EA0_RDREQ_DRAM_sum SQ_WAVES
                                                   SQ_INSTS_VMEM_RD SQ_INSTS_VMEM_WR SQ_INSTS_LDS SQ_LDS_BANK_CONFLICT
                                                   SQ_ACTIVE_INST_LDS SQ_BUSY_CYCLES SQ_WAVE_CYCLES TCP_TCC_READ_REQ_sum
                                                   TCP_TOTAL_CACHE_ACCESSES_sum TCP_TCC_WRITE_REQ_sum GRBM_GUI_ACTIVE   (optional)
  D/prof_W_ea/W_counter_collection.csv       --pmc TCC_EA0_RDREQ_sum TCC_EA0_RDREQ_32B_sum TCC_EA0_RDREQ_DRAM_32B_sum
                                                   TCC_EA0_WRREQ_WRITE_DRAM_32B_sum                                      (optional)

The 1 GiB device-to-device copy of `--calib-copy` scales the byte counters: whatever a counter reads for a copy of
known size gives its bytes per count on this chip.

usage: python -m paper_2411_01109_amd.profile_summary W "title of the workload" D out.md traffic.json workload_name [edges]
"""
import collections
import csv
import json
import os
import re
import sys

SETUP_KERNELS = ("validate", "expand", "iota", "source_rows", "offsets", "seg_rows", "compact", "scan_counts", "split_segs",
                 "block_fill", "block_cuts", "block_delta", "block_counts", "block_rowptr", "hub_zero", "group_", "coo_",
                 "list_length")
COPY = "__amd_rocclr_copyBuffer"
GIB_KIB = 1048576.0


def short(n):
    """hgnn::kernel<template arguments> from a mangled or demangled kernel name."""
    m = re.match(r"_ZN4hgnn(\d+)", n)
    if m:
        ln = int(m.group(1))
        st = m.end()
        name = n[st:st + ln]
        rest = n[st + ln:]
        args = []
        if rest.startswith("I"):
            for t, v in re.findall(r"L([ib])(\d+)E", rest.split("EEv")[0] + "E"):
                args.append(v if t == "i" else ("true" if v == "1" else "false"))
        return "hgnn::" + name + ("<" + ", ".join(args) + ">" if args else "")
    n = re.sub(r"^void ", "", n)
    n = re.sub(r"\(hgnn::\w+\)$", "", n)
    n = re.sub(r"\(.*$", "", n)
    return n[:76]


def read_counters(path):
    """{counter: {kernel: [values per dispatch]}}"""
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    if not os.path.exists(path):
        return None
    with open(path) as fh:
        for r in csv.DictReader(fh):
            acc[r.get("Counter_Name", "value")][short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return acc


def mean(v):
    return sum(v) / len(v) if v else 0.0


def is_compute(k):
    return k.startswith("hgnn::") and not any(s in k for s in SETUP_KERNELS)


def main(argv):
    W, title, D, out, traffic_path, wl_name = argv[:6]
    edges = float(argv[6]) if len(argv) > 6 else None
    base = lambda kind: os.path.join(D, f"prof_{W}_{kind}")
    with open(os.path.join(base("trace"), f"{W}_kernel_stats.csv")) as fh:
        stats = list(csv.DictReader(fh))
    fetch = read_counters(os.path.join(base("fetch"), f"{W}_counter_collection.csv"))
    write = read_counters(os.path.join(base("write"), f"{W}_counter_collection.csv"))
    cache = read_counters(os.path.join(base("cache"), f"{W}_counter_collection.csv"))
    ea = read_counters(os.path.join(base("ea"), f"{W}_counter_collection.csv"))
    fetch = fetch["FETCH_SIZE"] if fetch and "FETCH_SIZE" in fetch else next(iter(fetch.values()))
    write = write["WRITE_SIZE"] if write and "WRITE_SIZE" in write else next(iter(write.values()))
    cal_f, cal_w = max(fetch[COPY]), max(write[COPY])
    kf, kw = GIB_KIB / cal_f, GIB_KIB / cal_w  # true KiB per counted KiB
    bench_cmd = f"python3 $R/bench.py --workload {W} --steps {{n}} --warmup 1 --no-cpu-baseline --no-hbm-busy --calib-copy"
    L = [f"# rocprofv3 summary: hgnn kernels on {title} (one MI355X, bench.py step)\n",
         "Commands (run from /tmp with TMPDIR=/tmp, R = repository root; the tables are made from their CSV output by "
         "`python -m paper_2411_01109_amd.profile_summary`):\n", "```",
         f"rocprofv3 --kernel-trace --stats --output-format csv -d $R/gpurun_out/prof_{W}_trace -o {W} -- " + bench_cmd.format(n=5),
         f"rocprofv3 --pmc FETCH_SIZE --output-format csv -d $R/gpurun_out/prof_{W}_fetch -o {W} -- " + bench_cmd.format(n=2),
         f"rocprofv3 --pmc WRITE_SIZE --output-format csv -d $R/gpurun_out/prof_{W}_write -o {W} -- " + bench_cmd.format(n=2)]
    if cache:
        L.append(f"rocprofv3 --pmc {' '.join(sorted(cache))} --output-format csv -d $R/gpurun_out/prof_{W}_cache -o {W} -- " + bench_cmd.format(n=2))
    if ea:
        L.append(f"rocprofv3 --pmc {' '.join(sorted(ea))} --output-format csv -d $R/gpurun_out/prof_{W}_ea -o {W} -- " + bench_cmd.format(n=2))
    L.append("```\n")
    L.append(f"Counter calibration: the 1 GiB device-to-device copy of `--calib-copy` (`{COPY}`) reads FETCH_SIZE = {cal_f:.1f} KiB "
             f"and WRITE_SIZE = {cal_w:.1f} KiB for 1048576 KiB moved each way, so fetch bytes = FETCH_SIZE x {kf:.3f} KiB and write "
             f"bytes = WRITE_SIZE x {kw:.3f} KiB. FETCH_SIZE counts what the L2s request from the fabric: it includes reads that the "
             "Infinity Cache (the memory-side cache in front of HBM) serves, so it is an upper bound on HBM reads.\n")
    L.append("## Kernel durations (`*_kernel_stats.csv`, all launches of the run incl. warm-up)\n")
    L.append("| kernel | calls | avg us | min us | max us | % of GPU time |")
    L.append("|---|---:|---:|---:|---:|---:|")
    avg_us = {}
    for r in stats:
        k = short(r["Name"])
        avg_us[k] = float(r["AverageNs"]) / 1e3
        if float(r["Percentage"]) < 0.05:
            continue
        L.append(f"| `{k}` | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | {float(r['MinNs']) / 1e3:.1f} | "
                 f"{float(r['MaxNs']) / 1e3:.1f} | {float(r['Percentage']):.2f} |")
    L.append("\n## L2-miss traffic per launch (calibrated), hgnn compute kernels\n")
    L.append("| kernel | launches | fetch MB avg | fetch MB min | fetch MB max | write MB avg | (fetch+write) / avg time, TB/s |")
    L.append("|---|---:|---:|---:|---:|---:|---:|")
    tofb = lambda x: x * kf * 1024.0
    db = {}
    for k, v in sorted(fetch.items(), key=lambda kv: -mean(kv[1])):
        if not is_compute(k):
            continue
        wv = write.get(k, [0.0])
        fb, wb = tofb(mean(v)), mean(wv) * kw * 1024.0
        rate = (fb + wb) / (avg_us[k] * 1e-6) / 1e12 if avg_us.get(k) else float("nan")
        L.append(f"| `{k}` | {len(v)} | {fb / 1e6:.1f} | {tofb(min(v)) / 1e6:.1f} | {tofb(max(v)) / 1e6:.1f} | {wb / 1e6:.1f} | {rate:.2f} |")
        db[k] = {"fetch_bytes": round(fb), "write_bytes": round(wb), "launches_profiled": len(v), "avg_us": round(avg_us.get(k, 0.0), 2)}

    if ea:
        # bytes per counted request from the copy kernel: 1 GiB read / written
        rd32, wr32 = ea.get("TCC_EA0_RDREQ_DRAM_32B_sum"), ea.get("TCC_EA0_WRREQ_WRITE_DRAM_32B_sum")
        rq, rq32 = ea.get("TCC_EA0_RDREQ_sum"), ea.get("TCC_EA0_RDREQ_32B_sum")
        L.append("\n## Requests that leave the L2s for local memory (`TCC_EA0_*`), per launch\n")
        if rd32 and COPY in rd32 and max(rd32[COPY]) > 0:
            b_rd = GIB_KIB * 1024.0 / max(rd32[COPY])
            b_wr = GIB_KIB * 1024.0 / max(wr32[COPY]) if wr32 and COPY in wr32 and max(wr32[COPY]) > 0 else 32.0
            L.append(f"Calibration on the 1 GiB copy: `TCC_EA0_RDREQ_DRAM_32B_sum` = {max(rd32[COPY]):.0f} -> {b_rd:.1f} bytes per count; "
                     f"`TCC_EA0_WRREQ_WRITE_DRAM_32B_sum` -> {b_wr:.1f} bytes per count. \"DRAM\" in these counters names the "
                     "destination class of a request as the L2 sees it (local memory, as opposed to GMI = another device or "
                     "IO = the host): the Infinity Cache sits behind that interface, inside the memory side, so a request that it "
                     "serves is counted exactly like one that reaches an HBM stack. rocprofv3 on this machine offers no counter "
                     "of the memory controllers or of the data fabric (`rocprofv3 --list-avail`: blocks SQ, SQC, TA, TD, TCP, TCA, "
                     "TCC, SPI, CPC, CPF, GRBM only), so the split between Infinity-Cache hits and HBM accesses cannot be read "
                     "off a counter; what the tables give is the traffic between the L2s and the memory side.\n")
            L.append("| kernel | launches | read MB to local memory | write MB to local memory | read requests (M) | of them 32-byte (M) | read MB / FETCH_SIZE MB |")
            L.append("|---|---:|---:|---:|---:|---:|---:|")
            for k, v in sorted(rd32.items(), key=lambda kv: -mean(kv[1])):
                if not is_compute(k):
                    continue
                rb = mean(v) * b_rd
                wb = mean(wr32.get(k, [0.0])) * b_wr if wr32 else 0.0
                ratio = rb / db[k]["fetch_bytes"] if k in db and db[k]["fetch_bytes"] else float("nan")
                L.append(f"| `{k}` | {len(v)} | {rb / 1e6:.1f} | {wb / 1e6:.1f} | {mean(rq.get(k, [0.0])) / 1e6 if rq else 0:.2f} | "
                         f"{mean(rq32.get(k, [0.0])) / 1e6 if rq32 else 0:.2f} | {ratio:.3f} |")
                if k in db:
                    db[k]["local_memory_read_bytes"] = round(rb)
                    db[k]["local_memory_write_bytes"] = round(wb)

    if cache:
        hit, miss, req = cache.get("TCC_HIT_sum", {}), cache.get("TCC_MISS_sum", {}), cache.get("TCC_REQ_sum", {})
        waves, vrd, vwr = cache.get("SQ_WAVES", {}), cache.get("SQ_INSTS_VMEM_RD", {}), cache.get("SQ_INSTS_VMEM_WR", {})
        lds, conf, lact = cache.get("SQ_INSTS_LDS", {}), cache.get("SQ_LDS_BANK_CONFLICT", {}), cache.get("SQ_ACTIVE_INST_LDS", {})
        t_rd, t_acc = cache.get("TCP_TCC_READ_REQ_sum", {}), cache.get("TCP_TOTAL_CACHE_ACCESSES_sum", {})
        L.append("\n## Cache and wave counters per launch\n")
        L.append("L2 hit rate = TCC_HIT / (TCC_HIT + TCC_MISS); L1->L2 read requests = TCP_TCC_READ_REQ (per non-zero where the kernel "
                 "walks the graph's E edges once, E taken from the workload); L1 hit rate = 1 - TCP_TCC_READ_REQ / "
                 "TCP_TOTAL_CACHE_ACCESSES; LDS conflict share = SQ_LDS_BANK_CONFLICT / SQ_ACTIVE_INST_LDS (cycles).\n")
        L.append("| kernel | launches | L2 requests (M) | L2 hit rate | L1->L2 read req (M) | per non-zero | L1 accesses (M) | waves | "
                 "VMEM rd / wr instr (M) | LDS instr (M) | LDS conflict share |")
        L.append("|---|---:|---:|---:|---:|---:|---:|---:|---:|---:|---:|")
        for k, v in sorted(req.items(), key=lambda kv: -mean(kv[1])):
            if not is_compute(k):
                continue
            h, m_ = mean(hit.get(k, [0.0])), mean(miss.get(k, [0.0]))
            hr = h / (h + m_) if h + m_ > 0 else float("nan")
            rd = mean(t_rd.get(k, [0.0]))
            per_e = f"{rd / edges:.2f}" if edges else "-"
            la, lc = mean(lact.get(k, [0.0])), mean(conf.get(k, [0.0]))
            L.append(f"| `{k}` | {len(v)} | {mean(v) / 1e6:.1f} | {hr:.3f} | {rd / 1e6:.1f} | {per_e} | {mean(t_acc.get(k, [0.0])) / 1e6:.1f} | "
                     f"{mean(waves.get(k, [0.0])):.0f} | {mean(vrd.get(k, [0.0])) / 1e6:.2f} / {mean(vwr.get(k, [0.0])) / 1e6:.2f} | "
                     f"{mean(lds.get(k, [0.0])) / 1e6:.2f} | {lc / la if la > 0 else 0.0:.3f} |")
            if k in db:
                db[k].update({"l2_hit_rate": round(hr, 4), "l1_to_l2_read_requests": round(rd), "waves": round(mean(waves.get(k, [0.0])))})
    with open(out, "w") as fh:
        fh.write("\n".join(L) + "\n")
    try:
        with open(traffic_path) as fh:
            allw = json.load(fh)
    except (OSError, ValueError):
        allw = {}
    allw[wl_name] = db
    with open(traffic_path, "w") as fh:
        json.dump(allw, fh, indent=1, sort_keys=True)
        fh.write("\n")
    print("\n".join(L)[:6000])


if __name__ == "__main__":
    main(sys.argv[1:])
