"""Turns raw rocprofv3 output of the stand-alone profiling driver (agg_profile) into the short
summaries kept under profiles/.

Nothing here touches a GPU.  Input: a directory with one sub-directory per feature width, each
holding the output directories of up to four rocprofv3 passes over the same agg_profile command
plus the command's own output:

    DIR/meta.txt                 workload, op, dtype, options, source hash, date, the commands run
    DIR/F<width>/run.log         what agg_profile printed (its event timings)
    DIR/F<width>/stats/          rocprofv3 --kernel-trace --stats
    DIR/F<width>/fetch/          rocprofv3 --pmc FETCH_SIZE
    DIR/F<width>/write/          rocprofv3 --pmc WRITE_SIZE
    DIR/F<width>/tcc/            rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum

Output: profiles/aggregate_kernels_<workload>.md (tables) and profiles/hbm_traffic_<workload>.txt
(the figures bench.py prints as roofline.traffic, tagged with the hash of the kernel sources they
were measured on, so that a stale file is recognised).

    python -m paper_2104_06700_amd.profile_summary DIR [--out profiles]
    python -m paper_2104_06700_amd.profile_summary --source-hash
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import hashlib
import os
import re
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)

# kernels that make up one aggregation call (everything else in a trace is once-per-plan setup)
CALL_KERNELS = ("aggregate_kernel", "piece_kernel", "blk_finalize_kernel", "hub_finalize_kernel", "pad_rows_kernel",
                "pad_scale_rows_kernel")
CALIB_KERNEL = "copy16_kernel"
CALIB_BYTES = 1 << 30  # the calibration copy reads 1 GiB and writes 1 GiB


# sources of the aggregation calls (the layer, product and operator-table files do not change what they do)
AGGREGATION_SOURCES = ("aggregate.hip", "blocked.hip", "plan.hip", "graph.hip", "common.h")


def source_hash() -> str:
    """Hash of the sources of the aggregation kernels: identifies what a counter run measured."""
    h = hashlib.sha256()
    files = [os.path.join(PKG, "csrc", f) for f in AGGREGATION_SOURCES]
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def short_name(kernel: str) -> str:
    """'void (anonymous namespace)::aggregate_kernel<float, 4, 1, false>((anonymous namespace)::AggArgs)'
    -> 'aggregate_kernel<float, 4, 1, false>'."""
    k = kernel.replace("(anonymous namespace)::", "").replace("void ", "").strip()
    depth = 0
    for i, ch in enumerate(k):
        if ch == "<":
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0:
            return k[:i]
    return k[:60]


def _find(d: str, pattern: str):
    r = glob.glob(os.path.join(d, "**", pattern), recursive=True)
    return r[0] if r else None


def _counter_rows(d: str):
    p = _find(d, "*counter_collection.csv")
    return list(csv.DictReader(open(p))) if p else []


def _per_kernel(rows, counter):
    """{(kernel short name, grid): [values per dispatch]} for one counter."""
    out = collections.defaultdict(list)
    for r in rows:
        if r["Counter_Name"] == counter:
            out[(short_name(r["Kernel_Name"]), int(r["Grid_Size"]))].append(float(r["Counter_Value"]))
    return out


def _is_call_kernel(name: str) -> bool:
    return any(name.startswith(k) for k in CALL_KERNELS)


def read_meta(d: str) -> dict:
    meta = {"commands": []}
    p = os.path.join(d, "meta.txt")
    if os.path.exists(p):
        for line in open(p):
            line = line.rstrip("\n")
            if line.startswith("cmd: "):
                meta["commands"].append(line[5:])
            elif ": " in line:
                k, v = line.split(": ", 1)
                meta[k] = v
    return meta


def busy_ms(trace_csv: str, wanted) -> float:
    """Time during which at least one kernel accepted by `wanted(short name)` ran: the union of their
    [start, end] intervals.  Kernels of one call may run side by side on two streams (the short rows beside the
    source-blocked pieces), so their durations do not add up to the call's time; the union does."""
    spans = sorted((int(r["Start_Timestamp"]), int(r["End_Timestamp"])) for r in csv.DictReader(open(trace_csv))
                   if wanted(short_name(r["Kernel_Name"])))
    total, cur_a, cur_b = 0, None, None
    for a, b in spans:
        if cur_b is None or a > cur_b:
            if cur_b is not None:
                total += cur_b - cur_a
            cur_a, cur_b = a, b
        elif b > cur_b:
            cur_b = b
    if cur_b is not None:
        total += cur_b - cur_a
    return total / 1e6


def summarise_width(d: str) -> dict:
    """All figures of one width directory."""
    res = {"dir": d}
    # the driver's own timing
    log = os.path.join(d, "run.log")
    res["driver"] = [line.strip() for line in open(log) if line.startswith("N=") or line.startswith("source blocks")] \
        if os.path.exists(log) else []
    m = re.search(r"fwd ([\d.]+) ms\s+bwd ([\d.]+) ms", " ".join(res["driver"]))
    res["fwd_ms"], res["bwd_ms"] = (float(m.group(1)), float(m.group(2))) if m else (None, None)
    m = re.search(r"N=(\d+) E=(\d+) F=(\d+) (\w+)( weighted)?", " ".join(res["driver"]))
    if m:
        res.update(N=int(m.group(1)), E=int(m.group(2)), F=int(m.group(3)), esz=2 if m.group(4) == "bf16" else 4,
                   weighted=bool(m.group(5)))
    # kernel trace: mean duration and number of dispatches per (kernel, grid)
    trace = _find(os.path.join(d, "stats"), "*kernel_trace.csv")
    durations = collections.defaultdict(list)
    if trace:
        for r in csv.DictReader(open(trace)):
            grid = int(r["Grid_Size_X"]) * int(r.get("Grid_Size_Y", 1) or 1) * int(r.get("Grid_Size_Z", 1) or 1)
            durations[(short_name(r["Kernel_Name"]), grid)].append(
                (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6)
    res["durations"] = durations
    # calls in each pass: the driver prints how many it made (forward and backward, warm-up included)
    def calls_of(pass_name):
        p = os.path.join(d, pass_name + ".log")
        m2 = re.search(r"calls=(\d+)", open(p).read()) if os.path.exists(p) else None
        return int(m2.group(1)) if m2 else None
    n_calls = calls_of("stats")
    res["n_calls"] = n_calls
    counters = {}
    for sub, names in (("fetch", ["FETCH_SIZE"]), ("write", ["WRITE_SIZE"]), ("tcc", ["TCC_HIT_sum", "TCC_MISS_sum", "TCC_REQ_sum"])):
        rows = _counter_rows(os.path.join(d, sub))
        for n in names:
            counters[n] = _per_kernel(rows, n)
    res["counters"] = counters
    # calibration: what the counters read for the copy of known size
    scale = {}
    for n, true_kib in (("FETCH_SIZE", CALIB_BYTES / 1024), ("WRITE_SIZE", CALIB_BYTES / 1024)):
        vals = [v for (k, _), vs in counters.get(n, {}).items() if k.startswith(CALIB_KERNEL) for v in vs]
        scale[n] = (true_kib / (sum(vals) / len(vals))) if vals and sum(vals) > 0 else None
    res["scale"] = scale
    # per call totals over the kernels of a call
    def per_call(counter, factor):
        tot, seen = 0.0, False
        for (k, _), vs in counters.get(counter, {}).items():
            if _is_call_kernel(k):
                tot += sum(vs)
                seen = True
        n = calls_of({"FETCH_SIZE": "fetch", "WRITE_SIZE": "write"}.get(counter, "tcc"))
        return (tot * factor / n) if seen and n else None
    fs, ws = scale["FETCH_SIZE"], scale["WRITE_SIZE"]
    res["read_bytes_per_call"] = per_call("FETCH_SIZE", 1024.0 * fs) if fs else None
    res["write_bytes_per_call"] = per_call("WRITE_SIZE", 1024.0 * ws) if ws else None
    hit, miss, req = (per_call(c, 1.0) for c in ("TCC_HIT_sum", "TCC_MISS_sum", "TCC_REQ_sum"))
    res["tcc"] = (hit, miss, req)
    trace_ms = 0.0
    for (k, _), vs in durations.items():
        if _is_call_kernel(k):
            trace_ms += sum(vs)
    res["trace_ms_per_call"] = trace_ms / n_calls if n_calls else None
    res["busy_ms_per_call"] = busy_ms(trace, _is_call_kernel) / n_calls if trace and n_calls else None
    return res


def algorithmic_bytes(n, e, f, esz, ip_bytes, weighted, src_scaled):
    b = 2 * n * f * esz + 4 * e + (n + 1) * ip_bytes
    if weighted:
        b += 4 * e
    if src_scaled:
        b += 4 * n
    return b


def write_summary(d: str, out_dir: str) -> None:
    meta = read_meta(d)
    workload = meta.get("workload", os.path.basename(d.rstrip("/")).replace("prof_", ""))
    widths = sorted((int(os.path.basename(p)[1:]), p) for p in glob.glob(os.path.join(d, "F*")) if os.path.isdir(p))
    if not widths:
        sys.exit(f"no F<width> directories under {d}")
    results = [(f, summarise_width(p)) for f, p in widths]
    ip_bytes = int(meta.get("indptr_bytes", 4))
    lines = []
    r0 = results[0][1]
    lines.append(f"# Aggregation kernels on {workload} (N={r0.get('N')}, E={r0.get('E')}, op={meta.get('op', '?')}, "
                 f"{'bf16' if r0.get('esz') == 2 else 'fp32'}{', explicit edge weights' if r0.get('weighted') else ''})")
    lines.append("")
    lines.append(f"Written by `python -m paper_2104_06700_amd.profile_summary` from rocprofv3 output; kernel sources "
                 f"`{meta.get('source_hash', '?')}` (hash of the aggregation sources), {meta.get('date', '?')}.")
    lines.append("One agg_profile process per width and pass; a CALL = all kernels of one gnn_aggregate_fwd / _bwd "
                 "(copy into the plan's layout, piece / row / tail launches, finalisation).  Commands, from the repository root "
                 "on the MI355X box:")
    lines.append("")
    for c in meta["commands"]:
        lines.append(f"    {c}")
    lines.append("")
    traffic_lines = [f"# HBM-side traffic of one aggregation call on {workload}: (FETCH_SIZE x scale + WRITE_SIZE x scale) bytes summed",
                     "# over the kernels of a call, scale = 1 GiB / what the same counter reads for a 1 GiB copy in the same run.",
                     f"# Written by paper_2104_06700_amd.profile_summary from {os.path.basename(d.rstrip('/'))}; see aggregate_kernels_{workload}.md.",
                     f"source_hash {meta.get('source_hash', 'unknown')}"]
    for f, r in results:
        lines.append(f"## F = {f}")
        lines.append("")
        for t in r["driver"]:
            lines.append(f"    {t}")
        lines.append("")
        lines.append("    kernel                              grid  dispatches   mean ms   FETCH_SIZE KiB   WRITE_SIZE KiB      TCC_REQ      TCC_HIT   hit %")
        keys = sorted((k for k in r["durations"] if _is_call_kernel(k[0]) or k[0].startswith(CALIB_KERNEL)),
                      key=lambda k: (-sum(r["durations"][k]), k))
        for k in keys:
            dur = r["durations"][k]
            def mean(c):
                v = r["counters"].get(c, {}).get(k)
                return sum(v) / len(v) if v else None
            fe, wr, rq, hi = mean("FETCH_SIZE"), mean("WRITE_SIZE"), mean("TCC_REQ_sum"), mean("TCC_HIT_sum")
            fmt = lambda x, w: f"{x:{w},.0f}" if x is not None else " " * (w - 1) + "-"
            hitp = f"{100.0 * hi / rq:6.1f}" if rq and hi is not None else "     -"
            lines.append(f"    {k[0]:34s} {k[1]:>9d} {len(dur):>7d} {sum(dur) / len(dur):>10.3f} {fmt(fe, 16)} {fmt(wr, 16)} "
                         f"{fmt(rq, 12)} {fmt(hi, 12)}  {hitp}")
        lines.append("")
        sc = r["scale"]
        lines.append(f"    counter scale from the 1 GiB copy: FETCH_SIZE x {sc['FETCH_SIZE']:.3f}, WRITE_SIZE x {sc['WRITE_SIZE']:.3f}"
                     if sc["FETCH_SIZE"] and sc["WRITE_SIZE"] else "    counter scale: calibration copy not found in this run")
        if r.get("N") and r["read_bytes_per_call"] is not None and r["write_bytes_per_call"] is not None:
            n, e, esz = r["N"], r["E"], r["esz"]
            alg = algorithmic_bytes(n, e, f, esz, ip_bytes, r["weighted"], False)
            gathered = e * f * esz
            rd, wr = r["read_bytes_per_call"], r["write_bytes_per_call"]
            ms = (r["fwd_ms"] + r["bwd_ms"]) / 2 if r["fwd_ms"] else None
            hit, miss, req = r["tcc"]
            hitp = 100.0 * hit / req if req else None
            lines.append(f"    per call: L2-miss reads {rd / 1e9:.2f} GB + writes {wr / 1e9:.2f} GB = {(rd + wr) / 1e9:.2f} GB behind the L2s; "
                         f"compulsory {alg / 1e9:.2f} GB ({(rd + wr) / alg:.1f}x); gathered {gathered / 1e9:.1f} GB "
                         f"(reuse = gathered / fetched = {gathered / rd:.2f})")
            if ms:
                busy = r.get("busy_ms_per_call")
                overlap = (f"; their durations add up to {r['trace_ms_per_call']:.3f} ms because the short rows run beside the pieces on a "
                           f"second stream") if r["trace_ms_per_call"] > 1.02 * busy else ""
                lines.append(f"    per call: {ms:.3f} ms by the driver's events ({busy:.3f} ms of the kernel trace covered by at least one of "
                             f"the call's kernels{overlap}): "
                             f"{(rd + wr) / ms / 1e9:.2f} TB/s behind the L2s, {gathered / ms / 1e9:.2f} TB/s gathered, "
                             f"{alg / ms / 1e9 / 8.0 * 100:.2f} % of the 8 TB/s peak on compulsory bytes"
                             + (f"; L2 hit rate {hitp:.1f} %" if hitp is not None else ""))
            traffic_lines.append(f"traffic_bytes_F{f}_call {rd + wr:.4e}")
            if hitp is not None:
                traffic_lines.append(f"tcc_hit_pct_F{f} {hitp:.2f}")
            if ms:
                traffic_lines.append(f"ms_F{f}_call {ms:.4f}")
        lines.append("")
    os.makedirs(out_dir, exist_ok=True)
    with open(os.path.join(out_dir, f"aggregate_kernels_{workload}.md"), "w") as fh:
        fh.write("\n".join(lines) + "\n")
    with open(os.path.join(out_dir, f"hbm_traffic_{workload}.txt"), "w") as fh:
        fh.write("\n".join(traffic_lines) + "\n")
    print(f"wrote {out_dir}/aggregate_kernels_{workload}.md and hbm_traffic_{workload}.txt")


def write_bench_stats(d: str, out_dir: str) -> None:
    """rocprofv3 --kernel-trace --stats of the bench command itself (DIR holds its output and bench.json,
    the JSON line of the same run): the kernels of the aggregation calls, and whether their summed mean
    agrees with the call time the JSON line reports."""
    import json
    stats = _find(d, "*kernel_stats.csv")
    line = [l for l in open(os.path.join(d, "bench.json")) if l.startswith("{")][-1]
    res = json.loads(line)
    cmd = open(os.path.join(d, "cmd.txt")).read().strip() if os.path.exists(os.path.join(d, "cmd.txt")) else "?"
    workload = res["config"]["workload"].split(":")[0]
    rows = list(csv.DictReader(open(stats)))
    n_calls = (res["steps"] + res["warmup"]) * res["roofline"]["launches_per_step"]
    out = [f"# rocprofv3 kernel statistics of the bench command ({workload}, {res['steps']} steps + {res['warmup']} warm-up)", "",
           "Written by `python -m paper_2104_06700_amd.profile_summary --bench-stats`.  Command (repository root, MI355X box):", "",
           f"    {cmd}", "",
           "    kernel                                      calls    total ms     mean ms      %"]
    call_total = 0.0
    for r in rows:
        name = short_name(r["Name"])
        if not _is_call_kernel(name):
            continue
        call_total += float(r["TotalDurationNs"]) / 1e6
        out.append(f"    {name:42s} {int(r['Calls']):>6d} {float(r['TotalDurationNs']) / 1e6:>11.3f} {float(r['AverageNs']) / 1e6:>11.4f} "
                   f"{float(r['Percentage']):>6.2f}")
    trace = _find(d, "*kernel_trace.csv")
    busy = busy_ms(trace, _is_call_kernel) if trace else None
    busy_txt = (f"  At least one of them was running during {busy:.3f} ms = {busy / n_calls:.3f} ms per call (union of their intervals in "
                f"the kernel trace: the launches over the short rows run beside the source-blocked pieces on a second stream, so the "
                f"durations above overlap and do not add up to the call).") if busy is not None else ""
    out += ["", f"{n_calls} aggregation calls = ({res['steps']} + {res['warmup']}) steps x {res['roofline']['launches_per_step']} calls; "
                f"the kernels above sum to {call_total:.3f} ms = {call_total / n_calls:.3f} ms per call.{busy_txt}",
            f"The JSON line of the same run: value {res['value']} {res['unit']}, {res['ms_per_step']} ms per step, mean call "
            f"{res['roofline']['avg_launch_ms']} ms by events on the launch stream (`roofline.avg_launch_ms`; the unit the roofline is "
            f"taken over is the call = its copy into the plan's layout + piece / row / tail launches + finalisation), "
            f"roofline.frac {res['roofline']['frac']}.", "",
            "Per call (events, ms): " + ", ".join(f"{c['dir']} F={c['F']} {c['ms']}" for c in res["calls"]), ""]
    os.makedirs(out_dir, exist_ok=True)
    path = os.path.join(out_dir, f"bench_kernel_stats_{workload}.md")
    open(path, "w").write("\n".join(out))
    print(f"wrote {path}")


LAYER_KERNELS = CALL_KERNELS + ("gemm_kernel", "gemm_reduce_kernel", "mask_colsum_kernel", "colsum_reduce_kernel", "zero_kernel")


def write_layer_summary(d: str, out_dir: str) -> None:
    """Kernels and bytes of the GraphSAGE layer calls.  DIR holds one directory per variant (named for the
    GNN_LAYER_* flags it ran with), each with bench.json (the line of `bench.py --layers-only`), cmd.txt and
    the rocprofv3 output directories stats/ (--kernel-trace --stats), fetch/ and write/ (--pmc FETCH_SIZE /
    WRITE_SIZE) of that same command."""
    import json
    variants = sorted(x for x in os.listdir(d) if os.path.isdir(os.path.join(d, x)))
    out, workload = [], "?"
    fscale, wscale = 2.0, 1.0  # counter units per KiB, from the 1 GiB copy of the aggregation profiles of the same machine type
    for v in variants:
        vd = os.path.join(d, v)
        res = json.loads([l for l in open(os.path.join(vd, "bench.json")) if l.startswith("{")][-1])["layers"][0]
        workload = res["workload"]
        calls = res["calls_per_layer_and_direction"]
        cmd = open(os.path.join(vd, "cmd.txt")).read().strip()
        stats = {short_name(r["Name"]): r for r in csv.DictReader(open(_find(os.path.join(vd, "stats"), "*kernel_stats.csv")))}
        fetch, write = collections.defaultdict(float), collections.defaultdict(float)
        for sub, counter, acc in (("fetch", "FETCH_SIZE", fetch), ("write", "WRITE_SIZE", write)):
            for r in _counter_rows(os.path.join(vd, sub)):
                if r["Counter_Name"] == counter:
                    acc[short_name(r["Kernel_Name"])] += float(r["Counter_Value"])
        out += [f"## layer flags = {res['layer_flags']} ({v})", "", f"    {cmd}", "",
                f"    {'kernel':46s} {'calls':>6s} {'mean ms':>9s} {'ms/epoch':>9s} {'read GB/epoch':>14s} {'written GB/epoch':>17s}"]
        tot_ms = tot_r = tot_w = 0.0
        for name in sorted(stats, key=lambda k: -float(stats[k]["TotalDurationNs"])):
            if not any(name.startswith(k) for k in LAYER_KERNELS):
                continue
            r = stats[name]
            ms = float(r["TotalDurationNs"]) / 1e6 / calls
            rd, wr = fetch.get(name, 0.0) * fscale * 1024 / 1e9 / calls, write.get(name, 0.0) * wscale * 1024 / 1e9 / calls
            tot_ms += ms
            tot_r += rd
            tot_w += wr
            out.append(f"    {name:46s} {int(r['Calls']):>6d} {float(r['AverageNs']) / 1e6:>9.4f} {ms:>9.3f} {rd:>14.2f} {wr:>17.2f}")
        out += [f"    {'all kernels of the layer calls':46s} {'':>6s} {'':>9s} {tot_ms:>9.3f} {tot_r:>14.2f} {tot_w:>17.2f}", "",
                f"    per layer (events on the launch stream, ms; {calls} calls each): " +
                "; ".join(f"{l['layer']} fwd {l['fwd_ms']} bwd {l['bwd_ms']} (workspace {l['bwd_workspace_GB']} GB)" for l in res["layers"]),
                f"    model: forward {res['fwd_ms']} ms, backward {res['bwd_ms']} ms", ""]
    head = [f"# Kernels and bytes behind the L2s of the GraphSAGE layer calls ({workload})", "",
            f"Written by `python -m paper_2104_06700_amd.profile_summary --layers`; kernel sources `{source_hash()}`.",
            "An epoch here = one forward and one backward call of every layer of the model (no loss, no optimizer).  Three runs of",
            "the same command per variant: `rocprofv3 --kernel-trace --stats`, `--pmc FETCH_SIZE`, `--pmc WRITE_SIZE` (KiB per",
            f"dispatch, scaled x {fscale:.0f} / x {wscale:.0f} as calibrated with the 1 GiB copy of the aggregation profiles).  ms/epoch of a kernel =",
            "its total time / calls per layer and direction; kernels that run side by side on two streams (the weight-gradient",
            "product beside the backward aggregation) both count in full, so the sum exceeds the epoch's wall time.", ""]
    os.makedirs(out_dir, exist_ok=True)
    path = os.path.join(out_dir, f"layer_kernels_{workload}.md")
    open(path, "w").write("\n".join(head + out))
    print(f"wrote {path}")


def write_reuse_study(d: str, out_dir: str) -> None:
    """Reuse of gathered rows (the quantity of the paper's Table 3) per variant: DIR holds one directory per
    variant (NN_name/F<width>/{run.log, fetch/, tcc/}, plus variant.txt and order.txt) and meta.txt."""
    meta = read_meta(d)
    workload = meta.get("workload", "?")
    rows = []
    for v in sorted(p for p in glob.glob(os.path.join(d, "*")) if os.path.isdir(p)):
        fdirs = glob.glob(os.path.join(v, "F*"))
        if not fdirs:
            continue
        r = summarise_width(fdirs[0])
        name = os.path.basename(v).split("_", 1)[1].replace("_", " ")
        args = open(os.path.join(v, "variant.txt")).read().strip()
        order = open(os.path.join(v, "order.txt")).read().strip()
        rows.append((name, order, args, r))
    if not rows:
        sys.exit(f"no variants under {d}")
    r0 = rows[0][3]
    gathered = r0["E"] * r0["F"] * r0["esz"]
    out = [f"# Reuse of gathered rows on {workload} (N={r0['N']}, E={r0['E']}, F={r0['F']}, fp32 MEAN, forward and backward)", "",
           f"Written by `python -m paper_2104_06700_amd.profile_summary --reuse-study`; kernel sources `{meta.get('source_hash')}`, "
           f"{meta.get('date')}.  reuse = gathered bytes E*F*4 ({gathered / 1e9:.1f} GB) / bytes fetched past the L2s per call "
           f"(FETCH_SIZE x the scale a 1 GiB copy gives in the same run, all kernels of a call); the ideal is the average degree "
           f"{r0['E'] / r0['N']:.1f} (every row fetched once).  Commands:", ""]
    out += [f"    {c}" for c in meta["commands"]]
    out += ["", "    variant                                   vertex order   VARIANT arguments              ms/call   fetched GB   reuse   L2 hit %"]
    for name, order, args, r in rows:
        rd = r["read_bytes_per_call"]
        hit, miss, req = r["tcc"]
        ms = (r["fwd_ms"] + r["bwd_ms"]) / 2
        out.append(f"    {name:41s} {order:14s} {args:28s} {ms:>9.3f} {rd / 1e9:>12.2f} {gathered / rd:>7.2f} {100.0 * hit / req:>10.1f}")
    out.append("")
    os.makedirs(out_dir, exist_ok=True)
    path = os.path.join(out_dir, f"reuse_study_{workload}.md")
    open(path, "w").write("\n".join(out))
    print(f"wrote {path}")


def read_traffic(workload: str, widths) -> dict:
    """What bench.py reports next to its roofline: the mean HBM-side bytes per call over the calls of a
    step (two per width) and the L2 hit rate, or the reason why there is none."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return {"traffic": None, "reason": "no counter summary for this workload under profiles/"}
    vals = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()[:2]
        vals[k] = v
    if vals.get("source_hash") != source_hash():
        return {"traffic": None, "reason": f"profiles/hbm_traffic_{workload}.txt was measured on other kernel sources "
                                           f"({vals.get('source_hash')}, now {source_hash()})"}
    try:
        per = [float(vals[f"traffic_bytes_F{f}_call"]) for f in widths]
    except KeyError as err:
        return {"traffic": None, "reason": f"no counter run for width {err}"}
    hits = [float(vals[f"tcc_hit_pct_F{f}"]) for f in widths if f"tcc_hit_pct_F{f}" in vals]
    return {"traffic": sum(per) / len(per), "per_width": dict(zip(map(str, widths), per)),
            "tcc_hit_pct": round(sum(hits) / len(hits), 2) if hits else None, "source_hash": vals["source_hash"]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("dir", nargs="?")
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles"))
    ap.add_argument("--source-hash", action="store_true")
    ap.add_argument("--reuse-study", action="store_true", help="DIR holds one directory per variant of the reuse study")
    ap.add_argument("--bench-stats", action="store_true", help="DIR holds rocprofv3 --stats output of bench.py and its bench.json")
    ap.add_argument("--layers", action="store_true", help="DIR holds one directory per variant of `bench.py --layers-only`")
    args = ap.parse_args()
    if args.source_hash:
        print(source_hash())
        return
    if not args.dir:
        ap.error("DIR is required")
    if args.layers:
        write_layer_summary(args.dir, args.out)
    elif args.bench_stats:
        write_bench_stats(args.dir, args.out)
    elif args.reuse_study:
        write_reuse_study(args.dir, args.out)
    else:
        write_summary(args.dir, args.out)


if __name__ == "__main__":
    main()
