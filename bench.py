#!/usr/bin/env python3
"""Benchmark of the aggregation hot path on one MI355X.

A step = one pass of the aggregation stack of the workload: for every feature
width of the workload, one forward call (gnn_aggregate_fwd over the CSR) and one
backward call (gnn_aggregate_bwd over the transposed graph).  Graph generation,
the CSR/transpose build and the degree-binning plans are once-per-graph setup
(full-batch training reuses one static graph for every layer and epoch); they
run in the library too and are reported under "setup_ms", outside the timed
region.  All inputs are resident in HBM before the timed region starts.

Prints ONE JSON line (see the keys below).  `value` is edge-features per second
(edges x F, forward + backward), the unit of the paper's Table 8 work counts.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2104_06700_amd as gnn  # noqa: E402
import synth  # noqa: E402

HBM_PEAK_GBS = 8000.0  # MI355X published peak
OPS = {"sum": gnn.GNN_SUM, "mean": gnn.GNN_MEAN, "gcn": gnn.GNN_GCN_SYM}


def algorithmic_bytes(n, e, f, esz, ip_bytes, weighted, src_scaled):
    """Compulsory bytes of one aggregation call (one direction): every gathered
    row read once, every output row written once, the index stream (and the
    weight stream) read once, the row pointers read once, plus the per-vertex
    count array when the gathered rows carry a scale (MEAN backward, GCN)."""
    b = 2 * n * f * esz + 4 * e + (n + 1) * ip_bytes
    if weighted:
        b += 4 * e
    if src_scaled:
        b += 4 * n
    return b


def read_traffic_note(workload, widths):
    """HBM-side bytes per call and L2 hit rate measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE,
    TCC_*), from the summary that paper_2104_06700_amd.profile_summary wrote under profiles/ -- only if
    that summary was measured on the kernel sources of this tree (it records their hash)."""
    from paper_2104_06700_amd.profile_summary import read_traffic
    return read_traffic(workload, list(widths))


def calibrate(dev):
    """Measured ceilings printed next to the result: a streaming copy, and the aggregation
    kernel itself (no plan, rows gathered as they are) on synthetic gather patterns -- 2,449,029
    rows x 50 uniformly random neighbours, 400-byte rows -- whose neighbours all lie in the first
    5,000 rows of X (2 MB: L2-resident), the first 300,000 (120 MB: misses L2, fits the Infinity
    Cache), or anywhere (980 MB: HBM-resident)."""
    out = {}

    def timed(fn, reps=5):
        fn(); torch.cuda.synchronize()
        t0 = torch.cuda.Event(enable_timing=True); t1 = torch.cuda.Event(enable_timing=True)
        t0.record()
        for _ in range(reps):
            fn()
        t1.record(); torch.cuda.synchronize()
        return t0.elapsed_time(t1) / reps * 1e-3

    src = torch.empty(1 << 28, dtype=torch.float32, device=dev)  # 1 GiB
    dst = torch.empty_like(src)
    src.normal_()
    s = timed(lambda: gnn.gnn_calib_copy(src, dst))
    out["stream_copy_read_plus_write_GBs"] = round(2 * src.numel() * 4 / s / 1e9, 1)
    # bare gather of 128-byte lines (nothing accumulated into rows, nothing written but one float per thread):
    # what the memory system delivers per line request, from a table that fits every L2 and from one that does not
    ids = torch.empty(1 << 28, dtype=torch.int32, device=dev)
    probe_out = dst[: 1 << 23]
    for label, lines in (("line_gather_probe_L2_resident_GBs", 16_384), ("line_gather_probe_two_thirds_L2_hits_GBs", 49_152),
                         ("line_gather_probe_half_L2_hits_GBs", 65_536), ("line_gather_probe_L2_miss_infinity_cache_GBs", 1 << 20)):
        ids.random_(0, lines)
        n = gnn.gnn_calib_gather(src, lines, ids, probe_out)
        s = timed(lambda: gnn.gnn_calib_gather(src, lines, ids, probe_out), reps=3)
        out[label] = round(n * 128 / s / 1e9, 1)
    del dst, ids, probe_out
    n_rows, degree, f = 2_449_029, 50, 100
    x = src[: n_rows * f].view(n_rows, f)
    y = torch.empty((n_rows, f), dtype=torch.float32, device=dev)
    for label, rows in (("gather_L2_resident_GBs", 5_000), ("gather_L2_miss_infinity_cache_GBs", 300_000),
                        ("gather_L2_miss_hbm_GBs", n_rows)):
        indptr, idx = synth.regular_random_neighbours(n_rows, degree, rows, seed=rows, device=dev)
        s = timed(lambda: gnn.gnn_aggregate_fwd(indptr, idx, None, x, y, n_rows, f, gnn.GNN_SUM), reps=3)
        out[label] = round(n_rows * degree * f * 4 / s / 1e9, 1)  # gathered bytes per second
        del indptr, idx
    return out


def cpu_baseline(el, widths, op_name, target_seconds=20.0):
    """The oracle, as it stands, on this machine's host cores: the same step (forward and backward
    at every width) on a seeded sample of rows sized to about `target_seconds` of CPU work."""
    import oracle
    threads = oracle.max_threads()
    dst, src = synth.to_csr_numpy(el)
    indptr = oracle.csr_indptr(dst, el.n)
    indptr_t, indices_t, _ = oracle.transpose(indptr, src)
    din = np.diff(indptr)
    dout = np.diff(indptr_t)
    op = {"sum": oracle.OP_SUM, "mean": oracle.OP_MEAN, "gcn": oracle.OP_GCN_SYM}[op_name]
    rng = np.random.default_rng(12345)
    # probe for speed at the first width, then size the row sample to the time target
    f0 = widths[0]
    X0 = synth.normal_features(el.n, f0, 1).numpy()
    probe = rng.choice(el.n, size=min(el.n, 200000), replace=False)
    t0 = time.perf_counter()
    oracle.aggregate_fwd(indptr, src, X0, op=op, rows=probe, nthreads=threads, dout=dout)
    dt = max(time.perf_counter() - t0, 1e-4)
    rate = din[probe].sum() * f0 / dt                       # edge-features per second
    full_work = 2.0 * el.e * sum(widths)
    frac = min(1.0, rate * target_seconds / full_work)
    n_rows = max(1000, int(el.n * frac))
    rows = None if n_rows >= el.n else np.sort(rng.choice(el.n, size=n_rows, replace=False))
    ef = 0.0
    secs = 0.0
    for f in widths:
        X = X0 if f == f0 else synth.normal_features(el.n, f, 1).numpy()
        t0 = time.perf_counter()
        oracle.aggregate_fwd(indptr, src, X, op=op, rows=rows, nthreads=threads, dout=dout)
        oracle.aggregate_bwd(indptr_t, indices_t, X, op=op, rows=rows, nthreads=threads, din=din)
        secs += time.perf_counter() - t0
        ef += f * float((din.sum() + dout.sum()) if rows is None else (din[rows].sum() + dout[rows].sum()))
    what = "all rows" if rows is None else f"{n_rows} uniformly sampled rows per direction"
    # the same loops on ONE core, on a sample sized to a few seconds (forward at the first width)
    one_rows = np.sort(rng.choice(el.n, size=max(1000, min(el.n, int(el.n * min(1.0, rate / threads * 4.0 / (el.e * f0))))), replace=False))
    t0 = time.perf_counter()
    oracle.aggregate_fwd(indptr, src, X0, op=op, rows=one_rows, nthreads=1, dout=dout)
    one_secs = max(time.perf_counter() - t0, 1e-6)
    one_core = din[one_rows].sum() * f0 / one_secs / 1e9
    return {"value": round(ef / secs / 1e9, 4), "unit": "GEF/s", "cores": threads, "kind": "oracle",
            "sample": f"the same step (forward + backward {op_name}, widths {list(widths)}) on {what} of the same graph, "
                      f"{secs:.1f} s of CPU time, fp64 scalar loops, OpenMP dynamic over rows",
            "one_core_GEFs": round(float(one_core), 4),
            "one_core_sample": f"forward {op_name} at F={f0} on {len(one_rows)} sampled rows, {one_secs:.1f} s"}


def measure(workload, steps, warmup, scale, dev, dump_graph=None, flush=False, capture=False, relabel=None, packed_input=False):
    """Setup + warm-up + the timed region for one workload; returns (result dict, host edge list factory).
    flush: overwrite a 1 GiB scratch buffer before every call (outside the call's events), so that
    workloads whose matrices fit the caches start every call cold; value and ms_per_step are then
    the sums of the per-call event times instead of the wall clock over the steps.
    capture: also record one step into a HIP graph and time its replays (launch-bound workloads)."""
    w = synth.WORKLOADS[workload]
    widths = list(w["widths"])
    op_names = w["op"].split("+")
    dtype = torch.bfloat16 if w["dtype"] == "bf16" else torch.float32
    esz = 2 if dtype == torch.bfloat16 else 4

    # ---- setup (not timed as part of a step) ----
    t0 = time.perf_counter()
    el = synth.make_graph(workload, device=dev, scale=scale)
    if relabel:  # the same graph under another vertex order (reuse study)
        el = synth.relabel(el, relabel, seed=w["seed"])
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t0
    weights = synth.gcn_sym_edge_weights(el.dst, el.src, el.n) if w.get("weighted") else None
    t0 = time.perf_counter()
    dg = gnn.build_device_graph(el.dst, el.src, el.n, edge_w=weights, indptr64=w["indptr64"], with_plans=False)
    torch.cuda.synchronize()
    t_csr = time.perf_counter() - t0
    if dump_graph:
        os.makedirs(dump_graph, exist_ok=True)
        for name_, t in (("indptr", dg.indptr), ("indices", dg.indices), ("indptr_t", dg.indptr_t), ("indices_t", dg.indices_t)):
            t.cpu().numpy().tofile(os.path.join(dump_graph, name_ + ".bin"))
        with open(os.path.join(dump_graph, "meta.txt"), "w") as fh:
            fh.write(f"{el.n} {el.e} {1 if w['indptr64'] else 0}\n")
        print(f"dumped {workload} to {dump_graph}", file=sys.stderr)
        return None, None
    t0 = time.perf_counter()
    dg.plan_fwd = gnn.gnn_plan_create(dg.indptr, dg.indices, el.n)
    dg.plan_bwd = gnn.gnn_plan_create(dg.indptr_t, dg.indices_t, el.n)
    torch.cuda.synchronize()
    t_plan = time.perf_counter() - t0
    n, e = el.n, el.e
    fmax = max(widths)
    if weights is not None:  # the normalisation weights belong to the static graph: the plans keep them in piece order
        dg.plan_fwd.bind_edge_weights(dg.edge_w)
        dg.plan_bwd.bind_edge_weights(dg.edge_w_t)
    for op_name in op_names:
        for f in sorted(set(widths)):
            dg.plan_fwd.prepare(dg.indices, OPS[op_name], False, f, dtype)
            dg.plan_bwd.prepare(dg.indices_t, OPS[op_name], True, f, dtype)

    bufs = []  # one fresh set of inputs per layer of the stack
    for layer, f in enumerate(widths):
        X = synth.normal_features(n, f, 100 + layer, device=dev, dtype=dtype)
        dY = synth.normal_features(n, f, 200 + layer, device=dev, dtype=dtype)
        bufs.append((X, torch.empty_like(X), dY, torch.empty_like(dY)))
    torch.cuda.synchronize()

    calls = [(op_name, d, layer) for op_name in op_names for layer in range(len(widths)) for d in ("fwd", "bwd")]

    def one_call(op_name, d, layer):
        X, Y, dY, dX = bufs[layer]
        f = widths[layer]
        op = OPS[op_name]
        if d == "fwd":
            gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, dg.edge_w, X, Y, n, f, op, plan=dg.plan_fwd)
        else:
            gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, dg.edge_w_t, dY, dX, n, f, op, plan=dg.plan_bwd)

    scratch = torch.zeros(1 << 28, dtype=torch.float32, device=dev) if flush else None  # 1 GiB > L2 + Infinity Cache

    for _ in range(warmup):
        for op_name, d, layer in calls:
            one_call(op_name, d, layer)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps; events on the launch stream bracket every call ----
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in calls]
          for _ in range(steps)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(steps):
        for i, (op_name, d, layer) in enumerate(calls):
            if flush:
                scratch.add_(1.0)
            ev[k][i][0].record()
            one_call(op_name, d, layer)
            ev[k][i][1].record()
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t_start

    samples = [[ev[k][i][0].elapsed_time(ev[k][i][1]) for k in range(steps)] for i in range(len(calls))]
    per_call_ms = [float(np.mean(x)) for x in samples]
    if flush:  # the flushes are not part of a step
        t_total = sum(per_call_ms) * 1e-3 * steps
    ef_step = sum(2 * e * f for f in widths) * len(op_names)
    ms_per_step = t_total / steps * 1e3
    value = ef_step / (t_total / steps) / 1e9

    ip_bytes = 8 if w["indptr64"] else 4
    weighted = weights is not None
    call_rows = []
    for i, (op_name, d, layer) in enumerate(calls):
        f = widths[layer]
        src_scaled = (op_name in ("mean", "sage") and d == "bwd") or (op_name == "gcn" and not weighted)
        b = algorithmic_bytes(n, e, f, esz, ip_bytes, weighted, src_scaled)
        s = per_call_ms[i] * 1e-3
        call_rows.append({"op": op_name, "dir": d, "F": f, "ms": round(per_call_ms[i], 4),
                          "ms_median": round(float(np.median(samples[i])), 4), "ms_min": round(float(np.min(samples[i])), 4),
                          "GEF_per_s": round(e * f / s / 1e9, 2),
                          "algorithmic_GB": round(b / 1e9, 4), "algorithmic_GBs": round(b / s / 1e9, 1),
                          "frac_of_hbm_peak": round(b / s / 1e9 / HBM_PEAK_GBS, 4),
                          "gathered_TBs": round(e * f * esz / s / 1e12, 2)})
    # Dominant kernel = aggregate_kernel: one template instantiation serves every call of this
    # workload (forward and backward, all widths).  The unit timed is a CALL: the launches of that
    # kernel that cover the call's columns (one per group of up to 8 column slices, one for a dense
    # tail) plus, where the gathered rows are copied into padded rows first, the pad kernel, plus
    # the small hub finalisation; the events bracket the call, and the algorithmic bytes are the
    # call's.
    all_bytes = sum(r["algorithmic_GB"] for r in call_rows)
    all_s = sum(r["ms"] for r in call_rows) * 1e-3
    achieved = all_bytes / all_s
    tnote = read_traffic_note(workload, widths * len(op_names)) if scale == 1.0 else {"traffic": None, "reason": "scaled run"}
    traffic = tnote["traffic"]
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_GBs": None if traffic is None else round(traffic / (all_s / len(call_rows)) / 1e9, 1),
                "traffic_frac_of_peak": None if traffic is None else round(traffic / (all_s / len(call_rows)) / 1e9 / HBM_PEAK_GBS, 4),
                "traffic_note": tnote.get("reason") or f"rocprofv3 FETCH_SIZE + WRITE_SIZE per call, profiles/hbm_traffic_{workload}.txt "
                                                       f"(kernel sources {tnote.get('source_hash')})",
                "tcc_hit_pct": tnote.get("tcc_hit_pct"),
                "gathered_bytes_per_call": round(sum(e * r["F"] * esz for r in call_rows) / len(call_rows)),
                "line_requests_per_call": round(sum(e * ((r["F"] * esz + 127) // 128) for r in call_rows) / len(call_rows)),
                "kernel": "aggregate_kernel (all calls of one step: forward and backward at every width)",
                "per": "call (= its aggregate_kernel launches + pad copy + hub finalisation)",
                "launches_per_step": len(call_rows), "avg_launch_ms": round(all_s * 1e3 / len(call_rows), 4)}

    packed = None
    if packed_input and gnn.gnn_packed_bytes(n, widths[0], gnn.GNN_BF16 if esz == 2 else gnn.GNN_F32) > 0:
        # Layer 0 gathers the input features, which full-batch training never changes: the caller keeps their
        # packed copy and every epoch's forward call skips the copy.  Reported beside the step, not part of `value`.
        f0, op0 = widths[0], OPS[op_names[0]]
        X0, Y0 = bufs[0][0], bufs[0][1]
        buf = torch.empty(gnn.gnn_packed_bytes(n, f0, gnn.GNN_BF16 if esz == 2 else gnn.GNN_F32) // 4, dtype=torch.float32, device=dev)

        def timed(fn, reps=5):
            fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps

        t_pack = timed(lambda: gnn.gnn_pack_rows(dg.indptr, dg.indices, X0, buf, n, f0, op0, False, plan=dg.plan_fwd))
        t_packed = timed(lambda: gnn.gnn_aggregate_packed(dg.indptr, dg.indices, dg.edge_w, buf, Y0, n, f0, op0, False,
                                                          plan=dg.plan_fwd))
        t_plain = timed(lambda: one_call(op_names[0], "fwd", 0))
        packed = {"F": f0, "op": op_names[0], "dir": "fwd", "pack_once_ms": round(t_pack, 4), "ms_from_packed": round(t_packed, 4),
                  "ms_with_copy": round(t_plain, 4), "GEF_per_s_from_packed": round(e * f0 / (t_packed * 1e-3) / 1e9, 2),
                  "note": "input features kept packed by the caller (gnn_pack_rows once, gnn_aggregate_packed per epoch)"}
        del buf

    replay = None
    if capture:  # the same step as one captured graph: what is left when the launches cost nothing on the host
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for op_name, d, layer in calls:
                    one_call(op_name, d, layer)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        replay = {"ms_per_step": round(dt * 1e3, 4), "value": round(ef_step / dt / 1e9, 2), "unit": "GEF/s",
                  "note": "one step captured into a HIP graph and replayed; same kernels, no per-call host work"}

    result = {
        "metric": "aggregation GEdge-features/s (edges*F/s) fwd+bwd; % of HBM peak GB/s",
        "value": round(value, 2), "unit": "GEF/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if dtype == torch.bfloat16 else "f32", "data": "synthetic",
        "config": {"workload": f"{workload}: R-MAT/ER graph N={n} E={e}, op={w['op']}, widths={widths}, "
                               f"fwd+bwd per width" + ("" if scale == 1.0 else f" (SCALED x{scale}: not a result)"),
                   "N": n, "E": e, "widths": widths, "op": w["op"], "indptr_bits": ip_bytes * 8, "parallelism": "1 GPU",
                   "cache_flushed_before_every_call": bool(flush)},
        "roofline": roofline,
        "calls": call_rows,
        "setup_ms": {"graph_generation": round(t_gen * 1e3, 1), "csr_and_transpose": round(t_csr * 1e3, 1),
                     "plans_fwd_and_bwd": round(t_plan * 1e3, 1)},
    }
    if replay is not None:
        result["graph_replay"] = replay
    if packed is not None:
        result["static_input_packed"] = packed
    return result, (el, widths, op_names)


def measure_general_primitive(workload, dev, reps=5):
    """The general primitive (operator table, Table 1) and its gradients on the same graph: a
    few representative calls, each timed with events on the launch stream.  Not part of `value`."""
    w = synth.WORKLOADS[workload]
    el = synth.make_graph(workload, device=dev)
    n, e = el.n, el.e
    dg = gnn.build_device_graph(el.dst, el.src, n, indptr64=w["indptr64"], want_perm=True)
    ip = 8 if w["indptr64"] else 4
    rows = []

    def timed(name, d, bytes_, fn):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / reps
        rows.append({"call": name, "d": d, "ms": round(ms, 4), "GEF_per_s": round(e * d / ms / 1e6, 2),
                     "algorithmic_GB": round(bytes_ / 1e9, 4), "frac_of_hbm_peak": round(bytes_ / ms / 1e6 / HBM_PEAK_GBS, 4)})

    for d in (100, 32):
        fV = synth.normal_features(n, d, 301, device=dev)
        dO = synth.normal_features(n, d, 302, device=dev)
        fO = torch.empty_like(fV)
        dfV = torch.empty_like(fV)
        arg = torch.empty((n, d), dtype=torch.int32, device=dev)
        ws = synth.gcn_sym_edge_weights(el.dst, el.src, n).to(dev) + 0.5
        dws = torch.empty_like(ws)
        base = 2 * n * d * 4 + 4 * e + (n + 1) * ip
        B, R = gnn, gnn
        timed("fwd copylhs/max + winners", d, base + n * d * 4,
              lambda: gnn.gnn_ap_fwd(dg.indptr, dg.indices, fV, None, fO, arg, n, d, B.GNN_BIN_COPY_LHS, R.GNN_RED_MAX, plan=dg.plan_fwd))
        timed("vertex gradient of max (scatter to winners)", d, 4 * n * d * 4 + 4 * n * d,
              lambda: gnn.gnn_ap_bwd_vertex_arg(dg.indices, arg, dO, None, dfV, n, n, d, B.GNN_BIN_COPY_LHS))
        timed("fwd mul(scalar edge feature)/sum", d, base + 4 * e,
              lambda: gnn.gnn_ap_fwd(dg.indptr, dg.indices, fV, ws, fO, None, n, d, B.GNN_BIN_MUL, R.GNN_RED_SUM, plan=dg.plan_fwd))
        timed("edge gradient of mul(scalar)/sum (sampled dense-dense product)", d, 2 * n * d * 4 + 8 * e + (n + 1) * ip,
              lambda: gnn.gnn_ap_bwd_edge(dg.indptr, dg.indices, None, fV, ws, dO, dws, n, d, B.GNN_BIN_MUL, plan=dg.plan_fwd))
        if d == 32:
            fE = torch.rand((e, d), device=dev) + 0.5
            dfE = torch.empty_like(fE)
            timed("fwd mul(full-width edge features)/sum", d, base + e * d * 4,
                  lambda: gnn.gnn_ap_fwd(dg.indptr, dg.indices, fV, fE, fO, None, n, d, B.GNN_BIN_MUL, R.GNN_RED_SUM, plan=dg.plan_fwd))
            timed("fwd copyrhs/max + winners", d, n * d * 8 + 4 * e + e * d * 4 + (n + 1) * ip,
                  lambda: gnn.gnn_ap_fwd(dg.indptr, dg.indices, None, fE, fO, arg, n, d, B.GNN_BIN_COPY_RHS, R.GNN_RED_MAX, plan=dg.plan_fwd))
            timed("edge gradient of mul(full-width)/sum", d, 2 * n * d * 4 + 4 * e + e * d * 4 + (n + 1) * ip,
                  lambda: gnn.gnn_ap_bwd_edge(dg.indptr, dg.indices, None, fV, fE, dO, dfE, n, d, B.GNN_BIN_MUL, plan=dg.plan_fwd))
            timed("vertex gradient of mul(full-width)/sum (transposed graph, edge rows through perm)", d,
                  base + e * d * 4 + 8 * e,
                  lambda: gnn.gnn_ap_bwd_vertex(dg.indptr_t, dg.indices_t, dO, fE, dfV, n, d, B.GNN_BIN_MUL, plan=dg.plan_bwd, edge_ids=dg.perm))
            del fE, dfE
    return {"workload": workload, "reps": reps, "calls": rows,
            "note": "algorithmic_GB = operands read once + results written once; frac_of_hbm_peak = that / time / 8 TB/s"}


MODELS = {  # layer widths of the paper's GraphSAGE models (Section 6.1; Table 2 for inputs and classes)
    "rmat_sparse_stack": (100, 256, 256, 47),
    "rmat_dense_wide": (602, 16, 41),
}


def measure_layers(workload, dev, reps=5, flags=0):
    """Forward and backward of every layer of the paper's model for this graph shape (aggregation +
    dense update, gnn_sage_layer_*), each timed with events on the launch stream.  Not part of `value`."""
    dims = MODELS[workload]
    w = synth.WORKLOADS[workload]
    el = synth.make_graph(workload, device=dev)
    n, e = el.n, el.e
    dg = gnn.build_device_graph(el.dst, el.src, n, indptr64=w["indptr64"])
    rows = []

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    for li in range(len(dims) - 1):
        fi, fo = dims[li], dims[li + 1]
        relu = li < len(dims) - 2
        X = synth.normal_features(n, fi, 400 + li, device=dev)
        W = synth.normal_features(fi, fo, 410 + li, device=dev) / fi ** 0.5
        b = synth.normal_features(1, fo, 420 + li, device=dev).reshape(fo)
        dH = synth.normal_features(n, fo, 430 + li, device=dev)
        H = torch.empty((n, fo), device=dev)
        dX = torch.empty((n, fi), device=dev) if li else None
        dW, db = torch.empty((fi, fo), device=dev), torch.empty(fo, device=dev)
        saved = torch.empty(gnn.gnn_sage_layer_saved_elems(n, fi, fo), device=dev)
        ws_bytes = gnn.gnn_sage_layer_workspace_bytes(n, fi, fo, relu)
        if flags & gnn.GNN_LAYER_NO_GATE_FOLD:  # that route writes the masked gradient first and needs room for it
            ws_bytes += n * fo * 4 + 256
        ws = torch.empty(ws_bytes // 4, device=dev)
        tf = timed(lambda: gnn.gnn_sage_layer_fwd(dg.indptr, dg.indices, X, W, b, saved, H, dg.plan_fwd, relu=relu, flags=flags))
        tb = timed(lambda: gnn.gnn_sage_layer_bwd(dg.indptr_t, dg.indices_t, X, W, saved, H, dH, dX, dW, db, dg.plan_bwd, ws,
                                                  relu=relu, flags=flags))
        rows.append({"layer": f"{fi}->{fo}", "order": "aggregate first" if fi <= fo else "transform first",
                     "gathered_width": min(fi, fo), "fwd_ms": round(tf, 4), "bwd_ms": round(tb, 4),
                     "dense_GFLOP_fwd": round(2.0 * n * fi * fo / 1e9, 2), "input_gradient": li > 0,
                     "bwd_workspace_GB": round(ws_bytes / 1e9, 3)})
        del X, W, H, dH, dX, saved, ws
    return {"workload": workload, "widths": list(dims), "layers": rows, "calls_per_layer_and_direction": reps + 1, "layer_flags": flags,
            "fwd_ms": round(sum(r["fwd_ms"] for r in rows), 4), "bwd_ms": round(sum(r["bwd_ms"] for r in rows), 4),
            "note": "model compute of one full-batch epoch without loss and optimizer; the paper's epochs on one Xeon 8280 "
                    "socket: 0.88 s (232,965-vertex dataset, widths 602-16-41) and 11 s (2,449,029-vertex dataset, "
                    "widths 100-256-256-47), Sections 6.2 and 6.3 -- other hardware and real data, context only"}


def cpu_baseline_sampled(el, f, dtype, dev, n_rows=1_000_000):
    """The oracle on a bounded sample of a workload whose host copy would not fit: `n_rows` uniformly
    sampled destination rows become a compact sub-problem (their edges, the gathered vertices renumbered;
    pure index plumbing on the generator's edge list) on which the oracle runs the forward sum and mean."""
    import oracle
    rng = np.random.default_rng(777)
    rows = np.sort(rng.choice(el.n, size=min(n_rows, el.n), replace=False)).astype(np.int64)
    rows_t = torch.from_numpy(rows).to(dev).to(el.dst.dtype)
    lo = torch.searchsorted(el.dst, rows_t, right=False)
    hi = torch.searchsorted(el.dst, rows_t, right=True)
    cnt = hi - lo
    indptr = torch.zeros(len(rows) + 1, dtype=torch.int64, device=dev)
    indptr[1:] = torch.cumsum(cnt, 0)
    total = int(indptr[-1])
    owner = torch.repeat_interleave(torch.arange(len(rows), device=dev), cnt)
    pos = lo[owner] + (torch.arange(total, device=dev) - indptr[owner])
    used, inv = torch.unique(el.src[pos].long(), return_inverse=True)
    del owner, pos
    X = synth.normal_features(el.n, f, 100, device=dev, dtype=dtype)[used].float().cpu().numpy()
    ip, ix = indptr.cpu().numpy(), inv.to(torch.int32).cpu().numpy()
    threads = oracle.max_threads()
    secs = 0.0
    for op in (oracle.OP_SUM, oracle.OP_MEAN):
        t0 = time.perf_counter()
        oracle.aggregate_fwd(ip, ix, X, op=op, nthreads=threads)
        secs += time.perf_counter() - t0
    return {"value": round(2 * total * f / secs / 1e9, 4), "unit": "GEF/s", "cores": threads, "kind": "oracle",
            "sample": f"SAMPLED: forward sum and forward mean at F={f} on {len(rows)} uniformly sampled rows ({total} edges, "
                      f"{int(used.numel())} gathered vertices) of the same graph, {secs:.1f} s of CPU time, fp64 scalar loops, "
                      f"OpenMP dynamic over rows"}


BRIEF_KEYS = ("value", "unit", "ms_per_step", "steps", "dtype", "config", "roofline", "calls", "setup_ms", "graph_replay", "static_input_packed")


def brief(res):
    return {k: res[k] for k in BRIEF_KEYS if k in res}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="rmat_sparse_stack", choices=list(synth.WORKLOADS))
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the graph (debugging only; invalid as a result)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-calibration", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the brief runs of the other four workloads reported under 'workloads'")
    ap.add_argument("--no-general-primitive", action="store_true",
                    help="skip the operator-table calls (gnn_ap_*) reported under 'general_primitive'")
    ap.add_argument("--no-layers", action="store_true",
                    help="skip the GraphSAGE layer calls (gnn_sage_layer_*) reported under 'layers'")
    ap.add_argument("--layers-only", action="store_true",
                    help="run nothing but the layer calls of --workload (for profiling them); prints their section alone")
    ap.add_argument("--layer-flags", type=int, default=0, help="GNN_LAYER_* bits for the layer calls (A/B measurements)")
    ap.add_argument("--flush-cache", action="store_true",
                    help="overwrite a 1 GiB buffer before every call (for workloads that fit the caches); "
                         "value is then the sum of the calls' event times")
    ap.add_argument("--relabel", default=None, choices=["degree", "rmat_prefix", "random"],
                    help="rename the vertices of the workload's graph first (descending degree, the order of the R-MAT "
                         "recursion, or a random order): the vertex-reordering axis of the reuse study")
    ap.add_argument("--dump-graph", default=None, metavar="DIR",
                    help="write the CSR and transposed CSR as raw arrays for the stand-alone profiling driver, then exit")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1")
    if not torch.cuda.is_available():
        sys.exit("bench.py: needs a GPU")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    gnn.load_library()

    if args.layers_only:
        print(json.dumps({"layers": [measure_layers(args.workload, dev, flags=args.layer_flags)]}))
        return
    result, ctx = measure(args.workload, args.steps, args.warmup, args.scale, dev, args.dump_graph, args.flush_cache,
                          relabel=args.relabel, packed_input=args.scale == 1.0 and args.workload != "rmat_capacity")
    if result is None:
        return
    el, widths, op_names = ctx
    e = el.e
    full = args.scale == 1.0
    if not args.no_cpu_baseline and e <= 500_000_000:
        host_el = synth.EdgeList(el.n, el.src.cpu(), el.dst.cpu(), el.meta)
    del el, ctx
    torch.cuda.empty_cache()
    if not args.no_general_primitive and full and e <= 500_000_000:
        result["general_primitive"] = measure_general_primitive(args.workload, dev)
        torch.cuda.empty_cache()
    if not args.no_layers and full:
        result["layers"] = [measure_layers(wl, dev, flags=args.layer_flags) for wl in (args.workload, "rmat_dense_wide") if wl in MODELS]
        torch.cuda.empty_cache()
    if not args.no_calibration:
        result["ceilings"] = calibrate(dev)
        # the on-chip ceiling next to the roofline: every gathered byte crosses from an L2 to a compute unit at
        # least once; at the rate this kernel reaches on an L2-resident table that alone takes this share of a call
        l2 = result["ceilings"]["gather_L2_resident_GBs"] * 1e9
        rf = result["roofline"]
        rf["on_chip_ceiling_frac"] = round(rf["gathered_bytes_per_call"] / l2 / (rf["avg_launch_ms"] * 1e-3), 4)
        # the same against the bare probe: every gather is at least one request for a 128-byte line (a dense tail of
        # 16 bytes costs one too), and the probe shows how many of those the chip serves per second from its L2s
        probe = result["ceilings"]["line_gather_probe_L2_resident_GBs"] * 1e9 / 128
        rf["line_request_ceiling_frac"] = round(rf["line_requests_per_call"] / probe / (rf["avg_launch_ms"] * 1e-3), 4)
        torch.cuda.empty_cache()
    if not args.no_other_workloads and full:
        # the other four workloads, briefly, so that every configuration has a figure from this very run
        others = {}
        few = max(3, args.steps // 4)
        for name in synth.WORKLOADS:
            if name == args.workload:
                continue
            torch.cuda.empty_cache()
            if name == "er_tiny":
                res, _ = measure(name, 200, 20, 1.0, dev, capture=True)
                others[name] = brief(res)
                res, _ = measure(name, 20, 2, 1.0, dev, flush=True)  # its matrices fit an L2: every call from a cold cache
                others[name + " (caches flushed before every call)"] = brief(res)
            elif name == "rmat_weighted_narrow":
                res, _ = measure(name, few, 1, 1.0, dev)
                others[name] = brief(res)
                res, _ = measure(name, few, 1, 1.0, dev, flush=True)
                others[name + " (caches flushed before every call)"] = brief(res)
            elif name == "rmat_capacity":
                res, ctx2 = measure(name, 2, 1, 1.0, dev)
                others[name] = brief(res)
                if not args.no_cpu_baseline:
                    torch.cuda.empty_cache()
                    w5 = synth.WORKLOADS[name]
                    others[name]["cpu_baseline"] = cpu_baseline_sampled(ctx2[0], w5["widths"][0], torch.bfloat16, dev)
                del ctx2
            else:
                res, _ = measure(name, few, 1, 1.0, dev, packed_input=True)
                others[name] = brief(res)
            del res
        result["workloads"] = others
        torch.cuda.empty_cache()
    if not args.no_cpu_baseline and e > 500_000_000:
        result["cpu_baseline"] = None  # see 'workloads' for the sampled figure of such a workload when it is not the main one
    elif not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(host_el, widths, op_names[0])
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result))


if __name__ == "__main__":
    main()
