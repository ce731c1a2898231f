#!/usr/bin/env python3
"""Benchmark of the bulk minibatch sampler on one MI355X.

A step is one bulk sampling call over one batch of synthetic input: all hops of the
hot path (P = Q A, SAMPLE, EXTRACT) for k minibatches, with the CSR adjacency and the
seed batches already resident in HBM.  Prints ONE JSON line:
  value      sampled edges per second (sum of nnz over the hops / time per call)
  roofline   the dominant kernel's algorithmic bytes / its measured duration vs 8 TB/s
  cpu_baseline  the CPU oracle timed on this machine's host cores on the same workload
The dominant kernel's durations come from HIP events that the library records on the call's
own stream around its launches during the timed steps (BMS_PROFILE_MAIN); the other stages are
timed the same way in a few extra steps (BMS_PROFILE), because bracketing every stage costs
about 0.2 ms per call.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# Bytes that crossed from the L2 caches to the memory fabric (reads + writes), from rocprofv3 request counters:
# read requests by size (TCC_EA0_RDREQ_32B / _64B / _128B x 32 / 64 / 128 bytes) and write requests
# (TCC_EA0_WRREQ_64B x 64, the others x 32).  The counters sit between L2 and the fabric: a request that the
# 256 MB memory-side cache answers is counted like one that reaches HBM ("fabric traffic", an upper bound of the
# HBM traffic).  Keyed by (workload, kernel stage): bytes per step summed over the stage's launches.  Each value is
# the line "bench constant ..." of profiles/<workload>_hbm_traffic.txt (tests/test_bench_constants.py compares
# them); a kernel that has changed since its profile was taken has no entry (None in the output).
MEASURED_TRAFFIC = {
    ("dense_ladies", "ldw_accumulate"): 3_308_734_816,
    ("dense_ladies", "ldw_extract"): 2_026_395_190,
    ("dense_sage", "nw_sample"): 10_619_753_760,
    ("dense_sage", "nw_rows"): 1_379_272_096,
    ("dense_sage", "dd_split"): 1_138_991_268,
    ("dense_sage", "dd_unsplit"): 1_001_343_017,
    ("dense_sage", "dd_rank"): 875_271_634,
    ("dense_sage", "dd_front"): 616_770_066,
    ("large_sage", "nw_sample"): 5_716_071_922,
    ("large_sage", "nw_rows"): 1_649_649_339,
    ("large_sage", "dd_split"): 753_356_804,
    ("large_sage", "dd_unsplit"): 682_846_788,
    ("large_sage", "dd_rank"): 599_108_329,
    ("large_sage", "dd_front"): 473_554_418,
    ("mid_ladies", "ldw_accumulate"): 148_771_117,
    ("mid_ladies", "ldw_extract"): 85_080_091,
    ("mid_sage", "nw_sample"): 3_060_700_205,
    ("mid_sage", "dd_split"): 426_376_214,
    ("mid_sage", "dd_unsplit"): 366_985_101,
    ("mid_sage", "nw_rows"): 351_932_041,
    ("mid_sage", "dd_rank"): 314_712_068,
    ("mid_sage", "dd_front"): 204_159_766,
}
# the same summed over every kernel of one bulk call (bytes per step)
MEASURED_CALL_TRAFFIC = {
    "dense_ladies": 9_685_282_825,
    "dense_sage": 15_634_668_434,
    "large_sage": 9_878_498_779,
    "mid_ladies": 486_247_881,
    "mid_sage": 4_725_634_948,
}
OTHER_WORKLOADS = ("mid_sage", "dense_sage", "mid_ladies", "dense_ladies", "tiny_sage")


def algorithmic_bytes(stage: str, rows: int, nnz: int, ncols: int, pnnz: int = 0, gathered: int = 0) -> float:
    """Bytes the method itself must move in one launch of `stage` for a hop of the given sizes.

    Node-wise hop: 28 R + 16 E + 4 U in total (R stacked rows, E sampled edges, U distinct sampled
    vertices): frontier id 4 R + two adjacent rowptr entries 16 R (nw_rows); output rowptr 8 R,
    chosen neighbours read 4 E and staged 4 E (nw_sample); staged ids read 4 E, local columns
    written 4 E (nw_relabel); next frontier written 4 U (vset_rank).
    Layer-wise hop: 8 D + 8 C + 28 F + 4 nnz(A_S) + 4 S: frontier 4 F + rowptr 16 F (ld_rows); gathered
    neighbours 4 D (ldw_accumulate); P written 8 C (ldw_p_copy); sampled set 4 S (ldw_draw); second pass
    over the rows 4 D (ldw_extract); output 8 F + 4 nnz (ldw_extract_copy).
    Scratch traffic (degrees, vertex-set bitmaps, dense counters, tile sums) is not counted.
    """
    R, E, U = float(rows), float(nnz), float(ncols)
    table = {
        "nw_rows": 20 * R,
        "nw_sample": 8 * R + 8 * E,
        "nw_relabel": 8 * E,
        "nw_strip_self": 4 * R,   # BMS_UNION_DST: each row's own column; the rest of that pass is scratch
        "vset_rank": 4 * U,
        # EXTRACT by id-range segments: the staged ids are read once (4 E, charged to dd_split), the local
        # columns written once (4 E, dd_unsplit), the next frontier written once (4 U, dd_front); everything else
        # these kernels and dd_plan / dd_rank move is scratch.  dd_bins..dd_place: the per-minibatch kernel path
        "dd_split": 4 * E,
        "dd_unsplit": 4 * E,
        "dd_front": 4 * U,
        "dd_bins": 4 * E,
        "dd_place": 4 * E,
        "ld_rows": 20 * R,
        # LADIES by LDS windows (default): the neighbours are read once to build P (ldw_accumulate) and once
        # to extract (ldw_extract); ldw_bounds (the rows' window boundaries, copied from the per-graph index)
        # moves scratch only
        "ldw_accumulate": 4.0 * gathered,
        "ldw_p_copy": 8.0 * pnnz,
        "ldw_draw": 4 * U,
        "ldw_extract": 4.0 * gathered,
        "ldw_extract_copy": 8 * R + 4 * E,
        # LADIES with dense counters in HBM (BMS_LADIES_DENSE)
        "ld_accumulate": 4.0 * gathered,
        "ld_p_fill": 8.0 * pnnz,
        "ld_extract_count": 4.0 * gathered,
        "ld_extract_fill": 8 * R + 4 * E,
    }
    return table.get(stage, 0.0)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large_sage",
                    help="one of paper_2311_02909_amd.synth.WORKLOADS (default: the 111M-vertex node-wise config)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--no-feature-fetch", action="store_true",
                    help="skip the feature fetch of the last frontier that is timed after the sampling steps")
    ap.add_argument("--variant", default="none", choices=["none", "union_dst", "replace"],
                    help="node-wise variant: union_dst keeps the frontier's own vertices as columns (BMS_UNION_DST), "
                         "replace makes a row's draws independent (BMS_NODEWISE_REPLACE)")
    ap.add_argument("--relabel", default=None, choices=["degree"],
                    help="renumber the graph's vertices by descending degree (hubs first) instead of the recipe's random ids")
    ap.add_argument("--others", default="auto", choices=["auto", "yes", "no"],
                    help="also run the other workloads of the build's configs (fewer steps) and report them under "
                         "other_workloads; auto = only with the default workload")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run a plain device copy of MIB mebibytes 5 times "
                         "(calibrates rocprofv3's FETCH_SIZE / WRITE_SIZE counters against a known size)")
    ap.add_argument("--gather-probe", type=int, default=0, metavar="LOG2",
                    help="instead of the benchmark, time 2^28 random 4-byte reads (torch.index_select) over an int32 "
                         "array of 2^LOG2 elements, 5 launches: the chip's rate for reads that share no memory line")
    ap.add_argument("--line-probe", type=int, default=0, metavar="LOG2",
                    help="instead of the benchmark, time reads of 2^24 short rows (1 and 8 four-byte entries) that start "
                         "at random places of an int32 array of 2^LOG2 elements, one row per lane (libbms_probe.so): "
                         "the chip's rate of 128-byte memory lines for the access pattern of the node-wise kernels")
    ap.add_argument("--lds-probe", action="store_true",
                    help="instead of the benchmark, time LDS adds and stores at random places of 128 KB by 16 waves per "
                         "compute unit (libbms_probe.so): what one LDS instruction of a wave costs its compute unit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2311_02909_amd import bms, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.copy_probe:
        src = torch.arange(args.copy_probe * (1 << 18), dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read_per_launch": src.numel() * 4,
                          "copy_probe_bytes_written_per_launch": src.numel() * 4, "launches": 5}))
        return 0
    if args.line_probe or args.lds_probe:
        import ctypes as C
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2311_02909_amd", "libbms_probe.so")
        if not os.path.exists(path):
            print("bench.py: %s is not built (python paper_2311_02909_amd/build.py)" % path, file=sys.stderr)
            return 2
        P = C.CDLL(path)
        stream = torch.cuda.current_stream().cuda_stream
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        if args.line_probe:
            span, nrows = 1 << args.line_probe, 1 << 24
            array = torch.zeros(span + 64, dtype=torch.int32, device="cuda")
            start = torch.randint(0, span, (nrows,), dtype=torch.int64, device="cuda",
                                  generator=torch.Generator(device="cuda").manual_seed(1))
            sink = torch.zeros(1, dtype=torch.int32, device="cuda")
            P.bms_probe_random_rows.restype = C.c_int
            P.bms_probe_random_rows.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                                                C.c_void_p, C.c_void_p]
            out = {"line_probe_span_bytes": span * 4, "rows_per_launch": nrows, "launches": 6, "workgroups": cus * 8}
            for entries in (1, 8):
                def launch():
                    rc = P.bms_probe_random_rows(array.data_ptr(), span + 64, start.data_ptr(), nrows, entries, cus * 8,
                                                 sink.data_ptr(), stream)
                    assert rc == 0
                launch()
                torch.cuda.synchronize()
                e0.record()
                for _ in range(5):
                    launch()
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / 5
                # a row of 32 bytes at a random 4-byte aligned place lies in one line 100/128 of the time, else in two
                lines = nrows * (1.0 if entries == 1 else 1.0 + 28.0 / 128.0)
                out["rows_of_%d" % entries] = {"ms_per_launch": round(ms, 4), "rows_per_sec": nrows / ms * 1e3,
                                               "lines_per_sec": lines / ms * 1e3,
                                               "tb_per_sec_at_128B_per_line": lines * 128 / ms / 1e9}
            print(json.dumps(out))
            return 0
        P.bms_probe_lds_ops.restype = C.c_int
        P.bms_probe_lds_ops.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        ticks = torch.zeros(cus, dtype=torch.int32, device="cuda")
        iters, out = 200, {"lds_probe_waves_per_cu": 16, "wave_instructions_per_wave": 200 * 16, "lds_bytes": 131072}
        for mode, name in ((0, "add16_random"), (1, "store32_random")):
            for every in (1, 2, 4):
                for _ in range(2):
                    assert P.bms_probe_lds_ops(ticks.data_ptr(), cus, iters, mode, every, stream) == 0
                torch.cuda.synchronize()
                ns = float(ticks.to(torch.float64).mean().item()) * 10.0   # 100 MHz ticks
                out["%s_1_lane_in_%d" % (name, every)] = {"ns_per_wave_instruction_per_cu": round(ns / (16.0 * iters * 16), 3)}
        print(json.dumps(out))
        return 0
    if args.gather_probe:
        span, reads = 1 << args.gather_probe, 1 << 28
        src = torch.zeros(span, dtype=torch.int32, device="cuda")
        idx = torch.randint(0, span, (reads,), dtype=torch.int64, device="cuda",
                            generator=torch.Generator(device="cuda").manual_seed(1))
        out = torch.index_select(src, 0, idx)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            torch.index_select(src, 0, idx, out=out)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        print(json.dumps({"gather_probe_span_bytes": span * 4, "random_reads_per_launch": reads, "launches": 6,
                          "index_bytes_per_launch": reads * 8, "ms_per_launch": round(ms, 4),
                          "reads_per_sec": reads / ms * 1e3, "tb_per_sec_at_128B_per_read": reads * 128 / ms / 1e9}))
        return 0
    out = run_workload(args.workload, args.steps, args.warmup, args.variant, cpu=not args.no_cpu_baseline,
                       fetch=not args.no_feature_fetch, relabel=args.relabel)
    if out is None:
        return 2
    # the other workloads of the build's configs, each with its own dominant kernel, roofline and oracle time
    # (fewer steps; not part of `value`)
    if args.others == "yes" or (args.others == "auto" and args.workload == "large_sage" and args.variant == "none" and not args.relabel):
        others = {}
        for name in OTHER_WORKLOADS:
            if name == args.workload:
                continue
            torch.cuda.empty_cache()
            r = run_workload(name, max(5, args.steps // 2), 2, "none", cpu=not args.no_cpu_baseline, fetch=False)
            others[name] = {key: r[key] for key in ("value", "unit", "ms_per_step", "ms_per_step_min", "minibatches_per_sec",
                                                    "config", "roofline", "cpu_baseline") if key in r}
            if "gathered_neighbours_per_sec" in r:
                others[name]["gathered_neighbours_per_sec"] = r["gathered_neighbours_per_sec"]
        out["other_workloads"] = others
    print(json.dumps(out), flush=True)
    return 0


def run_workload(workload: str, steps: int, warmup: int, variant: str, cpu: bool, fetch: bool, relabel=None):
    """Times `steps` bulk calls of one workload (graph generated here, resident in HBM) and returns the record."""
    import functools

    import torch
    from paper_2311_02909_amd import bms, synth

    class args:  # the names the body below uses
        pass
    args.workload, args.steps, args.warmup, args.variant = workload, steps, warmup, variant
    args.no_cpu_baseline, args.no_feature_fetch = not cpu, not fetch
    t0 = time.time()
    g, batches, w = synth.make_workload(args.workload, device="cuda", relabel=relabel)
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    print("[bench] %s: %s (generated in %.1f s)" % (args.workload, g.describe(), gen_s), file=sys.stderr, flush=True)
    csr = bms.Csr(g.rowptr, g.col)
    nodewise = w["sampler"] == "nodewise"
    fn = bms.sample_nodewise if nodewise else bms.sample_ladies
    if args.variant != "none":
        if not nodewise:
            print("bench.py: --variant applies to node-wise workloads", file=sys.stderr)
            return None
        fn = functools.partial(fn, **{args.variant: True})
    traffic_key = args.workload if args.variant == "none" else args.workload + "+" + args.variant
    if relabel:
        traffic_key += "+" + relabel
    seed = synth.SAMPLING_SEED
    stream = torch.cuda.current_stream()

    res = None
    for _ in range(args.warmup):
        res = fn(csr, batches, w["params"], seed, recycle=res, profile="main")
    torch.cuda.synchronize()
    # timed region: exactly `steps` bulk calls, inputs resident in HBM.  The sampler's main kernel stage
    # (nw_sample / ldw_accumulate) is bracketed by HIP events on the call's stream in every timed step; timing
    # every stage costs ~0.2 ms per call in event records, so the full breakdown is taken in extra steps below.
    main_ms, main_n = {}, {}
    t_start = time.perf_counter()
    step_ms = []   # a call returns after its stream has drained, so the host clock around it times the step
    for _ in range(args.steps):
        t_step = time.perf_counter()
        res = fn(csr, batches, w["params"], seed, recycle=res, profile="main")
        step_ms.append((time.perf_counter() - t_step) * 1e3)
        for name, hop, ms in res.stages():
            main_ms[(name, hop)] = main_ms.get((name, hop), 0.0) + ms
            main_n[(name, hop)] = main_n.get((name, hop), 0) + 1
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed / args.steps * 1e3
    step_ms.sort()
    # per-stage breakdown: a few more steps with every stage timed (not part of `value`)
    stage_ms, stage_n = {}, {}
    for _ in range(max(3, min(args.steps, 10))):
        res = fn(csr, batches, w["params"], seed, recycle=res, profile=True)
        for name, hop, ms in res.stages():
            stage_ms[(name, hop)] = stage_ms.get((name, hop), 0.0) + ms
            stage_n[(name, hop)] = stage_n.get((name, hop), 0) + 1
    torch.cuda.synchronize()
    # the main stage keeps the durations measured inside the timed region
    for key, ms in main_ms.items():
        stage_ms[key] = ms
        stage_n[key] = main_n[key]

    sizes = res.sizes()
    edges = sum(nnz for _, nnz, _ in sizes)
    k = w["k"]
    value = edges / (ms_per_step * 1e-3)

    # per-kernel totals over the hops (each stage is one kernel launch per hop, except the few
    # multi-kernel stages named after their main kernel)
    per_stage = {}
    gathered_of_hop = {}
    if not nodewise:  # D_h = sum of the degrees of hop h's frontier rows (what LADIES has to read)
        deg = (g.rowptr[1:] - g.rowptr[:-1])
        for hop in range(len(sizes)):
            gathered_of_hop[hop] = int(deg[res.hop(hop).row_vertex.long()].sum().item())
    for (name, hop), ms in stage_ms.items():
        d = per_stage.setdefault(name, {"ms": 0.0, "launches": 0, "bytes": 0.0})
        d["ms"] += ms / stage_n[(name, hop)]
        d["launches"] += 1
        hv = res.hop(hop)
        gathered = gathered_of_hop.get(hop, 0)
        d["bytes"] += algorithmic_bytes(name, hv.rows, hv.nnz, hv.ncols, hv.pnnz, gathered)
    dominant = max(per_stage, key=lambda s: per_stage[s]["ms"])
    dom = per_stage[dominant]
    achieved = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9 if dom["ms"] > 0 else 0.0
    roofline = {
        "bound": "hbm", "kernel": dominant, "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 5),
        # measured HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated), average over the launches
        "traffic": (MEASURED_TRAFFIC[(traffic_key, dominant)] // dom["launches"])
        if (traffic_key, dominant) in MEASURED_TRAFFIC else None,
        "algorithmic_bytes_per_launch": int(dom["bytes"] / dom["launches"]),
        "avg_launch_ms": round(dom["ms"] / dom["launches"], 4), "launches_per_step": dom["launches"],
        "algorithmic_bytes_per_step": int(dom["bytes"]),
        "timed_in": "the timed steps" if any(name == dominant for name, _ in main_ms) else "extra steps after the timed ones",
        "timed_with_events": True,   # the timed steps carry the event records of the main stage (the value is conservative)
        "all_kernels_ms_per_step": {s: round(v["ms"], 4) for s, v in sorted(per_stage.items())},
    }
    if dominant == "nw_sample":
        # what bounds this kernel is memory lines per second, not bytes asked for: every sampled neighbour of a long
        # row is a 4-byte read that costs one 128-byte line.  Short rows at random places are read at 4.72e10 lines/s
        # on this chip (bench.py --line-probe 30, profiles/random_line_probe.txt); the kernel's own lines per
        # second follow from its fabric traffic
        lines = MEASURED_TRAFFIC.get((traffic_key, dominant))
        roofline["sampled_reads"] = {
            "per_sec": round(edges / (dom["ms"] * 1e-3), 1),
            "lines_per_sec": round(lines / 128.0 / (dom["ms"] * 1e-3), 1) if lines else None,
            "line_probe_lines_per_sec": 4.72e10,   # reads of short rows that share no line (measured ceiling)
        }
    # whole call: algorithmic bytes of all stages ("effective") and the profiled HBM bytes ("achieved"),
    # both over the sum of the kernel times measured in this run
    kernels_ms = sum(v["ms"] for v in per_stage.values())
    call_alg = sum(v["bytes"] for v in per_stage.values())
    roofline["call"] = {
        "kernels_ms_per_step": round(kernels_ms, 4),
        "effective_GBps": round(call_alg / (kernels_ms * 1e-3) / 1e9, 1),
        "effective_frac": round(call_alg / (kernels_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        # profiled bytes between L2 and the memory fabric (an upper bound of the HBM traffic) over the same time
        "fabric_traffic_bytes": MEASURED_CALL_TRAFFIC.get(traffic_key),
        "fabric_GBps": round(MEASURED_CALL_TRAFFIC[traffic_key] / (kernels_ms * 1e-3) / 1e9, 1)
        if traffic_key in MEASURED_CALL_TRAFFIC else None,
        "fabric_frac": round(MEASURED_CALL_TRAFFIC[traffic_key] / (kernels_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        if traffic_key in MEASURED_CALL_TRAFFIC else None,
    }

    # The step after sampling (not part of `value`): fetch the feature rows of the last frontier of all k
    # minibatches, H n x f fp32 resident in HBM.  Timed with HIP events on the stream the copy runs on.
    fetch = None
    if not args.no_feature_fetch:
        f = w["features"]
        last = res.hop(len(sizes) - 1)
        m = int(last.ncols)
        free_b = torch.cuda.mem_get_info()[0]
        need = (g.n + m) * f * 4
        if need < 0.8 * free_b and m > 0:
            H = torch.empty((g.n, f), dtype=torch.float32, device="cuda")
            H.view(-1)[:] = 1.0  # contents do not matter for a copy; avoid reading never-written pages
            out_rows = torch.empty((m, f), dtype=torch.float32, device="cuda")
            ids = last.col_vertex
            for _ in range(2):
                bms.fetch_features(H, ids, out=out_rows)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 5
            e0.record(stream)
            for _ in range(reps):
                bms.fetch_features(H, ids, out=out_rows)
            e1.record(stream)
            torch.cuda.synchronize()
            fetch_ms = e0.elapsed_time(e1) / reps
            fetch_bytes = m * (4 + 8 * f)  # ids read, rows read, rows written
            fetch = {"rows": m, "f": f, "ms": round(fetch_ms, 4), "bound": "hbm",
                     "achieved": round(fetch_bytes / (fetch_ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(fetch_bytes / (fetch_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "algorithmic_bytes": fetch_bytes}
            # ... and the first propagation step on it: mean aggregation over the last hop's sampled adjacency
            last_h = len(sizes) - 1
            agg_out = torch.empty((int(last.rows), f), dtype=torch.float32, device="cuda")
            for _ in range(2):
                bms.aggregate_hop(res, last_h, out_rows, out=agg_out)
            e0.record(stream)
            for _ in range(reps):
                bms.aggregate_hop(res, last_h, out_rows, out=agg_out)
            e1.record(stream)
            torch.cuda.synchronize()
            agg_ms = e0.elapsed_time(e1) / reps
            # every sampled edge reads one feature row, every row writes one; plus the CSR itself
            agg_bytes = int(last.nnz) * (4 * f + 4) + int(last.rows) * (4 * f + 8)
            fetch["aggregate_last_hop"] = {
                "rows": int(last.rows), "edges": int(last.nnz), "ms": round(agg_ms, 4), "bound": "hbm",
                "achieved": round(agg_bytes / (agg_ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(agg_bytes / (agg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "algorithmic_bytes": agg_bytes}
            del H, out_rows, agg_out
        else:
            fetch = {"skipped": "feature matrix of %d bytes does not fit beside the graph" % need}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import bms_oracle as O
        rp, cl, bt = g.rowptr.cpu().numpy(), g.col.cpu().numpy(), batches.cpu().numpy()
        cores = O.set_threads(0)
        ofn = O.sample_nodewise if nodewise else O.sample_ladies
        if args.variant != "none":
            ofn = functools.partial(ofn, **{args.variant: True})
        t1 = time.perf_counter()
        ofn(rp, cl, bt, w["params"], seed, collect=False)
        cpu_s = time.perf_counter() - t1
        cpu = {"value": round(edges / cpu_s, 1), "unit": "edges/s", "cores": cores, "kind": "oracle",
               "sample": "the same %d minibatches, one oracle call (%.2f s), OpenMP over minibatches" % (k, cpu_s)}
        # one thread, on the first minibatches only (their edges counted from the library's result of the same call)
        k1 = max(1, k // 16)
        edges1 = 0
        for hop in range(len(sizes)):
            hv = res.hop(hop)
            edges1 += int(hv.rowptr[int(hv.mb_rowoff[k1].item())].item())
        O.set_threads(1)
        t1 = time.perf_counter()
        ofn(rp, cl, bt[:k1], w["params"], seed, collect=False)
        cpu1_s = time.perf_counter() - t1
        O.set_threads(cores)
        cpu["single_thread"] = {"value": round(edges1 / cpu1_s, 1), "unit": "edges/s", "cores": 1,
                                "sample": "the first %d minibatches, one oracle call (%.2f s)" % (k1, cpu1_s)}

    out = {
        "metric": "sampled_edges_per_sec", "value": round(value, 1), "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(step_ms[len(step_ms) // 2], 4), "ms_per_step_min": round(step_ms[0], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32", "data": "synthetic",
        "minibatches_per_sec": round(k / (ms_per_step * 1e-3), 1),
        "config": {"workload": args.workload, "sampler": w["sampler"], "params": list(w["params"]),
                   "batch": w["batch"], "k": k, "n": g.n, "nnz": g.nnz, "max_degree": g.max_degree,
                   "variant": args.variant, "relabel": relabel or "random", "rows_nnz_cols_per_hop": [list(s) for s in sizes]},
        "roofline": roofline, "cpu_baseline": cpu, "feature_fetch": fetch,
    }
    if not nodewise:
        out["gathered_neighbours_per_sec"] = round(sum(gathered_of_hop.values()) / (ms_per_step * 1e-3), 1)
        out["config"]["gathered_per_hop"] = [gathered_of_hop[h] for h in sorted(gathered_of_hop)]
    del csr, res, g, batches
    return out


if __name__ == "__main__":
    sys.exit(main())
