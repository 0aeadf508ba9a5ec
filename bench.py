#!/usr/bin/env python3
"""Throughput of the segmented reduce / scan hot path on one MI355X.

One *step* is one pass of the whole hot path over one synthetic batch: the segment-length
sweep at n = 2^28 binary16 elements (uniform[0,1), seed 4) -- a segmented reduction and a
segmented inclusive scan for each seg_len in 2^4, 2^6, ..., 2^16, 2^20 (16 library calls).
That sweep crosses every stage: in-tile products, wavefront and workgroup combines, the
multi-workgroup carry, the partials pass of the long reductions, and the dispatch.

Printed: ONE JSON line.  `value` is input bytes consumed per second over the whole step
(16 x 512 MiB per step), inputs resident in HBM before the timed region starts.
`roofline` describes the kernel that takes the most time in the step; its duration is
measured with HIP events around each call on the launch stream in a second pass of the same
steps.  `cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload.
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
SWEEP = (4, 6, 8, 10, 12, 14, 16, 20)
LOG2N = 28


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--log2n", type=int, default=LOG2N, help="elements = 2^log2n (default: the headline size)")
    ap.add_argument("--formulation", default="mfma", choices=["mfma", "dpp"])
    ap.add_argument("--scan-carry", default="lookback", choices=["lookback", "reduce_then_scan", "scan_then_propagate"])
    ap.add_argument("--tile-load", default="direct", choices=["direct", "lds", "lds_dma"],
                    help="how tiles reach the matrix-core operands for seg_len 16..512 (measured alternatives to the default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tuning", default="", help="launch-shape choices to import first (tcr_tuning_import text)")
    ap.add_argument("--autotune", action="store_true",
                    help="let tcr_autotune re-pick the launch shape of every timed call first (default: shipped shapes)")
    ap.add_argument("--no-small-configs", action="store_true",
                    help="skip the context rows of configurations 1 and 2 (n = 2^20, 2^24), whose launches would mix with "
                         "those of the sweep in per-kernel profile statistics")
    ap.add_argument("--context-filter", default="", help="run only the context rows whose label contains this text")
    ap.add_argument("--no-context", action="store_true", help="skip the context rows (variants, library calls, full operations)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (read 1 GiB, write 1 GiB) three times before the timed "
                         "region, as the known-size reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--sustain", type=float, default=0.0,
                    help="instead of the benchmark, repeat ONE call (see --only) for this many seconds, for power "
                         "sampling with an external tool; prints calls per second")
    ap.add_argument("--only", default="segmented_scan:12", help="op:log2(seg_len) for --sustain")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (segmented reduce/scan needs no second one); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_1811_09736_amd import binding as tcr
    from paper_1811_09736_amd import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path", file=sys.stderr)
        return 3
    tcr.set_variant("reset")
    tcr.set_variant("formulation", args.formulation)
    tcr.set_variant("scan_carry", args.scan_carry)
    tcr.set_variant("tile_load", args.tile_load)

    n = 1 << args.log2n
    sweep = [e for e in SWEEP if e <= args.log2n]
    x_host = workloads.make_input(n, "uniform_01", 4)
    x = torch.from_numpy(x_host).cuda()
    out_scan = torch.empty(n, dtype=torch.float32, device="cuda")
    out_red = {e: torch.empty(n >> e, dtype=torch.float32, device="cuda") for e in sweep}
    calls = [("segmented_reduce", e) for e in sweep] + [("segmented_scan", e) for e in sweep]

    def run(op, e):
        if op == "segmented_reduce":
            tcr.segmented_reduce(x, 1 << e, out=out_red[e])
        else:
            tcr.segmented_scan(x, 1 << e, out=out_scan)

    def step():
        for op, e in calls:
            run(op, e)

    if args.sustain > 0:
        op, e = args.only.split(":")
        e = int(e)
        if op == "segmented_reduce" and e not in out_red:
            out_red[e] = torch.empty(n >> e, dtype=torch.float32, device="cuda")
        run(op, e)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        count = 0
        while time.perf_counter() - t0 < args.sustain:
            for _ in range(200):
                run(op, e)
            torch.cuda.synchronize()
            count += 200
        dt = time.perf_counter() - t0
        print(json.dumps({"sustain": args.only, "formulation": args.formulation, "calls": count, "seconds": round(dt, 3),
                          "us_per_call": round(dt / count * 1e6, 2)}))
        return 0
    if args.calibration_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.tuning:
        tcr.tuning_import(args.tuning)
    if args.autotune:
        ids = {"segmented_reduce": tcr.OP_SEGMENTED_REDUCE, "segmented_scan": tcr.OP_SEGMENTED_SCAN}
        for op, e in calls:
            tcr.autotune(ids[op], x, out_scan, 1 << e)
        tcr.autotune(tcr.OP_REDUCE, x, out_scan, 0)
        tcr.autotune(tcr.OP_SCAN, x, out_scan, 0)
        for seg in (12, 100, 196, 3000, 3001, 3584, 3 << 20):          # the lengths of the context rows without a tuned path
            m = (n // seg) * seg
            if m:
                tcr.autotune(tcr.OP_SEGMENTED_SCAN, x[:m], out_scan, seg)
                tcr.autotune(tcr.OP_SEGMENTED_REDUCE, x[:m], out_scan, seg)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    in_bytes_per_step = 2 * n * len(calls)
    value = in_bytes_per_step / (elapsed / args.steps) * 1e-9

    # second pass: HIP events around every call (same stream the kernels are launched on)
    stream = torch.cuda.current_stream()
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in calls]
          for _ in range(args.steps)]
    for s in range(args.steps):
        for c, (op, e) in enumerate(calls):
            ev[s][c][0].record(stream)
            run(op, e)
            ev[s][c][1].record(stream)
    torch.cuda.synchronize()
    tcr.check_device_flags()
    rows = []
    per_kernel = {}
    op_id = {"segmented_reduce": tcr.OP_SEGMENTED_REDUCE, "segmented_scan": tcr.OP_SEGMENTED_SCAN}
    for c, (op, e) in enumerate(calls):
        ms = [ev[s][c][0].elapsed_time(ev[s][c][1]) for s in range(args.steps)]
        avg = sum(ms) / len(ms)
        rd, wr = workloads.algorithmic_bytes(op, n, 1 << e)
        kname = tcr.kernel_name(op_id[op], n, 1 << e)
        rows.append({"op": op, "seg_len_log2": e, "kernel": kname, "avg_us": round(avg * 1e3, 2),
                     "median_us": round(sorted(ms)[len(ms) // 2] * 1e3, 2),
                     "min_us": round(min(ms) * 1e3, 2), "elem_per_s": n / (avg * 1e-3),
                     "input_GBps": round(2 * n / (avg * 1e-3) * 1e-9, 1),
                     "total_GBps": round((rd + wr) / (avg * 1e-3) * 1e-9, 1),
                     "pct_of_hbm_peak": round((rd + wr) / (avg * 1e-3) * 1e-9 / HBM_PEAK_GBS * 100, 1)})
        k = per_kernel.setdefault(kname, {"ms": 0.0, "bytes": 0, "launches": 0})
        k["ms"] += sum(ms)
        k["bytes"] += (rd + wr) * len(ms)
        k["launches"] += len(ms)
    dom_name, dom = max(per_kernel.items(), key=lambda kv: kv[1]["ms"])
    achieved = dom["bytes"] / (dom["ms"] * 1e-3) * 1e-9
    # HBM bytes per launch from the committed rocprofv3 counter runs -- null unless they were taken on exactly
    # these sources (a hash of csrc/) at the headline size and cover the dominant kernel
    from paper_1811_09736_amd import profiling
    traffic, traffic_note = (profiling.traffic_for(dom_name) if args.log2n == LOG2N
                             else (None, "the counter runs are for n = 2^%d" % LOG2N))
    roofline = {"bound": "hbm", "kernel": dom_name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_note": traffic_note,
                "avg_launch_us": round(dom["ms"] / dom["launches"] * 1e3, 2),
                "algorithmic_bytes_per_launch": dom["bytes"] // dom["launches"]}

    # context rows outside the step: the full (unsegmented) operations on the same input, and one segment
    # length without a tuned path
    extra = []
    out_one = torch.empty(1, dtype=torch.float32, device="cuda")
    big = 3 << 20
    nb = (n // big) * big
    n3 = (n // 3000) * 3000
    n35 = (n // 3584) * 3584
    n1, n100 = (n // 3001) * 3001, (n // 100) * 100
    n12 = (n // 12) * 12
    out_h12 = torch.empty(n12 // 12, dtype=torch.float32, device="cuda")
    out_g = torch.empty(n3 // 3000, dtype=torch.float32, device="cuda")
    out_h100 = torch.empty(n100 // 100, dtype=torch.float32, device="cuda")
    out_h = torch.empty(n, dtype=torch.float16, device="cuda")
    variant_rows = []
    for e in (8, 12, 16, 20):
        if e <= args.log2n and args.formulation == "mfma" and args.scan_carry != "scan_then_propagate":
            variant_rows.append((f"segmented_scan_ex seg_len=2^{e} binary16 output (the paper's precision, 4 B/elem)",
                                 (lambda e=e: tcr.segmented_scan_ex(x, 1 << e, tcr.OUT_F16, out=out_h)), n, (2 * n, 2 * n)))
    if args.formulation == "mfma":
        for e in (12, 20):
            if e <= args.log2n:
                variant_rows.append((f"segmented_scan_ex seg_len=2^{e} binary16 accumulator and output (the paper's half-precision "
                                     "mode, 4 B/elem; cross-lane binary16 adds, no matrix cores)",
                                     (lambda e=e: tcr.segmented_scan_ex(x, 1 << e, tcr.OUT_F16 | tcr.ACC_F16, out=out_h)), n,
                                     (2 * n, 2 * n)))
    variant_rows.append(("segmented_moments seg_len=2^12 (sum and sum of squares, X.X^T diagonal on the matrix cores)",
                         lambda: tcr.segmented_moments(x, 1 << 12), n, (2 * n, 8 * (n >> 12))))
    n196 = (n // 196) * 196
    variant_rows.append(("segmented_moments seg_len=196 (14x14 feature maps: masked row products, sums and sums of squares)",
                         lambda: tcr.segmented_moments(x[:n196], 196), n196, (2 * n196, 8 * (n196 // 196))))
    n24 = (n // 24) * 24
    variant_rows.append(("segmented_moments seg_len=24 (6x4 windows: rows of one segment each, masked constant matrix)",
                         lambda: tcr.segmented_moments(x[:n24], 24), n24, (2 * n24, 8 * (n24 // 24))))
    if args.formulation == "mfma":
        variant_rows.append(("segmented_scan_ex seg_len=2^12 exclusive",
                             lambda: tcr.segmented_scan_ex(x, 1 << 12, tcr.SCAN_EXCLUSIVE, out=out_scan), n, (2 * n, 4 * n)))
    out_r4 = torch.empty(n // 16, dtype=torch.float32, device="cuda")
    variant_rows.append(("segmented_reduce seg_len=2^4 called back to back", lambda: tcr.segmented_reduce(x, 16, out=out_r4), n,
                         (2 * n, n // 4)))
    variant_rows.append(("segmented_scan seg_len=2^4 called back to back (in the step it follows the reductions, whose "
                         "streaming loads leave the last scan's 256 MiB of dirty cache lines for it to write back)",
                         lambda: tcr.segmented_scan(x, 16, out=out_scan), n, (2 * n, 4 * n)))
    # library context (neither oracle nor target): the device copy this machine sustains -- the paper quotes its
    # results against the measured copy rate -- and torch's own sum / cumsum (rocPRIM) on the same input
    copy_src = out_scan
    copy_dst = torch.empty_like(out_scan)
    library_rows = [("context: device copy of 2^%d binary32 values (torch copy_)" % args.log2n,
                     lambda: copy_dst.copy_(copy_src), n, (4 * n, 4 * n)),
                    ("context: torch.sum(x, dtype=float32) (library full reduce)",
                     lambda: torch.sum(x, dtype=torch.float32), n, (2 * n, 4)),
                    ("context: torch.cumsum(x, 0, dtype=float32) (library full scan)",
                     lambda: torch.cumsum(x, 0, dtype=torch.float32, out=copy_dst), n, (2 * n, 4 * n))]
    # irregular segments (offsets array): three length mixes over the same input; the offsets are part of the
    # bytes the call must read
    irregular_rows = []
    if not args.no_context:
        import numpy as np
        for recipe, what in (("uniform16", "lengths uniform on 0..32"), ("lognormal256", "log-normal lengths, median 256, sigma 2"),
                             ("few7", "7 segments cut at random")):
            off = torch.from_numpy(workloads.make_offsets(n, recipe, 5).view(np.int64)).cuda()
            nseg = off.numel() - 1
            out_i = torch.empty(nseg, dtype=torch.float32, device="cuda")
            irregular_rows.append((f"irregular_reduce, {nseg} segments ({what})",
                                   (lambda off=off, out_i=out_i: tcr.irregular_reduce(x, off, out=out_i)), n,
                                   (2 * n + 8 * (nseg + 1), 4 * nseg)))
            irregular_rows.append((f"irregular_scan, {nseg} segments ({what})",
                                   (lambda off=off: tcr.irregular_scan(x, off, out=out_scan)), n, (2 * n + 8 * (nseg + 1), 4 * n)))
    # configurations 1 and 2 (n = 2^20 and 2^24): small enough to sit in the 256 MiB memory-side cache, so every call
    # takes the next slice of the 512 MiB input (256 resp. 16 distinct buffers); the figures are per call
    small_rows = []
    if args.log2n >= 25 and not args.no_context and not args.no_small_configs:
        k1 = n >> 20
        out1 = torch.empty((1 << 20) // 256, dtype=torch.float32, device="cuda")

        def cfg1():
            for i in range(k1):
                tcr.segmented_reduce(x[i << 20:(i + 1) << 20], 256, out=out1)
        small_rows.append((f"configuration 1: segmented_reduce n=2^20 seg_len=256, per call over {k1} rotating slices "
                           "(latency/cache-bound, not a roofline row)", cfg1, 1 << 20, (2 << 20, 4 * ((1 << 20) // 256)), k1))
        k2 = n >> 24
        for L in (16, 64, 256, 1024, 4096):
            def cfg2(L=L):
                for i in range(k2):
                    tcr.segmented_scan(x[i << 24:(i + 1) << 24], L, out=out_scan[i << 24:(i + 1) << 24])
            small_rows.append((f"configuration 2: segmented_scan n=2^24 seg_len={L}, per call over {k2} rotating slices "
                               "(latency/cache-bound, not a roofline row)", cfg2, 1 << 24, (2 << 24, 4 << 24), k2))
    for label, fn, nn, rd_wr, *per in [] if args.no_context else [row for row in small_rows + variant_rows + library_rows + irregular_rows + [
            ("reduce (full)", lambda: tcr.reduce(x, out=out_one), n, (2 * n, 4)),
            ("scan (full)", lambda: tcr.scan(x, out=out_scan), n, (2 * n, 4 * n)),
            ("segmented_reduce seg_len=3*2^20 (no power of two: masked pieces + second kernel)",
             lambda: tcr.segmented_reduce(x[:nb], big, out=out_g[: nb // big]), nb, (2 * nb, 4 * (nb // big))),
            ("segmented_scan seg_len=3*2^20 (no power of two: chain on a per-segment tile grid)",
             lambda: tcr.segmented_scan(x[:nb], big, out=out_scan[:nb]), nb, (2 * nb, 4 * nb)),
            ("segmented_reduce seg_len=3000 (no power of two: masked row products)", lambda: tcr.segmented_reduce(x[:n3], 3000, out=out_g), n3,
             (2 * n3, 4 * (n3 // 3000))),
            ("segmented_scan seg_len=3000 (no power of two: fixed tiles, segment starts marked)", lambda: tcr.segmented_scan(x[:n3], 3000, out=out_scan[:n3]), n3,
             (2 * n3, 4 * n3)),
            ("segmented_scan seg_len=3584 (aligned, seven eighths of 8 tiles: one workgroup per segment)",
             lambda: tcr.segmented_scan(x[:n35], 3584, out=out_scan[:n35]), n35, (2 * n35, 4 * n35)),
            ("segmented_scan seg_len=3001 (odd: fixed tiles, segment starts marked)", lambda: tcr.segmented_scan(x[:n1], 3001, out=out_scan[:n1]), n1,
             (2 * n1, 4 * n1)),
            ("segmented_scan seg_len=100 (fixed tiles, segment starts marked)", lambda: tcr.segmented_scan(x[:n100], 100, out=out_scan[:n100]), n100,
             (2 * n100, 4 * n100)),
            ("segmented_reduce seg_len=100 (no power of two: masked row products)", lambda: tcr.segmented_reduce(x[:n100], 100, out=out_h100), n100,
             (2 * n100, 4 * (n100 // 100))),
            ("segmented_reduce seg_len=12 (rows of two whole segments: one product with a masked constant matrix)",
             lambda: tcr.segmented_reduce(x[:n12], 12, out=out_h12), n12, (2 * n12, 4 * (n12 // 12)))] if args.context_filter in row[0]]:
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3 / (per[0] if per else 1)
        extra.append({"call": label, "avg_us": round(us, 2), "total_GBps": round(sum(rd_wr) / us * 1e-3, 1),
                      "pct_of_hbm_peak": round(sum(rd_wr) / us * 1e-3 / HBM_PEAK_GBS * 100, 1)})
    tcr.check_device_flags()
    del copy_dst
    copy_gbps = next((r["total_GBps"] for r in extra if r["call"].startswith("context: device copy")), None)
    for r in rows:
        if copy_gbps:
            r["pct_of_measured_copy"] = round(r["total_GBps"] / copy_gbps * 100, 1)

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        sample_log2 = min(args.log2n, 27)
        xs = np.ascontiguousarray(x_host[: 1 << sample_log2])
        t0 = time.perf_counter()
        for op, e in calls:
            if e > sample_log2:
                e = sample_log2
            if op == "segmented_reduce":
                oracle.segmented_reduce(xs, 1 << e)
            else:
                oracle.segmented_scan(xs, 1 << e)
        dt = time.perf_counter() - t0
        cpu = {"value": round(2 * (1 << sample_log2) * len(calls) / dt * 1e-9, 4), "unit": "GB/s", "cores": 1,
               "kind": "oracle",
               "sample": f"the same 16 calls on the first 2^{sample_log2} elements of the input (seg_len capped at the sample), "
                         f"sequential binary64 C loops, {dt:.1f} s"}

    cpu_openmp = None
    if not args.no_cpu_baseline:
        # the same loops with the segments shared among the host's cores (bit-identical results); context
        omp = oracle.openmp()
        threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or len(os.sched_getaffinity(0))
        t0 = time.perf_counter()
        for op, e in calls:
            e = min(e, sample_log2)
            (omp.segmented_reduce if op == "segmented_reduce" else omp.segmented_scan)(xs, 1 << e)
        dt = time.perf_counter() - t0
        cpu_openmp = {"value": round(2 * (1 << sample_log2) * len(calls) / dt * 1e-9, 4), "unit": "GB/s", "cores": threads,
                      "kind": "oracle, OpenMP over segments", "sample": f"as cpu_baseline, {dt:.1f} s"}

    props = torch.cuda.get_device_properties(0)
    device = {"name": props.name, "compute_units": props.multi_processor_count,
              "memory_GiB": round(props.total_memory / 2 ** 30, 1)}
    line = {
        "metric": "effective input GB/s (% of HBM peak) for seg-reduce/scan at N=2^" + str(args.log2n),
        "pct_of_hbm_peak": round(sum(sum(workloads.algorithmic_bytes(op, n, 1 << e)) for op, e in calls)
                                 / (elapsed / args.steps) * 1e-9 / HBM_PEAK_GBS * 100, 1),
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "cfg5 sweep: n=2^%d fp16 uniform[0,1) seed 4; segmented_reduce and segmented_scan at "
                               "seg_len=2^{%s}; fp32 accumulate and output" % (args.log2n, ",".join(map(str, sweep))),
                   "formulation": args.formulation, "scan_carry": args.scan_carry, "tile_load": args.tile_load,
                   "input_sha256": workloads.sha256(x_host)[:16]},
        "roofline": roofline, "cpu_baseline": cpu, "cpu_baseline_openmp": cpu_openmp, "measured_copy_GBps": copy_gbps, "device": device, "tuning": tcr.tuning_export(), "rows": rows, "context_rows": extra,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
