"""Turns rocprofv3 CSV output of `bench.py` runs into the short summaries kept under profiles/, and stamps the
traffic figures that `bench.py` quotes with the sources they were measured on.

Nothing here computes anything of the method: it reads profiler CSV files, averages counters per kernel, and
writes text.  Usage (the rocprofv3 commands themselves are quoted in every summary):

    python -m paper_1811_09736_amd.profiling kernel-stats  <dir of --kernel-trace --stats run>
    python -m paper_1811_09736_amd.profiling traffic       <dir of --pmc FETCH_SIZE run> <dir of --pmc WRITE_SIZE run>
    python -m paper_1811_09736_amd.profiling mix           <kernel-stats dir> <dir of SQ counters, mfma> <dir of SQ counters, dpp>
    python -m paper_1811_09736_amd.profiling irregular     <kt dir> <fetch dir> <write dir>  (three times, one per length mix)
    python -m paper_1811_09736_amd.profiling counters      <name> <title> <kernel-stats dir> <pmc dir> [<pmc dir> ...]
    python -m paper_1811_09736_amd.profiling chain-gap     <kernel-stats dir> <SQ counters dir> <TCC counters dir>
    python -m paper_1811_09736_amd.profiling irregular-counters <kernel-stats dir of the mix> <three SQ counter dirs>
    python -m paper_1811_09736_amd.profiling repeatability <bench JSON line file> ...
    python -m paper_1811_09736_amd.profiling tile-load     <five bench JSON line files>
"""
from __future__ import annotations

import collections
import csv
import hashlib
import json
import os
import re
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
PROFILES = os.path.join(ROOT, "profiles")
CSRC = os.path.join(_HERE, "csrc")
TRAFFIC_JSON = os.path.join(PROFILES, "pmc_traffic.json")
COPY_KERNEL = "__amd_rocclr_copyBuffer"


def source_stamp() -> str:
    """SHA-256 over the HIP sources (file names and contents, in name order): what a measurement was taken on."""
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".hpp")):
            h.update(name.encode())
            with open(os.path.join(CSRC, name), "rb") as fh:
                h.update(fh.read())
    return h.hexdigest()[:16]


def _commit() -> str:
    try:
        return subprocess.run(["git", "-C", ROOT, "rev-parse", "--short=12", "HEAD"], stdout=subprocess.PIPE, stderr=subprocess.DEVNULL,
                              text=True).stdout.strip()
    except OSError:
        return ""


def short(name: str) -> str:
    """A readable form of a (mangled) kernel name: tcr::kernel<template arguments>."""
    name = name.strip('"')
    m = re.match(r"_ZN3tcr(\d+)([a-z_0-9]+)I(.*?)EEv", name)
    if m:
        args = ",".join(re.findall(r"L[ib](\d+)E", m.group(3)))
        return f"tcr::{m.group(2)}<{args}>"
    m = re.match(r"_ZN3tcr(\d+)([a-z_0-9]+)E", name)
    if m:
        return f"tcr::{m.group(2)}"
    if name.startswith("tcr::"):
        return name.split("(")[0]
    return name[:70]


def _csv(directory: str, suffix: str):
    for f in sorted(os.listdir(directory)):
        if f.endswith(suffix):
            with open(os.path.join(directory, f)) as fh:
                return list(csv.DictReader(fh))
    raise FileNotFoundError(f"no *{suffix} in {directory}")


def _counters(directory: str):
    """{short kernel name: {counter: [value per dispatch]}} and {short name: set of raw names}."""
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    raw = collections.defaultdict(set)
    for r in _csv(directory, "counter_collection.csv"):
        k = short(r["Kernel_Name"])
        agg[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
        raw[k].add(r["Kernel_Name"].strip('"'))
    return agg, raw


def _write(name: str, lines) -> None:
    os.makedirs(PROFILES, exist_ok=True)
    with open(os.path.join(PROFILES, name), "w") as fh:
        fh.write("\n".join(lines) + "\n")
    print("wrote", os.path.join("profiles", name))


TEMPLATE_NOTE = [
    "Template arguments: reduce_small<FORM,LOG2L,U,W,LOAD>, scan_small<FORM,LOG2L,U,W,MODE,LOAD>, reduce_span<FORM,U,W,COMBINE,FINISH>,",
    "scan_block<FORM,U,W,CARRY,MODE>, scan_chain<FORM,U,W,MODE>, rows_reduce<KIND,U,W>, packed_rows_reduce<KIND,U,W>, scan_half<U,W,CARRY,EXCL>; FORM 0 = MFMA, 1 = DPP;",
    "CARRY 0 = none, 1 = look-back; irregular_scan<U,W,REGULAR,MODE>, irregular_reduce<U,W,REGULAR,KIND> (REGULAR 1: regular segments",
    "of an untuned length; the context rows mix three offset arrays).",
]


def kernel_stats(kt_dir: str) -> None:
    rows = _csv(kt_dir, "kernel_stats.csv")
    out = ["# rocprofv3 kernel statistics: bench.py, cfg5 sweep (n=2^28, seg_len 2^4..2^20) and its context rows", "",
           f"Sources: csrc stamp {source_stamp()}, commit {_commit()}.",
           "Command (run from /tmp with TMPDIR=/tmp on the MI355X box):", "",
           "    rocprofv3 --kernel-trace --stats --output-format csv -d <out> -o bench -- python3 bench.py --no-cpu-baseline --no-small-configs", "",
           *TEMPLATE_NOTE, "",
           "| kernel | calls | avg us | min us | max us | % of GPU time |", "|---|---:|---:|---:|---:|---:|"]
    for r in rows:
        out.append(f"| {short(r['Name'])} | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | {float(r['MinNs']) / 1e3:.1f} | "
                   f"{float(r['MaxNs']) / 1e3:.1f} | {float(r['Percentage']):.2f} |")
    _write("bench_cfg5_sweep_kernel_stats.md", out)


def dispatcher_names(k: str):
    """tcr_kernel_name strings under which a template instance runs in the bench sweep (plain binary32 calls)."""
    m = re.match(r"tcr::([a-z_0-9]+)<([\d,]*)>", k)
    if not m:
        return []
    name, args = m.group(1), [int(a) for a in m.group(2).split(",") if a]
    form = "mfma" if args and args[0] == 0 else "dpp"
    if name == "reduce_small_kernel":
        return [f"reduce_small_kernel<{form}>"]
    if name == "scan_small_kernel":
        return [f"scan_small_kernel<{form}>"] if args[4] == 0 else []
    if name == "scan_chain_kernel":
        return [f"scan_chain_kernel<{form}>"] if args[3] == 0 else []
    if name == "reduce_span_kernel":
        # (COMBINE 0: one result or partial per wavefront; the second kernel, where one runs, moves next to nothing)
        kind = "wave" if args[3] == 0 else "block"
        return [f"reduce_span_kernel<{form},{kind}>", f"reduce_span_kernel<{form},{kind}>+reduce_final_kernel"]
    if name == "scan_block_kernel":
        if args[4] != 0:
            return []
        return ([f"scan_block_kernel<{form},nocarry>"] if args[3] == 0
                else [f"scan_block_kernel<{form},ticket>", f"scan_block_kernel<{form},lookback>"])
    return []


def _copy_scale(agg, counter: str):
    """Scale of a traffic counter from the three 1 GiB device copies of the same run (small housekeeping copies
    share the kernel name and are left out)."""
    big = [v for v in agg[COPY_KERNEL][counter] if v > 100000.0]
    return 3 * 1048576.0 / sum(big), sum(big), len(big)


def traffic(fetch_dir: str, write_dir: str) -> None:
    fetch, raw = _counters(fetch_dir)
    write, _ = _counters(write_dir)
    f_scale, f_total, f_n = _copy_scale(fetch, "FETCH_SIZE")
    w_scale, w_total, _ = _copy_scale(write, "WRITE_SIZE")
    out = ["# HBM traffic per launch from rocprofv3 PMC counters: bench.py, cfg5 sweep (n=2^28)", "",
           f"Sources: csrc stamp {source_stamp()}, commit {_commit()}.",
           "Commands (each its own run, from /tmp with TMPDIR=/tmp):", "",
           "    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out> -o bench -- python3 bench.py --no-cpu-baseline --steps 2 --warmup 1 --no-context --calibration-copy",
           "    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <out> -o bench -- python3 bench.py --no-cpu-baseline --steps 2 --warmup 1 --no-context --calibration-copy", "",
           f"Calibration: three plain device copies of 1 GiB (`{COPY_KERNEL}`, {f_n} dispatches; 3 GiB read and 3 GiB written in all) read",
           f"FETCH_SIZE = {f_total:.0f} KiB and WRITE_SIZE = {w_total:.0f} KiB in total, so the counters are scaled by",
           f"{f_scale:.3f} (fetch) and {w_scale:.3f} (write).", "",
           "| kernel | FETCH_SIZE KiB | WRITE_SIZE KiB | scaled read MiB | scaled written MiB | algorithmic MiB (read + written) |",
           "|---|---:|---:|---:|---:|---|"]
    per_instance = {}
    for k in sorted(fetch):
        if not k.startswith("tcr::"):
            continue
        f = sum(fetch[k]["FETCH_SIZE"]) / len(fetch[k]["FETCH_SIZE"])
        wv = write.get(k, {}).get("WRITE_SIZE", [0.0])
        w = sum(wv) / len(wv)
        rd, wr = f * f_scale / 1024, w * w_scale / 1024
        alg = "512 + 1024" if "scan" in k else "512 + (1024 / seg_len)"
        out.append(f"| {k} | {f:.0f} | {w:.0f} | {rd:.1f} | {wr:.1f} | {alg} |")
        per_instance[k] = {"read_bytes": int(rd * 1048576), "written_bytes": int(wr * 1048576), "mangled": sorted(raw[k])}
    _write("bench_cfg5_sweep_pmc_traffic.md", out)

    groups = collections.defaultdict(list)
    for k, v in per_instance.items():
        for d in dispatcher_names(k):
            groups[d].append(v)
    kernels = {}
    for d, vs in groups.items():
        rd = sum(v["read_bytes"] for v in vs) // len(vs)
        wr = sum(v["written_bytes"] for v in vs) // len(vs)
        kernels[d] = {"read_bytes": rd, "written_bytes": wr, "total_bytes": rd + wr,
                      "mangled": sorted({m for v in vs for m in v["mangled"]})}
    doc = {"stamp": {"csrc_sha256_16": source_stamp(), "commit": _commit(),
                     "source": "profiles/bench_cfg5_sweep_pmc_traffic.md (rocprofv3 FETCH_SIZE and WRITE_SIZE scaled by the copy-kernel "
                               "calibration stated there; average over the launches of the kernel in one bench step)"},
           "kernels": kernels}
    with open(TRAFFIC_JSON, "w") as fh:
        json.dump(doc, fh, indent=1)
    print("wrote profiles/pmc_traffic.json")


def traffic_for(dispatch_name: str):
    """(total HBM bytes per launch or None, note) for bench.py: None with the reason when the committed figures
    were not measured on the sources at hand or do not cover the kernel."""
    if not os.path.exists(TRAFFIC_JSON):
        return None, "profiles/pmc_traffic.json is missing"
    with open(TRAFFIC_JSON) as fh:
        doc = json.load(fh)
    stamp = (doc.get("stamp") or {}).get("csrc_sha256_16")
    now = source_stamp()
    if stamp != now:
        return None, f"profiles/pmc_traffic.json was measured on other sources (stamp {stamp}, these sources {now})"
    entry = (doc.get("kernels") or {}).get(dispatch_name)
    if entry is None:
        return None, f"profiles/pmc_traffic.json has no entry for {dispatch_name}"
    return entry["total_bytes"], f"rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled; kernels {', '.join(entry['mangled'])}"


def _durations(kt_dir: str):
    return {short(r["Name"]): float(r["AverageNs"]) for r in _csv(kt_dir, "kernel_stats.csv")}


def instruction_mix(kt_dir: str, mfma_dir: str, dpp_dir: str) -> None:
    out = ["# Instruction mix per launch: MFMA formulation vs DPP (wavefront-primitive) formulation", "",
           f"Sources: csrc stamp {source_stamp()}, commit {_commit()}.",
           "bench.py, cfg5 sweep (n=2^28) and its context rows.  Commands (from /tmp with TMPDIR=/tmp), one run per formulation:", "",
           "    rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_MFMA SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_INSTS_SALU SQ_INSTS_VMEM_RD SQ_INSTS_VMEM_WR SQ_WAVES --output-format csv -d <out> -o bench -- python3 bench.py --no-cpu-baseline --no-small-configs --steps 2 --warmup 1 [--formulation dpp]", "",
           "Counts are wavefront-level instructions per launch, averaged over launches (millions).  `MFMA busy` is",
           "SQ_VALU_MFMA_BUSY_CYCLES (16 per product) divided by the SIMD-cycles of the launch: average duration from",
           "bench_cfg5_sweep_kernel_stats.md x 2.4 GHz x 1024 SIMDs (256 CUs x 4), i.e. the share of matrix-core time in use.",
           "SQ_INSTS_VALU includes the MFMA instructions.", *TEMPLATE_NOTE, "",
           "| kernel | waves | VALU (M) | of which MFMA (M) | SALU (M) | VMEM rd (M) | VMEM wr (M) | VALU per 512 elements | MFMA busy |",
           "|---|---:|---:|---:|---:|---:|---:|---:|---:|"]
    dur = _durations(kt_dir)
    tiles = (1 << 28) / 512
    seen = set()
    for directory in (mfma_dir, dpp_dir):
        agg, _ = _counters(directory)
        for k in sorted(agg):
            if not k.startswith("tcr::") or "final" in k or k in seen:
                continue                                          # kernels that do not depend on the formulation: listed once
            seen.add(k)
            a = {c: sum(v) / len(v) for c, v in agg[k].items()}
            busy = a.get("SQ_VALU_MFMA_BUSY_CYCLES", 0) / (dur[k] * 2.4 * 1024) if k in dur else 0.0
            out.append(f"| {k} | {a.get('SQ_WAVES', 0):.0f} | {a.get('SQ_INSTS_VALU', 0) / 1e6:.2f} | {a.get('SQ_INSTS_MFMA', 0) / 1e6:.2f} | "
                       f"{a.get('SQ_INSTS_SALU', 0) / 1e6:.2f} | {a.get('SQ_INSTS_VMEM_RD', 0) / 1e6:.2f} | {a.get('SQ_INSTS_VMEM_WR', 0) / 1e6:.2f} | "
                       f"{a.get('SQ_INSTS_VALU', 0) / tiles:.1f} | {100 * busy:.2f} % |")
    _write("bench_cfg5_sweep_instruction_mix.md", out)


IRREGULAR_MIXES = [("lengths uniform on 0..32", "uniform on 0..32", 16778647), ("log-normal lengths, median 256, sigma 2", "log-normal", 141593),
                   ("7 segments cut at random", "7 segments cut", 7)]


def irregular(dirs) -> None:
    out = ["# Irregular segments at n = 2^28: kernel times and HBM traffic per launch, one length mix per run", "",
           f"Sources: csrc stamp {source_stamp()}, commit {_commit()}.",
           "Commands (from /tmp with TMPDIR=/tmp; <mix> is the filter text given per table):", "",
           "    rocprofv3 --kernel-trace --stats --output-format csv -d <out> -o bench -- python3 bench.py --no-cpu-baseline --steps 1 --warmup 0 --context-filter <mix>",
           "    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out> -o bench -- python3 bench.py --no-cpu-baseline --steps 1 --warmup 0 --context-filter <mix> --calibration-copy",
           "    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <out> -o bench -- python3 bench.py --no-cpu-baseline --steps 1 --warmup 0 --context-filter <mix> --calibration-copy", "",
           "Counters scaled by the three 1 GiB device copies of the same run, as in bench_cfg5_sweep_pmc_traffic.md.",
           "Algorithmic bytes: input 512 MiB, offsets 8 B per entry, results 4 B per segment (reduce) or 1024 MiB (scan).",
           "irregular_scan_kernel<U,W,REGULAR,MODE>, irregular_reduce_kernel<U,W,REGULAR,KIND>: REGULAR 0 = offsets array.", ""]
    for i, (label, filt, nseg) in enumerate(IRREGULAR_MIXES):
        kt_dir, fetch_dir, write_dir = dirs[3 * i: 3 * i + 3]
        stats = {short(r["Name"]): r for r in _csv(kt_dir, "kernel_stats.csv")}
        fetch, _ = _counters(fetch_dir)
        write, _ = _counters(write_dir)
        f_scale = _copy_scale(fetch, "FETCH_SIZE")[0]
        w_scale = _copy_scale(write, "WRITE_SIZE")[0]
        off_mib = 8 * (nseg + 1) / 1048576
        out += [f"## {label}: {nseg} segments (`--context-filter \"{filt}\"`)", "",
                f"Algorithmic MiB: reduce {512 + off_mib + 4 * nseg / 1048576:.1f}, scan {512 + off_mib + 1024:.1f}.", "",
                "| kernel | calls | avg us | scaled read MiB | scaled written MiB |", "|---|---:|---:|---:|---:|"]
        for k in sorted(stats):
            if "irregular" not in k:
                continue
            fv = fetch.get(k, {}).get("FETCH_SIZE", [0.0])
            wv = write.get(k, {}).get("WRITE_SIZE", [0.0])
            out.append(f"| {k} | {stats[k]['Calls']} | {float(stats[k]['AverageNs']) / 1e3:.1f} | "
                       f"{sum(fv) / len(fv) * f_scale / 1024:.1f} | {sum(wv) / len(wv) * w_scale / 1024:.1f} |")
        out.append("")
    _write("irregular_n2^28_kernels_and_traffic.md", out)


def counters(name: str, title: str, kt_dir: str, pmc_dirs, commands=None, reading=None, only: str = "") -> None:
    """A table of arbitrary PMC counters per tcr kernel (averages per launch) next to the launch durations."""
    dur = _durations(kt_dir)
    table = collections.defaultdict(dict)
    names = []
    for d in pmc_dirs:
        agg, _ = _counters(d)
        for k, cs in agg.items():
            if not k.startswith("tcr::") or only not in k:
                continue
            for c, v in cs.items():
                table[k][c] = sum(v) / len(v)
                if c not in names:
                    names.append(c)
    out = [f"# {title}", "", f"Sources: csrc stamp {source_stamp()}, commit {_commit()}.", *(commands or []), "",
           "| kernel | avg us | " + " | ".join(names) + " |", "|---|---:|" + "---:|" * len(names)]
    for k in sorted(table):
        out.append(f"| {k} | {dur.get(k, 0.0) / 1e3:.1f} | " + " | ".join(f"{table[k].get(c, float('nan')):.4g}" for c in names) + " |")
    _write(name, out + (["", *reading] if reading else []))


def chain_gap(kt_dir: str, sq_dir: str, tcc_dir: str) -> None:
    """The counter table behind the statement of where scan_chain_kernel loses against the carry-free scans."""
    commands = ["Commands (each its own run, from /tmp with TMPDIR=/tmp; durations from the kernel-trace run of",
                "bench_cfg5_sweep_kernel_stats.md; counters are sums over the chip per launch, averaged over launches):", "",
                "    rocprofv3 --pmc SQ_WAVES SQ_WAVE_CYCLES SQ_BUSY_CU_CYCLES SQ_WAIT_ANY SQ_ACTIVE_INST_ANY SQ_WAIT_INST_LDS SQ_INSTS_VMEM_RD SQ_INSTS_VMEM_WR --output-format csv -d <out> -o bench -- python3 bench.py --no-cpu-baseline --steps 2 --warmup 1 --no-context",
                "    rocprofv3 --pmc TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum TCC_EA0_WRREQ_STALL_sum TCC_EA0_RD_UNCACHED_32B_sum TCC_ATOMIC --output-format csv -d <out> -o bench -- python3 bench.py --no-cpu-baseline --steps 2 --warmup 1 --no-context", "",
                *TEMPLATE_NOTE]
    reading = ["Reading (scan_chain_kernel<0,4,16,0,0>, seg_len 2^16 and 2^20, against scan_block_kernel<0,1,2,0,0> and <0,1,8,0,0>,",
               "seg_len 2^10 and 2^12, same bytes): the chain adds some 57 000 wavefront-level loads per launch (SQ_INSTS_VMEM_RD:",
               "the descriptor reads, one window of aggregates per tile) and 8 960 atomics (TCC_ATOMIC: the tickets) -- a",
               "hundredth of a percent of the traffic.  What differs is how much work is in flight: SQ_WAVE_CYCLES is about",
               "0.6e9 against 1.0-1.1e9, i.e. the persistent kernel keeps its 16 wavefronts per compute unit (three tiles, 96 KiB",
               "of loads and 192 KiB of stores) while the one-tile kernels average 26 short-lived wavefronts per compute unit, and",
               "the memory side shows it: the DRAM read-credit stalls are a tenth of the carry-free kernels' and the",
               "write-request stalls lower as well -- the chain does not press on the memory system as hard; it loses its 4-5 %",
               "to the two workgroup barriers per tile and the round trip of the carry between them, not to extra bytes.  More",
               "tiles in flight would need more registers than 16 wavefronts of 128 leave (three tiles take 122)."]
    counters("scan_chain_vs_block_counters_n2^28.md",
             "Where the chained scan loses against the carry-free one: SQ and L2 counters per launch (n = 2^28)", kt_dir,
             [sq_dir, tcc_dir], commands, reading)


def irregular_counters(kt_dir: str, sq1: str, sq2: str, sq3: str) -> None:
    """SQ counters of the irregular kernels on the mix with 16 elements per segment on average."""
    flt = '--context-filter "uniform on 0..32"'
    commands = ["Commands (each its own run, from /tmp with TMPDIR=/tmp; durations from the kernel-trace run of the same mix in",
                "irregular_n2^28_kernels_and_traffic.md; counters are sums over the chip per launch, averaged over launches):", "",
                f"    rocprofv3 --pmc SQ_WAVES SQ_WAVE_CYCLES SQ_BUSY_CYCLES SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS SQ_ACTIVE_INST_SCA SQ_WAIT_INST_LDS SQ_WAIT_ANY --output-format csv -d <out> -o bench -- python3 bench.py --no-cpu-baseline --steps 1 --warmup 0 {flt}",
                f"    rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_INSTS_VMEM_RD SQ_INSTS_VMEM_WR SQ_INSTS_SMEM SQ_INSTS_BRANCH SQ_WAIT_INST_ANY --output-format csv -d <out> -o bench -- python3 bench.py --no-cpu-baseline --steps 1 --warmup 0 {flt}",
                f"    rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_LDS_ADDR_CONFLICT SQ_INST_LEVEL_LDS SQ_INST_LEVEL_VMEM --output-format csv -d <out> -o bench -- python3 bench.py --no-cpu-baseline --steps 1 --warmup 0 {flt}", "",
                *TEMPLATE_NOTE]
    reading = ["Reading.  A launch covers 2^28 elements = 524288 sub-tiles of 512; irregular_reduce_kernel<4,4,0,0> runs 131072",
               "wavefronts of four sub-tiles.  SQ_INSTS_VALU / 524288 is the vector instructions per 512 elements, all of the",
               "kernel included (marking the segment starts, the sums, the walk over the segment ends); SQ_LDS_IDX_ACTIVE / 256 is",
               "the LDS busy cycles per compute unit, to be held against the launch's duration times the clock.  The same",
               "counters on earlier forms of this kernel, same input: with per-element selects for the restarts and the",
               "results corrected before staging, 7.8e7 vector instructions (149 per 512 elements), 4.0e7 LDS cycles of which",
               "2.4e7 bank conflicts, 156 us; with the fused multiply-adds but one LDS addition per segment end, 6.2e7 / 5.2e7 /",
               "2.6e7 and SQ_WAIT_INST_LDS up fivefold, 144 us -- the 64 additions to one LDS word per trip took 64 turns."]
    counters("irregular_uniform16_sq_counters_n2^28.md",
             "Irregular kernels on 16.8 million segments of 0..32 elements: SQ counters per launch (n = 2^28)", kt_dir, [sq1, sq2, sq3],
             commands, reading, only="irregular")


def repeatability(json_files) -> None:
    """Five (or more) JSON lines of `python bench.py --no-cpu-baseline --no-context`, run one after the other."""
    runs = []
    for f in json_files:
        with open(f) as fh:
            runs.append(json.loads(fh.read().strip().splitlines()[-1]))
    values = [r["value"] for r in runs]
    out = [f"# Repeatability of bench.py, cfg5 sweep (n=2^28): {len(runs)} runs in a row on one MI355X box", "",
           f"Sources: csrc stamp {source_stamp()}, commit {_commit()}.", f"Command, {len(runs)} times:", "",
           "    python bench.py --no-cpu-baseline --no-context", "",
           "`value` (input GB/s over the whole step): " + ", ".join(f"{v:.1f}" for v in values) +
           f"; spread {100 * (max(values) - min(values)) / min(values):.2f} %.", "",
           "Per call: average of the 20 HIP-event timings of a run (us); minimum, median and maximum over the runs.", "",
           "| op | seg_len | min | median | max | spread |", "|---|---|---:|---:|---:|---:|"]
    for i, row in enumerate(runs[0]["rows"]):
        t = sorted(r["rows"][i]["avg_us"] for r in runs)
        out.append(f"| {row['op']} | 2^{row['seg_len_log2']} | {t[0]:.1f} | {t[len(t) // 2]:.1f} | {t[-1]:.1f} | "
                   f"{100 * (t[-1] - t[0]) / t[0]:.1f} % |")
    _write("bench_cfg5_sweep_repeatability.md", out)


def tile_load(json_files) -> None:
    """JSON lines of bench.py --no-context with --tile-load direct | lds | lds_dma, --formulation dpp, and direct again."""
    names = ["direct", "lds", "lds_dma", "dpp (lane-ordered loads, no LDS)", "direct (again)"]
    runs = []
    for f in json_files:
        with open(f) as fh:
            runs.append(json.loads(fh.read().strip().splitlines()[-1]))
    out = ["# How a tile reaches the matrix-core operands: direct operand-layout loads vs LDS staging (n = 2^28)", "",
           f"Sources: csrc stamp {source_stamp()}, commit {_commit()}.",
           "Commands, one after the other on one MI355X box (HIP-event averages of the `rows` of each JSON line, us):", "",
           "    python bench.py --no-cpu-baseline --steps 10 --warmup 3 --no-context --tile-load direct",
           "    python bench.py --no-cpu-baseline --steps 10 --warmup 3 --no-context --tile-load lds",
           "    python bench.py --no-cpu-baseline --steps 10 --warmup 3 --no-context --tile-load lds_dma",
           "    python bench.py --no-cpu-baseline --steps 10 --warmup 3 --no-context --formulation dpp",
           "    python bench.py --no-cpu-baseline --steps 10 --warmup 3 --no-context --tile-load direct", "",
           "direct: lane (j, g) loads X[j][8g .. 8g+7], its MFMA operand, with one 128-bit load (the 64 loads of a wavefront",
           "cover one contiguous KiB in a permuted lane order).  lds: lanes load in lane order, write the tile to LDS and",
           "read their operand back (the shared-memory staging of the paper's kernels).  lds_dma: the same with gfx950's",
           "128-bit load from memory into LDS.  dpp: lane-ordered loads feeding the cross-lane formulation, no LDS.",
           "The variants exist for seg_len 16 .. 512 (`reduce_small_kernel`, `scan_small_kernel`); the other rows are the",
           "same kernels in every column and show the run-to-run spread.", "",
           "| op | seg_len | " + " | ".join(names) + " |", "|---|---|" + "---:|" * len(names)]
    for i, row in enumerate(runs[0]["rows"]):
        out.append(f"| {row['op']} | 2^{row['seg_len_log2']} | " + " | ".join(f"{r['rows'][i]['avg_us']:.1f}" for r in runs) + " |")
    out += ["", "Reading: staging through LDS buys nothing for the reductions (within the spread) and costs the scans 10-11 %",
            "(the LDS round trip sits between a wavefront's only load and its stores); the load from memory into LDS is",
            "slower still for short segments.  Operands are therefore loaded directly."]
    _write("tile_load_direct_vs_lds_n2^28.md", out)


def main(argv) -> int:
    if len(argv) < 2:
        print(__doc__)
        return 2
    kind, args = argv[1], argv[2:]
    if kind == "kernel-stats":
        kernel_stats(*args)
    elif kind == "traffic":
        traffic(*args)
    elif kind == "mix":
        instruction_mix(*args)
    elif kind == "irregular":
        irregular(args)
    elif kind == "counters":
        counters(args[0], args[1], args[2], args[3:])
    elif kind == "irregular-counters":
        irregular_counters(*args)
    elif kind == "chain-gap":
        chain_gap(*args)
    elif kind == "repeatability":
        repeatability(args)
    elif kind == "tile-load":
        tile_load(args)
    elif kind == "stamp":
        print(source_stamp())
    else:
        print(__doc__)
        return 2
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
