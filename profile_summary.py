#!/usr/bin/env python3
"""Turns the rocprofv3 CSVs of the benchmark's profiling runs into the short text summaries under profiles/.

Run the commands below from the repo root on the GPU machine; RAW = a scratch directory for the raw profiler output (each counter pass is a run of its own; rocprofv3 does not
split counters over passes), RAW being a scratch directory for the raw profiler output, then
`python3 profile_summary.py $RAW`.

  P="python3 bench.py --mode headline --no-cpu-baseline"
  rocprofv3 --kernel-trace --stats -d $RAW/trace -o trace --output-format csv -- $P --steps 20 --warmup 5
  rocprofv3 --pmc FETCH_SIZE --kernel-trace -d $RAW/fetch -o fetch --output-format csv -- $P --steps 3 --warmup 1 --copy-calibration
  rocprofv3 --pmc WRITE_SIZE --kernel-trace -d $RAW/write -o write --output-format csv -- $P --steps 3 --warmup 1 --copy-calibration
  rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 GRBM_GUI_ACTIVE --kernel-trace -d $RAW/mfma -o mfma --output-format csv -- $P --steps 3 --warmup 1
  rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_ACTIVE_INST_LDS SQ_WAVE_CYCLES --kernel-trace -d $RAW/lds -o lds --output-format csv -- $P --steps 3 --warmup 1
  S="python3 bench.py --mode streamed --no-cpu-baseline"      (the same step under DN_OPT_STREAMED_CHUNK_KERNEL)
  rocprofv3 --kernel-trace --stats -d $RAW/trace_s -o trace_s --output-format csv -- $S --steps 20 --warmup 5
  rocprofv3 --pmc FETCH_SIZE --kernel-trace -d $RAW/fetch_s -o fetch_s --output-format csv -- $S --steps 3 --warmup 1 --copy-calibration
  rocprofv3 --pmc WRITE_SIZE --kernel-trace -d $RAW/write_s -o write_s --output-format csv -- $S --steps 3 --warmup 1 --copy-calibration

  rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_ACTIVE_INST_LDS SQ_INSTS_LDS --kernel-trace -d $RAW/lds_patterns -o lds_patterns --output-format csv -- python3 bench_lds_patterns.py

  H="python3 bench_speedup_sweep.py --head-sizes 64 --lengths 2048 --only-kept --steps 20"      (head-size table; the same with 256 and hs256_*)
  rocprofv3 --kernel-trace --stats -d $RAW/hs64_trace -o hs64_trace --output-format csv -- $H
  rocprofv3 --pmc FETCH_SIZE --kernel-trace -d $RAW/hs64_fetch -o hs64_fetch --output-format csv -- $H
  rocprofv3 --pmc WRITE_SIZE --kernel-trace -d $RAW/hs64_write -o hs64_write --output-format csv -- $H
  rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 GRBM_GUI_ACTIVE --kernel-trace -d $RAW/hs64_mfma -o hs64_mfma --output-format csv -- $H

bench.py --mode headline runs the timed step (deltanet_fwd_save + deltanet_bwd_saved: k_wy_prep, k_scan_fwd_save,
k_scan_bwd, k_bwd_chunk) and the self-contained pair (deltanet_fwd + deltanet_bwd: k_wy_prep, k_scan_fwd; k_wy_prep,
k_scan_pair, k_bwd_chunk) and nothing else, so every row below belongs to one of the two.
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import re
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
PROF = os.path.abspath(sys.argv[1]) if len(sys.argv) > 1 else os.path.join(ROOT, "prof_raw")
OUT = os.path.join(ROOT, "profiles")
W = "bench.py --mode headline (configs[2]: bf16 fwd+bwd, B=8, L=2048, H=16, d=128, chunk 64), MI355X"
COPY = "__amd_rocclr_copyBuffer"
ALG_STEP_BYTES = 2824 * 8 * 2048 * 16   # inputs read once, outputs written once: 1026 + 1798 B per token and head
KEY = """kernel name key: k_wy_prep = T (Eq. 10) and, where a backward pass follows, X per chunk; k_scan_fwd_save = forward chain
scan (Eq. 8-9) that also leaves Ut and the chunk-initial states in the buffer; k_scan_bwd = reverse scan carrying dS;
k_bwd_chunk = chunk-local adjoint of Eq. 8-11.  These four are the timed step (deltanet_fwd_save + deltanet_bwd_saved).
The self-contained pair runs k_wy_prep twice (forward: T only; backward: T and X), k_scan_fwd (forward scan without the
stores), k_scan_pair (the backward pass's recompute scan and reverse scan in one grid) and k_bwd_chunk.  k_wy_prep rows are
split by what follows them in the dispatch order.  k_bwd_stream (streamed runs) = the chunk kernel that reads S and dS'
in blocks of 32 state columns and rebuilds Ut, dUt on chip; under that option the scans do not store Ut, dUt.
"""


def short(name: str) -> str:
    m = re.search(r"dn\d+(k_[a-z_]+?)I", name)
    return m.group(1) if m else name


def rows_of(sub: str, suffix: str):
    files = glob.glob(os.path.join(PROF, sub, "**", "*" + suffix), recursive=True)
    if not files:
        return None
    with open(files[0]) as f:
        return list(csv.DictReader(f))


def labelled(rows, name_key):
    """(label, row) per dispatch in dispatch order; k_wy_prep is split by the kernel that follows it"""
    rows = sorted(rows, key=lambda r: int(r["Dispatch_Id"]))
    out = []
    for i, r in enumerate(rows):
        nm = r[name_key]
        if "k_wy_prep" in nm:
            nxt = next((short(x[name_key]) for x in rows[i + 1:] if x[name_key].startswith("_ZN2dn") and "k_wy_prep" not in x[name_key]), "")
            lab = {"k_scan_fwd_save": "k_wy_prep", "k_scan_fwd": "k_wy_prep(fwd, T only)", "k_scan_pair": "k_wy_prep(bwd, T and X)"}.get(nxt, "k_wy_prep")
        elif nm.startswith("_ZN2dn"):
            lab = short(nm)
        elif COPY in nm:
            lab = COPY
        else:
            continue
        out.append((lab, r))
    return out


def counter_means(sub: str):
    """{counter: {label: mean per dispatch}}"""
    rows = rows_of(sub, "counter_collection.csv")
    if rows is None:
        return None
    by_disp = collections.OrderedDict()
    for r in rows:
        by_disp.setdefault(r["Dispatch_Id"], r)
    labels = {r["Dispatch_Id"]: lab for lab, r in labelled(list(by_disp.values()), "Kernel_Name")}
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in rows:
        lab = labels.get(r["Dispatch_Id"])
        if lab is not None:
            acc[r["Counter_Name"]][lab].append(float(r["Counter_Value"]))
    return {c: {k: sum(v) / len(v) for k, v in d.items()} for c, d in acc.items()}


def trace_means(sub: str):
    """{label: (calls, mean ns, min ns, max ns)} from the kernel trace (launch durations in dispatch order)"""
    rows = rows_of(sub, "kernel_trace.csv")
    if rows is None:
        return None
    acc = collections.defaultdict(list)
    for lab, r in labelled(rows, "Kernel_Name"):
        acc[lab].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    return {k: (len(v), sum(v) / len(v), min(v), max(v)) for k, v in acc.items()}


STEP = ["k_wy_prep", "k_scan_fwd_save", "k_scan_bwd", "k_bwd_chunk"]
STEP_S = ["k_wy_prep", "k_scan_fwd_save", "k_scan_bwd", "k_bwd_stream"]
PAIR = ["k_wy_prep(fwd, T only)", "k_scan_fwd", "k_wy_prep(bwd, T and X)", "k_scan_pair", "k_bwd_chunk"]


def write_trace():
    tr = trace_means("trace")
    if tr is None:
        return
    with open(os.path.join(OUT, "kernel_trace_cfg2_fwd_bwd.txt"), "w") as f:
        f.write("rocprofv3 kernel-trace summary: %s\n\ncommand (from the repo root on the GPU box; RAW = a scratch directory for the raw profiler output), then python3 profile_summary.py $RAW:\n"
                "  rocprofv3 --kernel-trace --stats -d $RAW/trace -o trace --output-format csv -- python3 bench.py --mode headline --no-cpu-baseline --steps 20 --warmup 5\n\n" % W)
        f.write("%-28s %7s %12s %10s %10s\n" % ("kernel", "calls", "avg_ns", "min_ns", "max_ns"))
        for k, (n, avg, lo, hi) in tr.items():
            if k != COPY:
                f.write("%-28s %7d %12.0f %10d %10d\n" % (k, n, avg, lo, hi))
        f.write("\nsum of kernel time per step (deltanet_fwd_save + deltanet_bwd_saved): %.1f us; per self-contained fwd+bwd: %.1f us\n"
                % (sum(tr[k][1] for k in STEP if k in tr) / 1e3, sum(tr[k][1] for k in PAIR if k in tr) / 1e3))
        ts = trace_means("trace_s")
        if ts is not None:
            f.write("\nthe same step under DN_OPT_STREAMED_CHUNK_KERNEL (bench.py --mode streamed, same flags, -d $RAW/trace_s -o trace_s):\n")
            for k in STEP_S:
                if k in ts:
                    f.write("%-28s %7d %12.0f %10d %10d\n" % ((k,) + ts[k]))
            f.write("sum of kernel time per step: %.1f us\n" % (sum(ts[k][1] for k in STEP_S if k in ts) / 1e3))
        f.write("\n" + KEY)


def traffic_table(fetch_sub, write_sub):
    fe, wr = counter_means(fetch_sub), counter_means(write_sub)
    if fe is None or wr is None:
        return None
    fe, wr = fe["FETCH_SIZE"], wr["WRITE_SIZE"]
    ff, wf = 262144.0 / fe[COPY], 262144.0 / wr[COPY]
    tab = {k: (fe[k] * ff, wr[k] * wf) for k in fe if k != COPY and k in wr}
    return tab, (fe[COPY], wr[COPY], ff, wf)


def write_traffic():
    res = traffic_table("fetch", "write")
    if res is None:
        return
    tab, (cf, cw, ff, wf) = res
    with open(os.path.join(OUT, "hbm_traffic_cfg2_fwd_bwd.txt"), "w") as f:
        f.write("rocprofv3 --pmc HBM traffic per launch: %s\n\ncommands (from the repo root on the GPU box; RAW = a scratch directory for the raw profiler output; one counter per run), then python3 profile_summary.py $RAW:\n"
                "  rocprofv3 --pmc FETCH_SIZE --kernel-trace -d $RAW/fetch -o fetch --output-format csv -- python3 bench.py --mode headline --no-cpu-baseline --steps 3 --warmup 1 --copy-calibration\n"
                "  rocprofv3 --pmc WRITE_SIZE --kernel-trace -d $RAW/write -o write --output-format csv -- python3 bench.py --mode headline --no-cpu-baseline --steps 3 --warmup 1 --copy-calibration\n\n" % W)
        f.write("calibration: a plain 256 MiB device copy (%s) reads FETCH_SIZE = %.1f and WRITE_SIZE = %.1f (KiB);\n"
                "it moves 262144 KiB each way, so the scale factors are %.3f (fetch) and %.3f (write).\n\n" % (COPY, cf, cw, ff, wf))
        f.write("%-28s %14s %14s %12s\n" % ("kernel", "fetch_KiB*f", "write_KiB*f", "total_MB"))
        mb = {}
        for k, (a, b) in tab.items():
            mb[k] = (a + b) * 1024 / 1e6
            f.write("%-28s %14.0f %14.0f %12.1f\n" % (k, a, b, mb[k]))
        step = sum(mb[k] for k in STEP if k in mb)
        pair = sum(mb[k] for k in PAIR if k in mb)
        f.write("\nHBM bytes per step (deltanet_fwd_save + deltanet_bwd_saved): %.1f MB; per self-contained fwd+bwd: %.1f MB;\n"
                "the algorithmic minimum (inputs read once, outputs written once) is 2824 B per token per head = %.1f MB.\n"
                % (step, pair, ALG_STEP_BYTES / 1e6))
        res_s = traffic_table("fetch_s", "write_s")
        if res_s is not None:
            tab_s = res_s[0]
            f.write("\nthe same step under DN_OPT_STREAMED_CHUNK_KERNEL (bench.py --mode streamed; -d $RAW/fetch_s -o fetch_s, write_s likewise):\n")
            tot = 0.0
            for k in STEP_S:
                if k in tab_s:
                    m = (tab_s[k][0] + tab_s[k][1]) * 1024 / 1e6
                    tot += m
                    f.write("%-28s %14.0f %14.0f %12.1f\n" % (k, tab_s[k][0], tab_s[k][1], m))
            f.write("HBM bytes per step: %.1f MB\n" % tot)
        f.write("\nbytes per launch as bench.py reads them (the headline step's kernels, and the self-contained pair's own two):\n")
        for k in STEP + ["k_scan_fwd", "k_scan_pair"]:
            if k in mb:
                f.write("traffic_bytes %s %d\n" % (k, round(mb[k] * 1e6)))
        if res_s is not None and "k_bwd_stream" in res_s[0]:
            a, b = res_s[0]["k_bwd_stream"]
            f.write("traffic_bytes k_bwd_stream %d\n" % round((a + b) * 1024))
        f.write("\n" + KEY)


def write_counters():
    mf, ld = counter_means("mfma"), counter_means("lds")
    if mf is None or ld is None:
        return
    with open(os.path.join(OUT, "mfma_lds_counters_cfg2_fwd_bwd.txt"), "w") as f:
        f.write("rocprofv3 --pmc MFMA and LDS counters per launch: %s\n\ncommands (from the repo root on the GPU box; RAW = a scratch directory for the raw profiler output; one pass per run), then python3 profile_summary.py $RAW:\n"
                "  rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 GRBM_GUI_ACTIVE --kernel-trace -d $RAW/mfma -o mfma --output-format csv -- python3 bench.py --mode headline --no-cpu-baseline --steps 3 --warmup 1\n"
                "  rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_ACTIVE_INST_LDS SQ_WAVE_CYCLES --kernel-trace -d $RAW/lds -o lds --output-format csv -- python3 bench.py --mode headline --no-cpu-baseline --steps 3 --warmup 1\n\n" % W)
        f.write("Averages per launch.  GRBM_GUI_ACTIVE is summed over the 8 XCDs; SQ_VALU_MFMA_BUSY_CYCLES over the 1024 SIMDs.\n"
                "mfma_util = SQ_VALU_MFMA_BUSY_CYCLES / 1024 / (GRBM_GUI_ACTIVE / 8): the share of the kernel's time in which a SIMD's matrix\n"
                "pipe is busy, averaged over the chip.  bf16_tflops = SQ_INSTS_VALU_MFMA_MOPS_BF16 x 512 FLOP / kernel time at 2.4 GHz.\n"
                "lds_conflict = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE: conflict cycles per cycle the LDS is indexing.\n\n")
        f.write("%-28s %12s %10s %12s %13s\n" % ("kernel", "active_cyc", "mfma_util", "bf16_tflops", "lds_conflict"))
        for k in mf["GRBM_GUI_ACTIVE"]:
            if k == COPY:
                continue
            act = mf["GRBM_GUI_ACTIVE"][k] / 8.0
            util = mf["SQ_VALU_MFMA_BUSY_CYCLES"][k] / 1024.0 / act if act else 0.0
            tfl = mf["SQ_INSTS_VALU_MFMA_MOPS_BF16"][k] * 512.0 / (act / 2.4e9) / 1e12 if act else 0.0
            idx = ld["SQ_LDS_IDX_ACTIVE"].get(k, 0.0)
            conf = ld["SQ_LDS_BANK_CONFLICT"].get(k, 0.0) / idx if idx else 0.0
            f.write("%-28s %12.0f %10.3f %12.1f %13.3f\n" % (k, act, util, tfl, conf))
        f.write("\nThe counters are taken under the profiler, where the kernels run a few percent slower than in the timed region.\n" + KEY)


def write_lds_patterns():
    rows = rows_of("lds_patterns", "counter_collection.csv")
    if rows is None:
        return
    sys.path.insert(0, ROOT)
    from bench_lds_patterns import PATTERNS  # the probe's pattern list (names only; importing it runs nothing)
    agg = collections.defaultdict(dict)
    for r in rows:
        m = re.search(r"k_lds_probe<(\d+)>", r["Kernel_Name"])
        if m:  # the long launch of each pattern (the short warm-up launch counts less)
            d = agg[int(m.group(1))]
            d[r["Counter_Name"]] = max(d.get(r["Counter_Name"], 0.0), float(r["Counter_Value"]))
    with open(os.path.join(OUT, "lds_conflicts_by_access_pattern.txt"), "w") as f:
        f.write("LDS counters of the access patterns the kernels are built from, one probe kernel per pattern (deltanet_lds_probe: the\n"
                "kernels' own helpers at the kernels' own leading dimensions, 8 wavefronts per workgroup, bf16 tiles), MI355X\n\n"
                "command (from the repo root on the GPU box; RAW = a scratch directory for the raw profiler output), then python3 profile_summary.py $RAW:\n"
                "  rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_ACTIVE_INST_LDS SQ_INSTS_LDS --kernel-trace -d $RAW/lds_patterns -o lds_patterns --output-format csv -- python3 bench_lds_patterns.py\n\n"
                "conflict = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE (the ratio profiles/mfma_lds_counters_cfg2_fwd_bwd.txt gives per kernel);\n"
                "idx/inst = SQ_LDS_IDX_ACTIVE / SQ_INSTS_LDS: cycles the LDS spends indexing one instruction of the pattern.  An instruction\n"
                "that moves 1024 bytes per wavefront (16 bytes per lane) occupies the 128-byte-per-clock data path for 8 cycles whatever its\n"
                "index cycles are, one that moves 512 bytes for 4.\n\n")
        f.write("%2s  %-92s %9s %9s\n" % ("#", "pattern", "conflict", "idx/inst"))
        for pat in sorted(agg):
            d = agg[pat]
            idx, inst = d.get("SQ_LDS_IDX_ACTIVE", 0.0), d.get("SQ_INSTS_LDS", 0.0)
            f.write("%2d  %-92s %9.3f %9.2f\n" % (pat, PATTERNS[pat][0], d.get("SQ_LDS_BANK_CONFLICT", 0.0) / idx if idx else 0.0,
                                                  idx / inst if inst else 0.0))
        f.write("\nReading: the 16-byte fragment reads are conflict-free at leading dimensions of 8 (mod 32) elements (136, 72) and take two\n"
                "index passes at 16 (mod 32) (144, 80): 8 index cycles, the same 8 cycles the data path needs for the instruction, so that\n"
                "conflict costs no time.  The transposing 8-byte reads take 4 index cycles against 4 data cycles at 144, 80 and 72, and 8 at 136,\n"
                "which is why tiles that are read in both orders carry the padding of 16 elements.  The 2-byte accumulator writes have no\n"
                "conflicts (they are bound by instruction issue).  The 8-byte transposed accumulator writes (issued in pairs, 16 bytes per\n"
                "lane) need 16 index cycles where 8 would do, and 31 at 144 or 80: the one pattern whose conflicts cost LDS time, about 30\n"
                "cycles per 32 x 32 tile and wavefront, at the better of the two paddings a 16-byte-aligned row allows.\n")


def write_head_sizes():
    base = traffic_table("fetch", "write")
    if base is None:
        return
    _, (_, _, ff, wf) = base
    subs = {64: "hs64_%s", 128: "%s", 256: "hs256_%s"}
    if trace_means(subs[64] % "trace") is None or trace_means(subs[256] % "trace") is None:
        return
    with open(os.path.join(OUT, "tiling_head_size_counters.txt"), "w") as f:
        f.write("Tiling study, head size: the training step that keeps the forward pass's tiles (deltanet_fwd_save + deltanet_bwd_saved) on\n"
                "16384 tokens of model width 2048 (B = 8, L = 2048, H = 2048 / d, bf16, chunk 64), per kernel, MI355X\n\n"
                "commands (from the repo root on the GPU box; RAW = a scratch directory for the raw profiler output; d = 64 and 256 shown, one pass per run; d = 128 is the headline step, whose\n"
                "passes are listed in profiles/kernel_trace_cfg2_fwd_bwd.txt and its neighbours), then python3 profile_summary.py $RAW:\n"
                "  P=\"python3 bench_speedup_sweep.py --head-sizes 64 --lengths 2048 --only-kept --steps 20\"     (and --head-sizes 256, hs256_*)\n"
                "  rocprofv3 --kernel-trace --stats -d $RAW/hs64_trace -o hs64_trace --output-format csv -- $P\n"
                "  rocprofv3 --pmc FETCH_SIZE --kernel-trace -d $RAW/hs64_fetch -o hs64_fetch --output-format csv -- $P\n"
                "  rocprofv3 --pmc WRITE_SIZE --kernel-trace -d $RAW/hs64_write -o hs64_write --output-format csv -- $P\n"
                "  rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 GRBM_GUI_ACTIVE --kernel-trace -d $RAW/hs64_mfma -o hs64_mfma --output-format csv -- $P\n\n"
                "HBM bytes = FETCH_SIZE x %.3f + WRITE_SIZE x %.3f (KiB per launch; factors from the 256 MiB copy of the headline run);\n"
                "mfma_util and bf16_tflops as in profiles/mfma_lds_counters_cfg2_fwd_bwd.txt.\n\n" % (ff, wf))
        f.write("%4s  %-20s %9s %9s %8s %10s %12s\n" % ("d", "kernel", "avg_us", "HBM_MB", "TB/s", "mfma_util", "bf16_tflops"))
        for d in (64, 128, 256):
            tr = trace_means(subs[d] % "trace")
            fe, wr, mf = counter_means(subs[d] % "fetch"), counter_means(subs[d] % "write"), counter_means(subs[d] % "mfma")
            step = ["k_wy_prep", "k_scan_fwd_save", "k_scan_bwd", "k_bwd_chunk_wide" if d == 256 else "k_bwd_chunk"]
            tot_us = tot_mb = 0.0
            for k in step:
                if k not in tr:
                    continue
                us = tr[k][1] / 1e3
                mb = (fe["FETCH_SIZE"][k] * ff + wr["WRITE_SIZE"][k] * wf) * 1024 / 1e6
                act = mf["GRBM_GUI_ACTIVE"][k] / 8.0
                util = mf["SQ_VALU_MFMA_BUSY_CYCLES"][k] / 1024.0 / act if act else 0.0
                tfl = mf["SQ_INSTS_VALU_MFMA_MOPS_BF16"][k] * 512.0 / (act / 2.4e9) / 1e12 if act else 0.0
                f.write("%4d  %-20s %9.1f %9.1f %8.2f %10.3f %12.1f\n" % (d, k, us, mb, mb / us, util, tfl))
                tot_us += us
                tot_mb += mb
            f.write("%4d  %-20s %9.1f %9.1f %8.2f\n\n" % (d, "step", tot_us, tot_mb, tot_mb / tot_us))
        f.write("TB/s = HBM_MB / avg_us.  At d = 64 a chain is one scan workgroup (256 chains), at d = 128 two (128 chains), at d = 256 eight\n"
                "workgroups of 32 state columns (64 chains, 512 workgroups in two rounds); the chunk kernel keeps a chunk's operands in LDS\n"
                "up to d = 128 and streams S and dS' in blocks of 32 state columns at d = 256 (k_bwd_chunk_wide).  Per token the matrix work\n"
                "grows with d (model FLOPs 6 d^2 + ... per token and head, H = 2048 / d heads) while the bytes per token stay the same for\n"
                "q, k, v, o and grow with d for the per-chunk states.\n")


def main() -> int:
    if not os.path.isdir(PROF):
        print("profile_summary.py: %s is missing; run the rocprofv3 commands in this file's header first" % PROF, file=sys.stderr)
        return 2
    os.makedirs(OUT, exist_ok=True)
    write_trace()
    write_traffic()
    write_counters()
    write_lds_patterns()
    write_head_sizes()
    return 0


if __name__ == "__main__":
    sys.exit(main())
