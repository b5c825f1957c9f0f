"""Runs the library's LDS access-pattern probe (deltanet_lds_probe) once per pattern, for a profiler to count.

  rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_ACTIVE_INST_LDS SQ_INSTS_LDS --kernel-trace \
      -d $RAW/lds_patterns -o lds_patterns --output-format csv -- python3 bench_lds_patterns.py

`python3 profile_summary.py $RAW` then writes profiles/lds_conflicts_by_access_pattern.txt from the counter file.  Without a
profiler the script only times the launches (HIP events on the current stream).
"""
import argparse
import json
import sys

import torch

import paper_2406_06484_amd as dn

# pattern -> (what it is in the kernels, LDS bytes one workgroup moves per repetition)
PATTERNS = {
    0: ("operand fragment, contraction contiguous (ds_read_b128), ld 136", 8 * 8 * 1024),
    1: ("operand fragment, contraction contiguous (ds_read_b128), ld 144", 8 * 8 * 1024),
    2: ("operand fragment, contraction contiguous (ds_read_b128), ld 72", 8 * 4 * 1024),
    3: ("operand fragment, contraction contiguous (ds_read_b128), ld 80", 8 * 4 * 1024),
    4: ("operand fragment, contraction strided (2 x ds_read_b64_tr_b16), ld 144", 8 * 4 * 1024),
    5: ("operand fragment, contraction strided (2 x ds_read_b64_tr_b16), ld 80", 8 * 4 * 1024),
    6: ("accumulator tile to the row-major staging tile (ds_write_b16), ld 40", 8 * 2048),
    7: ("accumulator tile to a row-major tile (ds_write_b16), ld 144", 8 * 2048),
    8: ("accumulator tile to a transposed tile (ds_write_b64), ld 136", 8 * 2048),
    9: ("accumulator tile to a transposed tile (ds_write_b64), ld 72", 8 * 2048),
    10: ("register tile to LDS, 512 threads (ds_write_b128), ld 144", 16384),
    11: ("register tile to LDS, 256 threads (ds_write_b128), ld 136", 16384),
    12: ("row segments of a 64 x 128 tile, 256 threads (ds_read_b128), ld 136", 16384),
    13: ("row segments of the staging tile (ds_read_b128), ld 40", 8 * 2048),
    14: ("operand fragment, contraction strided (2 x ds_read_b64_tr_b16), ld 136 (unused)", 8 * 4 * 1024),
    15: ("operand fragment, contraction strided (2 x ds_read_b64_tr_b16), ld 72 (unused)", 8 * 4 * 1024),
    16: ("accumulator tile to a transposed tile (ds_write_b64), ld 144 (unused)", 8 * 2048),
    17: ("accumulator tile to a transposed tile (ds_write_b64), ld 80 (unused)", 8 * 2048),
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=2000)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        sys.exit("bench_lds_patterns.py needs a GPU")
    torch.cuda.set_device(0)
    out = {}
    for pat, (what, nbytes) in PATTERNS.items():
        dn.deltanet_lds_probe(pat, 10)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        dn.deltanet_lds_probe(pat, args.iters)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        # 2.4 GHz: LDS bytes per clock and CU that the pattern sustains (the LDS moves at most 128 B per clock)
        out[pat] = {"pattern": what, "ms": round(ms, 4), "bytes_per_clk_per_cu": round(nbytes * args.iters / (ms * 1e-3 * 2.4e9), 1)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
