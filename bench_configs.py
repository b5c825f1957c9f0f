#!/usr/bin/env python3
"""Times the five benchmark configurations on one MI355X: forward, backward, and the training step as the
self-contained pair and as the pair that keeps the forward pass's tiles.  Inputs are the seeded synthetic
batches of ``synth.CONFIGS``, resident on the device; times are wall-clock per call over ``--steps`` calls.
Prints a table and, per configuration and mode, one JSON line (prefix ``JSON ``) with the same figures.

    python bench_configs.py [--steps 20]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=20)
    args = ap.parse_args()
    import numpy as np
    import torch

    import paper_2406_06484_amd as dn
    from paper_2406_06484_amd.synth import CONFIGS, make_config

    if not torch.cuda.is_available():
        print("config_timings: no GPU visible; there is no CPU fallback", file=sys.stderr)
        return 2
    dn.load_library()
    dev = torch.device("cuda:0")

    def timeit(f):
        for _ in range(3):
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            f()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t0) / args.steps

    lines = []
    print("%3s %-44s %8s | %8s %8s %10s %10s | %12s" % ("cfg", "shape", "tokens", "fwd ms", "bwd ms", "fwd+bwd ms", "kept ms", "M tokens/s"))
    for idx in sorted(CONFIGS):
        inp = make_config(idx)
        tdt = torch.bfloat16 if inp.dtype == "bf16" else torch.float32
        to = lambda a, t=tdt: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(torch.float32).to(t).to(dev)
        q, k, v, beta, d_o = (to(getattr(inp, n)) for n in ("q", "k", "v", "beta", "d_o"))
        S0, dST = to(inp.initial_state, torch.float32), to(inp.dfinal_state, torch.float32)
        cu = None if inp.cu_seqlens is None else torch.from_numpy(inp.cu_seqlens).to(dev)
        tokens = inp.meta["tokens"]
        _, _, saved = dn.deltanet_fwd_save(q, k, v, beta, S0, cu_seqlens=cu)
        ws = torch.empty_like(saved)
        t_f = timeit(lambda: dn.deltanet_fwd(q, k, v, beta, S0, cu_seqlens=cu, workspace=ws))
        t_b = timeit(lambda: dn.deltanet_bwd(q, k, v, beta, d_o, S0, dST, cu_seqlens=cu, workspace=ws))

        def kept():
            dn.deltanet_fwd_save(q, k, v, beta, S0, cu_seqlens=cu, saved=saved)
            dn.deltanet_bwd_saved(q, k, v, beta, d_o, saved, dST, cu_seqlens=cu)
        t_k = timeit(kept)
        c = CONFIGS[idx]
        shape = "%s %s H=%d d=%d" % (inp.dtype, ("packed %d seqs" % (len(inp.cu_seqlens) - 1)) if cu is not None else "B=%d L=%d" % (c["B"], c["L"]),
                                    c["H"], c["dk"])
        print("%3d %-44s %8d | %8.3f %8.3f %10.3f %10.3f | %12.2f" % (idx, shape, tokens, t_f, t_b, t_f + t_b, t_k, tokens / t_k / 1e3), flush=True)
        for mode, ms in (("fwd", t_f), ("bwd", t_b), ("fwd+bwd", t_f + t_b), ("fwd_save+bwd_saved", t_k)):
            lines.append(json.dumps({"config": idx, "shape": shape, "mode": mode, "tokens": tokens, "ms": round(ms, 4),
                                     "tokens_per_s": round(tokens / (ms * 1e-3), 1), "steps": args.steps}))
    for l in lines:
        print("JSON " + l)
    return 0


if __name__ == "__main__":
    sys.exit(main())
