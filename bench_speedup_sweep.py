#!/usr/bin/env python3
"""Chunkwise form against recurrent form on one MI355X, over sequence length and head size.

The workload is the one of the paper's speed-up figure (section 3.3): model width 2048 split into
heads of size d (H = 2048 / d), batch times length fixed at 16384 tokens, bf16, random unit-norm
q, k.  For each (d, L) it times the forward pass of both forms through the C ABI, the chunkwise
forward + backward as the self-contained pair and as the pair that keeps the forward pass's tiles,
and prints one table row.

    python bench_speedup_sweep.py [--steps 20]

With --only-kept it runs nothing but the training step that keeps the forward pass's tiles, --steps times per
(d, L): the form a profiler's counter passes use (profile_summary.py, head-size table).
"""
from __future__ import annotations

import argparse
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--tokens", type=int, default=16384)
    ap.add_argument("--width", type=int, default=2048)
    ap.add_argument("--head-sizes", type=int, nargs="+", default=[64, 128, 256])
    ap.add_argument("--lengths", type=int, nargs="+", default=[512, 1024, 2048, 4096, 8192, 16384])
    ap.add_argument("--only-kept", action="store_true", help="run only deltanet_fwd_save + deltanet_bwd_saved (for profiler passes)")
    args = ap.parse_args()
    import torch

    import paper_2406_06484_amd as dn
    from paper_2406_06484_amd.binding import _shape_of, deltanet_workspace_bytes

    if not torch.cuda.is_available():
        print("speedup_sweep: no GPU visible; there is no CPU fallback", file=sys.stderr)
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

    print("%5s %6s %4s %4s | %12s %12s %9s | %16s %16s" % ("d", "L", "B", "H", "recurrent ms", "chunkwise ms", "speed-up",
                                                        "fwd+bwd ms", "fwd+bwd kept ms"))
    for d in args.head_sizes:
        H = args.width // d
        for L in args.lengths:
            B = max(1, args.tokens // L)
            g = torch.Generator(device="cpu").manual_seed(L + d)
            unit = lambda: torch.nn.functional.normalize(torch.randn(B, L, H, d, generator=g), dim=-1).bfloat16().to(dev)
            q, k = unit(), unit()
            v = torch.randn(B, L, H, d, generator=g).bfloat16().to(dev)
            d_o = torch.randn(B, L, H, d, generator=g).bfloat16().to(dev)
            beta = torch.sigmoid(torch.randn(B, L, H, generator=g)).bfloat16().to(dev)
            o = torch.empty_like(v)
            ST = torch.empty(B, H, d, d, dtype=torch.float32, device=dev)
            ws = torch.empty(deltanet_workspace_bytes(_shape_of(q, v, None, 64, []), True), dtype=torch.uint8, device=dev)
            if args.only_kept:
                def kept_only():
                    dn.deltanet_fwd_save(q, k, v, beta, o=o, final_state=ST, saved=ws)
                    dn.deltanet_bwd_saved(q, k, v, beta, d_o, ws)
                print("%5d %6d %4d %4d | kept step %.3f ms" % (d, L, B, H, timeit(kept_only)), flush=True)
                continue
            t_rec = timeit(lambda: dn.deltanet_recurrent_fwd(q, k, v, beta, o=o, final_state=ST))
            t_chk = timeit(lambda: dn.deltanet_fwd(q, k, v, beta, o=o, final_state=ST, workspace=ws))

            def both():
                dn.deltanet_fwd(q, k, v, beta, o=o, final_state=ST, workspace=ws)
                dn.deltanet_bwd(q, k, v, beta, d_o, workspace=ws)

            def kept():
                dn.deltanet_fwd_save(q, k, v, beta, o=o, final_state=ST, saved=ws)
                dn.deltanet_bwd_saved(q, k, v, beta, d_o, ws)
            t_fb, t_kept = timeit(both), timeit(kept)
            print("%5d %6d %4d %4d | %12.3f %12.3f %8.2fx | %16.3f %16.3f" % (d, L, B, H, t_rec, t_chk, t_rec / t_chk, t_fb, t_kept),
                  flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
