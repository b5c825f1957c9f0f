#!/usr/bin/env python3
"""Benchmark of the DeltaNet layer hot path on one MI355X.

A "step" is one forward plus one backward pass of the layer over one batch of synthetic input shaped
like the paper's 1.3B-model layers: bf16, B=8, L=2048, H=16, d_k=d_v=128, chunk 64, through the C ABI
as a training step calls it: deltanet_fwd_save, which leaves its per-chunk tiles in a buffer, then
deltanet_bwd_saved, which reads them instead of recomputing them.  The self-contained pair
(deltanet_fwd + deltanet_bwd, backward recomputes everything from the inputs) is timed beside it and
reported as "recompute_fwd_bwd".  Inputs are resident in HBM before the timed region.  Prints ONE JSON line: tokens/s of the layer (B*L tokens per step), the dominant kernel's
roofline position (per-kernel time from HIP events recorded by the library on the launch stream),
and the fp64 CPU oracle timed on the host cores as a reported baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
PEAK_FP32_VECTOR_TFLOPS = 157.3  # published fp32 vector rate (counts packed FMA; plain FMA code reaches half)
C = 64


def model_flops_per_token_head(d: int, c: int = C):
    """Dense-tile FLOP count of the chunkwise algorithm per token per head (no recompute)."""
    fwd = 6 * d * d + 10 * c * d + (2.0 / 3.0) * c * c
    bwd = 12 * d * d + 20 * c * d + 4 * c * c
    return fwd, bwd


def kernel_flops_per_chunk_head(name: str, d: int, c: int = C) -> float:
    """Dense-tile FLOPs one (chunk, head) costs in each kernel (what that kernel contracts)."""
    if "k_wy_prep" in name:      # K K^T, forward substitution
        return 2 * c * c * d + (2.0 / 3.0) * c ** 3
    if "k_scan_fwd_save" in name:  # as k_scan_fwd
        return 6 * c * d * d + 8 * c * c * d
    if "k_scan_bwd" in name:     # T K, K Q^T, P^T dO (3 x 2C^2 d); K dS, Q^T dO, W^T dUt (3 x 2Cd^2)
        return 6 * c * d * d + 6 * c * c * d
    if "k_scan_pair" in name:    # recompute scan: T K, T V, W S, K^T Ut; reverse scan: T K, K Q^T, P^T dO, K dS, Q^T dO, W^T dUt
        return (4 * c * d * d + 4 * c * c * d) + (6 * c * d * d + 6 * c * c * d)
    if "k_scan_fwd" in name:     # T K, T V, Q K^T, P Ut (4 x 2C^2 d); W S, Q S, K^T Ut (3 x 2Cd^2)
        return 6 * c * d * d + 8 * c * c * d
    if "k_bwd_chunk" in name:
        # adjoint of Eq. 8-9: dO S^T, dUt S^T, Ut dS^T (3 x 2Cd^2); dO Ut^T, dP K, dP^T Q (3 x 2C^2 d)
        # adjoint of Eq. 10-11: K K^T, dW K^T, dU V^T, X^T dW, X^T dU, Ah K, Ah^T K (7 x 2C^2 d);
        #                       dX X^T, X^T M1 (2 x 2C^3); forward substitution (2/3 C^3)
        return 6 * c * d * d + 20 * c * c * d + 4 * c ** 3 + (2.0 / 3.0) * c ** 3
    return 0.0


def kernel_bytes_per_chunk_head(name: str, d: int, c: int = C, es: int = 2) -> float:
    """Operand bytes one (chunk, head) costs in each kernel: every tile it must read or write, once.

    tile = C x d elements, cc = C x C, st = d x d (states leave the scans in the element type)."""
    tile, cc, st, beta = c * d * es, c * c * es, d * d * es, c * es
    if "k_wy_prep" in name:      # mean of its two launches: K, beta -> T (forward) / T, X (backward)
        return tile + beta + 1.5 * cc
    if "k_scan_fwd_save" in name:  # Q, K, V, T -> O, Ut, S
        return 3 * tile + cc + 2 * tile + st
    if "k_scan_bwd" in name:     # Q, K, dO, T -> dUt, dS'
        return 3 * tile + cc + tile + st
    if "k_scan_pair" in name:    # K, V, T -> Ut, S   and   Q, K, dO, T -> dUt, dS'
        return (2 * tile + cc + tile + st) + (3 * tile + cc + tile + st)
    if "k_scan_fwd" in name:     # Q, K, V, T -> O
        return 3 * tile + cc + tile
    if "k_bwd_chunk" in name:    # dO, Ut, dUt, K, Q, V, S, dS', X, beta -> dQ, dK, dV, dbeta
        return 6 * tile + 2 * st + cc + beta + 3 * tile + c * 4
    return 0.0


# HBM bytes per launch of each kernel on this workload: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, each
# scaled by what the same counter reads for a plain 256 MiB device copy (factors 2.000 and 1.000);
# summary and commands in profiles/hbm_traffic_cfg2_fwd_bwd.txt.  The counters cannot be read from
# inside this script, so the figures are carried here and refreshed whenever the kernels change.
MEASURED_HBM_BYTES = {
    "k_wy_prep": 149.2e6,   # mean over the run's launches, those of the fused-prologue step (which also map q, k) included
    "k_scan_fwd_save": 512.0e6,
    "k_scan_bwd": 451.8e6,
    "k_scan_fwd": 310.5e6,
    "k_scan_pair": 824.3e6,
    "k_bwd_chunk": 919.8e6,
    "k_recurrent_fwd": 281.2e6,
}


def measured_traffic(name: str):
    for key, val in MEASURED_HBM_BYTES.items():
        if name.startswith(key):
            return val
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy, as the reference dispatch that scales the "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2406_06484_amd as dn
    from paper_2406_06484_amd.synth import CONFIGS, make_config

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    dn.load_library()
    cfg = CONFIGS[2]
    B, L, H, d = cfg["B"], cfg["L"], cfg["H"], cfg["dk"]
    inp = make_config(2)
    dev = torch.device("cuda:0")
    bf = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(torch.float32).to(torch.bfloat16).to(dev)
    q, k, v, beta, d_o = (bf(getattr(inp, n)) for n in ("q", "k", "v", "beta", "d_o"))
    from paper_2406_06484_amd.binding import _shape_of, deltanet_workspace_bytes
    shp = _shape_of(q, v, None, C, [])
    ws = torch.empty(deltanet_workspace_bytes(shp, True), dtype=torch.uint8, device=dev)
    o = torch.empty_like(v)
    ST = torch.empty((B, H, d, d), dtype=torch.float32, device=dev)

    def step():   # the training step: the forward pass leaves its per-chunk tiles in ws for the backward pass
        dn.deltanet_fwd_save(q, k, v, beta, o=o, final_state=ST, saved=ws)
        return dn.deltanet_bwd_saved(q, k, v, beta, d_o, ws)

    def recompute_step():   # the self-contained pair: nothing is kept between the two calls
        dn.deltanet_fwd(q, k, v, beta, o=o, final_state=ST, workspace=ws)
        return dn.deltanet_bwd(q, k, v, beta, d_o, workspace=ws)

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    tokens = B * L
    value = tokens * args.steps / dt

    # fwd / bwd split (untimed for `value`)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    fw = bw = 0.0
    for _ in range(args.steps):
        ev[0].record(); dn.deltanet_fwd_save(q, k, v, beta, o=o, final_state=ST, saved=ws)
        ev[1].record(); dn.deltanet_bwd_saved(q, k, v, beta, d_o, ws)
        ev[2].record(); torch.cuda.synchronize()
        fw += ev[0].elapsed_time(ev[1]); bw += ev[1].elapsed_time(ev[2])
    fw /= args.steps; bw /= args.steps

    # per-kernel device time from the library's own HIP events on the launch stream
    dn.deltanet_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = dn.deltanet_profile_collect()
    dn.deltanet_profile_enable(False)
    chunk_heads = B * H * (L // C)
    kernels = {}
    for name, (ms, n) in prof.items():
        nm = name.strip("()")
        avg = ms / n
        fl = kernel_flops_per_chunk_head(nm, d) * chunk_heads
        by = kernel_bytes_per_chunk_head(nm, d) * chunk_heads
        kernels[nm] = {"avg_ms": round(avg, 4), "launches_per_step": n // args.steps,
                       "tflops": round(fl / (avg * 1e-3) / 1e12, 2), "gbs": round(by / (avg * 1e-3) / 1e9, 1)}
    # k_wy_prep runs twice per step (forward and backward); weight by launches per step
    dom = max(kernels, key=lambda n: kernels[n]["avg_ms"] * kernels[n]["launches_per_step"])
    fwd_f, bwd_f = model_flops_per_token_head(d)
    model_tflops = (fwd_f + bwd_f) * H * value / 1e12
    # Every kernel of the path sits nearer the HBM roof than the MFMA roof (its operand bytes / 8 TB/s
    # exceed its FLOPs / 2.5 PFLOP/s), so the dominant kernel is placed against HBM; the same kernel
    # against the bf16 MFMA roof rides along.
    roofline = {"bound": "hbm", "kernel": dom, "achieved": kernels[dom]["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(kernels[dom]["gbs"] / PEAK_HBM_GBS, 4), "traffic": measured_traffic(dom),
                "mfma": {"achieved": kernels[dom]["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(kernels[dom]["tflops"] / PEAK_BF16_TFLOPS, 4)}}

    out = {
        "metric": "DeltaNet layer fwd+bwd tokens/s at H=16,d=128,L=2048; % bf16 MFMA peak",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[2]: bf16 fwd+bwd, B=8, L=2048, H=16, d_k=d_v=128, chunk=64; the forward pass keeps its per-chunk tiles for the backward pass",
                   "tokens_per_step": tokens},
        "fwd_ms": round(fw, 4), "bwd_ms": round(bw, 4),
        "model_tflops": round(model_tflops, 2),
        "pct_bf16_mfma_peak": round(100 * model_tflops / PEAK_BF16_TFLOPS, 3),
        # the same with the masked halves of the C x C tiles not counted (forward 6d^2 + 5Cd + 2/3 C^2), and with the FLOPs a
        # backward pass that recomputes the chunk states adds (4d^2 + 8Cd + 2/3 C^2; this step keeps them, so nothing is added)
        "pct_bf16_mfma_peak_triangle_aware": round(100 * (model_tflops - 5 * C * d * H * value / 1e12) / PEAK_BF16_TFLOPS, 3),
        "recompute_extra_flops_per_token_head": 4 * d * d + 8 * C * d + (2.0 / 3.0) * C * C,
        "algorithmic_hbm_gbs": round((1026 + 1798) * H * value / 1e9, 1),
        "measured_hbm_gbs": round(sum((measured_traffic(n) or 0.0) * k_["launches_per_step"] for n, k_ in kernels.items())
                                  / (ms_per_step * 1e-3) / 1e9, 1),
        "kernels": kernels,
        "roofline": roofline,
    }

    # The self-contained pair on the same workload (the backward pass recomputes T, X, the chunk states and
    # Ut from the inputs, as the paper's implementation does), with its own per-kernel times.
    for _ in range(args.warmup):
        recompute_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        recompute_step()
    torch.cuda.synchronize()
    rms = 1e3 * (time.perf_counter() - t0) / args.steps
    dn.deltanet_profile_enable(True)
    for _ in range(args.steps):
        recompute_step()
    torch.cuda.synchronize()
    rprof = dn.deltanet_profile_collect()
    dn.deltanet_profile_enable(False)
    out["recompute_fwd_bwd"] = {
        "ms_per_step": round(rms, 4), "tokens_per_s": round(tokens / (rms * 1e-3), 1), "steps": args.steps,
        "kernels": {name.strip("()"): {"avg_ms": round(ms / n, 4), "launches_per_step": n // args.steps}
                    for name, (ms, n) in rprof.items()}}

    # The same forward in the recurrent (token-serial) form, the baseline the paper times the chunkwise
    # form against; vector-ALU bound: 3 fused multiply-adds per state element per token.
    rec_steps = max(1, min(args.steps, 10))
    for _ in range(2):
        dn.deltanet_recurrent_fwd(q, k, v, beta, o=o, final_state=ST)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(rec_steps):
        dn.deltanet_recurrent_fwd(q, k, v, beta, o=o, final_state=ST)
    torch.cuda.synchronize()
    rec_ms = 1e3 * (time.perf_counter() - t0) / rec_steps
    t0 = time.perf_counter()
    for _ in range(rec_steps):
        dn.deltanet_fwd(q, k, v, beta, o=o, final_state=ST, workspace=ws)
    torch.cuda.synchronize()
    cfw = 1e3 * (time.perf_counter() - t0) / rec_steps
    rec_tflops = 6.0 * d * d * H * tokens / (rec_ms * 1e-3) / 1e12
    out["recurrent_fwd"] = {"ms": round(rec_ms, 4), "tokens_per_s": round(tokens / (rec_ms * 1e-3), 1), "steps": rec_steps,
                            "chunkwise_fwd_ms": round(cfw, 4), "chunkwise_speedup": round(rec_ms / cfw, 2),
                            "roofline": {"bound": "alu", "achieved": round(rec_tflops, 2), "peak": PEAK_FP32_VECTOR_TFLOPS,
                                         "unit": "TFLOP/s", "frac": round(rec_tflops / PEAK_FP32_VECTOR_TFLOPS, 4),
                                         "traffic": measured_traffic("k_recurrent_fwd")}}

    # The gated variant (scalar decay exp(g_t) on the transition) on the same workload: same kernels with
    # rescaled rows, plus the gate gradient.
    from paper_2406_06484_amd.binding import deltanet_gated_workspace_bytes
    from paper_2406_06484_amd.synth import make_gate
    g = torch.from_numpy(make_gate(2, (B, L, H), 0.9, 1.0)).to(dev)
    wsg = torch.empty(deltanet_gated_workspace_bytes(shp, True), dtype=torch.uint8, device=dev)

    def gated_step():
        dn.deltanet_gated_fwd_save(q, k, v, beta, g, o=o, final_state=ST, saved=wsg)
        return dn.deltanet_gated_bwd_saved(q, k, v, beta, g, d_o, wsg)
    for _ in range(args.warmup):
        gated_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        gated_step()
    torch.cuda.synchronize()
    gms = 1e3 * (time.perf_counter() - t0) / args.steps
    out["gated_fwd_bwd"] = {"ms": round(gms, 4), "tokens_per_s": round(tokens / (gms * 1e-3), 1), "steps": args.steps,
                            "vs_plain": round(gms / ms_per_step, 3)}

    # The same step with the layer's prologue fused into the load path (SiLU + L2 norm of q and k, sigmoid of the beta
    # logits, and the gradients through them in the store path), on pre-activations of the same shape.
    from paper_2406_06484_amd.synth import make_pre_activations
    pre = make_pre_activations(2, inp)
    qp, kp, bp = bf(pre.q), bf(pre.k), bf(pre.beta)

    from paper_2406_06484_amd.binding import deltanet_fused_workspace_bytes
    wsf = torch.empty(deltanet_fused_workspace_bytes(shp, True), dtype=torch.uint8, device=dev)

    def fused_step():
        dn.deltanet_fused_fwd_save(qp, kp, v, bp, o=o, final_state=ST, saved=wsf)
        return dn.deltanet_fused_bwd_saved(qp, kp, v, bp, d_o, wsf)
    for _ in range(args.warmup):
        fused_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        fused_step()
    torch.cuda.synchronize()
    fms = 1e3 * (time.perf_counter() - t0) / args.steps
    out["fused_prologue_fwd_bwd"] = {"ms": round(fms, 4), "tokens_per_s": round(tokens / (fms * 1e-3), 1), "steps": args.steps,
                                     "vs_plain": round(fms / ms_per_step, 3)}

    # The same number of tokens and the same model width at head size 256 (H / 2 heads): the scans own 32 state columns
    # per workgroup and the backward's chunk kernel streams S and dS' in column blocks.
    H2, d2 = max(1, H // 2), 2 * d
    gen = torch.Generator(device="cpu").manual_seed(7)
    unit2 = lambda: torch.nn.functional.normalize(torch.randn(B, L, H2, d2, generator=gen), dim=-1).bfloat16().to(dev)
    q2, k2 = unit2(), unit2()
    v2 = torch.randn(B, L, H2, d2, generator=gen).bfloat16().to(dev)
    do2 = torch.randn(B, L, H2, d2, generator=gen).bfloat16().to(dev)
    b2 = torch.sigmoid(torch.randn(B, L, H2, generator=gen)).bfloat16().to(dev)
    o2 = torch.empty_like(v2)
    _, _, ws2 = dn.deltanet_fwd_save(q2, k2, v2, b2, o=o2)

    def wide_step():
        dn.deltanet_fwd_save(q2, k2, v2, b2, o=o2, saved=ws2)
        return dn.deltanet_bwd_saved(q2, k2, v2, b2, do2, ws2)
    for _ in range(args.warmup):
        wide_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        wide_step()
    torch.cuda.synchronize()
    wms = 1e3 * (time.perf_counter() - t0) / args.steps
    out["head_size_256_fwd_bwd"] = {"ms": round(wms, 4), "tokens_per_s": round(tokens / (wms * 1e-3), 1), "steps": args.steps,
                                    "config": {"B": B, "L": L, "H": H2, "d_head": d2}, "vs_plain": round(wms / ms_per_step, 3)}
    del q2, k2, v2, do2, b2, o2, ws2

    if not args.no_cpu_baseline:
        import oracle
        nthr = oracle.max_threads()
        t0 = time.perf_counter()
        reps = 0
        while True:  # the whole workload through the fp64 oracle, repeated until >= 10 s of wall time
            oracle.fwd(inp.q, inp.k, inp.v, inp.beta)
            oracle.bwd(inp.q, inp.k, inp.v, inp.beta, inp.d_o)
            reps += 1
            if time.perf_counter() - t0 >= 10.0 or reps >= 12:
                break
        cdt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(tokens * reps / cdt, 1), "unit": "tokens/s", "cores": nthr, "kind": "oracle",
                               "sample": "the full workload (all %d chains x %d tokens), fwd+bwd, %d repetition(s), fp64, "
                                         "OpenMP over chains" % (B * H, L, reps)}
        # the same oracle on one core, on the first sequence of the batch (all heads)
        t0 = time.perf_counter()
        oracle.fwd(inp.q[:1], inp.k[:1], inp.v[:1], inp.beta[:1], nthreads=1)
        oracle.bwd(inp.q[:1], inp.k[:1], inp.v[:1], inp.beta[:1], inp.d_o[:1], nthreads=1)
        c1 = time.perf_counter() - t0
        out["cpu_baseline_one_core"] = {"value": round(L / c1, 1), "unit": "tokens/s", "cores": 1, "kind": "oracle",
                                        "sample": "the first sequence of the batch (%d chains x %d tokens), fwd+bwd, once" % (H, L)}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
