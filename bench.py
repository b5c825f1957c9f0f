#!/usr/bin/env python3
"""Benchmark of the DeltaNet layer hot path on one MI355X.

A "step" is one forward plus one backward pass of the layer over one batch of synthetic input shaped
like the paper's 1.3B-model layers: bf16, B=8, L=2048, H=16, d_k=d_v=128, chunk 64, through the C ABI
as a training step calls it: deltanet_fwd_save, which leaves its per-chunk tiles in a buffer, then
deltanet_bwd_saved, which reads them instead of recomputing them.  The self-contained pair
(deltanet_fwd + deltanet_bwd, backward recomputes everything from the inputs) is timed beside it and
reported as "recompute_fwd_bwd".  Inputs, outputs and the buffer are resident in HBM before the timed
region and the step allocates nothing.  Prints ONE JSON line: tokens/s of the layer (B*L tokens per
step), the dominant kernel's roofline position (per-kernel time from HIP events recorded by the
library on the launch stream), and the fp64 CPU oracle timed on the host cores as a reported baseline.

--mode headline runs only the step and the self-contained pair (the run the rocprofv3 summaries under
profiles/ are taken from); --mode streamed the same under DN_OPT_STREAMED_CHUNK_KERNEL.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
PEAK_FP32_VECTOR_TFLOPS = 157.3  # published fp32 vector rate (counts packed FMA; plain FMA code reaches half)
C = 64
PRECONDITION_STEPS = 150    # untimed steps ahead of the warm-up, to bring the chip to its steady clocks
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_cfg2_fwd_bwd.txt")


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
    if "k_bwd_stream" in name:
        # K S, K dS', dO S^T, Ut dS'^T, dV S^T (5 x 2Cd^2); T R, P^T dO, X^T dUt, dO Ut^T, dUt R^T, Q K^T, dP K, dP^T Q,
        # K K^T, Ah K, Ah^T K (11 x 2C^2 d); dX X^T, X^T M1 (2 x 2C^3)
        return 10 * c * d * d + 22 * c * c * d + 4 * c ** 3
    if "k_bwd_chunk" in name:
        # adjoint of Eq. 8-9: dO S^T, dUt S^T, Ut dS^T (3 x 2Cd^2); dO Ut^T, dP K, dP^T Q (3 x 2C^2 d)
        # adjoint of Eq. 10-11: K K^T, dW K^T, dU V^T, X^T dW, X^T dU, Ah K, Ah^T K (7 x 2C^2 d);
        #                       dX X^T, X^T M1 (2 x 2C^3); forward substitution (2/3 C^3)
        return 6 * c * d * d + 20 * c * c * d + 4 * c ** 3 + (2.0 / 3.0) * c ** 3
    return 0.0


def kernel_bytes_per_chunk_head(name: str, d: int, c: int = C, es: int = 2) -> float:
    """Operand bytes one (chunk, head) costs in each kernel: every tile it must read or write, once, the intermediates
    that cross kernels included (this is what the kernel as decomposed has to move, not what the method has to).

    tile = C x d elements, cc = C x C, st = d x d (states leave the scans in the element type)."""
    tile, cc, st, beta = c * d * es, c * c * es, d * d * es, c * es
    if "k_wy_prep" in name:      # K, beta -> T, X
        return tile + beta + 2 * cc
    if "k_scan_fwd_save" in name:  # Q, K, V, T -> O, Ut, S
        return 3 * tile + cc + 2 * tile + st
    if "k_scan_bwd" in name:     # Q, K, dO, T -> dUt, dS'
        return 3 * tile + cc + tile + st
    if "k_scan_pair" in name:    # K, V, T -> Ut, S   and   Q, K, dO, T -> dUt, dS'
        return (2 * tile + cc + tile + st) + (3 * tile + cc + tile + st)
    if "k_scan_fwd" in name:     # Q, K, V, T -> O
        return 3 * tile + cc + tile
    if "k_bwd_stream" in name:   # dO, K, Q, V, S, dS', X, beta -> dQ, dK, dV, dbeta
        return 4 * tile + 2 * st + cc + beta + 3 * tile + c * 4
    if "k_bwd_chunk" in name:    # dO, Ut, dUt, K, Q, V, S, dS', X, beta -> dQ, dK, dV, dbeta
        return 6 * tile + 2 * st + cc + beta + 3 * tile + c * 4
    return 0.0


def kernel_algorithmic_bytes_per_token_head(name: str, d: int, es: int = 2) -> float:
    """What the METHOD obliges a kernel to move per token and head: the layer's own tensors it reads and writes, once
    (forward: q, k, v, beta in, o out = 1026 B at d = 128 in bf16; backward: q, k, v, beta, do in, dq, dk, dv, dbeta out =
    1798 B).  Intermediates that cross kernels (T, X, Ut, dUt, the chunk states) count for nothing here: they are the
    price of the decomposition, and the roofline fraction reported against these bytes shows that price."""
    row, b_in, b_out = d * es, es, 4
    if "k_wy_prep" in name:                          # k, beta
        return row + b_in
    if "k_scan_fwd" in name:                         # the forward pass: q, k, v, beta -> o
        return 3 * row + b_in + row
    if "k_scan_bwd" in name:                         # q, k, do
        return 3 * row
    if "k_scan_pair" in name:                        # q, k, do and (recompute) k, v
        return 5 * row
    if "k_bwd_chunk" in name or "k_bwd_stream" in name:   # the backward pass: q, k, v, beta, do -> dq, dk, dv, dbeta
        return 4 * row + b_in + 3 * row + b_out
    return 0.0


def read_measured_traffic(path: str = TRAFFIC_FILE) -> dict:
    """{kernel name as in the summary: HBM bytes per launch} from the lines `traffic_bytes <kernel> <bytes>` of the
    rocprofv3 summary under profiles/ (written by profile_summary.py from the counter runs); {} if there is none."""
    out = {}
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 3 and parts[0] == "traffic_bytes":
                    out[parts[1]] = float(parts[2])
    except OSError:
        pass
    return out


def measured_traffic(name: str, table: dict | None = None):
    """bytes per launch of the kernel whose name (template arguments dropped) is `name`, or None"""
    table = read_measured_traffic() if table is None else table
    return table.get(name.split("<")[0].strip("()"))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mode", choices=("full", "headline", "streamed"), default="full",
                    help="headline: only the step and the self-contained pair; streamed: the same under DN_OPT_STREAMED_CHUNK_KERNEL")
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
    grads = dict(dq=torch.empty_like(q), dk=torch.empty_like(k), dv=torch.empty_like(v),
                 dbeta=torch.empty(beta.shape, dtype=torch.float32, device=dev), dinitial_state=torch.empty_like(ST))

    def step():   # the training step: the forward pass leaves its per-chunk tiles in ws for the backward pass
        dn.deltanet_fwd_save(q, k, v, beta, o=o, final_state=ST, saved=ws)
        return dn.deltanet_bwd_saved(q, k, v, beta, d_o, ws, **grads)

    def recompute_step():   # the self-contained pair: nothing is kept between the two calls
        dn.deltanet_fwd(q, k, v, beta, o=o, final_state=ST, workspace=ws)
        return dn.deltanet_bwd(q, k, v, beta, d_o, workspace=ws, **grads)

    def wall_ms(f, steps, warmup):
        for _ in range(warmup):
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            f()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t0) / steps

    def profile(f, steps):   # per-kernel device time from the library's own HIP events on the launch stream
        dn.deltanet_profile_enable(True)
        for _ in range(steps):
            f()
        torch.cuda.synchronize()
        prof = dn.deltanet_profile_collect()
        dn.deltanet_profile_enable(False)
        return {name.strip("()"): (ms, n) for name, (ms, n) in prof.items()}

    if args.mode == "streamed":
        dn.deltanet_set_option(dn.DN_OPT_STREAMED_CHUNK_KERNEL, 1)
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
    # The chip takes some tens of milliseconds of work to reach its steady clocks after the set-up above (the first steps
    # of a fresh process run ~10 % slower); a training job lives in the steady state, so the chip is brought there first.
    # These steps are neither the warm-up the caller asked for nor timed.
    for _ in range(PRECONDITION_STEPS):
        step()
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

    # every step between its own pair of events (they sit on the launch stream, torch's current one): median, and the
    # forward / backward split (untimed for `value`)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for e in ev:
        e[0].record(); dn.deltanet_fwd_save(q, k, v, beta, o=o, final_state=ST, saved=ws)
        e[1].record(); dn.deltanet_bwd_saved(q, k, v, beta, d_o, ws, **grads)
        e[2].record()
    torch.cuda.synchronize()
    step_ms = [e[0].elapsed_time(e[2]) for e in ev]
    fw = statistics.median(e[0].elapsed_time(e[1]) for e in ev)
    bw = statistics.median(e[1].elapsed_time(e[2]) for e in ev)

    prof = profile(step, args.steps)
    chunk_heads = B * H * (L // C)
    token_heads = B * H * L
    traffic_table = read_measured_traffic()
    kernels = {}
    for nm, (ms, n) in prof.items():
        avg = ms / n
        fl = kernel_flops_per_chunk_head(nm, d) * chunk_heads
        by = kernel_bytes_per_chunk_head(nm, d) * chunk_heads
        al = kernel_algorithmic_bytes_per_token_head(nm, d) * token_heads
        kernels[nm] = {"avg_ms": round(avg, 4), "launches_per_step": n // args.steps,
                       "tflops": round(fl / (avg * 1e-3) / 1e12, 2),
                       "algorithmic_gbs": round(al / (avg * 1e-3) / 1e9, 1),
                       "operand_gbs": round(by / (avg * 1e-3) / 1e9, 1),
                       "measured_bytes": measured_traffic(nm, traffic_table)}
    kernel_sum = sum(k_["avg_ms"] * k_["launches_per_step"] for k_ in kernels.values())
    dom = max(kernels, key=lambda n: kernels[n]["avg_ms"] * kernels[n]["launches_per_step"])
    fwd_f, bwd_f = model_flops_per_token_head(d)
    model_tflops = (fwd_f + bwd_f) * H * value / 1e12
    # The dominant kernel against the HBM roof.  `achieved` counts the ALGORITHMIC bytes of what the kernel is for (the
    # layer's own tensors, once); the bytes the kernel really has to move as the pass is decomposed (intermediates
    # included) are under `operand_model`, the rocprofv3 counter bytes under `traffic`.  The same kernel against the
    # bf16 MFMA roof rides along.
    dom_alg = kernel_algorithmic_bytes_per_token_head(dom, d) * token_heads
    dom_opd = kernel_bytes_per_chunk_head(dom, d) * chunk_heads
    dom_s = kernels[dom]["avg_ms"] * 1e-3
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(dom_alg / dom_s / 1e9, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(dom_alg / dom_s / 1e9 / PEAK_HBM_GBS, 4), "traffic": measured_traffic(dom, traffic_table),
                "algorithmic_bytes": dom_alg,
                "operand_model": {"bytes": dom_opd, "gbs": round(dom_opd / dom_s / 1e9, 1),
                                  "frac": round(dom_opd / dom_s / 1e9 / PEAK_HBM_GBS, 4)},
                "mfma": {"achieved": kernels[dom]["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(kernels[dom]["tflops"] / PEAK_BF16_TFLOPS, 4)}}
    step_measured = [k_["measured_bytes"] for k_ in kernels.values()]
    step_measured_bytes = (sum(m * k_["launches_per_step"] for m, k_ in zip(step_measured, kernels.values()))
                           if all(m is not None for m in step_measured) else None)

    out = {
        "metric": "DeltaNet layer fwd+bwd tokens/s at H=16,d=128,L=2048; % bf16 MFMA peak",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "precondition_steps": PRECONDITION_STEPS,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[2]: bf16 fwd+bwd, B=8, L=2048, H=16, d_k=d_v=128, chunk=64; the forward pass keeps its per-chunk tiles for the backward pass"
                               + ("; option DN_OPT_STREAMED_CHUNK_KERNEL" if args.mode == "streamed" else ""),
                   "tokens_per_step": tokens},
        "ms_per_step_median_of_events": round(statistics.median(step_ms), 4),
        "fwd_ms": round(fw, 4), "bwd_ms": round(bw, 4),
        "kernel_sum_ms": round(kernel_sum, 4), "non_kernel_ms": round(ms_per_step - kernel_sum, 4),
        "model_tflops": round(model_tflops, 2),
        "pct_bf16_mfma_peak": round(100 * model_tflops / PEAK_BF16_TFLOPS, 3),
        # the same with the masked halves of the C x C tiles not counted (forward 6d^2 + 5Cd + 2/3 C^2), and with the FLOPs a
        # backward pass that recomputes the chunk states adds (4d^2 + 8Cd + 2/3 C^2; this step keeps them, so nothing is added)
        "pct_bf16_mfma_peak_triangle_aware": round(100 * (model_tflops - 5 * C * d * H * value / 1e12) / PEAK_BF16_TFLOPS, 3),
        "recompute_extra_flops_per_token_head": 4 * d * d + 8 * C * d + (2.0 / 3.0) * C * C,
        "algorithmic_hbm_gbs": round((1026 + 1798) * H * value / 1e9, 1),
        # rocprofv3 counter bytes of the step's launches (profiles/hbm_traffic_cfg2_fwd_bwd.txt) over this run's step time
        "measured_hbm_bytes_per_step": step_measured_bytes,
        "measured_hbm_gbs": None if step_measured_bytes is None else round(step_measured_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "kernels": kernels,
        "roofline": roofline,
    }

    # The self-contained pair on the same workload (the backward pass recomputes T, X, the chunk states and
    # Ut from the inputs, as the paper's implementation does), with its own per-kernel times.
    rms = wall_ms(recompute_step, args.steps, args.warmup)
    rprof = profile(recompute_step, args.steps)
    out["recompute_fwd_bwd"] = {
        "ms_per_step": round(rms, 4), "tokens_per_s": round(tokens / (rms * 1e-3), 1), "steps": args.steps,
        "kernels": {name: {"avg_ms": round(ms / n, 4), "launches_per_step": n // args.steps} for name, (ms, n) in rprof.items()}}
    if args.mode != "full":
        if args.mode == "streamed":
            dn.deltanet_set_option(dn.DN_OPT_STREAMED_CHUNK_KERNEL, 0)
        print(json.dumps(out))
        return 0

    # The same step with the chunk kernel that streams S and dS' in column blocks and rebuilds Ut, dUt on chip (the
    # scans then do not store them): fewer bytes, more barrier intervals.
    dn.deltanet_set_option(dn.DN_OPT_STREAMED_CHUNK_KERNEL, 1)
    sms = wall_ms(step, args.steps, args.warmup)
    sprof = profile(step, args.steps)
    dn.deltanet_set_option(dn.DN_OPT_STREAMED_CHUNK_KERNEL, 0)
    out["streamed_chunk_kernel_fwd_bwd"] = {
        "ms_per_step": round(sms, 4), "tokens_per_s": round(tokens / (sms * 1e-3), 1), "steps": args.steps, "vs_plain": round(sms / ms_per_step, 3),
        "kernels": {name: {"avg_ms": round(ms / n, 4), "launches_per_step": n // args.steps} for name, (ms, n) in sprof.items()}}

    # The same forward in the recurrent (token-serial) form, the baseline the paper times the chunkwise
    # form against; vector-ALU bound: 3 fused multiply-adds per state element per token.
    rec_steps = max(1, min(args.steps, 10))
    rec_ms = wall_ms(lambda: dn.deltanet_recurrent_fwd(q, k, v, beta, o=o, final_state=ST), rec_steps, 2)
    cfw = wall_ms(lambda: dn.deltanet_fwd(q, k, v, beta, o=o, final_state=ST, workspace=ws), rec_steps, 2)
    rec_tflops = 6.0 * d * d * H * tokens / (rec_ms * 1e-3) / 1e12
    out["recurrent_fwd"] = {"ms": round(rec_ms, 4), "tokens_per_s": round(tokens / (rec_ms * 1e-3), 1), "steps": rec_steps,
                            "chunkwise_fwd_ms": round(cfw, 4), "chunkwise_speedup": round(rec_ms / cfw, 2),
                            "roofline": {"bound": "alu", "achieved": round(rec_tflops, 2), "peak": PEAK_FP32_VECTOR_TFLOPS,
                                         "unit": "TFLOP/s", "frac": round(rec_tflops / PEAK_FP32_VECTOR_TFLOPS, 4),
                                         "traffic": measured_traffic("k_recurrent_fwd", traffic_table)}}

    # The gated variant (scalar decay exp(g_t) on the transition) on the same workload: same kernels with
    # rescaled rows, plus the gate gradient.
    from paper_2406_06484_amd.binding import deltanet_gated_workspace_bytes
    from paper_2406_06484_amd.synth import make_gate
    g = torch.from_numpy(make_gate(2, (B, L, H), 0.9, 1.0)).to(dev)
    wsg = torch.empty(deltanet_gated_workspace_bytes(shp, True), dtype=torch.uint8, device=dev)
    dg = torch.empty_like(g)

    def gated_step():
        dn.deltanet_gated_fwd_save(q, k, v, beta, g, o=o, final_state=ST, saved=wsg)
        return dn.deltanet_gated_bwd_saved(q, k, v, beta, g, d_o, wsg, dg=dg, **grads)
    gms = wall_ms(gated_step, args.steps, args.warmup)
    out["gated_fwd_bwd"] = {"ms": round(gms, 4), "tokens_per_s": round(tokens / (gms * 1e-3), 1), "steps": args.steps,
                            "vs_plain": round(gms / ms_per_step, 3)}
    del wsg

    # The same step with the layer's prologue fused into the load path (SiLU + L2 norm of q and k, sigmoid of the beta
    # logits, and the gradients through them in the store path), on pre-activations of the same shape.
    from paper_2406_06484_amd.synth import make_pre_activations
    pre = make_pre_activations(2, inp)
    qp, kp, bp = bf(pre.q), bf(pre.k), bf(pre.beta)

    from paper_2406_06484_amd.binding import deltanet_fused_workspace_bytes
    wsf = torch.empty(deltanet_fused_workspace_bytes(shp, True), dtype=torch.uint8, device=dev)

    def fused_step():
        dn.deltanet_fused_fwd_save(qp, kp, v, bp, o=o, final_state=ST, saved=wsf)
        return dn.deltanet_fused_bwd_saved(qp, kp, v, bp, d_o, wsf, **grads)
    fms = wall_ms(fused_step, args.steps, args.warmup)
    out["fused_prologue_fwd_bwd"] = {"ms": round(fms, 4), "tokens_per_s": round(tokens / (fms * 1e-3), 1), "steps": args.steps,
                                     "vs_plain": round(fms / ms_per_step, 3)}
    del wsf, qp, kp, bp

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
    wms = wall_ms(wide_step, args.steps, args.warmup)
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
