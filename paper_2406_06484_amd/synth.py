"""Seeded synthetic inputs for the DeltaNet layer, shared by the tests, the smoke check and the benchmark.

This module holds none of the method's arithmetic: it only draws random tensors with the
structure the DeltaNet layer imposes on its operands (paper section 3.3: q and k are
L2-normalised per token; section 2.2: beta is a sigmoid, so it lies in (0,1)) and the shapes of
the paper's 1.3B-model layers (head dim 128, appendix A).  They stand in for real activations.

Draw order is fixed: q, k, v, beta-logits, do, S0, dS_final.  Everything is returned as float64
numpy arrays; in "bf16" mode the values are rounded to bf16 first, so that both the CPU oracle and
the GPU path consume exactly the same numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float values to the nearest bf16 (ties to even); returns float64 holding bf16 values."""
    f = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = ((u + 0x7FFF + lsb) >> 16) << 16
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(f.shape)


def round_to_f32(x: np.ndarray) -> np.ndarray:
    return np.asarray(x, dtype=np.float32).astype(np.float64)


@dataclass
class Inputs:
    q: np.ndarray            # [B,L,H,dk] or packed [T,H,dk]
    k: np.ndarray
    v: np.ndarray            # [.., dv]
    beta: np.ndarray         # [B,L,H] or [T,H]
    d_o: np.ndarray          # like v
    initial_state: Optional[np.ndarray]   # [N,H,dk,dv] float32-representable, or None
    dfinal_state: Optional[np.ndarray]
    cu_seqlens: Optional[np.ndarray]      # int32 [N+1] or None (dense)
    dtype: str               # "f32" or "bf16"
    meta: dict = field(default_factory=dict)


def draw_lengths(rng: np.random.Generator, total: int, lo: int, hi: int) -> np.ndarray:
    """Integer lengths uniform in [lo, hi], drawn in order until they cover `total`; the last one
    is cut so that the sum is exactly `total`.  Returns int32 cu_seqlens."""
    lens = []
    left = total
    while left > 0:
        n = int(rng.integers(lo, hi + 1))
        n = min(n, left)
        lens.append(n)
        left -= n
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)


def make_inputs(seed: int, *, B: int = 1, L: int = 0, H: int, dk: int, dv: int, dtype: str = "f32",
                with_initial_state: bool = False, with_dfinal_state: bool = False,
                cu_seqlens: Optional[np.ndarray] = None, varlen_total: int = 0,
                varlen_range=(128, 8192)) -> Inputs:
    rng = np.random.default_rng(seed)
    lead: tuple
    if varlen_total:
        cu = draw_lengths(np.random.default_rng(seed + 1_000_003), varlen_total, *varlen_range)
    else:
        cu = None if cu_seqlens is None else np.asarray(cu_seqlens, dtype=np.int32)
    if cu is not None:
        lead = (int(cu[-1]),)
        N = len(cu) - 1
    else:
        lead = (B, L)
        N = B
    rnd = round_to_bf16 if dtype == "bf16" else round_to_f32

    def unit_rows(shape):
        x = rng.standard_normal(shape)
        return x / np.linalg.norm(x, axis=-1, keepdims=True)

    q = rnd(unit_rows(lead + (H, dk)))
    k = rnd(unit_rows(lead + (H, dk)))
    v = rnd(rng.standard_normal(lead + (H, dv)))
    beta = rnd(1.0 / (1.0 + np.exp(-rng.standard_normal(lead + (H,)))))
    d_o = rnd(rng.standard_normal(lead + (H, dv)))
    S0 = round_to_f32(0.02 * rng.standard_normal((N, H, dk, dv))) if with_initial_state else None
    dST = round_to_f32(rng.standard_normal((N, H, dk, dv))) if with_dfinal_state else None
    return Inputs(q, k, v, beta, d_o, S0, dST, cu, dtype,
                  dict(seed=seed, B=B, L=L, H=H, dk=dk, dv=dv, N=N, tokens=int(np.prod(lead))))


# The five benchmark configurations (index = position in the benchmark's config list).
CONFIGS = {
    0: dict(seed=1, B=1, L=256, H=2, dk=64, dv=64, dtype="f32"),
    1: dict(seed=2, B=8, L=2048, H=16, dk=128, dv=128, dtype="bf16"),
    2: dict(seed=3, B=8, L=2048, H=16, dk=128, dv=128, dtype="bf16"),
    3: dict(seed=4, B=1, L=32768, H=16, dk=128, dv=128, dtype="bf16",
            with_initial_state=True, with_dfinal_state=True),
    4: dict(seed=5, H=16, dk=128, dv=128, dtype="bf16", varlen_total=65536, varlen_range=(128, 8192)),
}


def make_config(idx: int) -> Inputs:
    kw = dict(CONFIGS[idx])
    return make_inputs(kw.pop("seed"), **kw)


def make_gate(seed: int, shape, lo: float = 0.85, hi: float = 1.0) -> np.ndarray:
    """Log-decay g = log(alpha) of the gated variant, alpha ~ U(lo, hi) per token and head, as float32."""
    rng = np.random.default_rng(seed + 7_000_003)
    return np.log(rng.uniform(lo, hi, size=shape)).astype(np.float32)


def make_pre_activations(seed: int, inp: Inputs, scale: float = 1.0) -> Inputs:
    """The same batch with q, k replaced by pre-activations of the feature map (N(0, scale^2), what a
    projection followed by a short convolution hands over) and beta by logits (N(0, 1)), rounded to the
    batch's element type.  The values are drawn, nothing of the method is computed here."""
    rng = np.random.default_rng(seed + 9_000_011)
    rnd = round_to_bf16 if inp.dtype == "bf16" else round_to_f32
    q = rnd(scale * rng.standard_normal(inp.q.shape))
    k = rnd(scale * rng.standard_normal(inp.k.shape))
    b = rnd(rng.standard_normal(inp.beta.shape))
    return Inputs(q, k, inp.v, b, inp.d_o, inp.initial_state, inp.dfinal_state, inp.cu_seqlens, inp.dtype, dict(inp.meta))
