"""fp64 oracle of the layer's prologue in front of the delta rule: the query/key feature map and
normalisation of section 3.3 ("Feature map and normalization": q = SiLU(x) / ||SiLU(x)||_2 per token
and head, same for k) and the writing strength beta = sigmoid(b) of section 2.2, composed with the
token-level recurrence of this package, and the gradient of the composition by the chain rule.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Plain numpy in fp64.  The paper gives no
epsilon for the norm; a row whose SiLU image is exactly zero maps to zero (reading listed in the
design notes), every other row is divided by its exact norm.
"""
from __future__ import annotations

import numpy as np


def sigmoid(x):
    x = np.asarray(x, dtype=np.float64)
    return 1.0 / (1.0 + np.exp(-x))


def silu(x):
    x = np.asarray(x, dtype=np.float64)
    return x * sigmoid(x)


def feature_map(x):
    """Rows (last axis) of SiLU(x) divided by their Euclidean norm."""
    s = silu(x)
    n = np.sqrt(np.sum(s * s, axis=-1, keepdims=True))
    return np.divide(s, n, out=np.zeros_like(s), where=n > 0)


def feature_map_bwd(x, dy):
    """Gradient w.r.t. x of sum(feature_map(x) * dy).

    y = s / n with s = SiLU(x), n = ||s||:  ds = (dy - y (y . dy)) / n;  SiLU'(x) = sig (1 + x (1 - sig))."""
    x = np.asarray(x, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    sg = sigmoid(x)
    s = x * sg
    n = np.sqrt(np.sum(s * s, axis=-1, keepdims=True))
    y = np.divide(s, n, out=np.zeros_like(s), where=n > 0)
    ds = dy - y * np.sum(y * dy, axis=-1, keepdims=True)
    ds = np.divide(ds, n, out=np.zeros_like(ds), where=n > 0)
    return ds * sg * (1.0 + x * (1.0 - sg))


def fused_fwd(q_pre, k_pre, v, beta_logit, initial_state=None, cu_seqlens=None):
    """(o, final_state) of the delta rule on q = feature_map(q_pre), k = feature_map(k_pre), beta = sigmoid(beta_logit)."""
    import oracle
    return oracle.fwd(feature_map(q_pre), feature_map(k_pre), v, sigmoid(beta_logit), initial_state, cu_seqlens)


def fused_bwd(q_pre, k_pre, v, beta_logit, d_o, initial_state=None, dfinal_state=None, cu_seqlens=None):
    """(dq_pre, dk_pre, dv, dbeta_logit, dinitial_state) of the same composition."""
    import oracle
    beta = sigmoid(beta_logit)
    dq, dk, dv, dbeta, dS0 = oracle.bwd(feature_map(q_pre), feature_map(k_pre), v, beta, d_o, initial_state,
                                        dfinal_state, cu_seqlens)
    return (feature_map_bwd(q_pre, dq), feature_map_bwd(k_pre, dk), dv, dbeta * beta * (1.0 - beta), dS0)
