"""Independent numpy write-ups of the paper's OTHER formulations of DeltaNet, used only as pins for
the fp64 oracle (which is the plain per-token recurrence) and to check the chunkwise backward
algebra on the CPU.  Single chain, fp64, state orientation [d_k, d_v] as in the pseudocode listing.
Nothing here is imported by the oracle or by the product.
"""
import numpy as np


def pseudo_values(k, v, beta):
    """Eq. 3: u_t = beta_t (v_t - sum_{i<t} u_i (k_i . k_t)); S_t = sum_i k_i u_i^T (transposed)."""
    L = k.shape[0]
    u = np.zeros_like(v)
    for t in range(L):
        u[t] = beta[t] * (v[t] - (u[:t] * (k[:t] @ k[t])[:, None]).sum(0))
    return u


def wy_w(k, beta):
    """Eq. 7: w_t = beta_t (k_t - sum_{i<t} w_i (k_i . k_t)); prod_t (I - beta k k^T) = I - sum w k^T."""
    L = k.shape[0]
    w = np.zeros_like(k)
    for t in range(L):
        w[t] = beta[t] * (k[t] - (w[:t] * (k[:t] @ k[t])[:, None]).sum(0))
    return w


def ut_transform(k, beta):
    """Eq. 10: T = (I + tril(diag(beta) K K^T, -1))^{-1} diag(beta), with a library inverse."""
    C = k.shape[0]
    A = np.tril((beta[:, None] * k) @ k.T, -1)
    return np.linalg.inv(np.eye(C) + A) @ np.diag(beta)


def chunkwise_forward(q, k, v, beta, C, S0=None):
    """Eq. 8-11 with the state stored [d_k, d_v]; L must be a multiple of C."""
    L, dk = q.shape
    dv = v.shape[1]
    S = np.zeros((dk, dv)) if S0 is None else S0.copy()
    o = np.zeros((L, dv))
    for c0 in range(0, L, C):
        sl = slice(c0, c0 + C)
        T = ut_transform(k[sl], beta[sl])
        W, U = T @ k[sl], T @ v[sl]                      # Eq. 11
        Ut = U - W @ S                                   # inner term of Eq. 8-9
        o[sl] = q[sl] @ S + np.tril(q[sl] @ k[sl].T) @ Ut  # Eq. 9
        S = S + k[sl].T @ Ut                             # Eq. 8
    return o, S


def parallel_form(q, k, v, beta):
    """Fully parallel form (end of section 3.2): O = (Q K^T o M) T V with T over the whole sequence."""
    T = ut_transform(k, beta)
    return np.tril(q @ k.T) @ T @ v


def chunkwise_backward(q, k, v, beta, d_o, C, S0=None, dST=None):
    """Adjoint of chunkwise_forward, chunk by chunk (the algebra the GPU kernels implement)."""
    L, dk = q.shape
    dv = v.shape[1]
    nc = L // C
    S = np.zeros((dk, dv)) if S0 is None else S0.copy()
    states = []
    for c in range(nc):
        sl = slice(c * C, (c + 1) * C)
        states.append(S.copy())
        T = ut_transform(k[sl], beta[sl])
        S = S + k[sl].T @ (T @ v[sl] - T @ k[sl] @ S)
    dS = np.zeros((dk, dv)) if dST is None else dST.copy()
    dq, dk_, dv_, db = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v), np.zeros(L)
    I = np.eye(C)
    for c in reversed(range(nc)):
        sl = slice(c * C, (c + 1) * C)
        Q, K, V, b, dO, S = q[sl], k[sl], v[sl], beta[sl], d_o[sl], states[c]
        Kb, Vb = b[:, None] * K, b[:, None] * V
        X = np.linalg.inv(I + np.tril(Kb @ K.T, -1))
        W, U = X @ Kb, X @ Vb
        Ut = U - W @ S
        P = np.tril(Q @ K.T)
        dUt = P.T @ dO + K @ dS
        dP = np.tril(dO @ Ut.T)
        dq[sl] = dO @ S.T + dP @ K
        dK = dP.T @ Q + Ut @ dS.T
        dS_prev = dS + Q.T @ dO - W.T @ dUt
        dW = -dUt @ S.T
        dX = dW @ Kb.T + dUt @ Vb.T
        dKb, dVb = X.T @ dW, X.T @ dUt
        dA = -np.tril(X.T @ dX @ X.T, -1)
        dKb = dKb + dA @ K
        dK = dK + dA.T @ Kb + b[:, None] * dKb
        db[sl] = (dKb * K).sum(1) + (dVb * V).sum(1)
        dv_[sl] = b[:, None] * dVb
        dk_[sl] = dK
        dS = dS_prev
    return dq, dk_, dv_, db, dS
