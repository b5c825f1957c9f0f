"""Pins for the gated recurrence of the oracle (the "Gated DeltaNet" row of the paper's overview table,
S_t = S_{t-1} alpha_t (I - beta_t k_t k_t^T) + beta_t v_t k_t^T with alpha_t = exp(g_t)): special cases
with closed forms, the reduction to the plain delta rule, finite differences, and the two identities
the GPU path builds on (rescaling to the plain rule, and the gate gradient as a suffix sum)."""
import numpy as np
import pytest

import oracle


def rand_inputs(seed, B=2, L=11, H=2, dk=6, dv=5, gate_scale=1.0):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, L, H, dk))
    k = rng.standard_normal((B, L, H, dk)); k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = rng.standard_normal((B, L, H, dv))
    beta = rng.uniform(0.05, 0.95, (B, L, H))
    g = -gate_scale * rng.uniform(0.0, 1.0, (B, L, H))
    S0 = rng.standard_normal((B, H, dk, dv))
    return q, k, v, beta, g, S0


def test_zero_gate_is_the_plain_delta_rule_bitwise():
    q, k, v, beta, g, S0 = rand_inputs(1)
    o0, ST0 = oracle.fwd(q, k, v, beta, S0)
    o1, ST1 = oracle.gated_fwd(q, k, v, beta, np.zeros_like(g), S0)
    assert np.array_equal(o0, o1) and np.array_equal(ST0, ST1)
    do = np.ones_like(o0)
    a = oracle.bwd(q, k, v, beta, do, S0)
    b = oracle.gated_bwd(q, k, v, beta, np.zeros_like(g), do, S0)
    for x, y in zip(a, (b[0], b[1], b[2], b[3], b[5])):
        assert np.allclose(x, y, rtol=1e-13, atol=1e-13)


def test_beta_zero_is_pure_decay():
    # nothing is written: S_t = (prod_{i<=t} alpha_i) S_0 and o_t = S_t^T q_t
    q, k, v, beta, g, S0 = rand_inputs(2)
    o, ST = oracle.gated_fwd(q, k, v, np.zeros_like(beta), g, S0)
    gam = np.exp(np.cumsum(g, axis=1))                      # [B, L, H]
    assert np.allclose(ST, gam[:, -1][:, :, None, None] * S0, rtol=1e-13, atol=1e-13)
    want = np.einsum("blh,bhkv,blhk->blhv", gam, S0, q)
    assert np.allclose(o, want, rtol=1e-12, atol=1e-12)


def test_single_token_closed_form():
    # S_1 = alpha (I - beta k k^T) S_0 + beta k v^T in the listing orientation
    q, k, v, beta, g, S0 = rand_inputs(3, B=1, L=1, H=1)
    o, ST = oracle.gated_fwd(q, k, v, beta, g, S0)
    kk, vv, b, a = k[0, 0, 0], v[0, 0, 0], beta[0, 0, 0], np.exp(g[0, 0, 0])
    S1 = a * (np.eye(len(kk)) - b * np.outer(kk, kk)) @ S0[0, 0] + b * np.outer(kk, vv)
    assert np.allclose(ST[0, 0], S1, rtol=1e-13, atol=1e-13)
    assert np.allclose(o[0, 0, 0], S1.T @ q[0, 0, 0], rtol=1e-13, atol=1e-13)


def test_rescaling_to_the_plain_rule():
    # With gamma_t = prod_{i<=t} alpha_i: S_t / gamma_t follows the plain delta rule on values v_t / gamma_t,
    # so o_t = gamma_t * o~_t and S_L = gamma_L * S~_L.  (The chunkwise kernels use this per chunk.)
    q, k, v, beta, g, S0 = rand_inputs(4)
    gam = np.exp(np.cumsum(g, axis=1))
    o, ST = oracle.gated_fwd(q, k, v, beta, g, S0)
    ot, STt = oracle.fwd(q, k, v / gam[..., None], beta, S0)
    assert np.allclose(o, gam[..., None] * ot, rtol=1e-11, atol=1e-11)
    assert np.allclose(ST, gam[:, -1][:, :, None, None] * STt, rtol=1e-11, atol=1e-11)


@pytest.mark.parametrize("seed", [5, 6])
def test_gradients_by_central_differences(seed):
    q, k, v, beta, g, S0 = rand_inputs(seed, B=1, L=6, H=2, dk=4, dv=3)
    rng = np.random.default_rng(100 + seed)
    o, ST = oracle.gated_fwd(q, k, v, beta, g, S0)
    do, dST = rng.standard_normal(o.shape), rng.standard_normal(ST.shape)
    grads = oracle.gated_bwd(q, k, v, beta, g, do, S0, dST)
    args = [q, k, v, beta, g, S0]

    def loss():
        oo, SS = oracle.gated_fwd(*args)
        return (oo * do).sum() + (SS * dST).sum()
    order = {0: 0, 1: 1, 2: 2, 3: 3, 4: 4, 5: 5}  # positions of dq, dk, dv, dbeta, dg, dS0 in the result
    for idx, x in enumerate(args):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            mi = it.multi_index
            old = x[mi]
            x[mi] = old + 1e-6; lp = loss()
            x[mi] = old - 1e-6; lm = loss()
            x[mi] = old
            num[mi] = (lp - lm) / 2e-6
        assert np.max(np.abs(num - grads[order[idx]])) <= 1e-7 * max(1.0, np.max(np.abs(num))), idx


def test_gate_gradient_is_a_suffix_sum():
    # dg_t = <dS_L, S_L> + sum_{i >= t} (q_i . dq_i - v_i . dv_i): o_t is linear in q_t and S_t, so the
    # sensitivity to a rescaling of the state at time t can be read off the other gradients.
    q, k, v, beta, g, S0 = rand_inputs(7, B=2, L=40, H=3, dk=8, dv=6)
    rng = np.random.default_rng(70)
    o, ST = oracle.gated_fwd(q, k, v, beta, g, S0)
    do, dST = rng.standard_normal(o.shape), rng.standard_normal(ST.shape)
    dq, dk, dv, dbeta, dg, dS0 = oracle.gated_bwd(q, k, v, beta, g, do, S0, dST)
    c = (q * dq).sum(-1) - (v * dv).sum(-1)                          # [B, L, H]
    suffix = np.flip(np.cumsum(np.flip(c, axis=1), axis=1), axis=1)
    want = suffix + (dST * ST).sum(axis=(-1, -2))[:, None, :]
    assert np.allclose(dg, want, rtol=1e-10, atol=1e-10)


def test_adjoint_identity_mid_size():
    q, k, v, beta, g, S0 = rand_inputs(8, B=2, L=70, H=2, dk=16, dv=12, gate_scale=0.2)
    rng = np.random.default_rng(80)
    o, ST = oracle.gated_fwd(q, k, v, beta, g, S0)
    do, dST = rng.standard_normal(o.shape), rng.standard_normal(ST.shape)
    grads = oracle.gated_bwd(q, k, v, beta, g, do, S0, dST)
    args = [q, k, v, beta, g, S0]
    dirs = [rng.standard_normal(x.shape) for x in args]
    h = 1e-6
    op, Sp = oracle.gated_fwd(*[x + h * d for x, d in zip(args, dirs)])
    om, Sm = oracle.gated_fwd(*[x - h * d for x, d in zip(args, dirs)])
    lhs = ((op - om) * do).sum() / (2 * h) + ((Sp - Sm) * dST).sum() / (2 * h)
    rhs = sum((gr * d).sum() for gr, d in zip(grads, dirs))
    assert abs(lhs - rhs) <= 1e-6 * max(1.0, abs(lhs))


def test_chaining_and_packed_equal_separate_calls():
    q, k, v, beta, g, S0 = rand_inputs(9, B=1, L=30, H=2)
    o, ST = oracle.gated_fwd(q, k, v, beta, g, S0)
    o1, S1 = oracle.gated_fwd(q[:, :13], k[:, :13], v[:, :13], beta[:, :13], g[:, :13], S0)
    o2, S2 = oracle.gated_fwd(q[:, 13:], k[:, 13:], v[:, 13:], beta[:, 13:], g[:, 13:], S1)
    assert np.allclose(np.concatenate([o1, o2], axis=1), o, rtol=1e-13, atol=1e-13) and np.allclose(S2, ST, rtol=1e-13, atol=1e-13)
    cu = np.array([0, 13, 13, 30], dtype=np.int32)
    S0p = np.concatenate([S0, S0, S0], axis=0)
    op, STp = oracle.gated_fwd(q[0], k[0], v[0], beta[0], g[0], S0p, cu)
    oa, Sa = oracle.gated_fwd(q[:, :13], k[:, :13], v[:, :13], beta[:, :13], g[:, :13], S0)
    ob, Sb = oracle.gated_fwd(q[:, 13:], k[:, 13:], v[:, 13:], beta[:, 13:], g[:, 13:], S0)
    assert np.allclose(op[:13], oa[0]) and np.allclose(op[13:], ob[0])
    assert np.allclose(STp[0], Sa[0]) and np.allclose(STp[1], S0[0]) and np.allclose(STp[2], Sb[0])
