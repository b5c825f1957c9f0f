"""Pins for the fp64 oracle: things the paper and the mathematics fix, none of which is the oracle's
own formula retyped.  All CPU, all small."""
import os

import numpy as np
import pytest

import oracle
from tests import paper_forms as pf

RNG = np.random.default_rng(1234)


def chain(L, dk, dv, rng=RNG, unit=True, beta_range=(0.0, 1.0)):
    q = rng.standard_normal((1, L, 1, dk))
    k = rng.standard_normal((1, L, 1, dk))
    if unit:
        q /= np.linalg.norm(q, axis=-1, keepdims=True)
        k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = rng.standard_normal((1, L, 1, dv))
    beta = rng.uniform(*beta_range, size=(1, L, 1))
    return q, k, v, beta


def sq(x):  # [1,L,1,d] -> [L,d]
    return x[0, :, 0]


def test_golden_two_token_example():
    """Eq. 3 base case and inductive step, hand-computed (tests/golden/two_token_example.txt)."""
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "two_token_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, *nums = line.split()
            vals[name] = np.array([float(x) for x in nums])
    q = vals["q"].reshape(1, 2, 1, 2); k = vals["k"].reshape(1, 2, 1, 2)
    v = vals["v"].reshape(1, 2, 1, 2); beta = vals["beta"].reshape(1, 2, 1)
    o, S = oracle.fwd(q, k, v, beta)
    np.testing.assert_allclose(o.reshape(-1), vals["o"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(S.reshape(-1), vals["final_state"], rtol=0, atol=1e-14)


def test_one_step_is_sgd_on_regression_loss():
    """Section 2.2: S_t = S_{t-1} - beta * grad_S 0.5||S k - v||^2, gradient taken numerically."""
    dk, dv = 5, 3
    S0 = RNG.standard_normal((1, 1, dk, dv))
    q, k, v, beta = chain(1, dk, dv, unit=False)
    _, S1 = oracle.fwd(q, k, v, beta, initial_state=S0)
    loss = lambda S: 0.5 * np.sum((S.T @ k[0, 0, 0] - v[0, 0, 0]) ** 2)
    g = np.zeros((dk, dv)); h = 1e-6
    for i in range(dk):
        for j in range(dv):
            E = np.zeros((dk, dv)); E[i, j] = h
            g[i, j] = (loss(S0[0, 0] + E) - loss(S0[0, 0] - E)) / (2 * h)
    np.testing.assert_allclose(S1[0, 0], S0[0, 0] - beta[0, 0, 0] * g, atol=1e-8)


def test_remove_then_write_form():
    """Section 2.2: v_new = beta v + (1-beta) v_old; S_t = S_{t-1} - v_old k^T + v_new k^T."""
    dk, dv = 6, 4
    S0 = RNG.standard_normal((1, 1, dk, dv))
    q, k, v, beta = chain(1, dk, dv)
    o, S1 = oracle.fwd(q, k, v, beta, initial_state=S0)
    kk, vv, b = k[0, 0, 0], v[0, 0, 0], beta[0, 0, 0]
    v_old = S0[0, 0].T @ kk
    v_new = b * vv + (1 - b) * v_old
    ref = S0[0, 0] - np.outer(kk, v_old) + np.outer(kk, v_new)
    np.testing.assert_allclose(S1[0, 0], ref, atol=1e-13)
    np.testing.assert_allclose(o[0, 0, 0], ref.T @ q[0, 0, 0], atol=1e-13)  # read-out uses the UPDATED state


def test_beta_zero_leaves_state_unchanged():
    dk, dv, L = 7, 5, 9
    S0 = RNG.standard_normal((1, 1, dk, dv))
    q, k, v, _ = chain(L, dk, dv)
    o, S = oracle.fwd(q, k, v, np.zeros((1, L, 1)), initial_state=S0)
    assert np.array_equal(S, S0)  # bit-exact
    np.testing.assert_allclose(sq(o), sq(q) @ S0[0, 0], atol=1e-14)


def test_beta_one_onehot_keys_store_and_retrieve_exactly():
    """beta = 1 replaces the old value completely (section 2.2); with orthonormal keys every stored
    value is retrieved exactly and re-writing a key replaces its value."""
    d, dv = 8, 5
    perm = RNG.permutation(d)
    k = np.eye(d)[perm][None, :, None, :]
    v = RNG.standard_normal((1, d, 1, dv))
    o, S = oracle.fwd(k, k, v, np.ones((1, d, 1)))
    np.testing.assert_array_equal(S[0, 0], sq(k).T @ sq(v))
    np.testing.assert_array_equal(sq(o), sq(v))          # q_t = k_t reads back v_t
    np.testing.assert_array_equal(sq(k) @ S[0, 0], sq(v))  # every key still retrieves its value
    # overwrite key 0 with a new value
    k2 = np.concatenate([k, k[:, :1]], axis=1)
    v_new = RNG.standard_normal((1, 1, 1, dv))
    v2 = np.concatenate([v, v_new], axis=1)
    _, S2 = oracle.fwd(k2, k2, v2, np.ones((1, d + 1, 1)))
    np.testing.assert_allclose(sq(k)[0] @ S2[0, 0], v_new[0, 0, 0], atol=1e-15)
    np.testing.assert_allclose(sq(k)[1:] @ S2[0, 0], sq(v)[1:], atol=1e-15)


def test_beta_two_is_a_reflection():
    """Section 3.1 calls I - beta k k^T a generalized Householder matrix: beta = 2, ||k|| = 1 is a true
    reflection, so with v = 0 the state's Frobenius norm is preserved and S_L = (H_L ... H_1) S_0."""
    d, dv, L = 6, 4, 25
    S0 = RNG.standard_normal((1, 1, d, dv))
    q, k, _, _ = chain(L, d, dv)
    _, S = oracle.fwd(q, k, np.zeros((1, L, 1, dv)), 2 * np.ones((1, L, 1)), initial_state=S0)
    assert abs(np.linalg.norm(S) - np.linalg.norm(S0)) < 1e-12
    M = np.eye(d)
    for t in range(L):
        Hh = np.eye(d) - 2 * np.outer(sq(k)[t], sq(k)[t])
        np.testing.assert_allclose(Hh @ Hh.T, np.eye(d), atol=1e-14)
        M = Hh @ M
    np.testing.assert_allclose(S[0, 0], M @ S0[0, 0], atol=1e-12)


def test_transition_eigenstructure():
    """Section 3.3: I - beta k k^T has eigenvalue 1 - beta ||k||^2 on k and 1 on its complement;
    read off from the oracle by applying one step with v = 0 to S_0 = I."""
    d = 6
    _, k, _, _ = chain(1, d, d, unit=False)
    b = 0.7
    _, S = oracle.fwd(k, k, np.zeros((1, 1, 1, d)), np.full((1, 1, 1), b), initial_state=np.eye(d)[None, None])
    ev = np.sort(np.linalg.eigvalsh(S[0, 0]))
    kk = k[0, 0, 0]
    expect = np.sort(np.concatenate([[1 - b * kk @ kk], np.ones(d - 1)]))
    np.testing.assert_allclose(ev, expect, atol=1e-12)
    np.testing.assert_allclose(S[0, 0] @ kk, (1 - b * kk @ kk) * kk, atol=1e-12)


def test_wy_representation_of_P_and_S():
    """Eq. 6-7 / appendix B.1: prod (I - beta k k^T) = I - sum w k^T, and Eq. 3: S_n = sum u k^T."""
    d, dv, L = 7, 5, 12
    q, k, v, beta = chain(L, d, dv)
    # P: run the oracle with v = 0 from S_0 = I; in the listing's orientation S_L^T = P
    _, SP = oracle.fwd(q, k, np.zeros((1, L, 1, d)), beta, initial_state=np.eye(d)[None, None])
    w = pf.wy_w(sq(k), beta[0, :, 0])
    np.testing.assert_allclose(SP[0, 0].T, np.eye(d) - w.T @ sq(k), atol=1e-13)
    _, S = oracle.fwd(q, k, v, beta)
    u = pf.pseudo_values(sq(k), sq(v), beta[0, :, 0])
    np.testing.assert_allclose(S[0, 0], sq(k).T @ u, atol=1e-13)
    o, _ = oracle.fwd(q, k, v, beta)
    np.testing.assert_allclose(sq(o), np.tril(sq(q) @ sq(k).T) @ u, atol=1e-13)  # O = (QK^T o M) U


def test_ut_transform_closed_form_two_tokens():
    """Eq. 10 for C = 2: T = [[b1, 0], [-b1 b2 (k2.k1), b2]]."""
    _, k, _, _ = chain(2, 4, 4)
    b = np.array([0.3, 0.9])
    T = pf.ut_transform(sq(k), b)
    ref = np.array([[b[0], 0.0], [-b[0] * b[1] * (sq(k)[1] @ sq(k)[0]), b[1]]])
    np.testing.assert_allclose(T, ref, atol=1e-15)


@pytest.mark.parametrize("C", [1, 2, 4, 8, 16])
def test_chunkwise_form_equals_recurrence_for_any_chunk_size(C):
    """Eq. 8-11 vs the recurrence; d_k != d_v so a transposed state cannot hide; result independent of C."""
    L, dk, dv = 16, 6, 5
    q, k, v, beta = chain(L, dk, dv, rng=np.random.default_rng(7))
    S0 = np.random.default_rng(8).standard_normal((1, 1, dk, dv))
    o, S = oracle.fwd(q, k, v, beta, initial_state=S0)
    o_c, S_c = pf.chunkwise_forward(sq(q), sq(k), sq(v), beta[0, :, 0], C, S0[0, 0])
    np.testing.assert_allclose(sq(o), o_c, atol=1e-12)
    np.testing.assert_allclose(S[0, 0], S_c, atol=1e-12)


def test_fully_parallel_form():
    L, dk, dv = 12, 5, 7
    q, k, v, beta = chain(L, dk, dv)
    o, _ = oracle.fwd(q, k, v, beta)
    np.testing.assert_allclose(sq(o), pf.parallel_form(sq(q), sq(k), sq(v), beta[0, :, 0]), atol=1e-12)


def test_orthogonal_keys_reduce_to_linear_attention():
    """Mutually orthogonal keys: T = diag(beta), so O = tril(Q K^T) diag(beta) V - plain linear attention."""
    d, dv = 8, 6
    Qm, _ = np.linalg.qr(RNG.standard_normal((d, d)))
    k = Qm[None, :, None, :]
    q, _, v, beta = chain(d, d, dv)
    o, S = oracle.fwd(q, k, v, beta)
    np.testing.assert_allclose(sq(o), np.tril(sq(q) @ sq(k).T) @ (beta[0, :, 0, None] * sq(v)), atol=1e-13)
    np.testing.assert_allclose(S[0, 0], sq(k).T @ (beta[0, :, 0, None] * sq(v)), atol=1e-13)


def test_linearity_in_values_state_and_queries():
    L, dk, dv = 10, 5, 4
    q, k, v, beta = chain(L, dk, dv)
    q2, _, v2, _ = chain(L, dk, dv)
    S0a, S0b = RNG.standard_normal((2, 1, 1, dk, dv))
    a, b = 0.7, -1.3
    o1, S1 = oracle.fwd(q, k, v, beta, initial_state=S0a)
    o2, S2 = oracle.fwd(q, k, v2, beta, initial_state=S0b)
    o3, S3 = oracle.fwd(q, k, a * v + b * v2, beta, initial_state=a * S0a + b * S0b)
    np.testing.assert_allclose(o3, a * o1 + b * o2, atol=1e-12)
    np.testing.assert_allclose(S3, a * S1 + b * S2, atol=1e-12)
    o4, _ = oracle.fwd(q2, k, v, beta, initial_state=S0a)
    o5, _ = oracle.fwd(a * q + b * q2, k, v, beta, initial_state=S0a)
    np.testing.assert_allclose(o5, a * o1 + b * o4, atol=1e-12)


def test_state_chaining_and_packed_sequences():
    L, H, dk, dv = 37, 2, 6, 5
    rng = np.random.default_rng(5)
    q = rng.standard_normal((1, L, H, dk)); k = rng.standard_normal((1, L, H, dk)) / np.sqrt(dk)
    v = rng.standard_normal((1, L, H, dv)); beta = rng.uniform(size=(1, L, H))
    o, S = oracle.fwd(q, k, v, beta)
    t0 = 13
    o1, S1 = oracle.fwd(q[:, :t0], k[:, :t0], v[:, :t0], beta[:, :t0])
    o2, S2 = oracle.fwd(q[:, t0:], k[:, t0:], v[:, t0:], beta[:, t0:], initial_state=S1)
    np.testing.assert_allclose(np.concatenate([o1, o2], 1), o, atol=1e-12)
    np.testing.assert_allclose(S2, S, atol=1e-12)
    # packed: three sequences (one empty) in one call equal three separate calls
    cu = np.array([0, 13, 13, 30, 37], dtype=np.int32)
    op, Sp = oracle.fwd(q[0], k[0], v[0], beta[0], cu_seqlens=cu)
    for n in range(4):
        a, b = cu[n], cu[n + 1]
        if a == b:
            assert np.all(Sp[n] == 0)
            continue
        on, Sn = oracle.fwd(q[:, a:b], k[:, a:b], v[:, a:b], beta[:, a:b])
        np.testing.assert_allclose(op[a:b], on[0], atol=1e-13)
        np.testing.assert_allclose(Sp[n], Sn[0], atol=1e-13)


# ------------------------------------------------------------------ backward


def _loss(q, k, v, beta, S0, d_o, dST):
    o, S = oracle.fwd(q, k, v, beta, initial_state=S0)
    return np.sum(o * d_o) + np.sum(S * dST)


def test_backward_matches_central_finite_differences():
    B, L, H, dk, dv = 2, 7, 2, 4, 3
    rng = np.random.default_rng(11)
    q = rng.standard_normal((B, L, H, dk)); k = rng.standard_normal((B, L, H, dk)) / 2
    v = rng.standard_normal((B, L, H, dv)); beta = rng.uniform(0.1, 1.2, size=(B, L, H))
    S0 = rng.standard_normal((B, H, dk, dv)); d_o = rng.standard_normal((B, L, H, dv))
    dST = rng.standard_normal((B, H, dk, dv))
    grads = oracle.bwd(q, k, v, beta, d_o, initial_state=S0, dfinal_state=dST)
    args = [q, k, v, beta, S0]
    h = 1e-6
    for which, g in zip(range(5), grads):
        x = args[which]
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = x[idx]
            x[idx] = old + h; lp = _loss(*args, d_o, dST)
            x[idx] = old - h; lm = _loss(*args, d_o, dST)
            x[idx] = old
            num[idx] = (lp - lm) / (2 * h)
        np.testing.assert_allclose(g, num, rtol=1e-6, atol=1e-7, err_msg="gradient %d" % which)


def test_backward_adjoint_identity_midsize():
    """<do, J dx> = <J^T do, dx> with J dx from a central difference along a random direction."""
    B, L, H, dk, dv = 1, 150, 2, 16, 12
    rng = np.random.default_rng(12)
    x = chain_multi(rng, B, L, H, dk, dv)
    d_o = rng.standard_normal((B, L, H, dv)); dST = rng.standard_normal((B, H, dk, dv))
    grads = oracle.bwd(*x[:4], d_o, initial_state=x[4], dfinal_state=dST)
    dirs = [rng.standard_normal(a.shape) for a in x]
    h = 1e-5
    lp = _loss(*[a + h * d for a, d in zip(x, dirs)], d_o, dST)
    lm = _loss(*[a - h * d for a, d in zip(x, dirs)], d_o, dST)
    lhs = (lp - lm) / (2 * h)
    rhs = sum(np.sum(g * d) for g, d in zip(grads, dirs))
    assert abs(lhs - rhs) < 1e-6 * max(1.0, abs(rhs))


def chain_multi(rng, B, L, H, dk, dv):
    q = rng.standard_normal((B, L, H, dk)); q /= np.linalg.norm(q, axis=-1, keepdims=True)
    k = rng.standard_normal((B, L, H, dk)); k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = rng.standard_normal((B, L, H, dv)); beta = rng.uniform(size=(B, L, H))
    S0 = rng.standard_normal((B, H, dk, dv))
    return [q, k, v, beta, S0]


def test_backward_chaining_across_a_split_and_packed():
    B, L, H, dk, dv = 1, 90, 2, 8, 6   # 90 > SEG and not a multiple of it: exercises the checkpoint replay
    rng = np.random.default_rng(13)
    q, k, v, beta, S0 = chain_multi(rng, B, L, H, dk, dv)
    d_o = rng.standard_normal((B, L, H, dv)); dST = rng.standard_normal((B, H, dk, dv))
    full = oracle.bwd(q, k, v, beta, d_o, initial_state=S0, dfinal_state=dST)
    t0 = 41
    _, S1 = oracle.fwd(q[:, :t0], k[:, :t0], v[:, :t0], beta[:, :t0], initial_state=S0)
    g2 = oracle.bwd(q[:, t0:], k[:, t0:], v[:, t0:], beta[:, t0:], d_o[:, t0:], initial_state=S1, dfinal_state=dST)
    g1 = oracle.bwd(q[:, :t0], k[:, :t0], v[:, :t0], beta[:, :t0], d_o[:, :t0], initial_state=S0, dfinal_state=g2[4])
    for i in range(4):
        np.testing.assert_allclose(np.concatenate([g1[i], g2[i]], 1), full[i], atol=1e-11)
    np.testing.assert_allclose(g1[4], full[4], atol=1e-11)
    # packed layout with zero initial state equals separate calls
    cu = np.array([0, 41, 90], dtype=np.int32)
    gp = oracle.bwd(q[0], k[0], v[0], beta[0], d_o[0], cu_seqlens=cu)
    for n in range(2):
        a, b = cu[n], cu[n + 1]
        gn = oracle.bwd(q[:, a:b], k[:, a:b], v[:, a:b], beta[:, a:b], d_o[:, a:b])
        for i in range(4):
            np.testing.assert_allclose(gp[i][a:b], gn[i][0], atol=1e-12)
        np.testing.assert_allclose(gp[4][n], gn[4][0], atol=1e-12)


@pytest.mark.parametrize("C", [4, 16])
def test_chunkwise_backward_algebra_equals_oracle(C):
    """The chunk-level adjoint of Eq. 8-11 (what the GPU kernels evaluate) equals the token-level one."""
    L, dk, dv = 32, 6, 5
    rng = np.random.default_rng(14)
    q, k, v, beta, S0 = chain_multi(rng, 1, L, 1, dk, dv)
    d_o = rng.standard_normal((1, L, 1, dv)); dST = rng.standard_normal((1, 1, dk, dv))
    ref = oracle.bwd(q, k, v, beta, d_o, initial_state=S0, dfinal_state=dST)
    got = pf.chunkwise_backward(sq(q), sq(k), sq(v), beta[0, :, 0], sq(d_o), C, S0[0, 0], dST[0, 0])
    np.testing.assert_allclose(got[0], sq(ref[0]), atol=1e-11)
    np.testing.assert_allclose(got[1], sq(ref[1]), atol=1e-11)
    np.testing.assert_allclose(got[2], sq(ref[2]), atol=1e-11)
    np.testing.assert_allclose(got[3], ref[3][0, :, 0], atol=1e-11)
    np.testing.assert_allclose(got[4], ref[4][0, 0], atol=1e-11)


def test_thread_count_does_not_change_results():
    rng = np.random.default_rng(15)
    q, k, v, beta, S0 = chain_multi(rng, 3, 20, 3, 8, 8)
    a = oracle.fwd(q, k, v, beta, initial_state=S0, nthreads=1)
    b = oracle.fwd(q, k, v, beta, initial_state=S0, nthreads=4)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
