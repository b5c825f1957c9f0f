"""Pins for the oracle's prologue (section 3.3, "Feature map and normalization": q, k = SiLU(x) / ||SiLU(x)||_2;
section 2.2: beta = sigmoid(b)) and for its composition with the delta rule: known values, invariants of the
normalisation, limits, central differences of the composed loss, and the tangent-space property of the gradient."""
import math

import numpy as np

import oracle


def rand_pre(seed, B=2, L=9, H=2, dk=6, dv=5):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, L, H, dk)) * 1.5
    k = rng.standard_normal((B, L, H, dk)) * 1.5
    v = rng.standard_normal((B, L, H, dv))
    b = rng.standard_normal((B, L, H))
    S0 = rng.standard_normal((B, H, dk, dv)) * 0.3
    return q, k, v, b, S0


def test_known_values_of_silu_and_sigmoid():
    assert oracle.sigmoid(0.0) == 0.5
    assert abs(oracle.sigmoid(1.0) - 1.0 / (1.0 + math.exp(-1.0))) < 1e-16
    assert oracle.silu(0.0) == 0.0
    assert abs(oracle.silu(1.0) - 0.7310585786300049) < 1e-15       # 1 / (1 + e^-1)
    assert abs(oracle.silu(-1.0) + 0.2689414213699951) < 1e-15      # -1 / (1 + e)
    # SiLU(x) -> x for large x and -> 0 for very negative x
    assert abs(oracle.silu(40.0) - 40.0) < 1e-12 and abs(oracle.silu(-40.0)) < 1e-12


def test_feature_map_rows_have_unit_norm_and_the_direction_of_silu():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((3, 7, 2, 16)) * 2.0
    y = oracle.feature_map(x)
    assert np.allclose(np.linalg.norm(y, axis=-1), 1.0, rtol=0, atol=1e-14)
    s = x / (1.0 + np.exp(-x))
    # parallel to SiLU(x): y = s / ||s||, so y * ||s|| - s = 0 and the cosine is one
    assert np.allclose(y * np.linalg.norm(s, axis=-1, keepdims=True), s, rtol=0, atol=1e-14)
    # a hand-worked row: x = (1, -1, 0) -> s = (a, -b, 0), a = 0.7310585786, b = 0.2689414214
    a, b = 0.7310585786300049, 0.2689414213699951
    n = math.sqrt(a * a + b * b)
    assert np.allclose(oracle.feature_map(np.array([1.0, -1.0, 0.0])), [a / n, -b / n, 0.0], rtol=0, atol=1e-15)


def test_feature_map_limits_and_the_zero_row():
    e = np.zeros(8); e[3] = 50.0
    y = oracle.feature_map(e)          # one large coordinate: the unit vector
    assert abs(y[3] - 1.0) < 1e-15 and np.all(y[np.arange(8) != 3] == 0.0)
    assert np.array_equal(oracle.feature_map(np.zeros(8)), np.zeros(8))           # no 0 / 0
    assert np.array_equal(oracle.feature_map_bwd(np.zeros(8), np.ones(8)), np.zeros(8))
    # for large positive x SiLU is the identity, so the map is plain L2 normalisation
    x = np.array([30.0, 40.0, 50.0])
    assert np.allclose(oracle.feature_map(x), x / np.linalg.norm(x), rtol=0, atol=1e-12)


def test_feature_map_gradient_is_tangent_to_the_sphere():
    # y has unit norm whatever x is, so moving x along any direction keeps y on the sphere:
    # the gradient with respect to s = SiLU(x) is orthogonal to y
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 12)) * 1.3
    dy = rng.standard_normal((5, 12))
    dx = oracle.feature_map_bwd(x, dy)
    sg = 1.0 / (1.0 + np.exp(-x))
    ds = dx / (sg * (1.0 + x * (1.0 - sg)))
    y = oracle.feature_map(x)
    assert np.allclose(np.sum(ds * y, axis=-1), 0.0, rtol=0, atol=1e-13)
    # and a gradient along y itself maps to zero
    assert np.allclose(oracle.feature_map_bwd(x, 3.0 * y), 0.0, rtol=0, atol=1e-13)


def test_feature_map_bwd_matches_central_differences():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((4, 7)) * 1.2
    dy = rng.standard_normal((4, 7))
    got = oracle.feature_map_bwd(x, dy)
    h = 1e-6
    for idx in [(0, 0), (1, 3), (2, 6), (3, 2)]:
        xp, xm = x.copy(), x.copy()
        xp[idx] += h; xm[idx] -= h
        num = (np.sum(oracle.feature_map(xp) * dy) - np.sum(oracle.feature_map(xm) * dy)) / (2 * h)
        assert abs(num - got[idx]) < 1e-8, (idx, num, got[idx])


def test_fused_forward_is_the_delta_rule_on_the_mapped_inputs():
    q, k, v, b, S0 = rand_pre(4)
    o, ST = oracle.fused_fwd(q, k, v, b, S0)
    # written out independently of feature_map: explicit SiLU, norm and logistic
    sq, sk = q / (1 + np.exp(-q)), k / (1 + np.exp(-k))
    qn = sq / np.sqrt((sq ** 2).sum(-1, keepdims=True)); kn = sk / np.sqrt((sk ** 2).sum(-1, keepdims=True))
    beta = 1 / (1 + np.exp(-b))
    B, L, H, dk = q.shape
    S = S0.copy()
    for t in range(L):
        for bb in range(B):
            for h in range(H):
                kt, vt, bt = kn[bb, t, h], v[bb, t, h], beta[bb, t, h]
                S[bb, h] = S[bb, h] + bt * np.outer(kt, vt - S[bb, h].T @ kt)
                assert np.allclose(o[bb, t, h], S[bb, h].T @ qn[bb, t, h], rtol=1e-12, atol=1e-12)
    assert np.allclose(ST, S, rtol=1e-12, atol=1e-12)


def test_fused_gradients_match_central_differences_of_the_composed_loss():
    q, k, v, b, S0 = rand_pre(5, B=1, L=7, H=2, dk=5, dv=4)
    rng = np.random.default_rng(6)
    d_o = rng.standard_normal(v.shape)
    dST = rng.standard_normal(S0.shape)

    def loss(q_, k_, v_, b_, S0_):
        o, ST = oracle.fused_fwd(q_, k_, v_, b_, S0_)
        return float(np.sum(o * d_o) + np.sum(ST * dST))

    grads = oracle.fused_bwd(q, k, v, b, d_o, S0, dST)
    args = [q, k, v, b, S0]
    h = 1e-6
    for which, g in enumerate(grads):
        flat = np.arange(args[which].size)
        for pos in rng.choice(flat, size=min(6, flat.size), replace=False):
            idx = np.unravel_index(pos, args[which].shape)
            ap = [a.copy() for a in args]; am = [a.copy() for a in args]
            ap[which][idx] += h; am[which][idx] -= h
            num = (loss(*ap) - loss(*am)) / (2 * h)
            assert abs(num - g[idx]) < 2e-7 * max(1.0, abs(num)), (which, idx, num, g[idx])


def test_packed_layout_matches_separate_sequences():
    rng = np.random.default_rng(7)
    H, dk, dv = 2, 6, 4
    lens = [5, 0, 9, 3]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    q = rng.standard_normal((T, H, dk)); k = rng.standard_normal((T, H, dk))
    v = rng.standard_normal((T, H, dv)); b = rng.standard_normal((T, H)); d_o = rng.standard_normal((T, H, dv))
    o, ST = oracle.fused_fwd(q, k, v, b, None, cu)
    g = oracle.fused_bwd(q, k, v, b, d_o, None, None, cu)
    for n, ln in enumerate(lens):
        if ln == 0:
            continue
        sl = slice(cu[n], cu[n + 1])
        o1, ST1 = oracle.fused_fwd(q[sl][None], k[sl][None], v[sl][None], b[sl][None])
        g1 = oracle.fused_bwd(q[sl][None], k[sl][None], v[sl][None], b[sl][None], d_o[sl][None])
        assert np.allclose(o[sl], o1[0], atol=1e-13) and np.allclose(ST[n], ST1[0], atol=1e-13)
        for a, c in zip(g[:4], g1[:4]):
            assert np.allclose(a[sl], c[0], atol=1e-13)
