"""GPU parity (through the C ABI) against the fp64 oracle on small shapes that still span several
chunks, a ragged tail, both dtypes, d_k != d_v, packed sequences and the degenerate cases."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_06484_amd as dn
from paper_2406_06484_amd.synth import make_config, make_inputs
from tests.gpu_util import TOL, check_fwd_bwd, dev_inputs, gpu_bwd, gpu_fwd, nerr

pytestmark = pytest.mark.gpu


def test_config0_fp32_fwd_bwd():
    check_fwd_bwd(make_config(0), label="cfg0")


@pytest.mark.parametrize("dtype,dk,dv", [("f32", 64, 64), ("f32", 32, 64), ("f32", 64, 32),
                                         ("bf16", 64, 64), ("bf16", 128, 128), ("bf16", 64, 128), ("bf16", 128, 64)])
def test_ragged_multi_chunk_with_states(dtype, dk, dv):
    inp = make_inputs(100 + dk + dv, B=2, L=200, H=3, dk=dk, dv=dv, dtype=dtype,
                      with_initial_state=True, with_dfinal_state=True)
    inp.initial_state *= 10.0  # make the carried-in state matter
    check_fwd_bwd(inp, label="%s %dx%d" % (dtype, dk, dv))


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128)])
def test_packed_sequences(dtype, d):
    cu = np.array([0, 0, 5, 69, 199, 262, 263, 263, 520], dtype=np.int32)  # empty, tiny, exact-chunk, ragged
    inp = make_inputs(7, H=2, dk=d, dv=d, dtype=dtype, cu_seqlens=cu, with_initial_state=True, with_dfinal_state=True)
    check_fwd_bwd(inp, label="packed %s" % dtype)
    # the packed call equals separate dense calls, sequence by sequence
    o, ST = gpu_fwd(inp)
    for n in (2, 4):
        a, b = cu[n], cu[n + 1]
        sub = make_inputs(7, H=2, dk=d, dv=d, dtype=dtype, B=1, L=int(b - a))
        sub.q, sub.k, sub.v, sub.beta = (x[None, a:b] for x in (inp.q, inp.k, inp.v, inp.beta))
        sub.initial_state = inp.initial_state[n:n + 1]
        o1, ST1 = gpu_fwd(sub)
        assert nerr(o1[0], o[a:b]) < 1e-6 and nerr(ST1[0], ST[n]) < 1e-6


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_single_short_sequence_and_length_one(dtype):
    for L in (1, 17, 64, 65):
        inp = make_inputs(40 + L, B=1, L=L, H=1, dk=64, dv=64, dtype=dtype, with_dfinal_state=True)
        check_fwd_bwd(inp, label="L=%d %s" % (L, dtype))


def test_beta_zero_leaves_state_bitwise_unchanged():
    inp = make_inputs(3, B=1, L=130, H=2, dk=64, dv=64, dtype="f32", with_initial_state=True)
    inp.beta[:] = 0.0
    o, ST = gpu_fwd(inp)
    assert np.array_equal(ST, inp.initial_state.astype(np.float32))
    o_ref, _ = oracle.fwd(inp.q, inp.k, inp.v, inp.beta, inp.initial_state)
    assert nerr(o, o_ref) < 1e-5


def test_beta_one_onehot_keys_exact_in_bf16():
    """One-hot keys and small-integer values are exact in bf16, so store-and-retrieve must be exact."""
    d, L = 128, 128
    rng = np.random.default_rng(9)
    perm = rng.permutation(d)
    k = np.eye(d)[perm][None, :, None, :]
    inp = make_inputs(9, B=1, L=L, H=1, dk=d, dv=d, dtype="bf16")
    inp.q = k.copy(); inp.k = k.copy(); inp.beta[:] = 1.0
    inp.v = rng.integers(-8, 9, size=inp.v.shape).astype(np.float64)
    o, ST = gpu_fwd(inp)
    assert np.array_equal(o[0, :, 0], inp.v[0, :, 0])                       # q_t = k_t reads back v_t
    assert np.array_equal(ST[0, 0], k[0, :, 0].T @ inp.v[0, :, 0])          # S = sum k v^T


def test_state_chaining_on_gpu_matches_one_shot():
    inp = make_inputs(21, B=1, L=300, H=2, dk=64, dv=64, dtype="f32", with_dfinal_state=True)
    d = dev_inputs(inp)
    o, ST = dn.deltanet_fwd(d["q"], d["k"], d["v"], d["beta"])
    t0 = 150  # not a multiple of the chunk size
    cut = lambda x, a, b: x[:, a:b].contiguous()
    o1, S1 = dn.deltanet_fwd(cut(d["q"], 0, t0), cut(d["k"], 0, t0), cut(d["v"], 0, t0), cut(d["beta"], 0, t0))
    o2, S2 = dn.deltanet_fwd(cut(d["q"], t0, 300), cut(d["k"], t0, 300), cut(d["v"], t0, 300), cut(d["beta"], t0, 300), S1)
    assert nerr(torch.cat([o1, o2], 1).cpu().numpy(), o.cpu().numpy()) < 1e-5
    assert nerr(S2.cpu().numpy(), ST.cpu().numpy()) < 1e-5
    # gradients chain the same way: dS0 of part 2 is dfinal_state of part 1
    full = dn.deltanet_bwd(d["q"], d["k"], d["v"], d["beta"], d["d_o"], None, d["dST"])
    g2 = dn.deltanet_bwd(cut(d["q"], t0, 300), cut(d["k"], t0, 300), cut(d["v"], t0, 300), cut(d["beta"], t0, 300),
                         cut(d["d_o"], t0, 300), S1, d["dST"])
    g1 = dn.deltanet_bwd(cut(d["q"], 0, t0), cut(d["k"], 0, t0), cut(d["v"], 0, t0), cut(d["beta"], 0, t0),
                         cut(d["d_o"], 0, t0), None, g2[4])
    for i in range(4):
        assert nerr(torch.cat([g1[i], g2[i]], 1).cpu().numpy(), full[i].cpu().numpy()) < 2e-5
    assert nerr(g1[4].cpu().numpy(), full[4].cpu().numpy()) < 2e-5


def test_results_are_deterministic_and_ignore_workspace_contents():
    inp = make_inputs(5, B=2, L=192, H=2, dk=128, dv=128, dtype="bf16")
    d = dev_inputs(inp)
    outs = []
    for fill in (0, 255):
        from paper_2406_06484_amd.binding import _shape_of, deltanet_workspace_bytes
        s = _shape_of(d["q"], d["v"], None, 64, [])
        ws = torch.full((deltanet_workspace_bytes(s, True),), fill, dtype=torch.uint8, device="cuda")
        g = dn.deltanet_bwd(d["q"], d["k"], d["v"], d["beta"], d["d_o"], workspace=ws)
        outs.append([t.clone() for t in g])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_many_tiny_packed_sequences():
    # thousands of sequences of 0..3 tokens: every chain is one ragged chunk, the chunk-offset prefix and
    # the chunk -> sequence search see their extreme shape
    rng = np.random.default_rng(5)
    lens = rng.integers(0, 4, size=6000)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    inp = make_inputs(21, H=2, dk=64, dv=64, dtype="f32", cu_seqlens=cu, with_initial_state=True, with_dfinal_state=True)
    check_fwd_bwd(inp, label="6000 tiny sequences")


def test_many_heads_and_the_sequence_count_limit():
    inp = make_inputs(22, B=1, L=70, H=300, dk=64, dv=64, dtype="bf16", with_dfinal_state=True)
    check_fwd_bwd(inp, label="H=300")
    # more sequences than the grid mapping supports is refused before any launch
    q = torch.zeros((4, 1, 64), dtype=torch.float32, device="cuda")
    cu = torch.zeros(65537 + 1, dtype=torch.int32, device="cuda")
    cu[-1] = 4
    with pytest.raises(dn.DeltaNetError) as e:
        dn.deltanet_fwd(q, q, q, q[..., 0].contiguous(), cu_seqlens=cu)
    assert e.value.status == -2


def test_head_size_256():
    # d_k = d_v = 256: the scans own 32 state columns per workgroup, the backward's chunk kernel streams S and dS' in
    # column blocks
    from paper_2406_06484_amd.synth import make_gate
    inp = make_inputs(31, B=2, L=200, H=2, dk=256, dv=256, dtype="bf16", with_initial_state=True, with_dfinal_state=True)
    inp.initial_state *= 10.0
    check_fwd_bwd(inp, label="bf16 256x256")
    cu = np.array([0, 0, 5, 69, 199, 262, 263, 263, 520], dtype=np.int32)
    pk = make_inputs(32, H=2, dk=256, dv=256, dtype="bf16", cu_seqlens=cu, with_initial_state=True)
    check_fwd_bwd(pk, label="bf16 256x256 packed")
    plain = make_inputs(33, B=1, L=448, H=3, dk=256, dv=256, dtype="bf16")   # no optional state, whole chunks
    check_fwd_bwd(plain, label="bf16 256x256 no states")
    # more (chunk, head) tiles than compute units: the persistent workgroups of the chunk kernel walk over several tiles
    many = make_inputs(34, B=2, L=2048 + 37, H=5, dk=256, dv=256, dtype="bf16", with_initial_state=True, with_dfinal_state=True)
    check_fwd_bwd(many, label="bf16 256x256 330 tiles")
    # the gated rule at this head size: the gate gradient's per-token terms come from a second kernel
    from tests.test_gpu_gated import run_gated
    run_gated(inp, make_gate(5, inp.beta.shape, lo=0.6, hi=1.0), label="gated bf16 256x256")
    run_gated(many, make_gate(6, many.beta.shape, lo=0.9, hi=1.0), label="gated bf16 256x256 330 tiles")


def test_head_size_256_degenerate_cases():
    # beta = 0 (the token writes nothing) and beta = 1 (full overwrite) mixed into a batch, forward and backward
    inp = make_inputs(35, B=1, L=200, H=2, dk=256, dv=256, dtype="bf16", with_initial_state=True, with_dfinal_state=True)
    inp.beta[:, 0:70] = 0.0          # a whole chunk and a bit of the next one
    inp.beta[:, 100:110] = 1.0
    check_fwd_bwd(inp, label="bf16 256x256 beta in {0, 1}")
    # one-hot keys and small-integer values are exact in bf16: store-and-retrieve must be exact
    d, L = 256, 256
    rng = np.random.default_rng(10)
    k = np.eye(d)[rng.permutation(d)][None, :, None, :]
    one = make_inputs(36, B=1, L=L, H=1, dk=d, dv=d, dtype="bf16")
    one.q = k.copy(); one.k = k.copy(); one.beta[:] = 1.0
    one.v = rng.integers(-8, 9, size=one.v.shape).astype(np.float64)
    o, ST = gpu_fwd(one)
    assert np.array_equal(o[0, :, 0], one.v[0, :, 0])
    assert np.array_equal(ST[0, 0], k[0, :, 0].T @ one.v[0, :, 0])
    # the backward pass does not depend on what the workspace held before
    from paper_2406_06484_amd.binding import _shape_of, deltanet_workspace_bytes
    dd = dev_inputs(inp)
    outs = []
    for fill in (0, 255):
        ws = torch.full((deltanet_workspace_bytes(_shape_of(dd["q"], dd["v"], None, 64, []), True),), fill, dtype=torch.uint8, device="cuda")
        outs.append([t.clone() for t in dn.deltanet_bwd(dd["q"], dd["k"], dd["v"], dd["beta"], dd["d_o"], dd["S0"], dd["dST"], workspace=ws)])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


# (the last case cuts the forward pass only: 48 scan workgroups are too many for the backward rule)
@pytest.mark.parametrize("dtype,d,B,H,L", [("f32", 64, 1, 2, 2048), ("bf16", 128, 1, 3, 4096), ("bf16", 64, 2, 1, 1024), ("bf16", 128, 1, 24, 2048)])
def test_few_long_chains_take_the_segmented_scans(dtype, d, B, H, L):
    # few chains and a long sequence: both passes cut the sequence into segments, get each segment's start state (end
    # gradient) from the segments' affine maps, and scan the segments side by side
    from paper_2406_06484_amd.binding import _shape_of, deltanet_workspace_bytes
    inp = make_inputs(900 + d + L, B=B, L=L, H=H, dk=d, dv=d, dtype=dtype, with_initial_state=True, with_dfinal_state=True)
    inp.initial_state *= 10.0
    dd = dev_inputs(inp)
    # the workspace grows by the per-segment states exactly when the segmented path is taken
    one_chunk_tiles = (L // 64) * B * H * 64 * 64 * (2 if dtype == "bf16" else 4)
    assert deltanet_workspace_bytes(_shape_of(dd["q"], dd["v"], None, 64, []), False) > one_chunk_tiles
    check_fwd_bwd(inp, label="segmented %s d=%d B=%d H=%d L=%d" % (dtype, d, B, H, L))
    o, ST, saved = dn.deltanet_fwd_save(dd["q"], dd["k"], dd["v"], dd["beta"], dd["S0"])
    grads = dn.deltanet_bwd_saved(dd["q"], dd["k"], dd["v"], dd["beta"], dd["d_o"], saved, dd["dST"])
    o2, ST2 = dn.deltanet_fwd(dd["q"], dd["k"], dd["v"], dd["beta"], dd["S0"])
    grads2 = dn.deltanet_bwd(dd["q"], dd["k"], dd["v"], dd["beta"], dd["d_o"], dd["S0"], dd["dST"])
    torch.cuda.synchronize()
    assert torch.equal(o, o2) and torch.equal(ST, ST2)
    fwd_only_cut = B * H * (2 if (dtype == "bf16" and d == 128) else 1) > 32
    for a, b in zip(grads, grads2):
        if fwd_only_cut:   # kept tiles come from the cut forward pass, the self-contained backward recomputes them uncut
            assert nerr(a.float().cpu().numpy(), b.float().cpu().numpy()) < 1e-2   # two bf16 results, each within 5e-3 of the oracle
        else:              # the pair that keeps the forward's tiles runs the same segmented arithmetic
            assert torch.equal(a, b)


def test_segmented_scans_without_optional_states():
    # no initial state, no final-state gradient, and outputs for them not requested
    inp = make_inputs(77, B=1, L=2048, H=2, dk=128, dv=128, dtype="bf16")
    dd = dev_inputs(inp)
    o, _ = dn.deltanet_fwd(dd["q"], dd["k"], dd["v"], dd["beta"], output_final_state=False)
    grads = dn.deltanet_bwd(dd["q"], dd["k"], dd["v"], dd["beta"], dd["d_o"], want_dinitial_state=False)
    torch.cuda.synchronize()
    o_ref, _ = oracle.fwd(inp.q, inp.k, inp.v, inp.beta)
    g_ref = oracle.bwd(inp.q, inp.k, inp.v, inp.beta, inp.d_o)
    assert nerr(o.float().cpu().numpy(), o_ref) < TOL["bf16"]
    for a, b in zip(grads[:4], g_ref[:4]):
        assert nerr(a.float().cpu().numpy(), b) < TOL["bf16"]
    assert grads[4] is None


def test_seeded_random_shapes():
    # a handful of seeded random shapes, dense and packed (with empty and one-token sequences), both element types
    rng = np.random.default_rng(2024)
    for case in range(14):
        # (the first ten cases keep the shapes they always had; the last four add the largest head size)
        dtype, d = [("f32", 64), ("bf16", 128), ("bf16", 64)][case % 3] if case < 10 else ("bf16", 256)
        H = int(rng.integers(1, 4))
        if case % 2 == 0:
            B, L = int(rng.integers(1, 4)), int(rng.integers(1, 700))
            inp = make_inputs(3000 + case, B=B, L=L, H=H, dk=d, dv=d, dtype=dtype,
                              with_initial_state=bool(case % 4 == 0), with_dfinal_state=bool(case % 4 == 2))
            label = "random dense %s d=%d B=%d L=%d H=%d" % (dtype, d, B, L, H)
        else:
            lens = rng.integers(0, 300, size=int(rng.integers(1, 7)))
            lens[rng.integers(0, len(lens))] = 1
            cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
            inp = make_inputs(3000 + case, H=H, dk=d, dv=d, dtype=dtype, cu_seqlens=cu, with_initial_state=True, with_dfinal_state=True)
            label = "random packed %s d=%d lens=%s H=%d" % (dtype, d, lens.tolist(), H)
        check_fwd_bwd(inp, label=label)
