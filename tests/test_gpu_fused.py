"""GPU parity of the forward/backward pass with the layer's prologue in the load path (deltanet_fused_fwd / _bwd
and the pair that keeps the forward's tiles, through the C ABI) against the fp64 oracle of the composition:
q, k = SiLU(x) / ||SiLU(x)||_2 (section 3.3), beta = sigmoid(b) (section 2.2), then the delta rule."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_06484_amd as dn
from paper_2406_06484_amd.synth import make_config, make_inputs, make_pre_activations
from tests.gpu_util import TOL, check_tensors, dev_inputs, nerr

pytestmark = pytest.mark.gpu

NAMES = ("o", "final_state", "dq_pre", "dk_pre", "dv", "dbeta_logit", "dinitial_state")


def run_fused(inp, label, check_saved=True):
    d = dev_inputs(inp)
    o, ST = dn.deltanet_fused_fwd(d["q"], d["k"], d["v"], d["beta"], d["S0"], cu_seqlens=d["cu"])
    grads = dn.deltanet_fused_bwd(d["q"], d["k"], d["v"], d["beta"], d["d_o"], d["S0"], d["dST"], cu_seqlens=d["cu"])
    torch.cuda.synchronize()
    ref = list(oracle.fused_fwd(inp.q, inp.k, inp.v, inp.beta, inp.initial_state, inp.cu_seqlens))
    ref += list(oracle.fused_bwd(inp.q, inp.k, inp.v, inp.beta, inp.d_o, inp.initial_state, inp.dfinal_state, inp.cu_seqlens))
    check_tensors([(name, a.float().cpu().numpy(), b) for name, a, b in zip(NAMES, [o, ST] + list(grads), ref)], inp.dtype, label=label)
    if check_saved:  # the pair that keeps the forward's tiles does the same arithmetic
        o2, ST2, saved = dn.deltanet_fused_fwd_save(d["q"], d["k"], d["v"], d["beta"], d["S0"], cu_seqlens=d["cu"])
        grads2 = dn.deltanet_fused_bwd_saved(d["q"], d["k"], d["v"], d["beta"], d["d_o"], saved, d["dST"], cu_seqlens=d["cu"])
        torch.cuda.synchronize()
        assert torch.equal(o, o2) and torch.equal(ST, ST2), label
        for name, a, b in zip(NAMES[2:], grads, grads2):
            assert torch.equal(a, b), (label, name)


@pytest.mark.parametrize("dtype,dk,dv", [("f32", 64, 64), ("f32", 32, 64), ("bf16", 128, 128), ("bf16", 64, 128), ("bf16", 64, 64),
                                         ("bf16", 256, 256)])
def test_fused_ragged_multi_chunk_with_states(dtype, dk, dv):
    base = make_inputs(800 + dk + dv, B=2, L=200, H=3, dk=dk, dv=dv, dtype=dtype, with_initial_state=True, with_dfinal_state=True)
    run_fused(make_pre_activations(1, base), "fused %s %dx%d" % (dtype, dk, dv))


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128), ("bf16", 256)])
def test_fused_packed_with_empty_and_short_sequences(dtype, d):
    cu = np.array([0, 0, 5, 69, 199, 262, 263, 263, 520], dtype=np.int32)
    base = make_inputs(31, H=2, dk=d, dv=d, dtype=dtype, cu_seqlens=cu, with_initial_state=True, with_dfinal_state=True)
    run_fused(make_pre_activations(2, base), "fused packed %s" % dtype)


def test_fused_large_and_small_pre_activations():
    # wide pre-activations (SiLU nearly the identity on one side, nearly zero on the other) and tiny ones
    # (SiLU(x) ~ x / 2: the norm divides by a small number)
    for scale in (6.0, 0.01):
        base = make_inputs(32, B=1, L=130, H=2, dk=64, dv=64, dtype="f32", with_dfinal_state=True)
        run_fused(make_pre_activations(3, base, scale=scale), "fused scale %g" % scale)


def test_fused_equals_the_plain_path_on_the_mapped_inputs():
    # feeding the plain entry points with the oracle's mapped q, k, beta must give the same outputs up to the
    # rounding of q, k to the element type (fp32 here, so to 1e-5)
    base = make_inputs(33, B=1, L=150, H=2, dk=64, dv=64, dtype="f32", with_initial_state=True)
    inp = make_pre_activations(4, base)
    d = dev_inputs(inp)
    o, ST = dn.deltanet_fused_fwd(d["q"], d["k"], d["v"], d["beta"], d["S0"])
    f32 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float32)).cuda()
    o2, ST2 = dn.deltanet_fwd(f32(oracle.feature_map(inp.q)), f32(oracle.feature_map(inp.k)), d["v"], f32(oracle.sigmoid(inp.beta)), d["S0"])
    torch.cuda.synchronize()
    assert nerr(o.cpu().numpy(), o2.cpu().numpy()) < 1e-5 and nerr(ST.cpu().numpy(), ST2.cpu().numpy()) < 1e-5


@pytest.mark.parametrize("cfg", [2, 4])
def test_fused_full_size(cfg):
    # the benchmark shape and the packed variable-length batch (65536 tokens, lengths 128..8192)
    inp = make_pre_activations(5, make_config(cfg))
    run_fused(inp, "fused cfg%d" % cfg)


def test_fused_few_long_chains_take_the_segmented_scans():
    base = make_inputs(42, B=1, L=2048, H=2, dk=128, dv=128, dtype="bf16", with_initial_state=True, with_dfinal_state=True)
    run_fused(make_pre_activations(6, base), "fused segmented")
