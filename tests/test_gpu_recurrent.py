"""GPU parity of the token-serial forward (deltanet_recurrent_fwd, through the C ABI) against the fp64
oracle, which is the same per-token recurrence written out on the CPU: several head sizes, both
dtypes, d_k != d_v, packed sequences, carried-in state, and token-by-token decoding."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_06484_amd as dn
from paper_2406_06484_amd.synth import make_config, make_inputs
from tests.gpu_util import TOL, dev_inputs, nerr

pytestmark = pytest.mark.gpu


def rec_fwd(inp, d=None):
    d = d or dev_inputs(inp)
    o, ST = dn.deltanet_recurrent_fwd(d["q"], d["k"], d["v"], d["beta"], d["S0"], cu_seqlens=d["cu"])
    torch.cuda.synchronize()
    return o.float().cpu().numpy(), ST.cpu().numpy()


def check(inp, label):
    o, ST = rec_fwd(inp)
    o_ref, ST_ref = oracle.fwd(inp.q, inp.k, inp.v, inp.beta, inp.initial_state, inp.cu_seqlens)
    eo, es = nerr(o, o_ref), nerr(ST, ST_ref)
    print(label, "o=%.2e final_state=%.2e" % (eo, es), flush=True)
    assert eo < TOL[inp.dtype], (label, eo)
    # the state never leaves fp32, in either dtype
    assert es < (1e-4 if inp.dtype == "f32" else 2e-3), (label, es)


@pytest.mark.parametrize("dtype,dk,dv", [("f32", 32, 16), ("f32", 64, 64), ("f32", 128, 48), ("f32", 256, 64),
                                         ("bf16", 32, 64), ("bf16", 64, 128), ("bf16", 128, 128), ("bf16", 256, 256)])
def test_recurrent_matches_oracle(dtype, dk, dv):
    inp = make_inputs(500 + dk + dv, B=2, L=150, H=3, dk=dk, dv=dv, dtype=dtype, with_initial_state=True)
    inp.initial_state *= 10.0
    check(inp, "recurrent %s %dx%d" % (dtype, dk, dv))


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128)])
def test_recurrent_packed_sequences(dtype, d):
    cu = np.array([0, 0, 5, 69, 199, 262, 263, 263, 520], dtype=np.int32)
    inp = make_inputs(7, H=2, dk=d, dv=d, dtype=dtype, cu_seqlens=cu, with_initial_state=True)
    check(inp, "recurrent packed %s" % dtype)


def test_recurrent_config0():
    check(make_config(0), "recurrent cfg0")


def test_decode_token_by_token_equals_one_call():
    inp = make_inputs(11, B=2, L=24, H=2, dk=128, dv=128, dtype="bf16", with_initial_state=True)
    d = dev_inputs(inp)
    o_all, ST_all = dn.deltanet_recurrent_fwd(d["q"], d["k"], d["v"], d["beta"], d["S0"])
    S = d["S0"].clone()
    outs = []
    for t in range(24):  # one token per call, the state handed back in place
        sl = lambda x: x[:, t:t + 1].contiguous()
        o_t, S = dn.deltanet_recurrent_fwd(sl(d["q"]), sl(d["k"]), sl(d["v"]), sl(d["beta"]), S, final_state=S)
        outs.append(o_t)
    torch.cuda.synchronize()
    assert torch.equal(torch.cat(outs, dim=1), o_all)
    assert torch.equal(S, ST_all)


def test_recurrent_agrees_with_chunkwise_on_the_gpu():
    inp = make_inputs(12, B=2, L=300, H=4, dk=128, dv=128, dtype="bf16", with_initial_state=True)
    d = dev_inputs(inp)
    o_r, S_r = dn.deltanet_recurrent_fwd(d["q"], d["k"], d["v"], d["beta"], d["S0"])
    o_c, S_c = dn.deltanet_fwd(d["q"], d["k"], d["v"], d["beta"], d["S0"])
    torch.cuda.synchronize()
    assert nerr(o_c.float().cpu().numpy(), o_r.float().cpu().numpy()) < TOL["bf16"]
    assert nerr(S_c.cpu().numpy(), S_r.cpu().numpy()) < TOL["bf16"]


def test_recurrent_rejects_unsupported_head_sizes():
    inp = make_inputs(13, B=1, L=4, H=1, dk=96, dv=64, dtype="f32")
    d = dev_inputs(inp)
    with pytest.raises(dn.DeltaNetError) as e:
        dn.deltanet_recurrent_fwd(d["q"], d["k"], d["v"], d["beta"])
    assert e.value.status == -3
    inp = make_inputs(13, B=1, L=4, H=1, dk=64, dv=24, dtype="f32")
    d = dev_inputs(inp)
    with pytest.raises(dn.DeltaNetError) as e:
        dn.deltanet_recurrent_fwd(d["q"], d["k"], d["v"], d["beta"])
    assert e.value.status == -3


def test_recurrent_full_size_configs():
    # the benchmark shape and the packed variable-length batch, every element against the oracle
    check(make_config(1), "recurrent cfg1")
    check(make_config(4), "recurrent cfg4")
