"""GPU parity of the pair that keeps the forward pass's per-chunk results (deltanet_fwd_save /
deltanet_bwd_saved and the gated pair, through the C ABI): against the fp64 oracle, and against the
self-contained deltanet_fwd / deltanet_bwd, which must produce the very same numbers."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_06484_amd as dn
from paper_2406_06484_amd.synth import make_config, make_gate, make_inputs
from tests.gpu_util import TOL, check_tensors, dev_inputs, nerr

pytestmark = pytest.mark.gpu

NAMES = ("dq", "dk", "dv", "dbeta", "dinitial_state")


def run_saved(inp, label, saved=None, check_oracle=True):
    d = dev_inputs(inp)
    o, ST, saved = dn.deltanet_fwd_save(d["q"], d["k"], d["v"], d["beta"], d["S0"], cu_seqlens=d["cu"], saved=saved)
    grads = dn.deltanet_bwd_saved(d["q"], d["k"], d["v"], d["beta"], d["d_o"], saved, d["dST"], cu_seqlens=d["cu"])
    torch.cuda.synchronize()
    # the self-contained calls run the same kernels' arithmetic on the same tiles
    o2, ST2 = dn.deltanet_fwd(d["q"], d["k"], d["v"], d["beta"], d["S0"], cu_seqlens=d["cu"])
    grads2 = dn.deltanet_bwd(d["q"], d["k"], d["v"], d["beta"], d["d_o"], d["S0"], d["dST"], cu_seqlens=d["cu"])
    torch.cuda.synchronize()
    assert torch.equal(o, o2) and torch.equal(ST, ST2), label
    for name, a, b in zip(NAMES, grads, grads2):
        assert torch.equal(a, b), (label, name)
    if check_oracle:
        ref = list(oracle.fwd(inp.q, inp.k, inp.v, inp.beta, inp.initial_state, inp.cu_seqlens))
        ref += list(oracle.bwd(inp.q, inp.k, inp.v, inp.beta, inp.d_o, inp.initial_state, inp.dfinal_state, inp.cu_seqlens))
        check_tensors([(name, a.float().cpu().numpy(), b) for name, a, b in zip(("o", "final_state") + NAMES, [o, ST] + list(grads), ref)],
                      inp.dtype, label=label)
    return saved


@pytest.mark.parametrize("dtype,dk,dv", [("f32", 64, 64), ("f32", 32, 64), ("bf16", 128, 128), ("bf16", 64, 128), ("bf16", 128, 64),
                                         ("bf16", 256, 256)])
def test_saved_pair_ragged_multi_chunk_with_states(dtype, dk, dv):
    inp = make_inputs(700 + dk + dv, B=2, L=200, H=3, dk=dk, dv=dv, dtype=dtype, with_initial_state=True, with_dfinal_state=True)
    run_saved(inp, "saved %s %dx%d" % (dtype, dk, dv))


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128), ("bf16", 256)])
def test_saved_pair_packed_with_empty_and_short_sequences(dtype, d):
    cu = np.array([0, 0, 5, 69, 199, 262, 263, 263, 520], dtype=np.int32)
    inp = make_inputs(21, H=2, dk=d, dv=d, dtype=dtype, cu_seqlens=cu, with_initial_state=True, with_dfinal_state=True)
    run_saved(inp, "saved packed %s" % dtype)


def test_saved_buffer_serves_a_second_smaller_call():
    big = make_inputs(22, B=2, L=300, H=2, dk=128, dv=128, dtype="bf16", with_initial_state=True, with_dfinal_state=True)
    small = make_inputs(23, B=2, L=70, H=2, dk=128, dv=128, dtype="bf16")
    saved = run_saved(big, "saved big")
    saved2 = run_saved(small, "saved small, same buffer", saved=saved)
    assert saved2.data_ptr() == saved.data_ptr()


def test_saved_pair_without_optional_tensors():
    inp = make_inputs(24, B=1, L=130, H=2, dk=64, dv=64, dtype="f32")
    run_saved(inp, "saved, no states")


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128), ("bf16", 256)])
def test_gated_saved_pair(dtype, d):
    inp = make_inputs(25, B=2, L=200, H=2, dk=d, dv=d, dtype=dtype, with_initial_state=True, with_dfinal_state=True)
    g = make_gate(5, inp.beta.shape, lo=0.6, hi=1.0)
    dd = dev_inputs(inp)
    gd = torch.from_numpy(g).cuda()
    o, ST, saved = dn.deltanet_gated_fwd_save(dd["q"], dd["k"], dd["v"], dd["beta"], gd, dd["S0"])
    out = dn.deltanet_gated_bwd_saved(dd["q"], dd["k"], dd["v"], dd["beta"], gd, dd["d_o"], saved, dd["dST"])
    torch.cuda.synchronize()
    o2, ST2 = dn.deltanet_gated_fwd(dd["q"], dd["k"], dd["v"], dd["beta"], gd, dd["S0"])
    out2 = dn.deltanet_gated_bwd(dd["q"], dd["k"], dd["v"], dd["beta"], gd, dd["d_o"], dd["S0"], dd["dST"])
    torch.cuda.synchronize()
    assert torch.equal(o, o2) and torch.equal(ST, ST2)
    for a, b in zip(out, out2):
        assert torch.equal(a, b)
    ref = list(oracle.gated_fwd(inp.q, inp.k, inp.v, inp.beta, g, inp.initial_state))
    ref += list(oracle.gated_bwd(inp.q, inp.k, inp.v, inp.beta, g, inp.d_o, inp.initial_state, inp.dfinal_state))
    names = ("o", "final_state", "dq", "dk", "dv", "dbeta", "dg", "dinitial_state")
    check_tensors([(n, a.float().cpu().numpy(), b) for n, a, b in zip(names, [o, ST] + list(out), ref)], dtype, label="gated saved %s %d" % (dtype, d))


def test_saved_pair_rejects_what_it_cannot_do():
    inp = make_inputs(26, B=1, L=64, H=1, dk=128, dv=256, dtype="bf16")
    d = dev_inputs(inp)
    with pytest.raises(dn.DeltaNetError) as ei:   # a pair of head sizes that is not compiled
        dn.deltanet_fwd_save(d["q"], d["k"], d["v"], d["beta"])
    assert ei.value.status == -3
    inp = make_inputs(27, B=1, L=128, H=2, dk=128, dv=128, dtype="bf16")
    d = dev_inputs(inp)
    small = torch.empty(4096, dtype=torch.uint8, device="cuda")
    with pytest.raises(dn.DeltaNetError) as ei:
        dn.deltanet_fwd_save(d["q"], d["k"], d["v"], d["beta"], saved=small)
    assert ei.value.status == -5
    with pytest.raises(dn.DeltaNetError) as ei:
        dn.deltanet_bwd_saved(d["q"], d["k"], d["v"], d["beta"], d["d_o"], small)
    assert ei.value.status == -5


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_saved_pair_full_size(cfg):
    # the benchmark shape (the pair bench.py times), the long sequence with states at both ends, and the packed
    # variable-length batch: bit-equal to the self-contained pair, and held to the oracle directly
    run_saved(make_config(cfg), "saved cfg%d" % cfg)


def test_saved_pair_head_size_256_at_the_benchmark_size():
    # the d = 256 step that bench.py times beside the headline one (same tokens, half as many heads), against the oracle
    inp = make_inputs(28, B=8, L=2048, H=8, dk=256, dv=256, dtype="bf16")
    run_saved(inp, "saved bf16 256x256 B=8 L=2048 H=8")


@pytest.mark.parametrize("dk,dv", [(128, 128), (64, 128), (128, 64), (64, 64)])
def test_streamed_chunk_kernel_option(dk, dv):
    """DN_OPT_STREAMED_CHUNK_KERNEL: the backward pass through the chunk kernel that streams S and dS' in blocks of state
    columns and rebuilds U - W S and its gradient on chip (the scans then do not store them): against the oracle, for the
    self-contained pair and the pair that keeps the forward's tiles, dense ragged and packed, and at the benchmark size."""
    dn.deltanet_set_option(dn.DN_OPT_STREAMED_CHUNK_KERNEL, 1)
    try:
        inp = make_inputs(900 + dk + dv, B=2, L=200, H=3, dk=dk, dv=dv, dtype="bf16", with_initial_state=True, with_dfinal_state=True)
        run_saved(inp, "streamed bf16 %dx%d" % (dk, dv))
        cu = np.array([0, 0, 5, 69, 199, 262, 263, 263, 520], dtype=np.int32)
        inp = make_inputs(29, H=2, dk=dk, dv=dv, dtype="bf16", cu_seqlens=cu, with_initial_state=True, with_dfinal_state=True)
        run_saved(inp, "streamed packed bf16 %dx%d" % (dk, dv))
        if dk == dv == 128:
            run_saved(make_config(2), "streamed cfg2")
    finally:
        dn.deltanet_set_option(dn.DN_OPT_STREAMED_CHUNK_KERNEL, 0)
    with pytest.raises(dn.DeltaNetError):
        dn.deltanet_set_option(77, 1)
