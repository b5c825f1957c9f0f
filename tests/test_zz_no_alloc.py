"""The forward entry point that allocates nothing (deltanet_fwd_static: scratch from the library's own device array)
against deltanet_fwd on a caller-provided workspace and against the fp64 oracle, through the C ABI: two calls in a row,
the second with a smaller input, so that what the first call left in the array must not matter."""
import ctypes

import pytest
import torch

import oracle
import paper_2406_06484_amd as dn
from paper_2406_06484_amd.binding import _shape_of, load_library
from paper_2406_06484_amd.synth import make_inputs
from tests.gpu_util import check_tensors, dev_inputs

pytestmark = pytest.mark.gpu


def _static_fwd_raw(d):
    """deltanet_fwd_static called on the C symbol itself, every buffer allocated beforehand"""
    lib = load_library()
    keep = []
    s = _shape_of(d["q"], d["v"], d["cu"], 64, keep)
    o = torch.full_like(d["v"], float("nan"))
    N = s.num_seqs if d["cu"] is not None else s.B
    ST = torch.full((N, s.H, s.d_k, s.d_v), float("nan"), dtype=torch.float32, device="cuda")
    p = lambda t: ctypes.c_void_p(None if t is None else t.data_ptr())
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = lib.deltanet_fwd_static(ctypes.byref(s), p(d["q"]), p(d["k"]), p(d["v"]), p(d["beta"]), p(d["S0"]), p(o), p(ST),
                                 ctypes.c_void_p(torch.cuda.current_stream().cuda_stream or None))
    assert rc == 0, dn.deltanet_status_string(rc)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return o, ST


def test_static_scratch_forward_equals_the_workspace_forward_twice_in_a_row():
    big = make_inputs(91, B=3, L=700, H=4, dk=128, dv=128, dtype="bf16", with_initial_state=True)      # 11 chunks, the last ragged
    small = make_inputs(92, B=1, L=130, H=2, dk=128, dv=128, dtype="bf16")                              # fewer, smaller tiles
    packed = make_inputs(93, H=2, dk=64, dv=64, dtype="f32", with_initial_state=True,
                         cu_seqlens=__import__("numpy").array([0, 0, 5, 69, 199, 262], dtype="int32"))
    for inp, label in ((big, "static big"), (small, "static small after big"), (packed, "static packed fp32"), (big, "static big again")):
        d = dev_inputs(inp)
        o, ST = _static_fwd_raw(d)
        o_w, ST_w = dn.deltanet_fwd(d["q"], d["k"], d["v"], d["beta"], d["S0"], cu_seqlens=d["cu"])
        torch.cuda.synchronize()
        assert torch.equal(o, o_w) and torch.equal(ST, ST_w), label          # same kernels, same arithmetic
        o_ref, ST_ref = oracle.fwd(inp.q, inp.k, inp.v, inp.beta, inp.initial_state, inp.cu_seqlens)
        check_tensors([("o", o.float().cpu().numpy(), o_ref), ("final_state", ST.cpu().numpy(), ST_ref)], inp.dtype, label=label)


def test_static_scratch_forward_refuses_what_does_not_fit():
    lib = load_library()
    need, limit = ctypes.c_size_t(0), 36 << 20
    q = torch.zeros((8, 4096, 16, 128), dtype=torch.bfloat16, device="cuda")     # twice the tokens the array covers
    s = _shape_of(q, q, None, 64, [])
    assert lib.deltanet_workspace_bytes(ctypes.byref(s), 0, ctypes.byref(need)) == 0 and need.value > limit
    with pytest.raises(dn.DeltaNetError) as ei:
        dn.deltanet_fwd_static(q, q, q, q[..., 0].contiguous(), o=q.clone())
    assert ei.value.status == -5
    # the binding's own entry: the largest bf16 batch that fits, 16 384 tokens x 16 heads
    ok = make_inputs(94, B=2, L=512, H=16, dk=128, dv=128, dtype="bf16")
    d = dev_inputs(ok)
    o, ST = dn.deltanet_fwd_static(d["q"], d["k"], d["v"], d["beta"])
    o_w, ST_w = dn.deltanet_fwd(d["q"], d["k"], d["v"], d["beta"])
    assert torch.equal(o, o_w) and torch.equal(ST, ST_w)
