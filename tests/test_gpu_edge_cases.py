"""GPU edge cases of the C ABI: passes over no tokens at all, gradients written in place, and packed offsets that
no host copy was there to validate."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2406_06484_amd as dn
from paper_2406_06484_amd.binding import _shape_of, deltanet_workspace_bytes, load_library
from paper_2406_06484_amd.synth import make_inputs
from tests.gpu_util import dev_inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128), ("bf16", 256)])
def test_no_tokens_at_all_passes_the_state_through(dtype, d):
    """The recurrence over zero tokens leaves the state as it was (section 2.2): final_state = initial_state (zero
    without one), and the gradient passes through the other way."""
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    H = 2
    S0 = torch.randn(2, H, d, d, device="cuda")
    dST = torch.randn(2, H, d, d, device="cuda")
    # dense, L = 0
    z = lambda *shape: torch.zeros(shape, dtype=tdt, device="cuda")
    q, v, beta = z(2, 0, H, d), z(2, 0, H, d), z(2, 0, H)
    for fwd in (dn.deltanet_fwd, dn.deltanet_fwd_save):
        poison = torch.full((2, H, d, d), float("nan"), device="cuda")
        out = fwd(q, q, v, beta, S0, final_state=poison)
        assert torch.equal(out[1], S0) and out[0].numel() == 0
        poison = torch.full((2, H, d, d), float("nan"), device="cuda")
        out = fwd(q, q, v, beta, None, final_state=poison)
        assert torch.equal(out[1], torch.zeros_like(S0))
    g = dn.deltanet_bwd(q, q, v, beta, v, S0, dST)
    assert torch.equal(g[4], dST) and all(t.numel() == 0 for t in g[:4])
    # packed, every sequence empty
    cu = torch.zeros(3, dtype=torch.int32, device="cuda")
    q, v, beta = z(0, H, d), z(0, H, d), z(0, H)
    poison = torch.full((2, H, d, d), float("nan"), device="cuda")
    o, ST = dn.deltanet_fwd(q, q, v, beta, S0, cu_seqlens=cu, final_state=poison)
    assert torch.equal(ST, S0)
    g = dn.deltanet_bwd(q, q, v, beta, v, S0, dST, cu_seqlens=cu)
    assert torch.equal(g[4], dST)
    o, ST = dn.deltanet_recurrent_fwd(q, q, v, beta, S0, cu_seqlens=cu)
    assert torch.equal(ST, S0)


def test_gradients_written_in_place_equal_the_returned_ones():
    inp = make_inputs(61, B=2, L=150, H=2, dk=128, dv=128, dtype="bf16", with_initial_state=True, with_dfinal_state=True)
    d = dev_inputs(inp)
    ref = dn.deltanet_bwd(d["q"], d["k"], d["v"], d["beta"], d["d_o"], d["S0"], d["dST"])
    ws = torch.empty(deltanet_workspace_bytes(_shape_of(d["q"], d["v"], None, 64, []), True), dtype=torch.uint8, device="cuda")
    outs = dict(dq=torch.empty_like(d["q"]), dk=torch.empty_like(d["k"]), dv=torch.empty_like(d["v"]),
                dbeta=torch.empty(d["beta"].shape, dtype=torch.float32, device="cuda"), dinitial_state=torch.empty_like(d["S0"]))
    got = dn.deltanet_bwd(d["q"], d["k"], d["v"], d["beta"], d["d_o"], d["S0"], d["dST"], workspace=ws, **outs)
    for a, b, name in zip(got, ref, outs):
        assert a.data_ptr() == outs[name].data_ptr() and torch.equal(a, b), name
    with pytest.raises(ValueError):
        dn.deltanet_bwd(d["q"], d["k"], d["v"], d["beta"], d["d_o"], dq=torch.empty(3, device="cuda", dtype=torch.bfloat16))


def test_packed_offsets_without_a_host_copy_stay_in_bounds():
    """When the caller hands over no host copy of cu_seqlens the library cannot reject a malformed array; the kernels then
    work on its running maximum held inside [0, L], so every access stays inside the tensors and the workspace.  A valid
    array gives the same results with and without the host copy; a malformed one returns DN_OK and leaves finite numbers."""
    lib = load_library()
    H, dk, T = 2, 128, 520
    cu_good = np.array([0, 0, 5, 69, 199, 262, 263, 263, 520], dtype=np.int32)
    inp = make_inputs(7, H=H, dk=dk, dv=dk, dtype="bf16", cu_seqlens=cu_good, with_initial_state=True, with_dfinal_state=True)
    d = dev_inputs(inp)
    want_o, want_S = dn.deltanet_fwd(d["q"], d["k"], d["v"], d["beta"], d["S0"], cu_seqlens=d["cu"])
    want_g = dn.deltanet_bwd(d["q"], d["k"], d["v"], d["beta"], d["d_o"], d["S0"], d["dST"], cu_seqlens=d["cu"])

    def raw_call(cu_dev):
        keep = []
        s = _shape_of(d["q"], d["v"], cu_dev, 64, keep, cu_host=cu_good)
        s.cu_seqlens_host = None   # no host copy: nothing is validated
        ws = torch.empty(deltanet_workspace_bytes(s, True), dtype=torch.uint8, device="cuda")
        o, ST = torch.zeros_like(d["v"]), torch.zeros_like(d["S0"])
        p = lambda t: ctypes.c_void_p(t.data_ptr())
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream or None)
        rc = lib.deltanet_fwd(ctypes.byref(s), p(d["q"]), p(d["k"]), p(d["v"]), p(d["beta"]), p(d["S0"]), p(o), p(ST), p(ws),
                              ws.numel(), stream)
        assert rc == 0
        g = [torch.zeros_like(d["q"]), torch.zeros_like(d["k"]), torch.zeros_like(d["v"]),
             torch.zeros(d["beta"].shape, dtype=torch.float32, device="cuda"), torch.zeros_like(d["S0"])]
        rc = lib.deltanet_bwd(ctypes.byref(s), p(d["q"]), p(d["k"]), p(d["v"]), p(d["beta"]), p(d["S0"]), p(d["d_o"]), p(d["dST"]),
                              *[p(t) for t in g], p(ws), ws.numel(), stream)
        assert rc == 0
        torch.cuda.synchronize()
        return o, ST, g

    o, ST, g = raw_call(d["cu"])
    assert torch.equal(o, want_o) and torch.equal(ST, want_S)
    for a, b in zip(g, want_g):
        assert torch.equal(a, b)
    # decreasing, negative and beyond-the-end entries: bounded to [0, 0, 69, 69, 199, 262, 263, 520, 520]
    bad = torch.tensor([0, -7, 69, 5, 199, 262, 263, 9999, 520], dtype=torch.int32, device="cuda")
    o, ST, g = raw_call(bad)
    assert all(bool(torch.isfinite(t.float()).all()) for t in [o, ST] + g)
    bounded = torch.tensor([0, 0, 69, 69, 199, 262, 263, 520, 520], dtype=torch.int32, device="cuda")
    o2, ST2, g2 = raw_call(bounded)
    assert torch.equal(o, o2) and torch.equal(ST, ST2) and all(torch.equal(a, b) for a, b in zip(g, g2))


def test_lds_probe_launches_every_pattern_and_rejects_unknown_ones():
    """The measurement aid deltanet_lds_probe: every documented pattern launches and finishes; a pattern outside the list
    and a repeat count outside the documented range are refused before any launch."""
    for pattern in range(18):
        dn.deltanet_lds_probe(pattern, 3)
    torch.cuda.synchronize()
    with pytest.raises(dn.DeltaNetError):
        dn.deltanet_lds_probe(18, 3)
    with pytest.raises(dn.DeltaNetError):
        dn.deltanet_lds_probe(0, -1)
