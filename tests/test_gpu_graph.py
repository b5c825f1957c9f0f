"""The library allocates nothing and launches only on the caller's stream, so a training step can be captured
into a HIP graph: every replay must reproduce the eager results bit for bit, with eager work in between."""
import numpy as np
import pytest
import torch

import paper_2406_06484_amd as dn
from paper_2406_06484_amd.synth import make_inputs
from tests.gpu_util import dev_inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", ["dense bf16 d=128", "packed f32 d=64", "packed f32 d=64, host copy of cu_seqlens", "dense bf16 d=256"])
def test_captured_step_replays_bit_exactly(case):
    if case == "dense bf16 d=128":
        inp = make_inputs(41, B=2, L=300, H=2, dk=128, dv=128, dtype="bf16", with_initial_state=True, with_dfinal_state=True)
    elif case.startswith("packed f32 d=64"):
        cu = np.array([0, 0, 5, 69, 199, 262, 263, 263, 520], dtype=np.int32)
        inp = make_inputs(42, H=2, dk=64, dv=64, dtype="f32", cu_seqlens=cu, with_initial_state=True, with_dfinal_state=True)
    else:
        inp = make_inputs(43, B=1, L=200, H=2, dk=256, dv=256, dtype="bf16", with_dfinal_state=True)
    d = dev_inputs(inp)
    # packed batches: the binding validates cu_seqlens on the host; under capture it cannot copy them back, so it either
    # gets the caller's host copy or skips the check
    host = inp.cu_seqlens if "host copy" in case else None
    _, _, saved = dn.deltanet_fwd_save(d["q"], d["k"], d["v"], d["beta"], d["S0"], cu_seqlens=d["cu"])
    o = torch.empty_like(d["v"])
    N = len(inp.cu_seqlens) - 1 if inp.cu_seqlens is not None else inp.q.shape[0]
    ST = torch.empty((N,) + tuple(inp.q.shape[-2:]) + (inp.v.shape[-1],), dtype=torch.float32, device="cuda")

    def step():
        dn.deltanet_fwd_save(d["q"], d["k"], d["v"], d["beta"], d["S0"], cu_seqlens=d["cu"], cu_seqlens_host=host, o=o,
                             final_state=ST, saved=saved)
        return dn.deltanet_bwd_saved(d["q"], d["k"], d["v"], d["beta"], d["d_o"], saved, d["dST"], cu_seqlens=d["cu"],
                                     cu_seqlens_host=host)

    want = [t.clone() for t in step() if t is not None]
    want_o, want_ST = o.clone(), ST.clone()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()   # warm-up on the capture stream, as torch asks for
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        outs = [t for t in step() if t is not None]
    for replay in range(3):
        for t in outs + [o, ST]:
            t.zero_()
        saved.random_(0, 255)            # the buffer is rebuilt by the captured forward pass
        dn.deltanet_fwd(d["q"], d["k"], d["v"], d["beta"], cu_seqlens=d["cu"])   # eager work of the library between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, want_o) and torch.equal(ST, want_ST), (case, replay)
        for a, b in zip(outs, want):
            assert torch.equal(a, b), (case, replay)
