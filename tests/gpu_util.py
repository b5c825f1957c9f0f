"""Helpers for the GPU parity tests: move seeded inputs to the device, call the C ABI through the
binding, run the fp64 oracle on the same (already rounded) values, and compare."""
import numpy as np
import torch

import oracle
import paper_2406_06484_amd as dn

# "max relative error" of a tensor: max_i |x_i - ref_i| / max_i |ref_i|  (normalised max error)
TOL = {"f32": 1e-4, "bf16": 2e-2}


def nerr(x, ref):
    x = np.asarray(x, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    assert x.shape == ref.shape, (x.shape, ref.shape)
    assert np.all(np.isfinite(x)), "non-finite values in GPU output"
    den = np.max(np.abs(ref)) if ref.size else 1.0
    return float(np.max(np.abs(x - ref)) / den) if den > 0 else float(np.max(np.abs(x)))


def to_dev(a, dtype):
    if a is None:
        return None
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.float32).to(tdt).cuda().contiguous()


def dev_inputs(inp):
    d = {n: to_dev(getattr(inp, n), inp.dtype) for n in ("q", "k", "v", "beta", "d_o")}
    d["S0"] = to_dev(inp.initial_state, "f32")
    d["dST"] = to_dev(inp.dfinal_state, "f32")
    d["cu"] = None if inp.cu_seqlens is None else torch.from_numpy(inp.cu_seqlens).cuda()
    return d


def gpu_fwd(inp, d=None):
    d = d or dev_inputs(inp)
    o, ST = dn.deltanet_fwd(d["q"], d["k"], d["v"], d["beta"], d["S0"], cu_seqlens=d["cu"])
    torch.cuda.synchronize()
    return o.float().cpu().numpy(), ST.cpu().numpy()


def gpu_bwd(inp, d=None):
    d = d or dev_inputs(inp)
    out = dn.deltanet_bwd(d["q"], d["k"], d["v"], d["beta"], d["d_o"], d["S0"], d["dST"], cu_seqlens=d["cu"])
    torch.cuda.synchronize()
    return [t.float().cpu().numpy() for t in out]


def check_fwd_bwd(inp, tol=None, bwd=True, label=""):
    tol = tol or TOL[inp.dtype]
    o, ST = gpu_fwd(inp)
    o_ref, ST_ref = oracle.fwd(inp.q, inp.k, inp.v, inp.beta, inp.initial_state, inp.cu_seqlens)
    errs = {"o": nerr(o, o_ref), "final_state": nerr(ST, ST_ref)}
    if bwd:
        g = gpu_bwd(inp)
        g_ref = oracle.bwd(inp.q, inp.k, inp.v, inp.beta, inp.d_o, inp.initial_state, inp.dfinal_state, inp.cu_seqlens)
        for name, a, b in zip(("dq", "dk", "dv", "dbeta", "dinitial_state"), g, g_ref):
            errs[name] = nerr(a, b)
    print(label, " ".join("%s=%.2e" % kv for kv in errs.items()), flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, "normalised max error above %g: %s" % (tol, bad)
    return errs
