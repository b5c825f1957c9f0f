"""ctypes binding of ``libdeltanet_hip.so`` (declared in ``include/deltanet.h``).

Argument marshalling only: every step of the DeltaNet forward/backward runs in the HIP kernels.
PyTorch supplies device memory and the stream.  There is no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdeltanet_hip.so")
_lib = None

DN_F32, DN_BF16 = 0, 1


class DeltaNetError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__("deltanet: %s (status %d)" % (msg, status))
        self.status = status


class dn_shape(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("L", ctypes.c_int32), ("H", ctypes.c_int32),
        ("d_k", ctypes.c_int32), ("d_v", ctypes.c_int32), ("chunk", ctypes.c_int32),
        ("dtype", ctypes.c_int32), ("num_seqs", ctypes.c_int32),
        ("cu_seqlens", ctypes.c_void_p), ("cu_seqlens_host", ctypes.c_void_p),
    ]


class dn_kernel_time(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 96), ("total_ms", ctypes.c_double), ("launches", ctypes.c_int32)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the HIP library; raises if it has not been built (run ``__graft_entry__.build()``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                "%s is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`; "
                "there is no CPU fallback" % _LIB_PATH)
        lib = ctypes.CDLL(_LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        sp = ctypes.POINTER(dn_shape)
        lib.deltanet_workspace_bytes.restype = ctypes.c_int
        lib.deltanet_workspace_bytes.argtypes = [sp, ctypes.c_int, ctypes.POINTER(sz)]
        lib.deltanet_fwd.restype = ctypes.c_int
        lib.deltanet_fwd.argtypes = [sp] + [vp] * 7 + [vp, sz, vp]
        lib.deltanet_bwd.restype = ctypes.c_int
        lib.deltanet_bwd.argtypes = [sp] + [vp] * 12 + [vp, sz, vp]
        lib.deltanet_fwd_save.restype = ctypes.c_int
        lib.deltanet_fwd_save.argtypes = [sp] + [vp] * 7 + [vp, sz, vp]
        lib.deltanet_bwd_saved.restype = ctypes.c_int
        lib.deltanet_bwd_saved.argtypes = [sp] + [vp] * 11 + [vp, sz, vp]
        lib.deltanet_gated_fwd_save.restype = ctypes.c_int
        lib.deltanet_gated_fwd_save.argtypes = [sp] + [vp] * 8 + [vp, sz, vp]
        lib.deltanet_gated_bwd_saved.restype = ctypes.c_int
        lib.deltanet_gated_bwd_saved.argtypes = [sp] + [vp] * 13 + [vp, sz, vp]
        for name in ("deltanet_fused_fwd", "deltanet_fused_fwd_save"):
            getattr(lib, name).restype = ctypes.c_int
            getattr(lib, name).argtypes = [sp] + [vp] * 7 + [vp, sz, vp]
        lib.deltanet_fused_bwd.restype = ctypes.c_int
        lib.deltanet_fused_bwd.argtypes = [sp] + [vp] * 12 + [vp, sz, vp]
        lib.deltanet_fused_bwd_saved.restype = ctypes.c_int
        lib.deltanet_fused_bwd_saved.argtypes = [sp] + [vp] * 11 + [vp, sz, vp]
        lib.deltanet_fwd_static.restype = ctypes.c_int
        lib.deltanet_fwd_static.argtypes = [sp] + [vp] * 7 + [vp]
        lib.deltanet_recurrent_fwd.restype = ctypes.c_int
        lib.deltanet_recurrent_fwd.argtypes = [sp] + [vp] * 7 + [vp]
        lib.deltanet_gated_workspace_bytes.restype = ctypes.c_int
        lib.deltanet_gated_workspace_bytes.argtypes = [sp, ctypes.c_int, ctypes.POINTER(sz)]
        lib.deltanet_fused_workspace_bytes.restype = ctypes.c_int
        lib.deltanet_fused_workspace_bytes.argtypes = [sp, ctypes.c_int, ctypes.POINTER(sz)]
        lib.deltanet_gated_fwd.restype = ctypes.c_int
        lib.deltanet_gated_fwd.argtypes = [sp] + [vp] * 8 + [vp, sz, vp]
        lib.deltanet_gated_bwd.restype = ctypes.c_int
        lib.deltanet_gated_bwd.argtypes = [sp] + [vp] * 14 + [vp, sz, vp]
        lib.deltanet_gated_recurrent_fwd.restype = ctypes.c_int
        lib.deltanet_gated_recurrent_fwd.argtypes = [sp] + [vp] * 8 + [vp]
        lib.deltanet_set_option.restype = ctypes.c_int
        lib.deltanet_set_option.argtypes = [ctypes.c_int, ctypes.c_int]
        lib.deltanet_lds_probe.restype = ctypes.c_int
        lib.deltanet_lds_probe.argtypes = [ctypes.c_int, ctypes.c_int, vp]
        lib.deltanet_profile_enable.restype = ctypes.c_int
        lib.deltanet_profile_enable.argtypes = [ctypes.c_int]
        lib.deltanet_profile_collect.restype = ctypes.c_int
        lib.deltanet_profile_collect.argtypes = [ctypes.POINTER(dn_kernel_time), ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        lib.deltanet_status_string.restype = ctypes.c_char_p
        lib.deltanet_status_string.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def deltanet_status_string(status: int) -> str:
    return load_library().deltanet_status_string(int(status)).decode()


DN_OPT_STREAMED_CHUNK_KERNEL = 0


def deltanet_set_option(option: int, value: int) -> None:
    """Process-wide option of the library (see include/deltanet.h)."""
    _check(load_library().deltanet_set_option(int(option), int(value)))


def deltanet_lds_probe(pattern: int, iters: int) -> None:
    """Measurement aid: one launch of the probe kernel for LDS access pattern `pattern` (see include/deltanet.h)."""
    _check(load_library().deltanet_lds_probe(int(pattern), int(iters), ctypes.c_void_p(_stream(None))))


def deltanet_profile_enable(on: bool) -> None:
    _check(load_library().deltanet_profile_enable(int(bool(on))))


def deltanet_profile_collect(max_entries: int = 32) -> dict:
    """{kernel name: (total_ms, launches)} since profiling was enabled or last collected."""
    buf = (dn_kernel_time * max_entries)()
    n = ctypes.c_int(0)
    _check(load_library().deltanet_profile_collect(buf, max_entries, ctypes.byref(n)))
    return {buf[i].name.decode(): (buf[i].total_ms, buf[i].launches) for i in range(n.value)}


def _check(status: int):
    if status != 0:
        raise DeltaNetError(status, deltanet_status_string(status))


def _dt(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return DN_F32
    if t.dtype == torch.bfloat16:
        return DN_BF16
    raise TypeError("q/k/v/beta must be float32 or bfloat16, got %s" % t.dtype)


def _shape_of(q, v, cu_seqlens, chunk, cu_host_keepalive, cu_host=None):
    """cu_host: the caller's host copy of cu_seqlens (int32), which the library validates; without one the device
    tensor is copied back for that, except under stream capture, where no copy may run and validation is skipped."""
    import numpy as np
    import torch
    s = dn_shape()
    if cu_seqlens is None:
        if q.dim() != 4:
            raise ValueError("dense q must be [B, L, H, d_k]")
        s.B, s.L, s.H, s.d_k = q.shape
        s.num_seqs = 0
        s.cu_seqlens = None
        s.cu_seqlens_host = None
    else:
        if q.dim() != 3:
            raise ValueError("packed q must be [T, H, d_k]")
        s.B = 1
        s.L, s.H, s.d_k = q.shape
        s.num_seqs = cu_seqlens.numel() - 1
        s.cu_seqlens = cu_seqlens.data_ptr()
        if cu_host is not None:
            host = np.ascontiguousarray(np.asarray(cu_host, dtype=np.int32))
            if host.shape != (s.num_seqs + 1,):
                raise ValueError("cu_seqlens_host must have the shape of cu_seqlens")
        elif torch.cuda.is_current_stream_capturing():
            host = None
        else:
            host = np.ascontiguousarray(cu_seqlens.cpu().numpy().astype(np.int32))
        cu_host_keepalive.append(host)
        s.cu_seqlens_host = host.ctypes.data if host is not None else None
    s.d_v = v.shape[-1]
    s.chunk = chunk
    s.dtype = _dt(q)
    return s


def _p(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _req(t, name, dtype=None, shape=None):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("%s must be a contiguous device tensor" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s" % (name, dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))


def deltanet_workspace_bytes(shape: dn_shape, want_bwd: bool) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().deltanet_workspace_bytes(ctypes.byref(shape), int(bool(want_bwd)), ctypes.byref(out)))
    return int(out.value)


def deltanet_gated_workspace_bytes(shape: dn_shape, want_bwd: bool) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().deltanet_gated_workspace_bytes(ctypes.byref(shape), int(bool(want_bwd)), ctypes.byref(out)))
    return int(out.value)


def deltanet_fused_workspace_bytes(shape: dn_shape, want_bwd: bool) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().deltanet_fused_workspace_bytes(ctypes.byref(shape), int(bool(want_bwd)), ctypes.byref(out)))
    return int(out.value)


def _workspace(shape, want_bwd, workspace, device, gated=False, pro=False):
    import torch
    query = deltanet_fused_workspace_bytes if pro else (deltanet_gated_workspace_bytes if gated else deltanet_workspace_bytes)
    need = query(shape, want_bwd)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=device)
    return workspace, workspace.numel() * workspace.element_size()


def deltanet_fwd(q, k, v, beta, initial_state=None, *, cu_seqlens=None, cu_seqlens_host=None, chunk: int = 64,
                 output_final_state: bool = True, o=None, final_state=None, workspace=None,
                 stream=None, _g=None, _save=False, _pro=False) -> Tuple["torch.Tensor", Optional["torch.Tensor"]]:
    """Forward pass of the DeltaNet layer on the GPU; returns (o, final_state or None).  Packed batches: pass
    cu_seqlens_host (the int32 offsets on the host) as well, or the device tensor is copied back for validation on
    every call, which waits for the device."""
    import torch
    lib = load_library()
    keep = []
    if _g is not None:
        _req(_g, "g", torch.float32, beta.shape)
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (beta, "beta")):
        _req(t, n, q.dtype)
    s = _shape_of(q, v, cu_seqlens, chunk, keep, cu_seqlens_host)
    _req(k, "k", shape=q.shape); _req(v, "v", shape=tuple(q.shape[:-1]) + (s.d_v,))
    _req(beta, "beta", shape=q.shape[:-1])
    N = s.num_seqs if cu_seqlens is not None else s.B
    st_shape = (N, s.H, s.d_k, s.d_v)
    if initial_state is not None:
        _req(initial_state, "initial_state", torch.float32, st_shape)
    if o is None:
        o = torch.empty_like(v)
    _req(o, "o", q.dtype, v.shape)
    if final_state is None and output_final_state:
        final_state = torch.empty(st_shape, dtype=torch.float32, device=q.device)
    if final_state is not None:
        _req(final_state, "final_state", torch.float32, st_shape)
    workspace, wbytes = _workspace(s, _save, workspace, q.device, _g is not None, _pro)
    if _g is None:
        if _pro:
            fn = lib.deltanet_fused_fwd_save if _save else lib.deltanet_fused_fwd
        else:
            fn = lib.deltanet_fwd_save if _save else lib.deltanet_fwd
        _check(fn(ctypes.byref(s), _p(q), _p(k), _p(v), _p(beta), _p(initial_state), _p(o),
                  _p(final_state), _p(workspace), wbytes, _stream(stream)))
    else:
        fn = lib.deltanet_gated_fwd_save if _save else lib.deltanet_gated_fwd
        _check(fn(ctypes.byref(s), _p(q), _p(k), _p(v), _p(beta), _p(_g), _p(initial_state), _p(o),
                  _p(final_state), _p(workspace), wbytes, _stream(stream)))
    if _save:
        return o, final_state, workspace
    return o, final_state


def deltanet_fwd_static(q, k, v, beta, initial_state=None, *, cu_seqlens=None, cu_seqlens_host=None, chunk: int = 64,
                        output_final_state: bool = True, o=None, final_state=None, stream=None):
    """deltanet_fwd on the library's own scratch array instead of a workspace (for callers that cannot allocate: pass
    o and final_state in, and the call allocates nothing); returns (o, final_state or None)."""
    import torch
    lib = load_library()
    keep = []
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (beta, "beta")):
        _req(t, n, q.dtype)
    s = _shape_of(q, v, cu_seqlens, chunk, keep, cu_seqlens_host)
    _req(k, "k", shape=q.shape); _req(v, "v", shape=tuple(q.shape[:-1]) + (s.d_v,))
    _req(beta, "beta", shape=q.shape[:-1])
    N = s.num_seqs if cu_seqlens is not None else s.B
    st_shape = (N, s.H, s.d_k, s.d_v)
    if initial_state is not None:
        _req(initial_state, "initial_state", torch.float32, st_shape)
    if o is None:
        o = torch.empty_like(v)
    _req(o, "o", q.dtype, v.shape)
    if final_state is None and output_final_state:
        final_state = torch.empty(st_shape, dtype=torch.float32, device=q.device)
    if final_state is not None:
        _req(final_state, "final_state", torch.float32, st_shape)
    _check(lib.deltanet_fwd_static(ctypes.byref(s), _p(q), _p(k), _p(v), _p(beta), _p(initial_state), _p(o), _p(final_state),
                                   _stream(stream)))
    return o, final_state


def deltanet_fwd_save(q, k, v, beta, initial_state=None, *, saved=None, **kw):
    """Forward pass that keeps its per-chunk results for deltanet_bwd_saved; returns (o, final_state or None, saved).
    ``saved`` (optional) is a uint8 device tensor of deltanet_workspace_bytes(shape, True) bytes to reuse."""
    return deltanet_fwd(q, k, v, beta, initial_state, workspace=saved, _save=True, **kw)


def deltanet_gated_fwd_save(q, k, v, beta, g, initial_state=None, *, saved=None, **kw):
    """Gated forward pass that keeps its per-chunk results; returns (o, final_state or None, saved)."""
    return deltanet_fwd(q, k, v, beta, initial_state, workspace=saved, _save=True, _g=g, **kw)


def deltanet_gated_fwd(q, k, v, beta, g, initial_state=None, **kw):
    """Forward pass of the gated variant (decay exp(g) per token and head, g fp32); returns (o, final_state or None)."""
    return deltanet_fwd(q, k, v, beta, initial_state, _g=g, **kw)


def deltanet_recurrent_fwd(q, k, v, beta, initial_state=None, *, cu_seqlens=None, output_final_state: bool = True,
                           o=None, final_state=None, stream=None, _g=None):
    """Token-serial forward on the GPU (decode steps, and the baseline of the chunkwise form); returns (o, final_state or None)."""
    import torch
    lib = load_library()
    keep = []
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (beta, "beta")):
        _req(t, n, q.dtype)
    s = _shape_of(q, v, cu_seqlens, 64, keep)
    _req(k, "k", shape=q.shape); _req(v, "v", shape=tuple(q.shape[:-1]) + (s.d_v,))
    _req(beta, "beta", shape=q.shape[:-1])
    N = s.num_seqs if cu_seqlens is not None else s.B
    st_shape = (N, s.H, s.d_k, s.d_v)
    if initial_state is not None:
        _req(initial_state, "initial_state", torch.float32, st_shape)
    if o is None:
        o = torch.empty_like(v)
    _req(o, "o", q.dtype, v.shape)
    if final_state is None and output_final_state:
        final_state = torch.empty(st_shape, dtype=torch.float32, device=q.device)
    if final_state is not None:
        _req(final_state, "final_state", torch.float32, st_shape)
    if _g is None:
        _check(lib.deltanet_recurrent_fwd(ctypes.byref(s), _p(q), _p(k), _p(v), _p(beta), _p(initial_state), _p(o),
                                          _p(final_state), _stream(stream)))
    else:
        _req(_g, "g", torch.float32, beta.shape)
        _check(lib.deltanet_gated_recurrent_fwd(ctypes.byref(s), _p(q), _p(k), _p(v), _p(beta), _p(_g), _p(initial_state),
                                                _p(o), _p(final_state), _stream(stream)))
    return o, final_state


def deltanet_gated_recurrent_fwd(q, k, v, beta, g, initial_state=None, **kw):
    """Token-serial forward of the gated variant; returns (o, final_state or None)."""
    return deltanet_recurrent_fwd(q, k, v, beta, initial_state, _g=g, **kw)


def deltanet_bwd(q, k, v, beta, d_o, initial_state=None, dfinal_state=None, *, cu_seqlens=None, cu_seqlens_host=None,
                 chunk: int = 64, want_dinitial_state: bool = True, workspace=None, stream=None, dq=None, dk=None, dv=None,
                 dbeta=None, dinitial_state=None, dg=None, _g=None, _saved=False, _pro=False):
    """Backward pass; returns (dq, dk, dv, dbeta[fp32], dinitial_state[fp32] or None).  dq, dk, dv, dbeta,
    dinitial_state (and dg of the gated variant) may be passed in to be written in place; a call that is given all of
    them and a workspace allocates nothing.  Packed batches: pass cu_seqlens_host (the int32 offsets on the host) as
    well, or the device tensor is copied back for validation on every call, which waits for the device."""
    import torch
    lib = load_library()
    keep = []
    if _g is not None:
        _req(_g, "g", torch.float32, beta.shape)
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (beta, "beta"), (d_o, "d_o")):
        _req(t, n, q.dtype)
    s = _shape_of(q, v, cu_seqlens, chunk, keep, cu_seqlens_host)
    _req(k, "k", shape=q.shape); _req(v, "v", shape=tuple(q.shape[:-1]) + (s.d_v,))
    _req(beta, "beta", shape=q.shape[:-1]); _req(d_o, "d_o", shape=v.shape)
    N = s.num_seqs if cu_seqlens is not None else s.B
    st_shape = (N, s.H, s.d_k, s.d_v)
    for t, n in ((initial_state, "initial_state"), (dfinal_state, "dfinal_state")):
        if t is not None:
            _req(t, n, torch.float32, st_shape)
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    dbeta = torch.empty(beta.shape, dtype=torch.float32, device=q.device) if dbeta is None else dbeta
    dS0 = dinitial_state
    if dS0 is None and want_dinitial_state:
        dS0 = torch.empty(st_shape, dtype=torch.float32, device=q.device)
    _req(dq, "dq", q.dtype, q.shape); _req(dk, "dk", q.dtype, q.shape); _req(dv, "dv", q.dtype, v.shape)
    _req(dbeta, "dbeta", torch.float32, beta.shape)
    if dS0 is not None:
        _req(dS0, "dinitial_state", torch.float32, st_shape)
    if _saved and workspace is None:
        raise ValueError("saved must be the buffer returned by the matching forward call")
    workspace, wbytes = _workspace(s, True, workspace, q.device, _g is not None, _pro)
    if _saved and _g is None:
        fn = lib.deltanet_fused_bwd_saved if _pro else lib.deltanet_bwd_saved
        _check(fn(ctypes.byref(s), _p(q), _p(k), _p(v), _p(beta), _p(d_o), _p(dfinal_state),
                                      _p(dq), _p(dk), _p(dv), _p(dbeta), _p(dS0), _p(workspace), wbytes, _stream(stream)))
        return dq, dk, dv, dbeta, dS0
    if _g is None:
        fn = lib.deltanet_fused_bwd if _pro else lib.deltanet_bwd
        _check(fn(ctypes.byref(s), _p(q), _p(k), _p(v), _p(beta), _p(initial_state), _p(d_o),
                                _p(dfinal_state), _p(dq), _p(dk), _p(dv), _p(dbeta), _p(dS0), _p(workspace),
                                wbytes, _stream(stream)))
        return dq, dk, dv, dbeta, dS0
    dg = torch.empty(beta.shape, dtype=torch.float32, device=q.device) if dg is None else dg
    _req(dg, "dg", torch.float32, beta.shape)
    if _saved:
        _check(lib.deltanet_gated_bwd_saved(ctypes.byref(s), _p(q), _p(k), _p(v), _p(beta), _p(_g), _p(d_o),
                                            _p(dfinal_state), _p(dq), _p(dk), _p(dv), _p(dbeta), _p(dg), _p(dS0),
                                            _p(workspace), wbytes, _stream(stream)))
        return dq, dk, dv, dbeta, dg, dS0
    _check(lib.deltanet_gated_bwd(ctypes.byref(s), _p(q), _p(k), _p(v), _p(beta), _p(_g), _p(initial_state), _p(d_o),
                                  _p(dfinal_state), _p(dq), _p(dk), _p(dv), _p(dbeta), _p(dg), _p(dS0), _p(workspace),
                                  wbytes, _stream(stream)))
    return dq, dk, dv, dbeta, dg, dS0


def deltanet_gated_bwd(q, k, v, beta, g, d_o, initial_state=None, dfinal_state=None, **kw):
    """Backward pass of the gated variant; returns (dq, dk, dv, dbeta, dg, dinitial_state or None), dbeta and dg in fp32."""
    return deltanet_bwd(q, k, v, beta, d_o, initial_state, dfinal_state, _g=g, **kw)


def deltanet_bwd_saved(q, k, v, beta, d_o, saved, dfinal_state=None, **kw):
    """Backward pass from the buffer deltanet_fwd_save left for the same inputs; returns what deltanet_bwd returns."""
    return deltanet_bwd(q, k, v, beta, d_o, None, dfinal_state, workspace=saved, _saved=True, **kw)


def deltanet_gated_bwd_saved(q, k, v, beta, g, d_o, saved, dfinal_state=None, **kw):
    """Gated backward pass from the buffer deltanet_gated_fwd_save left; returns what deltanet_gated_bwd returns."""
    return deltanet_bwd(q, k, v, beta, d_o, None, dfinal_state, workspace=saved, _saved=True, _g=g, **kw)


def deltanet_fused_fwd(q_pre, k_pre, v, beta_logit, initial_state=None, **kw):
    """Forward pass with the layer's prologue in the load path: q, k = SiLU(x) / ||SiLU(x)||_2 of the given
    pre-activations, beta = sigmoid(beta_logit); returns (o, final_state or None)."""
    return deltanet_fwd(q_pre, k_pre, v, beta_logit, initial_state, _pro=True, **kw)


def deltanet_fused_bwd(q_pre, k_pre, v, beta_logit, d_o, initial_state=None, dfinal_state=None, **kw):
    """Backward pass of deltanet_fused_fwd; returns (dq_pre, dk_pre, dv, dbeta_logit[fp32], dinitial_state or None)."""
    return deltanet_bwd(q_pre, k_pre, v, beta_logit, d_o, initial_state, dfinal_state, _pro=True, **kw)


def deltanet_fused_fwd_save(q_pre, k_pre, v, beta_logit, initial_state=None, *, saved=None, **kw):
    """deltanet_fused_fwd that keeps its per-chunk results; returns (o, final_state or None, saved)."""
    return deltanet_fwd(q_pre, k_pre, v, beta_logit, initial_state, workspace=saved, _save=True, _pro=True, **kw)


def deltanet_fused_bwd_saved(q_pre, k_pre, v, beta_logit, d_o, saved, dfinal_state=None, **kw):
    """Backward pass from the buffer deltanet_fused_fwd_save left; returns what deltanet_fused_bwd returns."""
    return deltanet_bwd(q_pre, k_pre, v, beta_logit, d_o, None, dfinal_state, workspace=saved, _saved=True, _pro=True, **kw)
