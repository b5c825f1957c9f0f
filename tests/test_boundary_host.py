"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2406_06484_amd", "libdeltanet_hip.so")
pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="library not built (run __graft_entry__.build())")


def header_symbols():
    text = open(os.path.join(ROOT, "include", "deltanet.h")).read()
    return sorted(set(re.findall(r"\b(deltanet_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(LIB)
    syms = header_symbols()
    assert {"deltanet_fwd", "deltanet_bwd", "deltanet_recurrent_fwd", "deltanet_workspace_bytes",
            "deltanet_gated_fwd", "deltanet_gated_bwd", "deltanet_gated_recurrent_fwd",
            "deltanet_gated_workspace_bytes", "deltanet_status_string", "deltanet_fwd_save", "deltanet_bwd_saved",
            "deltanet_gated_fwd_save", "deltanet_gated_bwd_saved", "deltanet_fused_fwd", "deltanet_fused_bwd",
            "deltanet_fused_fwd_save", "deltanet_fused_bwd_saved"} <= set(syms)
    for s in syms:
        assert hasattr(lib, s), s


def _shape(**kw):
    from paper_2406_06484_amd.binding import dn_shape
    s = dn_shape()
    base = dict(B=2, L=256, H=4, d_k=128, d_v=128, chunk=64, dtype=1, num_seqs=0, cu_seqlens=None, cu_seqlens_host=None)
    base.update(kw)
    for k, v in base.items():
        setattr(s, k, v)
    return s


def test_workspace_query_and_validation_errors():
    from paper_2406_06484_amd.binding import load_library
    lib = load_library()
    out = ctypes.c_size_t(0)
    assert lib.deltanet_workspace_bytes(ctypes.byref(_shape()), 0, ctypes.byref(out)) == 0
    fwd_bytes = out.value
    assert lib.deltanet_workspace_bytes(ctypes.byref(_shape()), 1, ctypes.byref(out)) == 0
    assert out.value > fwd_bytes > 0
    # one C x C tile (T of Eq. 10) for every (chunk, head), bf16
    assert fwd_bytes == 2 * 256 * 4 * 64 * 2
    assert lib.deltanet_workspace_bytes(None, 0, ctypes.byref(out)) == -1
    assert lib.deltanet_workspace_bytes(ctypes.byref(_shape(H=0)), 0, ctypes.byref(out)) == -2
    assert lib.deltanet_workspace_bytes(ctypes.byref(_shape(d_k=96)), 0, ctypes.byref(out)) == -3
    assert lib.deltanet_workspace_bytes(ctypes.byref(_shape(chunk=32)), 0, ctypes.byref(out)) == -3
    assert lib.deltanet_workspace_bytes(ctypes.byref(_shape(dtype=7)), 0, ctypes.byref(out)) == -3
    # fp32 is compiled for head dim 64 only
    assert lib.deltanet_workspace_bytes(ctypes.byref(_shape(dtype=0)), 0, ctypes.byref(out)) == -3
    assert lib.deltanet_workspace_bytes(ctypes.byref(_shape(dtype=0, d_k=64, d_v=64)), 0, ctypes.byref(out)) == 0
    for code in range(0, -9, -1):
        assert lib.deltanet_status_string(code)
    # few long chains (16 of them, 32768 tokens): the scans are cut into 8 segments per sequence, and the workspace holds
    # five fp32 [segment, H, d_k, d_v] arrays for them (N, M, start state; R, end gradient)
    long_shape = _shape(B=1, L=32768, H=16)
    assert lib.deltanet_workspace_bytes(ctypes.byref(long_shape), 1, ctypes.byref(out)) == 0
    tiles = (32768 // 64) * 16
    base = tiles * (2 * 64 * 64 + 2 * 64 * 128 + 2 * 128 * 128) * 2          # T, X; Ut, dUt; S, dS' per chunk and head, bf16
    assert out.value == base + 5 * (1 * 8 * 16 * 128 * 128 * 4)
    # many chains: no cut, no such arrays
    assert lib.deltanet_workspace_bytes(ctypes.byref(_shape(B=8, L=2048, H=16)), 1, ctypes.byref(out)) == 0
    assert out.value == 8 * (2048 // 64) * 16 * (2 * 64 * 64 + 2 * 64 * 128 + 2 * 128 * 128) * 2


def test_fwd_bwd_reject_bad_arguments_before_any_launch():
    from paper_2406_06484_amd.binding import load_library
    lib = load_library()
    s = _shape()
    fake = ctypes.c_void_p(0x1000)  # never dereferenced: validation fails first
    args = [fake] * 4 + [None, fake, None]
    assert lib.deltanet_fwd(ctypes.byref(s), None, fake, fake, fake, None, fake, None, fake, 1 << 40, None) == -1
    odd = ctypes.c_void_p(0x1004)
    assert lib.deltanet_fwd(ctypes.byref(s), odd, fake, fake, fake, None, fake, None, fake, 1 << 40, None) == -4
    assert lib.deltanet_fwd(ctypes.byref(s), *args, fake, 16, None) == -5
    assert lib.deltanet_fwd(ctypes.byref(s), *args, None, 0, None) == -5
    rargs = [fake] * 4 + [None, fake, None, None]
    assert lib.deltanet_recurrent_fwd(ctypes.byref(s), None, fake, fake, fake, None, fake, None, None) == -1
    assert lib.deltanet_recurrent_fwd(ctypes.byref(s), odd, fake, fake, fake, None, fake, None, None) == -4
    assert lib.deltanet_recurrent_fwd(ctypes.byref(_shape(d_k=96)), *rargs) == -3
    assert lib.deltanet_recurrent_fwd(ctypes.byref(_shape(d_v=72)), *rargs) == -3
    # gated entry points: g (and dg in the backward) are required, same checks otherwise
    gout = ctypes.c_size_t(0)
    assert lib.deltanet_gated_workspace_bytes(ctypes.byref(s), 1, ctypes.byref(gout)) == 0
    plain = ctypes.c_size_t(0)
    assert lib.deltanet_workspace_bytes(ctypes.byref(s), 1, ctypes.byref(plain)) == 0
    assert gout.value > plain.value  # the per-chunk decay table rides along
    assert lib.deltanet_gated_fwd(ctypes.byref(s), fake, fake, fake, fake, None, None, fake, None, fake, 1 << 40, None) == -1
    assert lib.deltanet_gated_fwd(ctypes.byref(s), fake, fake, fake, fake, odd, None, fake, None, fake, 1 << 40, None) == -4
    assert lib.deltanet_gated_fwd(ctypes.byref(s), fake, fake, fake, fake, fake, None, fake, None, fake, 16, None) == -5
    gb = [fake] * 5 + [None, fake, None, fake, fake, fake, fake, None, None]  # dg missing
    assert lib.deltanet_gated_bwd(ctypes.byref(s), *gb, fake, 1 << 40, None) == -1
    assert lib.deltanet_gated_recurrent_fwd(ctypes.byref(s), fake, fake, fake, fake, None, None, fake, None, None) == -1
    bargs = [fake] * 4 + [None, fake, None, fake, fake, fake, fake, None]
    assert lib.deltanet_bwd(ctypes.byref(s), *bargs, fake, 16, None) == -5
    bargs[10] = None  # dbeta is required
    assert lib.deltanet_bwd(ctypes.byref(s), *bargs, fake, 1 << 40, None) == -1
    # the pair that keeps the forward pass's tiles: the buffer has the backward pass's size
    assert lib.deltanet_fwd_save(ctypes.byref(s), *args, fake, fwd_only_bytes(lib, s), None) == -5
    assert lib.deltanet_fwd_save(ctypes.byref(s), None, fake, fake, fake, None, fake, None, fake, 1 << 40, None) == -1
    # d = 256 has all three variants; a pair of head sizes that is not compiled is refused
    assert lib.deltanet_fwd_save(ctypes.byref(_shape(d_k=256, d_v=256)), *args, fake, 16, None) == -5
    assert lib.deltanet_fused_fwd_save(ctypes.byref(_shape(d_k=256, d_v=256)), *args, fake, 16, None) == -5
    assert lib.deltanet_gated_fwd_save(ctypes.byref(_shape(d_k=256, d_v=256)), fake, fake, fake, fake, fake, None, fake, None,
                                       fake, 16, None) == -5
    assert lib.deltanet_fwd_save(ctypes.byref(_shape(d_k=128, d_v=256)), *args, fake, 1 << 40, None) == -3
    sargs = [fake] * 4 + [fake, None, fake, fake, fake, fake, None]
    assert lib.deltanet_bwd_saved(ctypes.byref(s), *sargs, fake, 16, None) == -5
    assert lib.deltanet_bwd_saved(ctypes.byref(s), *sargs, odd, 1 << 40, None) == -4
    sargs[4] = None  # d_o is required
    assert lib.deltanet_bwd_saved(ctypes.byref(s), *sargs, fake, 1 << 40, None) == -1
    assert lib.deltanet_gated_fwd_save(ctypes.byref(s), fake, fake, fake, fake, None, None, fake, None, fake, 1 << 40, None) == -1
    gs = [fake] * 5 + [fake, None, fake, fake, fake, fake, None, None]  # dg missing
    assert lib.deltanet_gated_bwd_saved(ctypes.byref(s), *gs, fake, 1 << 40, None) == -1
    # the entry points with the prologue in the load path validate like the plain ones
    assert lib.deltanet_fused_fwd(ctypes.byref(s), None, fake, fake, fake, None, fake, None, fake, 1 << 40, None) == -1
    assert lib.deltanet_fused_fwd(ctypes.byref(s), *args, fake, 16, None) == -5
    fb = [fake] * 4 + [None, fake, None, fake, fake, fake, fake, None]
    assert lib.deltanet_fused_bwd(ctypes.byref(s), *fb, fake, 16, None) == -5
    assert lib.deltanet_fused_bwd(ctypes.byref(_shape(d_k=256, d_v=256)), *fb, fake, 16, None) == -5
    assert lib.deltanet_gated_bwd(ctypes.byref(_shape(d_k=128, d_v=256)), *gb, fake, 1 << 40, None) == -3
    assert lib.deltanet_fused_fwd_save(ctypes.byref(s), *args, fake, fwd_only_bytes(lib, s), None) == -5
    fs = [fake] * 4 + [fake, None, fake, fake, fake, None, None]  # dbeta_logit missing
    assert lib.deltanet_fused_bwd_saved(ctypes.byref(s), *fs, fake, 1 << 40, None) == -1


def fwd_only_bytes(lib, s):
    out = ctypes.c_size_t(0)
    assert lib.deltanet_workspace_bytes(ctypes.byref(s), 0, ctypes.byref(out)) == 0
    return out.value


def test_cu_seqlens_host_is_validated():
    from paper_2406_06484_amd.binding import load_library
    lib = load_library()
    out = ctypes.c_size_t(0)
    fake = 0x1000
    good = np.array([0, 10, 10, 300, 512], dtype=np.int32)
    for arr, rc in ((good, 0), (np.array([0, 10, 5, 300, 512], np.int32), -6), (np.array([1, 10, 20, 300, 512], np.int32), -6),
                    (np.array([0, 10, 20, 300, 500], np.int32), -6)):
        s = _shape(B=1, L=512, num_seqs=4, cu_seqlens=fake, cu_seqlens_host=arr.ctypes.data)
        assert lib.deltanet_workspace_bytes(ctypes.byref(s), 1, ctypes.byref(out)) == rc
    s = _shape(B=2, L=512, num_seqs=4, cu_seqlens=fake, cu_seqlens_host=good.ctypes.data)
    assert lib.deltanet_workspace_bytes(ctypes.byref(s), 1, ctypes.byref(out)) == -2  # packed needs B = 1
