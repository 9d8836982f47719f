"""C-ABI checks that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2603_04127_amd as dk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "dark.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(dark_[a-z_]+)\s*\(", src)))


def test_header_symbols_exported():
    names = _declared()
    assert {"dark_featurize", "dark_attn_fwd", "dark_attn_causal_fwd", "dark_attn_bwd",
            "dark_workspace_bytes", "dark_status_string"} <= set(names)
    L = dk.lib()
    for n in names:
        assert hasattr(L, n), n
    assert L.dark_version() >= 100
    assert dk.status_string(dk.DARK_OK) == "ok"
    assert "workspace" in dk.status_string(dk.DARK_EWORKSPACE)


def _p(**kw):
    base = dict(B=1, H=1, L=64, d=16, r=16, m=32, dv=8)
    base.update(kw)
    return dk.make_params(**base)


def test_workspace_query():
    p = _p()
    for op in (dk.OP_FEATURIZE, dk.OP_ATTN_FWD, dk.OP_ATTN_CAUSAL_FWD, dk.OP_ATTN_BWD):
        n = dk.workspace_bytes(p, op)
        assert n > 0 and n % 256 == 0
    assert dk.workspace_bytes(_p(L=0), dk.OP_ATTN_FWD) == 0
    assert dk.workspace_bytes(_p(d=0), dk.OP_ATTN_FWD) == 0          # invalid -> 0
    assert dk.workspace_bytes(_p(L=128), dk.OP_ATTN_FWD) > dk.workspace_bytes(_p(L=64), dk.OP_ATTN_FWD)
    assert dk.workspace_bytes(p, 17) == 0


def test_argument_errors_before_any_device_work():
    L = dk.lib()
    p = _p()
    A = 1 << 20        # fake, aligned, never dereferenced: every call below must fail in the checks
    ws = 1 << 24
    big = 1 << 30
    f = L.dark_attn_fwd
    assert f(None, A, A, A, A, A, A, ws, big, None) == dk.DARK_EINVAL
    assert f(ctypes.byref(p), None, A, A, A, A, A, ws, big, None) == dk.DARK_EINVAL
    assert f(ctypes.byref(p), A, A, A, A, A, None, ws, big, None) == dk.DARK_EINVAL
    assert f(ctypes.byref(p), A + 4, A, A, A, A, A, ws, big, None) == dk.DARK_EALIGN
    assert f(ctypes.byref(p), A, A, A, A, A, A, None, 0, None) == dk.DARK_EWORKSPACE
    assert f(ctypes.byref(p), A, A, A, A, A, A, ws, 16, None) == dk.DARK_EWORKSPACE
    assert f(ctypes.byref(p), A, A, A, A, A, A, ws + 16, big, None) == dk.DARK_EALIGN
    for bad in (dict(m=0), dict(H=0), dict(L=-1), dict(io_dtype=7), dict(path=9), dict(scale=-1.0), dict(chunk=-2),
                dict(sched={"kv_wgs": -1})):
        q = _p(**bad)
        assert f(ctypes.byref(q), A, A, A, A, A, A, ws, big, None) == dk.DARK_EINVAL, bad
    assert f(ctypes.byref(_p(chunk=4096)), A, A, A, A, A, A, ws, big, None) == dk.DARK_EUNSUPPORTED
    # empty problems are valid and enqueue nothing
    assert f(ctypes.byref(_p(L=0)), A, A, A, A, A, A, None, 0, None) == dk.DARK_OK
    assert L.dark_attn_causal_fwd(ctypes.byref(_p(B=0)), A, A, A, A, A, A, None, 0, None) == dk.DARK_OK
    assert L.dark_featurize(ctypes.byref(p), A, A, A, 1, None, A, ws, big, None) == dk.DARK_EINVAL
    assert L.dark_featurize(ctypes.byref(p), A, A, A, 1, A, A, None, 0, None) == dk.DARK_EWORKSPACE
    assert L.dark_attn_bwd(ctypes.byref(p), 1, A, A, A, A, A, None, A, A, A, A, ws, big, None) == dk.DARK_EINVAL
    assert L.dark_attn_bwd(ctypes.byref(p), 1, A, A, A, A, A, A, A, A, A, A, None, 0, None) == dk.DARK_EWORKSPACE
    # a shape the fused kernels cannot take, with the fused path forced
    q = _p(d=24, io_dtype=dk.DARK_BF16, path=dk.PATH_FUSED)
    assert f(ctypes.byref(q), A, A, A, A, A, A, ws, big, None) == dk.DARK_EUNSUPPORTED


def test_argument_errors_of_the_later_entry_points():
    L = dk.lib()
    p = _p()
    A = 1 << 20
    ws = 1 << 24
    big = 1 << 30
    P = ctypes.byref(p)
    # whitening: needs rows, Q and M_out; K and cov_out are optional
    assert dk.workspace_bytes(p, dk.OP_WHITEN) > 0
    assert L.dark_whiten(ctypes.byref(_p(L=0)), A, A, A, A, ws, big, None) == dk.DARK_EINVAL
    assert L.dark_whiten(P, None, A, A, A, ws, big, None) == dk.DARK_EINVAL
    assert L.dark_whiten(P, A, A, None, A, ws, big, None) == dk.DARK_EINVAL
    assert L.dark_whiten(P, A, A + 8, A, A, ws, big, None) == dk.DARK_EALIGN
    assert L.dark_whiten(ctypes.byref(_p(d=256, r=256)), A, A, A, A, ws, big, None) == dk.DARK_EUNSUPPORTED
    assert L.dark_whiten(ctypes.byref(_p(r=32)), A, A, A, A, ws, big, None) == dk.DARK_EUNSUPPORTED
    assert L.dark_whiten(P, A, None, A, None, None, 0, None) == dk.DARK_EWORKSPACE
    # decode step: every state pointer is required; M may be NULL only when r == d
    f = L.dark_decode_step
    assert f(ctypes.byref(_p(B=0)), A, A, A, A, A, A, A, A, A, None) == dk.DARK_OK
    assert f(P, A, A, A, A, A, None, A, A, A, None) == dk.DARK_EINVAL
    assert f(P, A, A, A, A, A, A, A, None, A, None) == dk.DARK_EINVAL
    assert f(ctypes.byref(_p(r=8)), A, A, A, None, A, A, A, A, A, None) == dk.DARK_EINVAL
    assert f(P, A, A, A, A, A, A + 4, A, A, A, None) == dk.DARK_EALIGN
    # hand-over pair: parameters without a hand-over report 0 bytes and ignore the buffer
    assert dk.saved_bytes(p) == 0
    q = dk.make_params(B=1, H=2, L=1024, d=64, r=64, m=256, dv=64, io_dtype=dk.DARK_BF16)
    n = dk.saved_bytes(q)
    assert n > 0
    Q = ctypes.byref(q)
    g = L.dark_attn_causal_fwd_save
    assert g(Q, A, A, A, A, A, A, None, 0, ws, big, None) == dk.DARK_EWORKSPACE
    assert g(Q, A, A, A, A, A, A, ws, n - 1, ws, big, None) == dk.DARK_EWORKSPACE
    assert g(Q, A, A, A, A, A, A, ws + 64, n, ws, big, None) == dk.DARK_EALIGN
    h = L.dark_attn_bwd_saved
    assert h(Q, A, A, A, A, A, A, None, 0, A, A, A, A, A, ws, big, None) == dk.DARK_EWORKSPACE
    assert h(Q, A, A, A, A, A, None, ws, n, A, A, A, A, A, ws, big, None) == dk.DARK_EINVAL
    # identity geometry (M == NULL) needs r == d on every entry point
    assert L.dark_attn_fwd(ctypes.byref(_p(r=8)), A, A, A, None, A, A, ws, big, None) == dk.DARK_EINVAL
    assert L.dark_attn_bwd_dw(ctypes.byref(_p(r=8)), 0, A, A, A, None, A, A, A, A, A, A, A, ws, big, None) \
        == dk.DARK_EINVAL


def test_timing_slots_named():
    L = dk.lib()
    n = L.dark_timing_slots()
    assert n > 4
    name = ctypes.c_char_p()
    assert L.dark_timing_read(0, ctypes.byref(name), None, None) == dk.DARK_OK and name.value
    assert L.dark_timing_read(n, None, None, None) == dk.DARK_EINVAL


def test_timeline_is_a_build_option():
    """The ordinary library records no timeline: the call validates its arguments and says so (no HIP call)."""
    L = dk.lib()
    buf = (ctypes.c_int64 * 16)()
    assert L.dark_timeline_read(0, buf, 16) == dk.DARK_EUNSUPPORTED
    assert L.dark_timeline_read(2, buf, 16) == dk.DARK_EINVAL
    assert L.dark_timeline_read(1, None, 16) == dk.DARK_EINVAL
    assert L.dark_timeline_read(1, buf, 10 ** 9) == dk.DARK_EINVAL
