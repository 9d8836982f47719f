"""Python binding over the C-ABI DARK attention library (libdark.so).

Argument marshalling only: every step of the computation runs in the HIP
kernels behind ``include/dark.h``.  PyTorch supplies device memory (tensors)
and the current HIP stream.  There is no CPU fallback: if the shared library is
missing the import of this binding's functions raises.
"""
from __future__ import annotations

import ctypes
import math
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdark.so")

DARK_OK, DARK_EINVAL, DARK_EUNSUPPORTED, DARK_EWORKSPACE, DARK_EALIGN, DARK_EHIP, DARK_ESCRATCH = range(7)
DARK_F32, DARK_BF16 = 0, 1
OP_FEATURIZE, OP_ATTN_FWD, OP_ATTN_CAUSAL_FWD, OP_ATTN_BWD, OP_WHITEN = range(5)
PATH_AUTO, PATH_F32, PATH_FUSED = range(3)


class DarkParams(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("L", ctypes.c_int32),
        ("d", ctypes.c_int32), ("r", ctypes.c_int32), ("m", ctypes.c_int32), ("dv", ctypes.c_int32),
        ("chunk", ctypes.c_int32), ("io_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("scale", ctypes.c_float), ("w_shared", ctypes.c_int32), ("path", ctypes.c_int32),
        ("sched_kv_wgs", ctypes.c_int32), ("sched_ro_wgs", ctypes.c_int32), ("sched_cs_wgs", ctypes.c_int32),
        ("sched_cs_state", ctypes.c_int32),
    ]


class DarkError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libdark.so (built in-tree by ``build.py``); raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it first (python -m paper_2603_04127_amd.build or __graft_entry__.build())")
    L = ctypes.CDLL(LIB_PATH)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    pp = ctypes.POINTER(DarkParams)
    L.dark_version.restype = i32
    L.dark_status_string.restype = ctypes.c_char_p
    L.dark_status_string.argtypes = [i32]
    L.dark_workspace_bytes.restype = sz
    L.dark_workspace_bytes.argtypes = [pp, i32, i32]
    L.dark_featurize.restype = i32
    L.dark_featurize.argtypes = [pp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    for f in (L.dark_attn_fwd, L.dark_attn_causal_fwd):
        f.restype = i32
        f.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.dark_attn_fwd_static.restype = i32
    L.dark_attn_fwd_static.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp]
    L.dark_static_scratch_bytes.restype = sz
    L.dark_attn_bwd.restype = i32
    L.dark_attn_bwd.argtypes = [pp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.dark_attn_bwd_dw.restype = i32
    L.dark_attn_bwd_dw.argtypes = [pp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.dark_decode_step.restype = i32
    L.dark_decode_step.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.dark_whiten.restype = i32
    L.dark_whiten.argtypes = [pp, vp, vp, vp, vp, vp, sz, vp]
    L.dark_saved_bytes.restype = sz
    L.dark_saved_bytes.argtypes = [pp]
    L.dark_attn_causal_fwd_save.restype = i32
    L.dark_attn_causal_fwd_save.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, sz, vp, sz, vp]
    L.dark_attn_bwd_saved.restype = i32
    L.dark_attn_bwd_saved.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp, vp, vp, vp, vp, sz, vp]
    L.dark_timing_enable.argtypes = [i32]
    L.dark_timing_enable.restype = None
    L.dark_timing_reset.restype = None
    L.dark_timing_slots.restype = i32
    L.dark_timing_read.restype = i32
    L.dark_timing_read.argtypes = [i32, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_int64),
                                   ctypes.POINTER(ctypes.c_double)]
    L.dark_timeline_read.restype = i32
    L.dark_timeline_read.argtypes = [i32, ctypes.POINTER(ctypes.c_int64), sz]
    L.dark_ceiling_copy.restype = i32
    L.dark_ceiling_copy.argtypes = [vp, vp, sz, vp]
    L.dark_ceiling_read.restype = i32
    L.dark_ceiling_read.argtypes = [vp, sz, vp, vp]
    L.dark_ceiling_mfma.restype = i32
    L.dark_ceiling_mfma.argtypes = [i32, vp, ctypes.POINTER(ctypes.c_double), vp]
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().dark_status_string(int(status)).decode()


def make_params(B, H, L, d, r, m, dv, *, io_dtype=DARK_F32, out_dtype=None, chunk=0, scale=0.0, w_shared=False,
                path=PATH_AUTO, sched=None) -> DarkParams:
    """`sched`: optional dict of the schedule overrides of dark_params (kv_wgs, ro_wgs, cs_wgs, cs_state)."""
    sched = sched or {}
    unknown = set(sched) - {"kv_wgs", "ro_wgs", "cs_wgs", "cs_state"}
    if unknown:
        raise ValueError(f"unknown schedule override(s) {sorted(unknown)}")
    return DarkParams(B, H, L, d, r, m, dv, chunk, io_dtype, io_dtype if out_dtype is None else out_dtype,
                      float(scale), int(bool(w_shared)), path, int(sched.get("kv_wgs", 0)), int(sched.get("ro_wgs", 0)),
                      int(sched.get("cs_wgs", 0)), int(sched.get("cs_state", 0)))


def workspace_bytes(p: DarkParams, op: int, causal: bool = False) -> int:
    return int(lib().dark_workspace_bytes(ctypes.byref(p), op, int(causal)))


# ----------------------------------------------------------------------------
# torch-facing helpers
# ----------------------------------------------------------------------------
def _torch():
    import torch
    return torch


def _dtype_code(t) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return DARK_F32
    if t.dtype == torch.bfloat16:
        return DARK_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous device tensors")
    return t.data_ptr()


def _stream() -> int:
    return _torch().cuda.current_stream().cuda_stream


_ws_cache = {}


def _workspace(nbytes: int, device):
    """A cached device byte buffer of at least nbytes (torch owns the memory)."""
    torch = _torch()
    key = (device.type, device.index)
    buf = _ws_cache.get(key)
    if buf is None or buf.numel() < nbytes:
        _ws_cache.pop(key, None)
        buf = None
        buf = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        _ws_cache[key] = buf
    return buf


def _params_from(Q, V, M, W, *, out_dtype=None, chunk=0, scale=0.0, path=PATH_AUTO, sched=None) -> DarkParams:
    B, H, L, d = Q.shape
    dv = V.shape[-1] if V is not None else 1
    r = M.shape[-2] if M is not None else d      # M = None: the identity (isotropic features), r = d
    w_shared = W.dim() == 2
    m = W.shape[-2]
    torch = _torch()
    if (M is not None and M.dtype != torch.float32) or W.dtype != torch.float32:
        raise TypeError("M and W must be float32")
    if (M is not None and tuple(M.shape) != (H, r, d)) or W.shape[-1] != r or (not w_shared and W.shape[0] != H):
        raise ValueError("M must be [H, r, d] (or None) and W [H, m, r] or [m, r]")
    io = _dtype_code(Q)
    od = io if out_dtype is None else (DARK_BF16 if out_dtype == torch.bfloat16 else DARK_F32)
    return make_params(B, H, L, d, r, m, dv, io_dtype=io, out_dtype=od, chunk=chunk, scale=scale, w_shared=w_shared,
                       path=path, sched=sched)


def _check(status: int, where: str):
    if status != DARK_OK:
        raise DarkError(status, where)


def dark_featurize(X, M, W, is_query: bool, *, scale=0.0, path=PATH_AUTO):
    """phi_Sigma of every row of X [B,H,L,d] -> (phi [B,H,L,m], stab)."""
    torch = _torch()
    p = _params_from(X, None, M, W, scale=scale, path=path)
    B, H, L, _ = X.shape
    phi = torch.empty((B, H, L, p.m), dtype=X.dtype, device=X.device)
    stab = torch.empty((B, H, L) if is_query else (B, H), dtype=torch.float32, device=X.device)
    nb = workspace_bytes(p, OP_FEATURIZE)
    ws = _workspace(nb, X.device)
    _check(lib().dark_featurize(ctypes.byref(p), _ptr(X), _ptr(M), _ptr(W), int(is_query), _ptr(phi), _ptr(stab),
                                ws.data_ptr(), ws.numel(), _stream()), "dark_featurize")
    return phi, stab


def _attn(fn_name, op, Q, K, V, M, W, out, chunk, scale, path, out_dtype, sched=None):
    torch = _torch()
    p = _params_from(Q, V, M, W, out_dtype=out_dtype, chunk=chunk, scale=scale, path=path, sched=sched)
    if K.shape != Q.shape or V.shape[:3] != Q.shape[:3] or K.dtype != Q.dtype or V.dtype != Q.dtype:
        raise ValueError("Q, K, V shapes/dtypes disagree")
    if out is None:
        od = Q.dtype if out_dtype is None else out_dtype
        out = torch.empty(V.shape, dtype=od, device=Q.device)
    nb = workspace_bytes(p, op)
    ws = _workspace(nb, Q.device)
    fn = getattr(lib(), fn_name)
    _check(fn(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(M), _ptr(W), _ptr(out), ws.data_ptr(), ws.numel(),
              _stream()), fn_name)
    return out


def dark_attn_fwd(Q, K, V, M, W, *, out=None, scale=0.0, path=PATH_AUTO, out_dtype=None, sched=None):
    """Bidirectional random-feature attention, out [B,H,L,dv]."""
    return _attn("dark_attn_fwd", OP_ATTN_FWD, Q, K, V, M, W, out, 0, scale, path, out_dtype, sched)


def dark_attn_fwd_static(Q, K, V, M, W, out, *, scale=0.0, path=PATH_AUTO):
    """dark_attn_fwd on the library's static scratch: no workspace, no allocation (``out`` is the caller's)."""
    p = _params_from(Q, V, M, W, out_dtype=out.dtype, scale=scale, path=path)
    if K.shape != Q.shape or V.shape[:3] != Q.shape[:3] or K.dtype != Q.dtype or V.dtype != Q.dtype:
        raise ValueError("Q, K, V shapes/dtypes disagree")
    if tuple(out.shape) != tuple(V.shape):
        raise ValueError("out must have the shape of V")
    _check(lib().dark_attn_fwd_static(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(M), _ptr(W), _ptr(out),
                                      _stream()), "dark_attn_fwd_static")
    return out


def static_scratch_bytes() -> int:
    return int(lib().dark_static_scratch_bytes())


def dark_attn_causal_fwd(Q, K, V, M, W, *, out=None, chunk=0, scale=0.0, path=PATH_AUTO, out_dtype=None, sched=None):
    """Causal random-feature attention (keys l <= i), out [B,H,L,dv]."""
    return _attn("dark_attn_causal_fwd", OP_ATTN_CAUSAL_FWD, Q, K, V, M, W, out, chunk, scale, path, out_dtype, sched)


def decode_state(B, H, m, dv, device="cuda"):
    """Empty recurrent state (S, z, c) of dark_decode_step."""
    torch = _torch()
    return (torch.zeros((B, H, m, dv), dtype=torch.float32, device=device),
            torch.zeros((B, H, m), dtype=torch.float32, device=device),
            torch.full((B, H), float("-inf"), dtype=torch.float32, device=device))


def dark_decode_step(q, k, v, M, W, state, *, out=None, scale=0.0):
    """One token: q, k [B,H,d], v [B,H,dv]; state = (S, z, c) is updated in place; returns out [B,H,dv]."""
    torch = _torch()
    B, H, d = q.shape
    S, z, c = state
    p = _params_from(q[:, :, None, :], v[:, :, None, :], M, W, scale=scale)
    if out is None:
        out = torch.empty(v.shape, dtype=q.dtype, device=q.device)
    _check(lib().dark_decode_step(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(M), _ptr(W), _ptr(S), _ptr(z), _ptr(c),
                                  _ptr(out), _stream()), "dark_decode_step")
    return out


def dark_whiten(Q, K=None, *, r=None, want_cov=False):
    """Whitening geometry M [H, r, d] (float32) from the rows of Q and K [B, H, L, d]; with want_cov also the
    covariance estimate [H, d, d]."""
    torch = _torch()
    B, H, L, d = Q.shape
    r = d if r is None else int(r)
    p = make_params(B, H, L, d, r, 64, 1, io_dtype=_dtype_code(Q))
    M = torch.empty((H, r, d), dtype=torch.float32, device=Q.device)
    cov = torch.empty((H, d, d), dtype=torch.float32, device=Q.device) if want_cov else None
    ws = _workspace(workspace_bytes(p, OP_WHITEN), Q.device)
    _check(lib().dark_whiten(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(M), _ptr(cov), ws.data_ptr(), ws.numel(),
                             _stream()), "dark_whiten")
    return (M, cov) if want_cov else M


def saved_bytes(p: DarkParams) -> int:
    return int(lib().dark_saved_bytes(ctypes.byref(p)))


def dark_attn_causal_fwd_save(Q, K, V, M, W, *, out=None, saved=None, chunk=0, scale=0.0, path=PATH_AUTO, out_dtype=None):
    """Causal forward that leaves what the backward can take over in `saved` (a uint8 device tensor of at
    least saved_bytes(p) bytes; allocated here when not given).  Returns (out, saved); `saved` is None for
    parameters that have no hand-over."""
    torch = _torch()
    p = _params_from(Q, V, M, W, out_dtype=out_dtype, chunk=chunk, scale=scale, path=path)
    if out is None:
        out = torch.empty(V.shape, dtype=Q.dtype if out_dtype is None else out_dtype, device=Q.device)
    ns = saved_bytes(p)
    if ns and saved is None:
        saved = torch.empty(ns, dtype=torch.uint8, device=Q.device)
    ws = _workspace(workspace_bytes(p, OP_ATTN_CAUSAL_FWD), Q.device)
    _check(lib().dark_attn_causal_fwd_save(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(M), _ptr(W), _ptr(out),
                                           _ptr(saved) if ns else None, saved.numel() if ns else 0,
                                           ws.data_ptr(), ws.numel(), _stream()), "dark_attn_causal_fwd_save")
    return out, (saved if ns else None)


def dark_attn_bwd(Q, K, V, M, W, dOut, causal: bool, *, chunk=0, scale=0.0, path=PATH_AUTO, need=("dQ", "dK", "dV", "dM"),
                  saved=None, grads=None):
    """Gradients of sum(out*dOut): returns dict with the float32 gradients named in `need`
    ("dQ", "dK", "dV", "dM", and "dW", the gradient with respect to the draws).  `saved`: the hand-over
    buffer of dark_attn_causal_fwd_save for the same inputs (causal only).  `grads`: a dict of preallocated
    output tensors to write into instead of allocating."""
    torch = _torch()
    p = _params_from(Q, V, M, W, chunk=chunk, scale=scale, path=path)
    f32 = dict(dtype=torch.float32, device=Q.device)
    H, d = Q.shape[1], Q.shape[3]
    if grads is not None:
        g = {k: grads.get(k) for k in ("dQ", "dK", "dV", "dM", "dW")}
    else:
        g = {
            "dQ": torch.empty(Q.shape, **f32) if "dQ" in need else None,
            "dK": torch.empty(K.shape, **f32) if "dK" in need else None,
            "dV": torch.empty(V.shape, **f32) if "dV" in need else None,
            "dM": torch.empty(M.shape if M is not None else (H, d, d), **f32) if "dM" in need else None,
        }
        if "dW" in need:
            g["dW"] = torch.empty(W.shape, **f32)
    nb = workspace_bytes(p, OP_ATTN_BWD, causal)
    ws = _workspace(nb, Q.device)
    if saved is not None:
        if not causal:
            raise ValueError("saved state exists for the causal form only")
        _check(lib().dark_attn_bwd_saved(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(M), _ptr(W), _ptr(dOut),
                                         _ptr(saved), saved.numel(), _ptr(g.get("dQ")), _ptr(g.get("dK")),
                                         _ptr(g.get("dV")), _ptr(g.get("dM")), _ptr(g.get("dW")), ws.data_ptr(),
                                         ws.numel(), _stream()), "dark_attn_bwd_saved")
        return g
    if g.get("dW") is not None:
        _check(lib().dark_attn_bwd_dw(ctypes.byref(p), int(causal), _ptr(Q), _ptr(K), _ptr(V), _ptr(M), _ptr(W),
                                      _ptr(dOut), _ptr(g["dQ"]), _ptr(g["dK"]), _ptr(g["dV"]), _ptr(g["dM"]),
                                      _ptr(g["dW"]), ws.data_ptr(), ws.numel(), _stream()), "dark_attn_bwd_dw")
        return g
    _check(lib().dark_attn_bwd(ctypes.byref(p), int(causal), _ptr(Q), _ptr(K), _ptr(V), _ptr(M), _ptr(W), _ptr(dOut),
                               _ptr(g["dQ"]), _ptr(g["dK"]), _ptr(g["dV"]), _ptr(g["dM"]), ws.data_ptr(), ws.numel(),
                               _stream()), "dark_attn_bwd")
    return g


# ----------------------------------------------------------------------------
# per-kernel timing (benchmarks)
# ----------------------------------------------------------------------------
def timing_enable(on: bool):
    lib().dark_timing_enable(int(on))


def timing_reset():
    lib().dark_timing_reset()


def timing_read() -> dict:
    """{kernel name: (launches, total_ms)} for kernels launched since the last reset."""
    L = lib()
    out = {}
    for k in range(L.dark_timing_slots()):
        name = ctypes.c_char_p()
        n = ctypes.c_int64()
        ms = ctypes.c_double()
        _check(L.dark_timing_read(k, ctypes.byref(name), ctypes.byref(n), ctypes.byref(ms)), "dark_timing_read")
        if n.value:
            out[name.value.decode()] = (n.value, ms.value)
    return out


def timeline_read(which: int, n: int):
    """The wall-clock stamps of the last launch of the key/value pass (which = 0) or the readout (which = 1)
    as a list of n int64 ticks; raises unless the loaded library was built with -DDARK_TIMELINE."""
    buf = (ctypes.c_int64 * n)()
    _check(lib().dark_timeline_read(int(which), buf, n), "dark_timeline_read")
    return list(buf)


# ----------------------------------------------------------------------------
# measured ceilings of the device (benchmarks)
# ----------------------------------------------------------------------------
def ceiling_copy(dst, src):
    """One launch of the plain copy kernel: src -> dst (same byte size, a multiple of 16)."""
    nb = src.numel() * src.element_size()
    _check(lib().dark_ceiling_copy(_ptr(dst), _ptr(src), nb, _stream()), "dark_ceiling_copy")
    return nb


def ceiling_read(src, sink):
    """One launch of the plain read kernel over src."""
    nb = src.numel() * src.element_size()
    _check(lib().dark_ceiling_read(_ptr(src), nb, _ptr(sink), _stream()), "dark_ceiling_read")
    return nb


def ceiling_mfma(iters, sink) -> float:
    """One launch of the MFMA loop kernel; returns the floating-point operations it performs."""
    fl = ctypes.c_double()
    _check(lib().dark_ceiling_mfma(int(iters), _ptr(sink), ctypes.byref(fl), _stream()), "dark_ceiling_mfma")
    return fl.value
