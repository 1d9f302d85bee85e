"""Thin ctypes binding of libsbattn.so (include/sb_attn.h, include/sb_diag.h): same names, argument
marshalling only.  torch is used to own device memory and to name the stream;
every step of the computation runs inside the library's kernels.

There is no fallback: if the library is missing or a call fails, this raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsbattn.so")

EXPORTS = (
    "sb_attn_fwd", "sb_attn_fwd_halt", "sb_attn_fwd_train", "sb_attn_fwd_f32",
    "sb_attn_bwd_workspace_bytes", "sb_attn_bwd", "sb_attn_bwd_dq", "sb_attn_bwd_dkdv",
    "sb_attn_fwd_rb", "sb_attn_bwd_rb", "sb_attn_fwd_gqa", "sb_attn_bwd_gqa",
    "sb_attn_varlen_fwd", "sb_attn_varlen_bwd_workspace_bytes", "sb_attn_varlen_bwd",
    "sb_attn_decode_workspace_bytes", "sb_attn_decode", "sb_attn_decode_static",
    "sb_diag_mfma_rate", "sb_diag_stream_read", "sb_diag_fwd_clock", "sb_diag_fwd_tri",
    "sb_status_string", "sb_version",
)

_lib = None


class SbAttnError(RuntimeError):
    pass


def load(build_if_missing: bool = True):
    """Load libsbattn.so (building it first only when no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise SbAttnError(f"{LIB_PATH} not built; run `python -m paper_2410_17980_amd.build`")
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, fp = ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p
    lib.sb_attn_fwd.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, vp]
    lib.sb_attn_fwd.restype = ci
    lib.sb_attn_fwd_halt.argtypes = [vp, vp, vp, vp, ctypes.c_float, vp, ci, ci, ci, ci, vp]
    lib.sb_attn_fwd_halt.restype = ci
    lib.sb_attn_fwd_train.argtypes = [vp, vp, vp, vp, fp, ci, ci, ci, ci, vp]
    lib.sb_attn_fwd_train.restype = ci
    lib.sb_attn_fwd_f32.argtypes = [fp, fp, fp, fp, fp, ci, ci, ci, ci, vp]
    lib.sb_attn_fwd_f32.restype = ci
    lib.sb_attn_bwd_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.sb_attn_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.sb_attn_bwd.argtypes = [vp, vp, vp, fp, vp, fp, fp, fp, vp, ctypes.c_size_t, ci, ci, ci, ci, vp]
    lib.sb_attn_bwd.restype = ci
    lib.sb_attn_bwd_dq.argtypes = [vp, vp, vp, fp, vp, fp, vp, ctypes.c_size_t, ci, ci, ci, ci, vp]
    lib.sb_attn_bwd_dq.restype = ci
    lib.sb_attn_bwd_dkdv.argtypes = [vp, vp, vp, vp, fp, fp, vp, ctypes.c_size_t, ci, ci, ci, ci, vp]
    lib.sb_attn_bwd_dkdv.restype = ci
    lib.sb_attn_fwd_rb.argtypes = [vp, vp, vp, vp, vp, fp, ci, ci, ci, ci, vp]
    lib.sb_attn_fwd_rb.restype = ci
    lib.sb_attn_bwd_rb.argtypes = [vp, vp, vp, vp, fp, vp, fp, fp, fp, fp, vp, ctypes.c_size_t, ci, ci, ci, ci, vp]
    lib.sb_attn_bwd_rb.restype = ci
    lib.sb_attn_fwd_gqa.argtypes = [vp, vp, vp, vp, vp, fp, ci, ci, ci, ci, ci, vp]
    lib.sb_attn_fwd_gqa.restype = ci
    lib.sb_attn_bwd_gqa.argtypes = [vp, vp, vp, vp, fp, vp, fp, fp, fp, fp, vp, ctypes.c_size_t,
                                    ci, ci, ci, ci, ci, vp]
    lib.sb_attn_bwd_gqa.restype = ci
    lib.sb_attn_varlen_fwd.argtypes = [vp, vp, vp, vp, vp, fp, vp, ci, ci, ci, ci, ci, ci, vp]
    lib.sb_attn_varlen_fwd.restype = ci
    lib.sb_attn_varlen_bwd_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.sb_attn_varlen_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.sb_attn_varlen_bwd.argtypes = [vp, vp, vp, vp, fp, vp, fp, fp, fp, fp, vp, ci, ci, ci, ci, ci, ci,
                                       vp, ctypes.c_size_t, vp]
    lib.sb_attn_varlen_bwd.restype = ci
    lib.sb_attn_decode_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.sb_attn_decode_workspace_bytes.restype = ctypes.c_size_t
    lib.sb_attn_decode.argtypes = [vp, vp, vp, vp, vp, fp, vp, ctypes.c_size_t, ci, ci, ci, ci, ci, ci, vp]
    lib.sb_attn_decode.restype = ci
    lib.sb_attn_decode_static.argtypes = [vp, vp, vp, vp, vp, fp, ci, ci, ci, ci, ci, ci, vp]
    lib.sb_attn_decode_static.restype = ci
    lib.sb_diag_mfma_rate.argtypes = [vp, ctypes.c_size_t, ci, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.sb_diag_mfma_rate.restype = ci
    lib.sb_diag_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    lib.sb_diag_stream_read.restype = ci
    lib.sb_diag_fwd_clock.argtypes = [vp, vp, vp, vp, fp, ci, ci, ci, ci, vp, vp]
    lib.sb_diag_fwd_clock.restype = ci
    lib.sb_diag_fwd_tri.argtypes = [vp, vp, vp, vp, fp, ci, ci, ci, ci, vp]
    lib.sb_diag_fwd_tri.restype = ci
    lib.sb_status_string.argtypes = [ci]
    lib.sb_status_string.restype = ctypes.c_char_p
    lib.sb_version.argtypes = []
    lib.sb_version.restype = ci
    _lib = lib
    return lib


def sb_status_string(status: int) -> str:
    return load().sb_status_string(int(status)).decode()


def sb_version() -> int:
    return int(load().sb_version())


def _check(rc: int, what: str):
    if rc != 0:
        raise SbAttnError(f"{what} failed: {sb_status_string(rc)} ({rc})")


def _dims(t: torch.Tensor):
    if t.dim() != 4:
        raise SbAttnError("expected a [B, H, T, d] tensor")
    return tuple(int(x) for x in t.shape)


def _ptr(t, dtype, shape=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise SbAttnError(f"{name} must live on the GPU")
    if t.dtype != dtype:
        raise SbAttnError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise SbAttnError(f"{name} must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise SbAttnError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def sb_attn_fwd(q, k, v, o=None, stream=None):
    """bf16 forward.  Returns o (allocated when not given)."""
    B, H, T, d = _dims(q)
    if o is None:
        o = torch.empty_like(q)
    rc = load().sb_attn_fwd(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, q.shape, "k"),
                            _ptr(v, torch.bfloat16, q.shape, "v"), _ptr(o, torch.bfloat16, q.shape, "o"),
                            B, H, T, d, _stream(stream))
    _check(rc, "sb_attn_fwd")
    return o


def sb_attn_fwd_halt(q, k, v, eps, o=None, tile_counts=None, stream=None):
    """bf16 forward with early halt.  tile_counts: optional int64 tensor of 2 on the GPU (added to)."""
    B, H, T, d = _dims(q)
    if o is None:
        o = torch.empty_like(q)
    tc = _ptr(tile_counts, torch.int64, (2,), "tile_counts") if tile_counts is not None else None
    rc = load().sb_attn_fwd_halt(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, q.shape, "k"),
                                 _ptr(v, torch.bfloat16, q.shape, "v"), _ptr(o, torch.bfloat16, q.shape, "o"),
                                 ctypes.c_float(eps), tc, B, H, T, d, _stream(stream))
    _check(rc, "sb_attn_fwd_halt")
    return o


def sb_attn_fwd_train(q, k, v, o=None, m=None, stream=None):
    """bf16 forward that also returns m[B,H,T] (fp32) for the backward."""
    B, H, T, d = _dims(q)
    if o is None:
        o = torch.empty_like(q)
    if m is None:
        m = torch.empty((B, H, T), dtype=torch.float32, device=q.device)
    rc = load().sb_attn_fwd_train(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, q.shape, "k"),
                                  _ptr(v, torch.bfloat16, q.shape, "v"), _ptr(o, torch.bfloat16, q.shape, "o"),
                                  _ptr(m, torch.float32, (B, H, T), "m"), B, H, T, d, _stream(stream))
    _check(rc, "sb_attn_fwd_train")
    return o, m


def sb_attn_fwd_f32(q, k, v, o=None, m=None, want_m=False, stream=None):
    """fp32 forward.  Returns o, or (o, m) when m is given or want_m is set."""
    B, H, T, d = _dims(q)
    if o is None:
        o = torch.empty_like(q)
    if m is None and want_m:
        m = torch.empty((B, H, T), dtype=torch.float32, device=q.device)
    rc = load().sb_attn_fwd_f32(_ptr(q, torch.float32, None, "q"), _ptr(k, torch.float32, q.shape, "k"),
                                _ptr(v, torch.float32, q.shape, "v"), _ptr(o, torch.float32, q.shape, "o"),
                                _ptr(m, torch.float32, (B, H, T), "m"), B, H, T, d, _stream(stream))
    _check(rc, "sb_attn_fwd_f32")
    return (o, m) if m is not None else o


def sb_attn_bwd_workspace_bytes(B, H, T, d) -> int:
    return int(load().sb_attn_bwd_workspace_bytes(B, H, T, d))


def sb_attn_bwd(q, k, v, m, dout, dq=None, dk=None, dv=None, workspace=None, stream=None):
    """bf16 backward.  Returns (dq, dk, dv) in fp32."""
    B, H, T, d = _dims(q)
    mk = lambda: torch.empty(q.shape, dtype=torch.float32, device=q.device)
    dq = mk() if dq is None else dq
    dk = mk() if dk is None else dk
    dv = mk() if dv is None else dv
    need = sb_attn_bwd_workspace_bytes(B, H, T, d)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_ptr = ctypes.c_void_p(workspace.data_ptr()) if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load().sb_attn_bwd(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, q.shape, "k"),
                            _ptr(v, torch.bfloat16, q.shape, "v"), _ptr(m, torch.float32, (B, H, T), "m"),
                            _ptr(dout, torch.bfloat16, q.shape, "dout"),
                            _ptr(dq, torch.float32, q.shape, "dq"), _ptr(dk, torch.float32, q.shape, "dk"),
                            _ptr(dv, torch.float32, q.shape, "dv"), ws_ptr, ws_bytes,
                            B, H, T, d, _stream(stream))
    _check(rc, "sb_attn_bwd")
    return dq, dk, dv


def sb_attn_fwd_rb(q, k, v, r, o=None, m=None, want_m=True, stream=None):
    """bf16 forward with remainder bias r [H,d] (bf16).  Returns (o, m), or o when want_m is off."""
    B, H, T, d = _dims(q)
    if o is None:
        o = torch.empty_like(q)
    if m is None and want_m:
        m = torch.empty((B, H, T), dtype=torch.float32, device=q.device)
    rc = load().sb_attn_fwd_rb(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, q.shape, "k"),
                               _ptr(v, torch.bfloat16, q.shape, "v"), _ptr(r, torch.bfloat16, (H, d), "r"),
                               _ptr(o, torch.bfloat16, q.shape, "o"), _ptr(m, torch.float32, (B, H, T), "m"),
                               B, H, T, d, _stream(stream))
    _check(rc, "sb_attn_fwd_rb")
    return (o, m) if m is not None else o


def sb_attn_bwd_rb(q, k, v, r, m, dout, dq=None, dk=None, dv=None, dr=None, workspace=None, stream=None):
    """bf16 backward with remainder bias.  Returns (dq, dk, dv, dr) in fp32; dr is [H,d]."""
    B, H, T, d = _dims(q)
    mk = lambda: torch.empty(q.shape, dtype=torch.float32, device=q.device)
    dq = mk() if dq is None else dq
    dk = mk() if dk is None else dk
    dv = mk() if dv is None else dv
    dr = torch.empty((H, d), dtype=torch.float32, device=q.device) if dr is None else dr
    workspace, ws_ptr, ws_bytes = _workspace(workspace, B, H, T, d, q.device)
    rc = load().sb_attn_bwd_rb(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, q.shape, "k"),
                               _ptr(v, torch.bfloat16, q.shape, "v"), _ptr(r, torch.bfloat16, (H, d), "r"),
                               _ptr(m, torch.float32, (B, H, T), "m"),
                               _ptr(dout, torch.bfloat16, q.shape, "dout"),
                               _ptr(dq, torch.float32, q.shape, "dq"), _ptr(dk, torch.float32, q.shape, "dk"),
                               _ptr(dv, torch.float32, q.shape, "dv"), _ptr(dr, torch.float32, (H, d), "dr"),
                               ws_ptr, ws_bytes, B, H, T, d, _stream(stream))
    _check(rc, "sb_attn_bwd_rb")
    return dq, dk, dv, dr


def sb_attn_fwd_gqa(q, k, v, r=None, o=None, m=None, want_m=True, stream=None):
    """bf16 forward with grouped kv heads: q [B,H,T,d], k, v [B,Hkv,T,d]; optional remainder
    bias r [H,d].  Returns (o, m), or o when want_m is off."""
    B, H, T, d = _dims(q)
    Hkv = _dims(k)[1]
    if o is None:
        o = torch.empty_like(q)
    if m is None and want_m:
        m = torch.empty((B, H, T), dtype=torch.float32, device=q.device)
    kv_shape = (B, Hkv, T, d)
    rc = load().sb_attn_fwd_gqa(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, kv_shape, "k"),
                                _ptr(v, torch.bfloat16, kv_shape, "v"), _ptr(r, torch.bfloat16, (H, d), "r"),
                                _ptr(o, torch.bfloat16, q.shape, "o"), _ptr(m, torch.float32, (B, H, T), "m"),
                                B, H, Hkv, T, d, _stream(stream))
    _check(rc, "sb_attn_fwd_gqa")
    return (o, m) if m is not None else o


def sb_attn_bwd_gqa(q, k, v, m, dout, r=None, dq=None, dk=None, dv=None, dr=None, workspace=None, stream=None):
    """bf16 backward with grouped kv heads.  Returns (dq, dk, dv) in fp32 (dk, dv [B,Hkv,T,d]),
    and dr [H,d] as a fourth item when r is given."""
    B, H, T, d = _dims(q)
    Hkv = _dims(k)[1]
    kv_shape = (B, Hkv, T, d)
    mk = lambda shape: torch.empty(shape, dtype=torch.float32, device=q.device)
    dq = mk(q.shape) if dq is None else dq
    dk = mk(kv_shape) if dk is None else dk
    dv = mk(kv_shape) if dv is None else dv
    if r is not None and dr is None:
        dr = mk((H, d))
    workspace, ws_ptr, ws_bytes = _workspace(workspace, B, H, T, d, q.device)
    rc = load().sb_attn_bwd_gqa(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, kv_shape, "k"),
                                _ptr(v, torch.bfloat16, kv_shape, "v"), _ptr(r, torch.bfloat16, (H, d), "r"),
                                _ptr(m, torch.float32, (B, H, T), "m"),
                                _ptr(dout, torch.bfloat16, q.shape, "dout"),
                                _ptr(dq, torch.float32, q.shape, "dq"), _ptr(dk, torch.float32, kv_shape, "dk"),
                                _ptr(dv, torch.float32, kv_shape, "dv"), _ptr(dr, torch.float32, (H, d), "dr"),
                                ws_ptr, ws_bytes, B, H, Hkv, T, d, _stream(stream))
    _check(rc, "sb_attn_bwd_gqa")
    return (dq, dk, dv, dr) if r is not None else (dq, dk, dv)


def _dims3(t, name):
    if t.dim() != 3:
        raise SbAttnError(f"{name}: expected a packed [H, Ttot, d] tensor")
    return tuple(int(x) for x in t.shape)


def sb_attn_varlen_fwd(q, k, v, cu_seqlens, max_T, r=None, o=None, m=None, want_m=True, stream=None):
    """bf16 forward on a packed variable-length batch: q [H,Ttot,d], k, v [Hkv,Ttot,d],
    cu_seqlens int32 [nseq+1] on the GPU, max_T >= the longest sequence.  Returns (o, m) or o."""
    H, Ttot, d = _dims3(q, "q")
    Hkv = _dims3(k, "k")[0]
    nseq = int(cu_seqlens.numel()) - 1
    if o is None:
        o = torch.empty_like(q)
    if m is None and want_m:
        m = torch.empty((H, Ttot), dtype=torch.float32, device=q.device)
    kv_shape = (Hkv, Ttot, d)
    rc = load().sb_attn_varlen_fwd(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, kv_shape, "k"),
                                   _ptr(v, torch.bfloat16, kv_shape, "v"), _ptr(r, torch.bfloat16, (H, d), "r"),
                                   _ptr(o, torch.bfloat16, q.shape, "o"), _ptr(m, torch.float32, (H, Ttot), "m"),
                                   _ptr(cu_seqlens, torch.int32, None, "cu_seqlens"),
                                   nseq, H, Hkv, Ttot, int(max_T), d, _stream(stream))
    _check(rc, "sb_attn_varlen_fwd")
    return (o, m) if m is not None else o


def sb_attn_varlen_bwd_workspace_bytes(nseq, H, Ttot, max_T, d) -> int:
    return int(load().sb_attn_varlen_bwd_workspace_bytes(nseq, H, Ttot, max_T, d))


def sb_attn_varlen_bwd(q, k, v, m, dout, cu_seqlens, max_T, r=None, dq=None, dk=None, dv=None, dr=None,
                       workspace=None, stream=None):
    """bf16 backward on a packed variable-length batch.  Returns (dq, dk, dv[, dr]) in fp32."""
    H, Ttot, d = _dims3(q, "q")
    Hkv = _dims3(k, "k")[0]
    nseq = int(cu_seqlens.numel()) - 1
    kv_shape = (Hkv, Ttot, d)
    mk = lambda shape: torch.empty(shape, dtype=torch.float32, device=q.device)
    dq = mk(q.shape) if dq is None else dq
    dk = mk(kv_shape) if dk is None else dk
    dv = mk(kv_shape) if dv is None else dv
    if r is not None and dr is None:
        dr = mk((H, d))
    need = sb_attn_varlen_bwd_workspace_bytes(nseq, H, Ttot, int(max_T), d)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_ptr = ctypes.c_void_p(workspace.data_ptr()) if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load().sb_attn_varlen_bwd(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, kv_shape, "k"),
                                   _ptr(v, torch.bfloat16, kv_shape, "v"), _ptr(r, torch.bfloat16, (H, d), "r"),
                                   _ptr(m, torch.float32, (H, Ttot), "m"),
                                   _ptr(dout, torch.bfloat16, q.shape, "dout"),
                                   _ptr(dq, torch.float32, q.shape, "dq"), _ptr(dk, torch.float32, kv_shape, "dk"),
                                   _ptr(dv, torch.float32, kv_shape, "dv"), _ptr(dr, torch.float32, (H, d), "dr"),
                                   _ptr(cu_seqlens, torch.int32, None, "cu_seqlens"),
                                   nseq, H, Hkv, Ttot, int(max_T), d, ws_ptr, ws_bytes, _stream(stream))
    _check(rc, "sb_attn_varlen_bwd")
    return (dq, dk, dv, dr) if r is not None else (dq, dk, dv)


def sb_attn_decode(q, k, v, T=None, r=None, o=None, m=None, want_m=False, workspace=None, stream=None):
    """Single-token decode: q [B,H,d], cache k, v [B,Hkv,Tcap,d] with the first T rows valid
    (T defaults to Tcap).  Returns o [B,H,d] (bf16), or (o, m) when m is wanted."""
    if q.dim() != 3:
        raise SbAttnError("q: expected [B, H, d]")
    B, H, d = (int(x) for x in q.shape)
    _, Hkv, Tcap, _ = _dims(k)
    T = Tcap if T is None else int(T)
    if o is None:
        o = torch.empty_like(q)
    if m is None and want_m:
        m = torch.empty((B, H), dtype=torch.float32, device=q.device)
    need = int(load().sb_attn_decode_workspace_bytes(B, H, T, d))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_ptr = ctypes.c_void_p(workspace.data_ptr()) if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    kv_shape = (B, Hkv, Tcap, d)
    rc = load().sb_attn_decode(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, kv_shape, "k"),
                               _ptr(v, torch.bfloat16, kv_shape, "v"), _ptr(r, torch.bfloat16, (H, d), "r"),
                               _ptr(o, torch.bfloat16, q.shape, "o"), _ptr(m, torch.float32, (B, H), "m"),
                               ws_ptr, ws_bytes, B, H, Hkv, T, Tcap, d, _stream(stream))
    _check(rc, "sb_attn_decode")
    return (o, m) if m is not None else o


def sb_attn_decode_static(q, k, v, o, T=None, r=None, m=None, stream=None):
    """sb_attn_decode on the library's own static device scratch: nothing is allocated, so the
    caller passes every output (o [B,H,d] bf16, optionally m [B,H] fp32)."""
    if q.dim() != 3:
        raise SbAttnError("q: expected [B, H, d]")
    B, H, d = (int(x) for x in q.shape)
    _, Hkv, Tcap, _ = _dims(k)
    T = Tcap if T is None else int(T)
    kv_shape = (B, Hkv, Tcap, d)
    rc = load().sb_attn_decode_static(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, kv_shape, "k"),
                                      _ptr(v, torch.bfloat16, kv_shape, "v"), _ptr(r, torch.bfloat16, (H, d), "r"),
                                      _ptr(o, torch.bfloat16, q.shape, "o"), _ptr(m, torch.float32, (B, H), "m"),
                                      B, H, Hkv, T, Tcap, d, _stream(stream))
    _check(rc, "sb_attn_decode_static")
    return (o, m) if m is not None else o


def _workspace(workspace, B, H, T, d, device):
    need = sb_attn_bwd_workspace_bytes(B, H, T, d)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    ws_ptr = ctypes.c_void_p(workspace.data_ptr()) if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    return workspace, ws_ptr, ws_bytes


def sb_attn_bwd_dq(q, k, v, m, dout, dq=None, workspace=None, stream=None):
    """Query-stationary pass of the backward.  Returns (dq, workspace)."""
    B, H, T, d = _dims(q)
    dq = torch.empty(q.shape, dtype=torch.float32, device=q.device) if dq is None else dq
    workspace, ws_ptr, ws_bytes = _workspace(workspace, B, H, T, d, q.device)
    rc = load().sb_attn_bwd_dq(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, q.shape, "k"),
                               _ptr(v, torch.bfloat16, q.shape, "v"), _ptr(m, torch.float32, (B, H, T), "m"),
                               _ptr(dout, torch.bfloat16, q.shape, "dout"),
                               _ptr(dq, torch.float32, q.shape, "dq"), ws_ptr, ws_bytes,
                               B, H, T, d, _stream(stream))
    _check(rc, "sb_attn_bwd_dq")
    return dq, workspace


def sb_attn_bwd_dkdv(q, k, v, dout, workspace, dk=None, dv=None, stream=None):
    """Key-stationary pass of the backward (after sb_attn_bwd_dq on the same workspace).  Returns (dk, dv)."""
    B, H, T, d = _dims(q)
    mk = lambda: torch.empty(q.shape, dtype=torch.float32, device=q.device)
    dk = mk() if dk is None else dk
    dv = mk() if dv is None else dv
    _, ws_ptr, ws_bytes = _workspace(workspace, B, H, T, d, q.device)
    rc = load().sb_attn_bwd_dkdv(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, q.shape, "k"),
                                 _ptr(v, torch.bfloat16, q.shape, "v"), _ptr(dout, torch.bfloat16, q.shape, "dout"),
                                 _ptr(dk, torch.float32, q.shape, "dk"), _ptr(dv, torch.float32, q.shape, "dv"),
                                 ws_ptr, ws_bytes, B, H, T, d, _stream(stream))
    _check(rc, "sb_attn_bwd_dkdv")
    return dk, dv


def sb_diag_mfma_rate(operands, iters=2000, stream=None):
    """MFMA-only rate on the given bf16 operand data.  Returns (TFLOP/s, shader clock in MHz)."""
    if not operands.is_cuda or operands.dtype != torch.bfloat16 or not operands.is_contiguous():
        raise SbAttnError("operands must be a contiguous bf16 tensor on the GPU")
    ticks = torch.zeros(4, dtype=torch.int64, device=operands.device)
    flop = ctypes.c_double(0.0)
    nbytes = operands.numel() * 2
    run = lambda: _check(load().sb_diag_mfma_rate(ctypes.c_void_p(operands.data_ptr()), nbytes, int(iters),
                                                  ctypes.c_void_p(ticks.data_ptr()), ctypes.byref(flop),
                                                  _stream(stream)), "sb_diag_mfma_rate")
    run()
    s = torch.cuda.current_stream() if stream is None else stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(s)
    run()
    e1.record(s)
    e1.synchronize()
    ms = e0.elapsed_time(e1)
    t = ticks.cpu().tolist()
    mhz = t[0] / (t[1] / 100e6) / 1e6 if t[1] > 0 else float("nan")
    return flop.value / (ms * 1e-3) / 1e12, mhz


def sb_diag_stream_read(data, iters=10, stream=None):
    """Read bandwidth (GB/s) of a kernel that only loads `data` (any contiguous GPU tensor)."""
    if not data.is_cuda or not data.is_contiguous():
        raise SbAttnError("data must be a contiguous tensor on the GPU")
    nbytes = (data.numel() * data.element_size()) // 16 * 16
    sink = torch.zeros(4, dtype=torch.int32, device=data.device)
    run = lambda: _check(load().sb_diag_stream_read(ctypes.c_void_p(data.data_ptr()), nbytes,
                                                    ctypes.c_void_p(sink.data_ptr()), _stream(stream)),
                         "sb_diag_stream_read")
    for _ in range(2):
        run()
    s = torch.cuda.current_stream() if stream is None else stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(s)
    for _ in range(iters):
        run()
    e1.record(s)
    e1.synchronize()
    return nbytes * iters / (e0.elapsed_time(e1) * 1e-3) / 1e9


def sb_diag_fwd_clock(q, k, v, o, m, stream=None):
    """sb_attn_fwd_train that also returns the shader clock (MHz) its first workgroup saw."""
    B, H, T, d = _dims(q)
    clocks = torch.zeros(4, dtype=torch.int64, device=q.device)
    rc = load().sb_diag_fwd_clock(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, q.shape, "k"),
                                  _ptr(v, torch.bfloat16, q.shape, "v"), _ptr(o, torch.bfloat16, q.shape, "o"),
                                  _ptr(m, torch.float32, (B, H, T), "m"), B, H, T, d,
                                  ctypes.c_void_p(clocks.data_ptr()), _stream(stream))
    _check(rc, "sb_diag_fwd_clock")
    c = clocks.cpu().tolist()
    ref = c[3] - c[1]
    return (c[2] - c[0]) / (ref / 100e6) / 1e6 if ref > 0 else float("nan")


def sb_diag_fwd_tri(q, k, v, o=None, m=None, stream=None):
    """Training forward with the in-tile cumulative sum taken by triangular MFMA (d = 128)."""
    B, H, T, d = _dims(q)
    if o is None:
        o = torch.empty_like(q)
    if m is None:
        m = torch.empty((B, H, T), dtype=torch.float32, device=q.device)
    rc = load().sb_diag_fwd_tri(_ptr(q, torch.bfloat16, None, "q"), _ptr(k, torch.bfloat16, q.shape, "k"),
                                _ptr(v, torch.bfloat16, q.shape, "v"), _ptr(o, torch.bfloat16, q.shape, "o"),
                                _ptr(m, torch.float32, (B, H, T), "m"), B, H, T, d, _stream(stream))
    _check(rc, "sb_diag_fwd_tri")
    return o, m
