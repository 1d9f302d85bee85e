"""ctypes front end of the CPU float64 oracle (oracle/sb_oracle.c).

TEST INFRASTRUCTURE: only tests/, the smoke check and the benchmark's
cpu_baseline leg import this.  Nothing here touches the GPU library and the
GPU library never touches this.

All arrays are numpy float64, layout [B, H, T, d] (or [T, d] for one head).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sb_oracle.c")
_LIB = os.path.join(_HERE, "libsb_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-ffp-contract=off", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ci = ctypes.c_int
        lib.sb_oracle_num_threads.restype = ci
        lib.sb_oracle_weights.argtypes = [dp, dp, ci, ci, dp, dp, dp]
        lib.sb_oracle_weights.restype = ci
        lib.sb_oracle_fwd.argtypes = [dp, dp, dp, dp, dp, dp, ci, ci, ci, ci, ci, ci]
        lib.sb_oracle_fwd.restype = ci
        lib.sb_oracle_bwd.argtypes = [dp, dp, dp, dp, dp, dp, dp, dp, dp, ci, ci, ci, ci]
        lib.sb_oracle_bwd.restype = ci
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if a is not None else None


def _as4(x):
    x = np.ascontiguousarray(np.asarray(x, dtype=np.float64))
    if x.ndim == 2:
        x = x[None, None]
    elif x.ndim == 3:
        x = x[None]
    assert x.ndim == 4, "expected [T,d], [H,T,d] or [B,H,T,d]"
    return x


def num_threads() -> int:
    return int(_load().sb_oracle_num_threads())


def weights(q, k):
    """One head, q,k [T,d] -> (A, beta, rem): A[j,i] is the paper's A[i,j]
    (query row j, key column i), zero for i >= j; rem[j] = prod_{k<j}(1-beta)."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    k = np.ascontiguousarray(k, dtype=np.float64)
    T, d = q.shape
    A = np.empty((T, T))
    beta = np.empty((T, T))
    rem = np.empty(T)
    rc = _load().sb_oracle_weights(_p(q), _p(k), T, d, _p(A), _p(beta), _p(rem))
    if rc != 0:
        raise RuntimeError(f"sb_oracle_weights failed: {rc}")
    return A, beta, rem


def _as_r(r, H, d):
    if r is None:
        return None
    r = np.ascontiguousarray(np.asarray(r, dtype=np.float64)).reshape(H, d)
    return r


def fwd(q, k, v, rows=None, r=None):
    """Forward.  Returns (o, rem) with the input's leading shape; with
    rows=(r0, r1) only query rows r0 <= j < r1 are computed and returned.
    r ([H,d], or [d] for one head): remainder-bias embeddings (Appendix C)."""
    shape = np.asarray(q).shape
    q4, k4, v4 = _as4(q), _as4(k), _as4(v)
    B, H, T, d = q4.shape
    r0, r1 = (0, T) if rows is None else rows
    o = np.zeros((B, H, T, d))
    rem = np.ones((B, H, T))
    rr = _as_r(r, H, d)
    rc = _load().sb_oracle_fwd(_p(q4), _p(k4), _p(v4), _p(rr), _p(o), _p(rem), B, H, T, d, r0, r1)
    if rc != 0:
        raise RuntimeError(f"sb_oracle_fwd failed: {rc}")
    o = o[:, :, r0:r1].reshape(shape[:-2] + (r1 - r0, d))
    rem = rem[:, :, r0:r1].reshape(shape[:-2] + (r1 - r0,))
    return o, rem


def bwd(q, k, v, dout, r=None):
    """Backward for upstream gradient dout = dL/do.  Returns (dq, dk, dv), and with
    remainder-bias embeddings r also dr ([H,d], summed over the batch)."""
    shape = np.asarray(q).shape
    q4, k4, v4, g4 = _as4(q), _as4(k), _as4(v), _as4(dout)
    B, H, T, d = q4.shape
    dq = np.empty((B, H, T, d))
    dk = np.empty((B, H, T, d))
    dv = np.empty((B, H, T, d))
    rr = _as_r(r, H, d)
    dr = np.empty((H, d)) if rr is not None else None
    rc = _load().sb_oracle_bwd(_p(q4), _p(k4), _p(v4), _p(rr), _p(g4), _p(dq), _p(dk), _p(dv), _p(dr), B, H, T, d)
    if rc != 0:
        raise RuntimeError(f"sb_oracle_bwd failed: {rc}")
    out = (dq.reshape(shape), dk.reshape(shape), dv.reshape(shape))
    return out + (dr.reshape(np.asarray(r).shape),) if rr is not None else out


def _expand_kv(x, H):
    """[B,Hkv,T,d] -> [B,H,T,d]: query head h reads kv head h // (H // Hkv)."""
    x = np.asarray(x, dtype=np.float64)
    Hkv = x.shape[1]
    assert H % Hkv == 0, "query heads must be a multiple of kv heads"
    return np.repeat(x, H // Hkv, axis=1)


def fwd_gqa(q, k, v, rows=None, r=None):
    """Grouped kv heads (the paper's larger models pair 12 query heads with 4 kv heads,
    Appendix C model table): q [B,H,T,d], k,v [B,Hkv,T,d]; consecutive groups of H/Hkv
    query heads attend to the same keys and values.  Plain definition: copy each kv
    head to its group and run Eq. 1."""
    H = np.asarray(q).shape[1]
    return fwd(q, _expand_kv(k, H), _expand_kv(v, H), rows=rows, r=r)


def bwd_gqa(q, k, v, dout, r=None):
    """Gradients for grouped kv heads: dq per query head; dk, dv [B,Hkv,T,d] are the sums
    over the group of the per-head gradients (a shared tensor collects every use)."""
    q = np.asarray(q, dtype=np.float64)
    B, H, T, d = q.shape
    Hkv = np.asarray(k).shape[1]
    out = bwd(q, _expand_kv(k, H), _expand_kv(v, H), dout, r=r)
    dk = out[1].reshape(B, Hkv, H // Hkv, T, d).sum(axis=2)
    dv = out[2].reshape(B, Hkv, H // Hkv, T, d).sum(axis=2)
    return (out[0], dk, dv) + tuple(out[3:])


def _seq_bounds(cu_seqlens, Ttot):
    cu = [int(x) for x in cu_seqlens]
    assert len(cu) >= 1 and cu[0] == 0 and cu[-1] == Ttot, "cu_seqlens must run from 0 to the packed length"
    assert all(a <= b for a, b in zip(cu, cu[1:])), "cu_seqlens must not decrease"
    return list(zip(cu, cu[1:]))


def fwd_varlen(q, k, v, cu_seqlens, r=None):
    """Packed variable-length batch (padding-free training, section 5 set-up): q [H,Ttot,d],
    k, v [Hkv,Ttot,d] hold the sequences one after the other along T; sequence s occupies
    rows cu_seqlens[s] .. cu_seqlens[s+1]-1 and attends only inside itself.  Plain
    definition: Eq. 1 on every sequence separately.  Returns (o [H,Ttot,d], rem [H,Ttot])."""
    q = np.asarray(q, dtype=np.float64)
    H, Ttot, d = q.shape
    o = np.zeros((H, Ttot, d))
    rem = np.ones((H, Ttot))
    for a, b in _seq_bounds(cu_seqlens, Ttot):
        if b > a:
            os_, rs = fwd_gqa(q[None, :, a:b], np.asarray(k)[None, :, a:b], np.asarray(v)[None, :, a:b], r=r)
            o[:, a:b] = os_[0]
            rem[:, a:b] = rs[0]
    return o, rem


def bwd_varlen(q, k, v, dout, cu_seqlens, r=None):
    """Gradients of fwd_varlen: every sequence on its own; dr adds up over the sequences."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    H, Ttot, d = q.shape
    dq = np.zeros(q.shape)
    dk = np.zeros(k.shape)
    dv = np.zeros(k.shape)
    dr = np.zeros((H, d)) if r is not None else None
    for a, b in _seq_bounds(cu_seqlens, Ttot):
        if b > a:
            out = bwd_gqa(q[None, :, a:b], k[None, :, a:b], np.asarray(v)[None, :, a:b],
                          np.asarray(dout)[None, :, a:b], r=r)
            dq[:, a:b], dk[:, a:b], dv[:, a:b] = out[0][0], out[1][0], out[2][0]
            if r is not None:
                dr += out[3].reshape(H, d)
    return (dq, dk, dv, dr) if r is not None else (dq, dk, dv)


def decode(q, k, v, r=None):
    """Single-token decode (inference on a key/value cache): q [B,H,d] is the query of the
    position after the T cached tokens k, v [B,Hkv,T,d], so every cached key is visible.
    Plain definition: the last row of Eq. 1 on the sequence extended by that position
    (its own key and value never enter: Eq. 1 is strictly causal).
    Returns (o [B,H,d], rem [B,H])."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, H, d = q.shape
    _, Hkv, T, _ = k.shape
    qf = np.zeros((B, H, T + 1, d))
    qf[:, :, T] = q
    pad = np.zeros((B, Hkv, 1, d))
    o, rem = fwd_gqa(qf, np.concatenate([k, pad], axis=2), np.concatenate([v, pad], axis=2),
                     rows=(T, T + 1), r=r)
    return o[:, :, 0], rem[:, :, 0]
