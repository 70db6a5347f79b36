"""CPU oracle (test infrastructure only): ctypes binding of ``ulysses_oracle.c``.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
The GPU library never does, and this module never imports the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ulysses_oracle.c")
_LIB = os.path.join(_HERE, "libulysses_oracle.so")
_lib = None

LAYOUT_SEQ_HEAD = 0   # [N, Hl, d]
LAYOUT_HEAD_SEQ = 1   # [Hl, N, d]


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, i64, ci, dbl = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_double
        lib.oracle_pack.argtypes = [vp, vp, i64, ci, ci, ci]
        lib.oracle_unpack.argtypes = [vp, vp, i64, ci, ci, ci, ci]
        lib.oracle_pack_rev.argtypes = [vp, vp, i64, ci, ci, ci, ci]
        lib.oracle_unpack_rev.argtypes = [vp, vp, i64, ci, ci, ci]
        lib.oracle_bf16_to_f64.argtypes = [vp, vp, i64]
        for f in (lib.oracle_pack, lib.oracle_unpack, lib.oracle_pack_rev, lib.oracle_unpack_rev,
                  lib.oracle_bf16_to_f64):
            f.restype = None
        lib.oracle_attn_fwd.argtypes = [vp, vp, vp, vp, vp, i64, ci, ci, dbl, ci, ci]
        lib.oracle_attn_fwd_rows.argtypes = [vp, vp, vp, vp, i64, vp, vp, i64, ci, ci, dbl, ci, ci]
        lib.oracle_attn_bwd_rows.argtypes = [vp, vp, vp, vp, vp, i64, vp, vp, vp, i64, ci, ci, dbl, ci, ci]
        lib.oracle_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, ci, ci, dbl, ci, ci]
        lib.oracle_xattn_fwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, ci, ci, dbl, ci]
        lib.oracle_xattn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, ci, ci, dbl, ci]
        lib.oracle_sparse_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, ci, ci, dbl, ci]
        lib.oracle_sparse_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, ci, ci, dbl, ci]
        for f in (lib.oracle_attn_fwd, lib.oracle_attn_fwd_rows, lib.oracle_attn_bwd_rows, lib.oracle_attn_bwd,
                  lib.oracle_xattn_fwd, lib.oracle_xattn_bwd, lib.oracle_sparse_attn_fwd, lib.oracle_sparse_attn_bwd):
            f.restype = ci
        lib.oracle_num_threads.restype = ci
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16
    return a


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _check_heads(H, P):
    if P <= 0 or H <= 0 or H % P:
        raise ValueError("H must be a positive multiple of P")


# ---- layout transforms ------------------------------------------------------------------------
def pack(x: np.ndarray, P: int) -> np.ndarray:
    """x:[nl,H,d] uint16 -> send:[P,nl,H/P,d]."""
    x = _u16(x); nl, H, d = x.shape; _check_heads(H, P)
    out = np.empty((P, nl, H // P, d), np.uint16)
    _load().oracle_pack(x.ctypes.data, out.ctypes.data, nl, H, d, P)
    return out


def unpack(recv: np.ndarray, layout: int = LAYOUT_SEQ_HEAD) -> np.ndarray:
    """recv:[P,nl,Hl,d] uint16 -> y:[P*nl,Hl,d] (or [Hl,P*nl,d])."""
    recv = _u16(recv); P, nl, Hl, d = recv.shape
    shape = (P * nl, Hl, d) if layout == LAYOUT_SEQ_HEAD else (Hl, P * nl, d)
    out = np.empty(shape, np.uint16)
    _load().oracle_unpack(recv.ctypes.data, out.ctypes.data, nl, Hl * P, d, P, layout)
    return out


def pack_rev(o: np.ndarray, P: int, layout: int = LAYOUT_SEQ_HEAD) -> np.ndarray:
    """o:[N,Hl,d] (or [Hl,N,d]) uint16 -> send:[P,N/P,Hl,d]."""
    o = _u16(o)
    N, Hl, d = o.shape if layout == LAYOUT_SEQ_HEAD else (o.shape[1], o.shape[0], o.shape[2])
    if N % P:
        raise ValueError("N must be a multiple of P")
    out = np.empty((P, N // P, Hl, d), np.uint16)
    _load().oracle_pack_rev(o.ctypes.data, out.ctypes.data, N // P, Hl * P, d, P, layout)
    return out


def unpack_rev(recv: np.ndarray) -> np.ndarray:
    """recv:[P,nl,Hl,d] uint16 -> y:[nl,P*Hl,d]."""
    recv = _u16(recv); P, nl, Hl, d = recv.shape
    out = np.empty((nl, P * Hl, d), np.uint16)
    _load().oracle_unpack_rev(recv.ctypes.data, out.ctypes.data, nl, Hl * P, d, P)
    return out


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    bits = _u16(bits)
    out = np.empty(bits.shape, np.float64)
    _load().oracle_bf16_to_f64(bits.ctypes.data, out.ctypes.data, bits.size)
    return out


# ---- attention ----------------------------------------------------------------------------------
def _dims(q, layout):
    if layout == LAYOUT_SEQ_HEAD:
        N, Hl, d = q.shape
    else:
        Hl, N, d = q.shape
    return N, Hl, d


def attn_fwd(q, k, v, scale: float, causal: bool = True, layout: int = LAYOUT_SEQ_HEAD):
    """fp64 inputs in ``layout`` -> (O in ``layout``, LSE [Hl,N])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    N, Hl, d = _dims(q, layout)
    o = np.empty_like(q); lse = np.empty((Hl, N), np.float64)
    rc = _load().oracle_attn_fwd(q.ctypes.data, k.ctypes.data, v.ctypes.data, o.ctypes.data,
                                 lse.ctypes.data, N, Hl, d, scale, int(causal), layout)
    if rc:
        raise MemoryError("oracle_attn_fwd")
    return o, lse


def attn_fwd_rows(q, k, v, rows, scale: float, causal: bool = True, layout: int = LAYOUT_SEQ_HEAD):
    """-> (O_rows [n_rows,Hl,d], LSE_rows [Hl,n_rows])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    N, Hl, d = _dims(q, layout)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    o = np.empty((rows.size, Hl, d), np.float64); lse = np.empty((Hl, rows.size), np.float64)
    rc = _load().oracle_attn_fwd_rows(q.ctypes.data, k.ctypes.data, v.ctypes.data, rows.ctypes.data,
                                      rows.size, o.ctypes.data, lse.ctypes.data, N, Hl, d, scale,
                                      int(causal), layout)
    if rc:
        raise MemoryError("oracle_attn_fwd_rows")
    return o, lse


def attn_bwd(q, k, v, dout, scale: float, causal: bool = True, layout: int = LAYOUT_SEQ_HEAD):
    """-> (dQ, dK, dV) in ``layout``, fp64."""
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    N, Hl, d = _dims(q, layout)
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    rc = _load().oracle_attn_bwd(q.ctypes.data, k.ctypes.data, v.ctypes.data, dout.ctypes.data,
                                 dq.ctypes.data, dk.ctypes.data, dv.ctypes.data, N, Hl, d, scale,
                                 int(causal), layout)
    if rc:
        raise MemoryError("oracle_attn_bwd")
    return dq, dk, dv


def _xdims(q, k, layout):
    Nq, Hl, d = _dims(q, layout)
    Nk, Hk, dk = _dims(k, layout)
    if (Hk, dk) != (Hl, d):
        raise ValueError("q and k must agree in heads and head dim")
    if Nk <= 0:
        raise ValueError("cross-attention needs at least one key")
    return Nq, Nk, Hl, d


def xattn_fwd(q, k, v, scale: float, layout: int = LAYOUT_SEQ_HEAD):
    """Cross-attention, no mask: q has Nq tokens, k and v have Nk.  -> (O like q, LSE [Hl,Nq])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    Nq, Nk, Hl, d = _xdims(q, k, layout)
    o = np.empty_like(q); lse = np.empty((Hl, Nq), np.float64)
    rc = _load().oracle_xattn_fwd(q.ctypes.data, k.ctypes.data, v.ctypes.data, o.ctypes.data, lse.ctypes.data,
                                  Nq, Nk, Hl, d, scale, layout)
    if rc:
        raise MemoryError("oracle_xattn_fwd")
    return o, lse


def xattn_bwd(q, k, v, dout, scale: float, layout: int = LAYOUT_SEQ_HEAD):
    """-> (dQ like q, dK, dV like k), fp64."""
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    Nq, Nk, Hl, d = _xdims(q, k, layout)
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(k)
    rc = _load().oracle_xattn_bwd(q.ctypes.data, k.ctypes.data, v.ctypes.data, dout.ctypes.data,
                                  dq.ctypes.data, dk.ctypes.data, dv.ctypes.data, Nq, Nk, Hl, d, scale, layout)
    if rc:
        raise MemoryError("oracle_xattn_bwd")
    return dq, dk, dv


def _block_mask(mask, N, B):
    nb = (N + B - 1) // B
    m = np.ascontiguousarray(np.asarray(mask) != 0, dtype=np.uint8)
    if m.shape != (nb, nb):
        raise ValueError(f"block mask must be {nb} x {nb}")
    return m


def sparse_attn_fwd(q, k, v, mask, B: int, scale: float, layout: int = LAYOUT_SEQ_HEAD):
    """Causal attention restricted to the blocks set in ``mask`` [ceil(N/B), ceil(N/B)] (diagonal required)."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    N, Hl, d = _dims(q, layout)
    m = _block_mask(mask, N, B)
    o = np.empty_like(q); lse = np.empty((Hl, N), np.float64)
    rc = _load().oracle_sparse_attn_fwd(q.ctypes.data, k.ctypes.data, v.ctypes.data, o.ctypes.data, lse.ctypes.data,
                                        m.ctypes.data, B, N, Hl, d, scale, layout)
    if rc == 3:
        raise ValueError("every diagonal block must be set")
    if rc:
        raise MemoryError("oracle_sparse_attn_fwd")
    return o, lse


def sparse_attn_bwd(q, k, v, dout, mask, B: int, scale: float, layout: int = LAYOUT_SEQ_HEAD):
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    N, Hl, d = _dims(q, layout)
    m = _block_mask(mask, N, B)
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    rc = _load().oracle_sparse_attn_bwd(q.ctypes.data, k.ctypes.data, v.ctypes.data, dout.ctypes.data,
                                        dq.ctypes.data, dk.ctypes.data, dv.ctypes.data, m.ctypes.data, B, N, Hl, d,
                                        scale, layout)
    if rc == 3:
        raise ValueError("every diagonal block must be set")
    if rc:
        raise MemoryError("oracle_sparse_attn_bwd")
    return dq, dk, dv


def attn_bwd_rows(q, k, v, dout, rows, scale: float, causal: bool = True, layout: int = LAYOUT_SEQ_HEAD):
    """-> (dQ_rows [n_rows,Hl,d], dK, dV for the dO that is zero outside ``rows``)."""
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    N, Hl, d = _dims(q, layout)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    if rows.size > 1 and not (np.diff(rows) > 0).all():
        raise ValueError("rows must be strictly increasing")
    dq = np.empty((rows.size, Hl, d), np.float64); dk, dv = np.empty_like(q), np.empty_like(q)
    rc = _load().oracle_attn_bwd_rows(q.ctypes.data, k.ctypes.data, v.ctypes.data, dout.ctypes.data,
                                      rows.ctypes.data, rows.size, dq.ctypes.data, dk.ctypes.data,
                                      dv.ctypes.data, N, Hl, d, scale, int(causal), layout)
    if rc:
        raise MemoryError("oracle_attn_bwd_rows")
    return dq, dk, dv
