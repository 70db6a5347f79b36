"""Python binding of libulysses (MI355X / gfx950): argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their device pointers and
the current HIP stream through the C ABI declared in ``include/ulysses.h`` and returns the output
tensors.  PyTorch is used for device memory and streams; all computation happens in the library's
kernels.  There is no CPU fallback: if the library is missing or a call fails, an exception is
raised.
"""
from __future__ import annotations

import ctypes
import os

from . import build as _build

LAYOUT_SEQ_HEAD = 0   # [N, Hl, d]
LAYOUT_HEAD_SEQ = 1   # [Hl, N, d]

EXPORTS = ("ulysses_pack", "ulysses_unpack", "ulysses_pack_rev", "ulysses_unpack_rev",
           "ulysses_pack_qkv", "ulysses_unpack_qkv", "ulysses_pack_rev_qkv", "ulysses_unpack_rev_qkv",
           "ulysses_xattn_fwd_workspace_bytes", "ulysses_xattn_fwd", "ulysses_xattn_bwd_workspace_bytes",
           "ulysses_xattn_bwd",
           "ulysses_sparse_attn_fwd_workspace_bytes", "ulysses_sparse_attn_fwd",
           "ulysses_sparse_attn_bwd_workspace_bytes", "ulysses_sparse_attn_bwd",
           "ulysses_probe_mfma", "ulysses_probe_mfma_lds",
           "ulysses_attn_fwd", "ulysses_attn_fwd_workspace_bytes", "ulysses_attn_fwd_ws",
           "ulysses_attn_bwd_workspace_bytes", "ulysses_attn_bwd", "ulysses_attn_bwd_stage",
           "ulysses_status_string", "ulysses_abi_version")

_lib = None


class UlyssesError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


def load(path: str | None = None):
    """Load libulysses.so (built in-tree by ``build.build_library``).  Raises if it is absent."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or _build.LIB
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: build it with __graft_entry__.build() "
                                "(python -m paper_2309_14509_amd.build)")
    lib = ctypes.CDLL(path)
    vp, i64, ci, cf, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.ulysses_pack.argtypes = [vp, vp, i64, ci, ci, ci, ci, vp]
    lib.ulysses_unpack.argtypes = [vp, vp, i64, ci, ci, ci, ci, ci, vp]
    lib.ulysses_pack_rev.argtypes = [vp, vp, i64, ci, ci, ci, ci, ci, vp]
    lib.ulysses_unpack_rev.argtypes = [vp, vp, i64, ci, ci, ci, ci, vp]
    p3 = ctypes.POINTER(ctypes.c_void_p)      # host array of three device pointers
    lib.ulysses_pack_qkv.argtypes = [p3, p3, i64, ci, ci, ci, ci, vp]
    lib.ulysses_unpack_qkv.argtypes = [p3, p3, i64, ci, ci, ci, ci, ci, vp]
    lib.ulysses_pack_rev_qkv.argtypes = [p3, p3, i64, ci, ci, ci, ci, ci, vp]
    lib.ulysses_unpack_rev_qkv.argtypes = [p3, p3, i64, ci, ci, ci, ci, vp]
    lib.ulysses_attn_fwd.argtypes = [vp, vp, vp, vp, vp, i64, ci, ci, cf, ci, ci, vp]
    lib.ulysses_attn_fwd_workspace_bytes.argtypes = [i64, ci, ci, ci]
    lib.ulysses_attn_fwd_workspace_bytes.restype = sz
    lib.ulysses_attn_fwd_ws.argtypes = [vp, vp, vp, vp, vp, vp, sz, i64, ci, ci, cf, ci, ci, vp]
    lib.ulysses_attn_bwd_workspace_bytes.argtypes = [i64, ci, ci]
    lib.ulysses_attn_bwd_workspace_bytes.restype = sz
    lib.ulysses_attn_bwd.argtypes = [vp] * 10 + [sz, i64, ci, ci, cf, ci, ci, vp]
    lib.ulysses_attn_bwd_stage.argtypes = [ci] + [vp] * 10 + [sz, i64, ci, ci, cf, ci, ci, vp]
    lib.ulysses_xattn_fwd_workspace_bytes.argtypes = [i64, i64, ci, ci]
    lib.ulysses_xattn_fwd_workspace_bytes.restype = sz
    lib.ulysses_xattn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, sz, i64, i64, ci, ci, cf, ci, vp]
    lib.ulysses_xattn_bwd_workspace_bytes.argtypes = [i64, i64, ci, ci]
    lib.ulysses_xattn_bwd_workspace_bytes.restype = sz
    lib.ulysses_xattn_bwd.argtypes = [vp] * 10 + [sz, i64, i64, ci, ci, cf, ci, vp]
    lib.ulysses_sparse_attn_fwd_workspace_bytes.argtypes = [i64, ci, ci]
    lib.ulysses_sparse_attn_fwd_workspace_bytes.restype = sz
    lib.ulysses_sparse_attn_fwd.argtypes = [vp] * 8 + [sz, i64, ci, ci, cf, ci, vp]
    lib.ulysses_sparse_attn_bwd_workspace_bytes.argtypes = [i64, ci, ci]
    lib.ulysses_sparse_attn_bwd_workspace_bytes.restype = sz
    lib.ulysses_sparse_attn_bwd.argtypes = [vp] * 14 + [sz, i64, ci, ci, cf, ci, vp]
    lib.ulysses_probe_mfma.argtypes = [vp, sz, vp, sz, ci, ci, vp]
    lib.ulysses_probe_mfma.restype = ci
    lib.ulysses_probe_mfma_lds.argtypes = [vp, sz, vp, sz, ci, ci, vp]
    lib.ulysses_probe_mfma_lds.restype = ci
    lib.ulysses_status_string.argtypes = [ci]
    lib.ulysses_status_string.restype = ctypes.c_char_p
    for name in ("ulysses_pack", "ulysses_unpack", "ulysses_pack_rev", "ulysses_unpack_rev",
                 "ulysses_pack_qkv", "ulysses_unpack_qkv", "ulysses_xattn_fwd", "ulysses_xattn_bwd",
                 "ulysses_sparse_attn_fwd", "ulysses_sparse_attn_bwd", "ulysses_attn_fwd", "ulysses_attn_bwd", "ulysses_attn_bwd_stage", "ulysses_abi_version"):
        getattr(lib, name).restype = ci
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().ulysses_status_string(status).decode()


def _check(rc: int, where: str):
    if rc != 0:
        raise UlyssesError(rc, where)


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, where):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{where}: tensors must be contiguous GPU tensors")
    return ctypes.c_void_p(t.data_ptr())


# ---- layout transforms ------------------------------------------------------------------------
def ulysses_pack(x, P: int):
    """x [n_local, H, d] -> send [P, n_local, H/P, d]."""
    import torch
    nl, H, d = x.shape
    send = torch.empty((P, nl, H // max(P, 1) if P > 0 else 0, d), dtype=x.dtype, device=x.device)
    _check(load().ulysses_pack(_dev(x, "pack"), _dev(send, "pack"), nl, H, d, P, x.element_size(), _stream()),
           "ulysses_pack")
    return send


def ulysses_unpack(recv, out_layout: int = LAYOUT_SEQ_HEAD):
    """recv [P, n_local, Hl, d] -> y [P*n_local, Hl, d] (or [Hl, P*n_local, d])."""
    import torch
    P, nl, Hl, d = recv.shape
    shape = (Hl, P * nl, d) if out_layout == LAYOUT_HEAD_SEQ else (P * nl, Hl, d)
    y = torch.empty(shape, dtype=recv.dtype, device=recv.device)
    _check(load().ulysses_unpack(_dev(recv, "unpack"), _dev(y, "unpack"), nl, Hl * P, d, P, recv.element_size(),
                                 out_layout, _stream()), "ulysses_unpack")
    return y


def _ptr3(tensors, where):
    if len(tensors) != 3:
        raise ValueError(f"{where}: exactly three tensors (q, k, v) are expected")
    return (ctypes.c_void_p * 3)(*[t.data_ptr() if _dev(t, where) is not None else None for t in tensors])


def ulysses_pack_qkv(xs, P: int):
    """Three tensors x [n_local, H, d] of one shape and dtype -> three send buffers, in one launch."""
    import torch
    nl, H, d = xs[0].shape
    if any(x.shape != xs[0].shape or x.dtype != xs[0].dtype for x in xs):
        raise ValueError("ulysses_pack_qkv: the three tensors must share shape and dtype")
    sends = [torch.empty((P, nl, H // max(P, 1) if P > 0 else 0, d), dtype=x.dtype, device=x.device) for x in xs]
    _check(load().ulysses_pack_qkv(_ptr3(xs, "pack_qkv"), _ptr3(sends, "pack_qkv"), nl, H, d, P,
                                   xs[0].element_size(), _stream()), "ulysses_pack_qkv")
    return sends


def ulysses_unpack_qkv(recvs, out_layout: int = LAYOUT_SEQ_HEAD):
    """Three receive buffers [P, n_local, Hl, d] -> three tensors [P*n_local, Hl, d] (or head-major), in one launch."""
    import torch
    P, nl, Hl, d = recvs[0].shape
    if any(r.shape != recvs[0].shape or r.dtype != recvs[0].dtype for r in recvs):
        raise ValueError("ulysses_unpack_qkv: the three tensors must share shape and dtype")
    shape = (Hl, P * nl, d) if out_layout == LAYOUT_HEAD_SEQ else (P * nl, Hl, d)
    ys = [torch.empty(shape, dtype=r.dtype, device=r.device) for r in recvs]
    _check(load().ulysses_unpack_qkv(_ptr3(recvs, "unpack_qkv"), _ptr3(ys, "unpack_qkv"), nl, Hl * P, d, P,
                                     recvs[0].element_size(), out_layout, _stream()), "ulysses_unpack_qkv")
    return ys


def ulysses_pack_rev(o, P: int, in_layout: int = LAYOUT_SEQ_HEAD):
    """o [N, Hl, d] (or [Hl, N, d]) -> send [P, N/P, Hl, d]."""
    import torch
    if in_layout == LAYOUT_HEAD_SEQ:
        Hl, N, d = o.shape
    else:
        N, Hl, d = o.shape
    if P <= 0 or N % P:
        raise ValueError("N must be a multiple of P")
    send = torch.empty((P, N // P, Hl, d), dtype=o.dtype, device=o.device)
    _check(load().ulysses_pack_rev(_dev(o, "pack_rev"), _dev(send, "pack_rev"), N // P, Hl * P, d, P,
                                   o.element_size(), in_layout, _stream()), "ulysses_pack_rev")
    return send


def ulysses_unpack_rev(recv):
    """recv [P, n_local, Hl, d] -> y [n_local, P*Hl, d]."""
    import torch
    P, nl, Hl, d = recv.shape
    y = torch.empty((nl, P * Hl, d), dtype=recv.dtype, device=recv.device)
    _check(load().ulysses_unpack_rev(_dev(recv, "unpack_rev"), _dev(y, "unpack_rev"), nl, Hl * P, d, P,
                                     recv.element_size(), _stream()), "ulysses_unpack_rev")
    return y


def ulysses_pack_rev_qkv(gs, P: int, in_layout: int = LAYOUT_SEQ_HEAD):
    """Three tensors [N, Hl, d] (or [Hl, N, d]) of one shape and dtype -> three send buffers [P, N/P, Hl, d]."""
    import torch
    if any(g.shape != gs[0].shape or g.dtype != gs[0].dtype for g in gs):
        raise ValueError("ulysses_pack_rev_qkv: the three tensors must share shape and dtype")
    if in_layout == LAYOUT_HEAD_SEQ:
        Hl, N, d = gs[0].shape
    else:
        N, Hl, d = gs[0].shape
    if P <= 0 or N % P:
        raise ValueError("N must be a multiple of P")
    sends = [torch.empty((P, N // P, Hl, d), dtype=g.dtype, device=g.device) for g in gs]
    _check(load().ulysses_pack_rev_qkv(_ptr3(gs, "pack_rev_qkv"), _ptr3(sends, "pack_rev_qkv"), N // P, Hl * P, d, P,
                                       gs[0].element_size(), in_layout, _stream()), "ulysses_pack_rev_qkv")
    return sends


def ulysses_unpack_rev_qkv(recvs):
    """Three receive buffers [P, n_local, Hl, d] -> three tensors [n_local, P*Hl, d], in one launch."""
    import torch
    P, nl, Hl, d = recvs[0].shape
    if any(r.shape != recvs[0].shape or r.dtype != recvs[0].dtype for r in recvs):
        raise ValueError("ulysses_unpack_rev_qkv: the three tensors must share shape and dtype")
    ys = [torch.empty((nl, P * Hl, d), dtype=r.dtype, device=r.device) for r in recvs]
    _check(load().ulysses_unpack_rev_qkv(_ptr3(recvs, "unpack_rev_qkv"), _ptr3(ys, "unpack_rev_qkv"), nl, Hl * P, d, P,
                                         recvs[0].element_size(), _stream()), "ulysses_unpack_rev_qkv")
    return ys


# ---- attention ----------------------------------------------------------------------------------
def _attn_dims(q, layout):
    if layout == LAYOUT_HEAD_SEQ:
        Hl, N, d = q.shape
    else:
        N, Hl, d = q.shape
    return N, Hl, d


ELEM_BF16, ELEM_F16 = 0, 0x100


def _elem_flag(*tensors):
    """The element-type flag the attention entry points take on their layout argument: all tensors
    bfloat16 -> 0, all float16 -> ELEM_F16."""
    import torch
    kinds = {t.dtype for t in tensors}
    if kinds == {torch.bfloat16}:
        return ELEM_BF16
    if kinds == {torch.float16}:
        return ELEM_F16
    raise ValueError("attention tensors must all be bfloat16 or all be float16")


def ulysses_attn_fwd_workspace_bytes(N: int, Hl: int, d: int, causal: bool = True) -> int:
    return int(load().ulysses_attn_fwd_workspace_bytes(N, Hl, d, int(causal)))


def ulysses_attn_fwd(q, k, v, scale: float, causal: bool = True, layout: int = LAYOUT_SEQ_HEAD, out=None, lse=None,
                     workspace=None):
    """bf16 (or fp16) q, k, v in ``layout`` -> (o of the same type in ``layout``, lse fp32 [Hl, N]).  With a
    ``workspace`` (uint8, ulysses_attn_fwd_workspace_bytes) the call goes through ulysses_attn_fwd_ws."""
    import torch
    elem = _elem_flag(q, k, v)
    N, Hl, d = _attn_dims(q, layout)
    o = torch.empty_like(q) if out is None else out
    lse = torch.empty((Hl, N), dtype=torch.float32, device=q.device) if lse is None else lse
    if workspace is not None:
        _check(load().ulysses_attn_fwd_ws(_dev(q, "attn_fwd"), _dev(k, "attn_fwd"), _dev(v, "attn_fwd"), _dev(o, "attn_fwd"),
                                          _dev(lse, "attn_fwd"), _dev(workspace, "attn_fwd"), workspace.numel(), N, Hl, d,
                                          scale, int(causal), layout | elem, _stream()), "ulysses_attn_fwd_ws")
        return o, lse
    _check(load().ulysses_attn_fwd(_dev(q, "attn_fwd"), _dev(k, "attn_fwd"), _dev(v, "attn_fwd"), _dev(o, "attn_fwd"),
                                   _dev(lse, "attn_fwd"), N, Hl, d, scale, int(causal), layout | elem, _stream()),
           "ulysses_attn_fwd")
    return o, lse


def ulysses_attn_bwd_workspace_bytes(N: int, Hl: int, d: int) -> int:
    return int(load().ulysses_attn_bwd_workspace_bytes(N, Hl, d))


BWD_STAGE_DELTA, BWD_STAGE_DKV, BWD_STAGE_DQ = 0, 1, 2


def ulysses_attn_bwd(q, k, v, o, dout, lse, scale: float, causal: bool = True, layout: int = LAYOUT_SEQ_HEAD,
                     workspace=None, out=None, stage=None):
    """-> (dq, dk, dv) bf16 in ``layout``.  ``stage`` (one of BWD_STAGE_*) runs a single stage of the
    backward pass through ulysses_attn_bwd_stage; the caller then supplies ``workspace`` and ``out``."""
    import torch
    elem = _elem_flag(q, k, v, o, dout)
    N, Hl, d = _attn_dims(q, layout)
    need = ulysses_attn_bwd_workspace_bytes(N, Hl, d)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    dq, dk, dv = (torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)) if out is None else out
    args = (_dev(q, "attn_bwd"), _dev(k, "attn_bwd"), _dev(v, "attn_bwd"), _dev(o, "attn_bwd"),
            _dev(dout, "attn_bwd"), _dev(lse, "attn_bwd"), _dev(dq, "attn_bwd"), _dev(dk, "attn_bwd"),
            _dev(dv, "attn_bwd"), _dev(workspace, "attn_bwd"), workspace.numel() * workspace.element_size(),
            N, Hl, d, scale, int(causal), layout | elem, _stream())
    if stage is None:
        _check(load().ulysses_attn_bwd(*args), "ulysses_attn_bwd")
    else:
        _check(load().ulysses_attn_bwd_stage(int(stage), *args), "ulysses_attn_bwd_stage")
    return dq, dk, dv


def ulysses_xattn_fwd(q, k, v, scale: float, layout: int = LAYOUT_SEQ_HEAD):
    """Cross-attention, no mask: bf16 q (Nq tokens), k, v (Nk tokens) in ``layout`` -> (o like q, lse fp32 [Hl, Nq])."""
    import torch
    elem = _elem_flag(q, k, v)
    Nq, Hl, d = _attn_dims(q, layout)
    Nk = _attn_dims(k, layout)[0]
    o = torch.empty_like(q)
    lse = torch.empty((Hl, Nq), dtype=torch.float32, device=q.device)
    need = int(load().ulysses_xattn_fwd_workspace_bytes(Nq, Nk, Hl, d))
    workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    _check(load().ulysses_xattn_fwd(_dev(q, "xattn_fwd"), _dev(k, "xattn_fwd"), _dev(v, "xattn_fwd"),
                                    _dev(o, "xattn_fwd"), _dev(lse, "xattn_fwd"), _dev(workspace, "xattn_fwd"),
                                    workspace.numel(), Nq, Nk, Hl, d, scale, layout | elem, _stream()),
           "ulysses_xattn_fwd")
    return o, lse


def ulysses_xattn_bwd(q, k, v, o, dout, lse, scale: float, layout: int = LAYOUT_SEQ_HEAD):
    """-> (dq like q, dk, dv like k) bf16."""
    import torch
    elem = _elem_flag(q, k, v, o, dout)
    Nq, Hl, d = _attn_dims(q, layout)
    Nk = _attn_dims(k, layout)[0]
    need = int(load().ulysses_xattn_bwd_workspace_bytes(Nq, Nk, Hl, d))
    workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(k)
    w = "xattn_bwd"
    _check(load().ulysses_xattn_bwd(_dev(q, w), _dev(k, w), _dev(v, w), _dev(o, w), _dev(dout, w), _dev(lse, w),
                                    _dev(dq, w), _dev(dk, w), _dev(dv, w), _dev(workspace, w), workspace.numel(),
                                    Nq, Nk, Hl, d, scale, layout | elem, _stream()), "ulysses_xattn_bwd")
    return dq, dk, dv


SPARSE_BLOCK = 256


class SparsePattern:
    """A block-sparse causal pattern in the compressed form the library takes (device int32 arrays).
    ``mask`` is a [nb, nb] boolean array over 256-token blocks; only its lower triangle is used and every
    diagonal block must be set.  Built and checked on the host."""

    def __init__(self, mask, device="cuda"):
        import numpy as np
        import torch
        m = np.asarray(mask).astype(bool)
        if m.ndim != 2 or m.shape[0] != m.shape[1]:
            raise ValueError("block mask must be square")
        m = np.tril(m)
        if not m.diagonal().all():
            raise ValueError("every diagonal block must be set")
        self.nb = m.shape[0]
        rows, cols = np.nonzero(m)                      # row-major order: ascending columns inside a row
        self.row_ptr = np.concatenate([[0], np.cumsum(m.sum(1))]).astype(np.int32)
        self.col_idx = cols.astype(np.int32)
        cols_t, rows_t = np.nonzero(m.T)                # column-major: ascending rows inside a column
        self.col_ptr = np.concatenate([[0], np.cumsum(m.sum(0))]).astype(np.int32)
        self.row_idx = rows_t.astype(np.int32)
        self.nnz = int(m.sum())
        self.dev = {n: torch.from_numpy(getattr(self, n)).to(device)
                    for n in ("row_ptr", "col_idx", "col_ptr", "row_idx")}


def _pattern_for(pattern, N):
    if pattern.nb != (N + SPARSE_BLOCK - 1) // SPARSE_BLOCK:
        raise ValueError("pattern does not match the sequence length")
    return pattern.dev


def ulysses_sparse_attn_fwd_workspace_bytes(N: int, Hl: int, d: int) -> int:
    return int(load().ulysses_sparse_attn_fwd_workspace_bytes(N, Hl, d))


def ulysses_sparse_attn_fwd(q, k, v, pattern: SparsePattern, scale: float, layout: int = LAYOUT_SEQ_HEAD,
                            out=None, lse=None, workspace=None):
    """Causal attention restricted to the blocks of ``pattern`` -> (o, lse).  ``workspace`` (uint8,
    ulysses_sparse_attn_fwd_workspace_bytes) is allocated here unless the caller brings it."""
    import torch
    elem = _elem_flag(q, k, v)
    N, Hl, d = _attn_dims(q, layout)
    p = _pattern_for(pattern, N)
    o = torch.empty_like(q) if out is None else out
    lse = torch.empty((Hl, N), dtype=torch.float32, device=q.device) if lse is None else lse
    if workspace is None:
        workspace = torch.empty(max(ulysses_sparse_attn_fwd_workspace_bytes(N, Hl, d), 16), dtype=torch.uint8,
                                device=q.device)
    w = "sparse_attn_fwd"
    _check(load().ulysses_sparse_attn_fwd(_dev(q, w), _dev(k, w), _dev(v, w), _dev(o, w), _dev(lse, w),
                                          _dev(p["row_ptr"], w), _dev(p["col_idx"], w), _dev(workspace, w),
                                          workspace.numel(), N, Hl, d, scale, layout | elem, _stream()),
           "ulysses_sparse_attn_fwd")
    return o, lse


def ulysses_sparse_attn_bwd_workspace_bytes(N: int, Hl: int, d: int) -> int:
    return int(load().ulysses_sparse_attn_bwd_workspace_bytes(N, Hl, d))


def ulysses_sparse_attn_bwd(q, k, v, o, dout, lse, pattern: SparsePattern, scale: float,
                            layout: int = LAYOUT_SEQ_HEAD, workspace=None, out=None):
    """-> (dq, dk, dv) in ``layout``.  ``workspace`` (uint8, ulysses_sparse_attn_bwd_workspace_bytes) and ``out``
    are allocated here unless the caller brings them."""
    import torch
    elem = _elem_flag(q, k, v, o, dout)
    N, Hl, d = _attn_dims(q, layout)
    p = _pattern_for(pattern, N)
    if workspace is None:
        workspace = torch.empty(max(ulysses_sparse_attn_bwd_workspace_bytes(N, Hl, d), 16), dtype=torch.uint8,
                                device=q.device)
    dq, dk, dv = (torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)) if out is None else out
    w = "sparse_attn_bwd"
    _check(load().ulysses_sparse_attn_bwd(_dev(q, w), _dev(k, w), _dev(v, w), _dev(o, w), _dev(dout, w), _dev(lse, w),
                                          _dev(dq, w), _dev(dk, w), _dev(dv, w), _dev(p["row_ptr"], w),
                                          _dev(p["col_idx"], w), _dev(p["col_ptr"], w), _dev(p["row_idx"], w),
                                          _dev(workspace, w), workspace.numel(), N, Hl, d, scale, layout | elem,
                                          _stream()),
           "ulysses_sparse_attn_bwd")
    return dq, dk, dv
