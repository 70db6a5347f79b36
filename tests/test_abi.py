"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and rejects
bad arguments before touching the device (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

import paper_2309_14509_amd as uly
from paper_2309_14509_amd import build as uly_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if uly_build.is_stale():
        uly_build.build_library()
    return uly.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "ulysses.h")).read()
    declared = set(re.findall(r"\b(ulysses_[a-z_]+)\s*\(", header))
    assert declared == set(uly.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.ulysses_abi_version() == 1


def test_status_strings(lib):
    seen = {uly.status_string(s) for s in range(8)}
    assert len(seen) == 8 and uly.status_string(0) == "ok"
    assert uly.status_string(1234) == "unknown status"


A, B, C_, D_ = 0x10000, 0x20000000, 0x40000000, 0x60000000   # fake, aligned, far apart "device" addresses


def _pack(lib, x=A, s=B, nl=16, H=8, d=64, P=4, eb=2):
    return lib.ulysses_pack(x, s, nl, H, d, P, eb, None)


def test_layout_validation_happens_before_any_device_call(lib):
    assert _pack(lib, x=None) == 1 and _pack(lib, s=None) == 1
    assert _pack(lib, P=3) == 2 and _pack(lib, P=0) == 2 and _pack(lib, nl=-1) == 2 and _pack(lib, d=0) == 2
    assert _pack(lib, P=16) == 2                       # more ranks than heads
    assert _pack(lib, eb=3) == 3 and _pack(lib, eb=8) == 3
    assert _pack(lib, x=A + 2) == 4 and _pack(lib, s=B + 8) == 4
    assert _pack(lib, s=A) == 5 and _pack(lib, s=A + 16 * 8 * 64 * 2 - 16) == 5
    assert lib.ulysses_unpack(A, B, 16, 8, 64, 4, 2, 7, None) == 3
    assert lib.ulysses_pack_rev(A, B, 16, 8, 64, 4, 2, -1, None) == 3
    assert lib.ulysses_unpack_rev(A, A, 16, 8, 64, 4, 2, None) == 5
    assert lib.ulysses_pack(A, B, 1 << 61, 8, 64, 4, 2, None) == 2          # size overflow


def test_qkv_transform_validation(lib):
    """Three tensors in one launch: the pointer arrays are host arrays of device pointers."""
    import ctypes as ct
    arr = lambda *p: (ct.c_void_p * 3)(*p)
    size = 16 * 8 * 64 * 2
    ins, outs = arr(A, A + size, A + 2 * size), arr(B, B + size, B + 2 * size)
    assert lib.ulysses_pack_qkv(None, outs, 16, 8, 64, 4, 2, None) == 1
    assert lib.ulysses_pack_qkv(arr(A, None, A + 2 * size), outs, 16, 8, 64, 4, 2, None) == 1
    assert lib.ulysses_pack_qkv(ins, outs, 16, 8, 64, 3, 2, None) == 2
    assert lib.ulysses_pack_qkv(ins, outs, 16, 8, 64, 4, 3, None) == 3
    assert lib.ulysses_pack_qkv(arr(A, A + size + 4, A + 2 * size), outs, 16, 8, 64, 4, 2, None) == 4
    # an output of one tensor overlapping the input of another, or another output
    assert lib.ulysses_pack_qkv(ins, arr(B, A + 2 * size, B + 2 * size), 16, 8, 64, 4, 2, None) == 5
    assert lib.ulysses_pack_qkv(ins, arr(B, B + size - 16, B + 2 * size), 16, 8, 64, 4, 2, None) == 5
    assert lib.ulysses_unpack_qkv(ins, outs, 16, 8, 64, 4, 2, 9, None) == 3
    # empty tensors: nothing to do, pointers inside the arrays are not looked at
    assert lib.ulysses_pack_qkv(arr(None, None, None), arr(None, None, None), 0, 8, 64, 4, 2, None) == 0
    assert lib.ulysses_unpack_qkv(arr(None, None, None), arr(None, None, None), 0, 8, 64, 4, 2, 0, None) == 0
    # the reverse direction (dQ, dK, dV): same checks
    assert lib.ulysses_pack_rev_qkv(ins, None, 16, 8, 64, 4, 2, 0, None) == 1
    assert lib.ulysses_pack_rev_qkv(ins, outs, 16, 8, 64, 4, 2, 7, None) == 3
    assert lib.ulysses_pack_rev_qkv(ins, arr(B, B + size - 16, B + 2 * size), 16, 8, 64, 4, 2, 1, None) == 5
    assert lib.ulysses_unpack_rev_qkv(arr(A, A + size, None), outs, 16, 8, 64, 4, 2, None) == 1
    assert lib.ulysses_unpack_rev_qkv(ins, outs, 16, 8, 64, 3, 2, None) == 2
    assert lib.ulysses_unpack_rev_qkv(arr(None, None, None), arr(None, None, None), 0, 8, 64, 4, 2, None) == 0


def _fwd(lib, q=A, k=B, v=C_, o=D_, lse=0x7000000, N=128, Hl=2, d=64, scale=0.125, causal=1, layout=0):
    return lib.ulysses_attn_fwd(q, k, v, o, lse, N, Hl, d, scale, causal, layout, None)


def test_attention_forward_validation(lib):
    assert _fwd(lib, q=None) == 1 and _fwd(lib, lse=None) == 1
    assert _fwd(lib, N=-5) == 2 and _fwd(lib, Hl=0) == 2 and _fwd(lib, N=1 << 31) == 2
    assert _fwd(lib, Hl=(1 << 16) + 1, N=8) == 2                              # a token row of more than 2^22 elements
    assert _fwd(lib, d=96) == 3 and _fwd(lib, layout=2) == 3
    assert _fwd(lib, scale=0.0) == 3 and _fwd(lib, scale=-1.0) == 3
    assert _fwd(lib, scale=float("nan")) == 3 and _fwd(lib, scale=float("inf")) == 3
    assert _fwd(lib, k=B + 4) == 4
    assert _fwd(lib, o=A) == 5 and _fwd(lib, lse=D_) == 5
    assert _fwd(lib, N=0) == 0                                               # empty: ok, no launch


def test_attention_forward_with_workspace_validation(lib):
    wb = lib.ulysses_attn_fwd_workspace_bytes
    assert wb(131072, 4, 128, 1) == 0                   # 2048 query tiles: nothing would be cut
    need = wb(32768, 2, 128, 1)                         # 256 query tiles: long rows are cut
    assert 0 < need <= 600 << 20 and wb(32768, 2, 256, 1) == 0 and wb(0, 2, 128, 1) == 0 and wb(-4, 2, 128, 1) == 0
    assert wb(2048, 4, 128, 0) == lib.ulysses_xattn_fwd_workspace_bytes(2048, 2048, 4, 128)

    def call(ws=0xB0000000, wsb=need, N=32768, Hl=2, d=128, causal=1, q=A):
        return lib.ulysses_attn_fwd_ws(q, B, C_, D_, 0x7000000, ws, wsb, N, Hl, d, 0.1, causal, 0, None)
    assert call(ws=None) == 6 and call(wsb=need - 1) == 6 and call(ws=0xB0000008) == 4 and call(ws=A) == 5
    assert call(q=None) == 1 and call(N=-1) == 2 and call(d=80) == 3
    assert call(N=0, ws=None, wsb=0) == 0               # empty: nothing to do


def test_attention_backward_validation(lib):
    ws_need = lib.ulysses_attn_bwd_workspace_bytes(128, 2, 64)
    assert ws_need >= 2 * 128 * 2 * 4
    assert lib.ulysses_attn_bwd_workspace_bytes(0, 2, 64) == 0
    base = dict(q=A, k=B, v=C_, o=D_, dout=0x80000000, lse=0x7000000, dq=0xA0000000, dk=0xC0000000,
                dv=0xE0000000, ws=0x9000000, wsb=ws_need, N=128, Hl=2, d=64, scale=0.125, causal=1, layout=0)

    def call(**kw):
        a = dict(base); a.update(kw)
        return lib.ulysses_attn_bwd(a["q"], a["k"], a["v"], a["o"], a["dout"], a["lse"], a["dq"], a["dk"], a["dv"],
                                    a["ws"], a["wsb"], a["N"], a["Hl"], a["d"], a["scale"], a["causal"],
                                    a["layout"], None)
    assert call(dout=None) == 1 and call(dv=None) == 1
    assert call(d=32) == 3 and call(scale=-0.5) == 3
    assert call(ws=None) == 6 and call(wsb=ws_need - 1) == 6
    assert call(dq=0xA0000008) == 4
    assert call(dk=A) == 5 and call(dq=0xC0000000) == 5 and call(ws=0x7000000) == 5
    assert call(N=0, ws=None, wsb=0) == 0


def test_element_type_flag(lib):
    """ULY_ELEM_F16 rides on the layout word of the attention entry points; validation is the same for both
    element types, unknown bits stay unsupported, and the layout transforms (elem_bytes) refuse the flag."""
    F16 = 0x100
    assert uly.ELEM_F16 == F16
    for layout in (0 | F16, 1 | F16):
        assert _fwd(lib, layout=layout, N=0) == 0
        assert _fwd(lib, layout=layout, q=None) == 1 and _fwd(lib, layout=layout, o=A) == 5
    assert _fwd(lib, layout=2 | F16) == 3 and _fwd(lib, layout=0x200) == 3
    assert lib.ulysses_unpack(A, B, 64, 8, 64, 4, 2, F16, None) == 3
    assert lib.ulysses_pack_rev(A, B, 64, 8, 64, 4, 2, F16, None) == 3


def test_binding_refuses_a_missing_library(tmp_path):
    with pytest.raises(FileNotFoundError):
        uly.load(str(tmp_path / "nope.so"))


def test_build_scratch_report_parser():
    """The build refuses attention kernels that use scratch memory; this checks the parser it relies on."""
    from paper_2309_14509_amd import build
    text = (
        "a.hip:1:1: remark: Function Name: _Zk1 [-Rpass-analysis=kernel-resource-usage]\n"
        "a.hip:1:1: remark:     VGPRs: 254 [-Rpass-analysis=kernel-resource-usage]\n"
        "a.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]\n"
        "a.hip:9:1: remark: Function Name: _Zk2 [-Rpass-analysis=kernel-resource-usage]\n"
        "a.hip:9:1: remark:     ScratchSize [bytes/lane]: 120 [-Rpass-analysis=kernel-resource-usage]\n"
    )
    assert build.scratch_bytes(text) == {"_Zk1": 0, "_Zk2": 120}
    assert build.scratch_bytes("no remarks here") == {}


def test_cross_attention_validation(lib):
    f = lambda **kw: lib.ulysses_xattn_fwd(*[{**dict(q=A, k=B, v=C_, o=D_, lse=0x7000000, ws=None, wsb=0, Nq=128, Nk=96,
                                                      Hl=2, d=64, scale=0.125, layout=0), **kw}[n]
                                             for n in ("q", "k", "v", "o", "lse", "ws", "wsb", "Nq", "Nk", "Hl", "d",
                                                       "scale", "layout")],
                                           None)
    assert f(q=None) == 1 and f(k=None) == 1
    assert f(Nq=-1) == 2 and f(Nk=-3) == 2 and f(Nk=0) == 2       # no keys: softmax undefined
    assert f(Nq=0, Nk=0) == 0 and f(Nq=0) == 0
    assert f(d=96) == 3 and f(scale=0.0) == 3 and f(layout=5) == 3
    assert f(v=C_ + 4) == 4
    assert f(o=B + 96 * 2 * 64 * 2 - 32) == 5                      # o overlaps the end of k (sized by Nk)
    # workspaces: nothing extra while both sides have enough (or too few) tokens to cut; few queries over many
    # keys take a forward workspace and a larger backward one, bounded whatever the sizes
    assert lib.ulysses_xattn_fwd_workspace_bytes(128, 96, 2, 64) == 0
    assert lib.ulysses_xattn_bwd_workspace_bytes(128, 96, 2, 64) == lib.ulysses_attn_bwd_workspace_bytes(128, 2, 64)
    assert lib.ulysses_xattn_fwd_workspace_bytes(1 << 17, 1 << 17, 4, 128) == 0
    fw = lib.ulysses_xattn_fwd_workspace_bytes(2048, 1 << 17, 4, 128)
    assert 0 < fw <= 600 << 20
    assert lib.ulysses_xattn_bwd_workspace_bytes(2048, 1 << 17, 4, 128) > lib.ulysses_attn_bwd_workspace_bytes(2048, 4, 128)
    for shape in ((2048, 1 << 20, 1, 128), (1 << 20, 2048, 1, 128), (300, 1 << 20, 3, 64), (1 << 20, 130, 2, 128)):
        assert lib.ulysses_xattn_bwd_workspace_bytes(*shape) <= 600 << 20 and lib.ulysses_xattn_fwd_workspace_bytes(*shape) <= 600 << 20
    big = dict(Nq=2048, Nk=1 << 17, Hl=4, d=128)
    assert f(**big, ws=None, wsb=0) == 6 and f(**big, ws=0xB0000000, wsb=fw - 1) == 6
    assert f(**big, ws=0xB0000008, wsb=fw) == 4
    assert lib.ulysses_xattn_fwd_workspace_bytes(0, 5, 2, 64) == 0 and lib.ulysses_xattn_fwd_workspace_bytes(5, 5, 2, 100) == 0
    g = lambda **kw: lib.ulysses_xattn_bwd(*[{**dict(q=A, k=B, v=C_, o=D_, do=0x70000000, lse=0x7800000, dq=0x80000000,
                                                      dk=0x90000000, dv=0xA0000000, ws=0xB0000000, wsb=1 << 20, Nq=128,
                                                      Nk=96, Hl=2, d=64, scale=0.125, layout=0), **kw}[n]
                                             for n in ("q", "k", "v", "o", "do", "lse", "dq", "dk", "dv", "ws", "wsb",
                                                       "Nq", "Nk", "Hl", "d", "scale", "layout")], None)
    assert g(dk=None) == 1 and g(Nk=0) == 2 and g(Nq=0) == 2 and g(Nq=0, Nk=0) == 0
    assert g(wsb=16) == 6 and g(ws=None) == 6
    assert g(dv=B + 64) == 5


def test_sparse_attention_validation(lib):
    RP, CI, CP, RI = 0xC0000000, 0xC1000000, 0xC2000000, 0xC3000000
    f = lambda **kw: lib.ulysses_sparse_attn_fwd(*[{**dict(q=A, k=B, v=C_, o=D_, lse=0x7000000, rp=RP, ci=CI, ws=0xB0000000,
                                                            wsb=4 << 20, N=600, Hl=2, d=64, scale=0.125, layout=0), **kw}[n]
                                                   for n in ("q", "k", "v", "o", "lse", "rp", "ci", "ws", "wsb", "N", "Hl", "d",
                                                             "scale", "layout")], None)
    fneed = lib.ulysses_sparse_attn_fwd_workspace_bytes(600, 2, 64)
    assert 0 < fneed <= 4 << 20 and f(ws=None) == 6 and f(wsb=fneed - 1) == 6 and f(ws=0xB0000004) == 4 and f(ws=A) == 5
    assert lib.ulysses_sparse_attn_fwd_workspace_bytes(1 << 20, 4, 128) <= 2048 * 256 * 130 * 4 + (4 << 20)
    assert lib.ulysses_sparse_attn_fwd_workspace_bytes(0, 2, 64) == 0 and f(N=8000001) == 2
    assert f(rp=None) == 1 and f(ci=None) == 1 and f(v=None) == 1
    assert f(N=-1) == 2 and f(d=100) == 3 and f(scale=-1.0) == 3
    assert f(d=256) == 3 and _fwd(lib, d=256, N=0) == 0         # d = 256: dense attention only
    assert f(rp=RP + 2) == 4 and f(q=A + 8) == 4
    assert f(o=A) == 5 and f(N=0, rp=None, ci=None) == 0
    # statistics as for the dense backward, plus a work plan and a bounded number of fp32 partial-sum slots
    assert lib.ulysses_sparse_attn_bwd_workspace_bytes(600, 2, 64) > lib.ulysses_attn_bwd_workspace_bytes(600, 2, 64)
    big, slot = lib.ulysses_sparse_attn_bwd_workspace_bytes(1 << 20, 4, 128), 2 * 128 * 128 * 4
    # dK/dV: at most 8192 slots of two 128 x d fp32 tensors; dQ: at most 4096 slots of one; plans and tables: a few MiB
    assert big - lib.ulysses_attn_bwd_workspace_bytes(1 << 20, 4, 128) <= 8192 * slot + 4096 * slot // 2 + (4 << 20)
    assert lib.ulysses_sparse_attn_bwd_workspace_bytes(0, 4, 128) == 0
    assert lib.ulysses_sparse_attn_bwd_workspace_bytes(600, 2, 100) == 0
    g = lambda **kw: lib.ulysses_sparse_attn_bwd(*[{**dict(q=A, k=B, v=C_, o=D_, do=0x70000000, lse=0x7800000,
                                                            dq=0x80000000, dk=0x90000000, dv=0xA0000000, rp=RP, ci=CI,
                                                            cp=CP, ri=RI, ws=0xB0000000, wsb=4 << 20, N=600, Hl=2, d=64,
                                                            scale=0.125, layout=0), **kw}[n]
                                                   for n in ("q", "k", "v", "o", "do", "lse", "dq", "dk", "dv", "rp", "ci",
                                                             "cp", "ri", "ws", "wsb", "N", "Hl", "d", "scale", "layout")],
                                                 None)
    assert g(N=8000001) == 2 and lib.ulysses_sparse_attn_bwd_workspace_bytes(8000001, 2, 64) == 0
    assert g(cp=None) == 1 and g(ri=None) == 1 and g(wsb=8) == 6 and g(ri=RI + 1) == 4 and g(dq=A) == 5


def test_probe_validation(lib):
    ok = dict(data=A, db=65536, sink=B, sb=256 * 256 * 4, blocks=256, iters=10)
    for entry in (lib.ulysses_probe_mfma, lib.ulysses_probe_mfma_lds):
        f = lambda **kw: entry(*[{**ok, **kw}[n] for n in ("data", "db", "sink", "sb", "blocks", "iters")], None)
        assert f(data=None) == 1 and f(sink=None) == 1 and f(blocks=0) == 2 and f(db=1000) == 6
    f = lambda **kw: lib.ulysses_probe_mfma(*[{**ok, **kw}[n] for n in ("data", "db", "sink", "sb", "blocks", "iters")], None)
    assert f(data=None) == 1 and f(sink=None) == 1
    assert f(blocks=0) == 2 and f(iters=0) == 2 and f(blocks=1 << 20) == 2
    assert f(data=A + 4) == 4
    assert f(db=1000) == 6 and f(sb=1024) == 6
