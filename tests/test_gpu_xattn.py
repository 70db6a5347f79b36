"""GPU parity of cross-attention (Nq queries over Nk keys, no mask) against the fp64 oracle, through
the C ABI.  Same tolerances as self-attention (see test_gpu_attention.py)."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as synth
from _util import f64_of, max_abs, o_within_tolerance, rel_l2, to_gpu_bf16

pytestmark = pytest.mark.gpu

TOL_O, TOL_G, TOL_LSE = 1e-2, 2e-2, 2e-3

SHAPES = [(1, 1), (1, 300), (300, 1), (64, 200), (257, 129), (129, 257), (700, 333), (333, 1100), (1500, 40)]


def _inputs(Nq, Nk, Hl, d, seed, layout):
    q, _, _, do = synth.attention_inputs(Nq, Hl, d, seed)
    _, k, v, _ = synth.attention_inputs(Nk, Hl, d, seed + 1)
    arrs = [q, k, v, do]
    if layout == 1:
        arrs = [np.ascontiguousarray(a.transpose(1, 0, 2)) for a in arrs]
    return arrs


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("Nq,Nk", SHAPES)
def test_cross_attention_parity(gpu_lib, Nq, Nk, d, layout):
    Hl, scale = 2, 1.0 / np.sqrt(d)
    q, k, v, do = _inputs(Nq, Nk, Hl, d, 1000 + Nq + Nk, layout)
    tq, tk, tv, tdo = (to_gpu_bf16(a) for a in (q, k, v, do))
    o, lse = gpu_lib.ulysses_xattn_fwd(tq, tk, tv, scale, layout)
    dq, dk, dv = gpu_lib.ulysses_xattn_bwd(tq, tk, tv, o, tdo, lse, scale, layout)
    torch.cuda.synchronize()
    fq, fk, fv, fdo = (oracle.bf16_to_f64(a) for a in (q, k, v, do))
    o_ref, lse_ref = oracle.xattn_fwd(fq, fk, fv, scale, layout)
    o_abs, _ = oracle.xattn_fwd(fq, fk, np.abs(fv), scale, layout)
    ok, worst, n_bad = o_within_tolerance(f64_of(o), o_ref, o_abs, TOL_O)
    assert ok, (worst, n_bad)
    assert max_abs(f64_of(lse), lse_ref) <= TOL_LSE
    for name, got, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), oracle.xattn_bwd(fq, fk, fv, fdo, scale, layout)):
        assert got.shape == ref.shape
        err = rel_l2(f64_of(got), ref)
        assert err <= TOL_G, (name, err)


def _parity(gpu_lib, Nq, Nk, Hl, d, layout, seed):
    scale = 1.0 / np.sqrt(d)
    q, k, v, do = _inputs(Nq, Nk, Hl, d, seed, layout)
    tq, tk, tv, tdo = (to_gpu_bf16(a) for a in (q, k, v, do))
    o, lse = gpu_lib.ulysses_xattn_fwd(tq, tk, tv, scale, layout)
    grads = gpu_lib.ulysses_xattn_bwd(tq, tk, tv, o, tdo, lse, scale, layout)
    again = gpu_lib.ulysses_xattn_bwd(tq, tk, tv, o, tdo, lse, scale, layout)
    torch.cuda.synchronize()
    fq, fk, fv, fdo = (oracle.bf16_to_f64(a) for a in (q, k, v, do))
    o_ref, lse_ref = oracle.xattn_fwd(fq, fk, fv, scale, layout)
    o_abs, _ = oracle.xattn_fwd(fq, fk, np.abs(fv), scale, layout)
    ok, worst, n_bad = o_within_tolerance(f64_of(o), o_ref, o_abs, TOL_O)
    assert ok, (worst, n_bad)
    assert max_abs(f64_of(lse), lse_ref) <= TOL_LSE
    for name, got, rep, ref in zip(("dq", "dk", "dv"), grads, again, oracle.xattn_bwd(fq, fk, fv, fdo, scale, layout)):
        err = rel_l2(f64_of(got), ref)
        assert err <= TOL_G, (name, err)
        assert torch.equal(got, rep), name                  # partial sums are added in a fixed order


@pytest.mark.parametrize("Nq,Nk,Hl,d,layout", [(5000, 200, 2, 128, 0), (200, 5000, 2, 128, 0), (3000, 3000, 2, 64, 0),
                                               (2100, 4100, 3, 128, 1), (4500, 129, 1, 64, 1), (131, 6000, 3, 64, 0)])
def test_few_tiles_on_one_side_are_cut_into_work_items(gpu_lib, Nq, Nk, Hl, d, layout):
    """With few key tiles (query tiles) and a long other side, the backward cuts each tile's walk into several
    work items whose fp32 partial sums a second kernel adds: every (query, key) pair must be counted once."""
    _parity(gpu_lib, Nq, Nk, Hl, d, layout, 40 + Nq)


@pytest.mark.parametrize("Nq,Nk", [(2048, 65536), (65536, 2048), (300, 40000)])
def test_many_work_items_per_tile(gpu_lib, Nq, Nk):
    """A short side against a long one: every tile of the short side is cut into 20 to 64 work items."""
    _parity(gpu_lib, Nq, Nk, 1, 128, 0, 5)


@pytest.mark.parametrize("Nq,Nk,layout", [(300, 1000, 0), (1000, 77, 1), (129, 257, 0), (2000, 2500, 0)])
def test_head_dimension_256(gpu_lib, Nq, Nk, layout):
    _parity(gpu_lib, Nq, Nk, 2, 256, layout, 70 + Nq)


def test_square_case_matches_self_attention_bits(gpu_lib):
    """Nq == Nk must give exactly what the non-causal self-attention entry points give."""
    q, k, v, do = _inputs(300, 300, 3, 128, 5, 0)
    tq, tk, tv, tdo = (to_gpu_bf16(a) for a in (q, k, v, do))
    o, lse = gpu_lib.ulysses_xattn_fwd(tq, tk, tv, 0.09)
    o2, lse2 = gpu_lib.ulysses_attn_fwd(tq, tk, tv, 0.09, False)
    assert torch.equal(o, o2) and torch.equal(lse, lse2)
    for a, b in zip(gpu_lib.ulysses_xattn_bwd(tq, tk, tv, o, tdo, lse, 0.09),
                    gpu_lib.ulysses_attn_bwd(tq, tk, tv, o, tdo, lse, 0.09, False)):
        assert torch.equal(a, b)
