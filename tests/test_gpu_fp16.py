"""GPU parity of the fp16 build of the attention kernels (layout | ULY_ELEM_F16) against the fp64 oracle.

The paper states no precision; bf16 is the default element type here and fp16 the alternative.  Inputs are
the seeded bf16 samples rounded to fp16 (the oracle gets exactly the values the GPU gets).  fp16 carries
11 significand bits, so the stated max-abs 1e-2 on O holds without the large-|O| allowance the bf16 path
needs (half an fp16 ulp is below 4e-3 for |O| < 8); gradients: relative L2 2e-2; LSE: max-abs 2e-3.
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as synth
from _util import f64_of, max_abs, rel_l2

pytestmark = pytest.mark.gpu

TOL_O, TOL_G, TOL_LSE = 1e-2, 2e-2, 2e-3


def _inputs(N, Hl, d, seed, mult=1.0, layout=0, n=4):
    arrs = synth.attention_inputs(N, Hl, d, seed, mult)[:n]
    if layout == 1:
        arrs = [np.ascontiguousarray(a.transpose(1, 0, 2)) for a in arrs]
    h = [oracle.bf16_to_f64(a).astype(np.float16) for a in arrs]          # what the GPU gets
    return h, [a.astype(np.float64) for a in h], [torch.from_numpy(a).cuda() for a in h]


def _compare(o, lse, grads, o_ref, lse_ref, grads_ref):
    assert o.dtype == torch.float16 and all(g.dtype == torch.float16 for g in grads)
    assert max_abs(f64_of(o), o_ref) <= TOL_O
    assert max_abs(f64_of(lse), lse_ref) <= TOL_LSE
    for name, got, ref in zip(("dq", "dk", "dv"), grads, grads_ref):
        err = rel_l2(f64_of(got), ref)
        assert err <= TOL_G, (name, err)


def _dense(uly, N, Hl, d, causal=True, layout=0, seed=1, mult=1.0):
    scale = 1.0 / np.sqrt(d)
    _, (fq, fk, fv, fdo), (tq, tk, tv, tdo) = _inputs(N, Hl, d, seed, mult, layout)
    o, lse = uly.ulysses_attn_fwd(tq, tk, tv, scale, causal, layout)
    grads = uly.ulysses_attn_bwd(tq, tk, tv, o, tdo, lse, scale, causal, layout)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attn_fwd(fq, fk, fv, scale, causal, layout)
    _compare(o, lse, grads, o_ref, lse_ref, oracle.attn_bwd(fq, fk, fv, fdo, scale, causal, layout))


@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("N", [1, 33, 128, 257, 700, 1021, 2177])
def test_causal(gpu_lib, N, d):
    _dense(gpu_lib, N, 2, d, seed=N + d)


@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("N", [65, 777])
def test_non_causal(gpu_lib, N, d):
    _dense(gpu_lib, N, 3, d, causal=False, seed=N)


def test_head_major_and_wide_logits(gpu_lib):
    _dense(gpu_lib, 900, 3, 128, layout=1, seed=5)
    _dense(gpu_lib, 1024, 2, 128, seed=8, mult=3.0)


def test_tiny_config(gpu_lib):
    c = synth.CONFIGS["tiny"]
    _dense(gpu_lib, c["N"], c["H"] // c["P"], c["d"], seed=synth.config_seed("tiny"))


@pytest.mark.parametrize("Nq,Nk,d", [(300, 1000, 128), (1000, 77, 64), (513, 513, 128), (200, 5000, 128), (5000, 200, 64)])
def test_cross_attention(gpu_lib, Nq, Nk, d):
    scale = 1.0 / np.sqrt(d)
    _, (fq, _, _, fdo), (tq, _, _, tdo) = _inputs(Nq, 2, d, 21)
    _, (_, fk, fv), (_, tk, tv) = _inputs(Nk, 2, d, 22, n=3)
    o, lse = gpu_lib.ulysses_xattn_fwd(tq, tk, tv, scale)
    grads = gpu_lib.ulysses_xattn_bwd(tq, tk, tv, o, tdo, lse, scale)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.xattn_fwd(fq, fk, fv, scale)
    _compare(o, lse, grads, o_ref, lse_ref, oracle.xattn_bwd(fq, fk, fv, fdo, scale))


@pytest.mark.parametrize("N,d", [(1300, 128), (2300, 64)])
def test_block_sparse(gpu_lib, N, d):
    scale, B = 1.0 / np.sqrt(d), gpu_lib.SPARSE_BLOCK
    nb = (N + B - 1) // B
    i, j = np.indices((nb, nb))
    mask = np.tril((i - j < 2) | (j == 0))
    _, (fq, fk, fv, fdo), (tq, tk, tv, tdo) = _inputs(N, 2, d, 31)
    pat = gpu_lib.SparsePattern(mask)
    o, lse = gpu_lib.ulysses_sparse_attn_fwd(tq, tk, tv, pat, scale)
    grads = gpu_lib.ulysses_sparse_attn_bwd(tq, tk, tv, o, tdo, lse, pat, scale)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.sparse_attn_fwd(fq, fk, fv, mask, B, scale, 0)
    _compare(o, lse, grads, o_ref, lse_ref, oracle.sparse_attn_bwd(fq, fk, fv, fdo, mask, B, scale, 0))


def test_fp16_is_closer_than_bf16(gpu_lib):
    """The same values through both builds: the fp16 output must carry the extra significand bits
    (a build that silently ran the bf16 kernels on fp16 bits would fail both this and the parity above)."""
    N, Hl, d, scale = 1024, 2, 128, 1.0 / np.sqrt(128)
    _, (fq, fk, fv, _), (tq, tk, tv, _) = _inputs(N, Hl, d, 3)
    o_ref, _ = oracle.attn_fwd(fq, fk, fv, scale, True, 0)
    o16, _ = gpu_lib.ulysses_attn_fwd(tq, tk, tv, scale, True)
    obf, _ = gpu_lib.ulysses_attn_fwd(tq.bfloat16(), tk.bfloat16(), tv.bfloat16(), scale, True)
    e16, ebf = rel_l2(f64_of(o16), o_ref), rel_l2(f64_of(obf), o_ref)
    assert e16 < 0.5 * ebf, (e16, ebf)


def test_mixed_element_types_are_refused(gpu_lib):
    q = torch.zeros((64, 1, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(ValueError):
        gpu_lib.ulysses_attn_fwd(q, q.bfloat16(), q.clone(), 0.1)
    with pytest.raises(ValueError):
        gpu_lib.ulysses_attn_fwd(q.float(), q.float(), q.float(), 0.1)
