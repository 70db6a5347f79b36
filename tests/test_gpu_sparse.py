"""GPU parity of block-sparse causal attention (256-token blocks, caller-given pattern) against the fp64
oracle, through the C ABI.  Same tolerances as dense attention (see test_gpu_attention.py)."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as synth
from _util import f64_of, max_abs, o_within_tolerance, rel_l2, to_gpu_bf16

pytestmark = pytest.mark.gpu

TOL_O, TOL_G, TOL_LSE = 1e-2, 2e-2, 2e-3
B = 256


def _mask(nb, kind, seed):
    rng = np.random.default_rng(seed)
    if kind == "full":
        m = np.ones((nb, nb), bool)
    elif kind == "diagonal":
        m = np.eye(nb, dtype=bool)
    elif kind == "window_global":          # local window of 2 blocks plus the first block column
        i, j = np.indices((nb, nb))
        m = (i - j < 2) | (j == 0)
    elif kind == "global_rows":            # local window of 2 blocks; every fifth block row sees everything before it
        i, j = np.indices((nb, nb))
        m = (i - j < 2) | (i % 5 == 4)
    else:
        m = rng.random((nb, nb)) < 0.4
    m = np.tril(m)
    np.fill_diagonal(m, True)
    return m


def _check(gpu_lib, N, Hl, d, kind, layout=0, seed=0):
    scale = 1.0 / np.sqrt(d)
    q, k, v, do = synth.attention_inputs(N, Hl, d, 500 + N + seed)
    if layout == 1:
        q, k, v, do = (np.ascontiguousarray(a.transpose(1, 0, 2)) for a in (q, k, v, do))
    mask = _mask((N + B - 1) // B, kind, N + seed)
    pat = gpu_lib.SparsePattern(mask)
    tq, tk, tv, tdo = (to_gpu_bf16(a) for a in (q, k, v, do))
    o, lse = gpu_lib.ulysses_sparse_attn_fwd(tq, tk, tv, pat, scale, layout)
    dq, dk, dv = gpu_lib.ulysses_sparse_attn_bwd(tq, tk, tv, o, tdo, lse, pat, scale, layout)
    torch.cuda.synchronize()
    fq, fk, fv, fdo = (oracle.bf16_to_f64(a) for a in (q, k, v, do))
    o_ref, lse_ref = oracle.sparse_attn_fwd(fq, fk, fv, mask, B, scale, layout)
    o_abs, _ = oracle.sparse_attn_fwd(fq, fk, np.abs(fv), mask, B, scale, layout)
    ok, worst, n_bad = o_within_tolerance(f64_of(o), o_ref, o_abs, TOL_O)
    assert ok, (worst, n_bad)
    assert max_abs(f64_of(lse), lse_ref) <= TOL_LSE
    refs = oracle.sparse_attn_bwd(fq, fk, fv, fdo, mask, B, scale, layout)
    for name, got, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), refs):
        err = rel_l2(f64_of(got), ref)
        assert err <= TOL_G, (name, err)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("N", [1, 200, 256, 257, 700, 1024, 1300, 2300])
@pytest.mark.parametrize("kind", ["random", "window_global"])
def test_sparse_parity(gpu_lib, N, d, kind):
    _check(gpu_lib, N, 2, d, kind)


@pytest.mark.parametrize("kind", ["full", "diagonal"])
def test_extreme_patterns(gpu_lib, kind):
    """Every lower-triangular block (= dense causal attention) and diagonal blocks only (= block-local)."""
    _check(gpu_lib, 1500, 2, 128, kind)


@pytest.mark.parametrize("N,Hl,d,kind", [(6000, 3, 128, "window_global"), (5000, 1, 64, "full"),
                                         (7700, 2, 128, "random")])
def test_long_block_columns_are_cut_into_several_work_items(gpu_lib, N, Hl, d, kind):
    """Block columns of 20 to 31 visible blocks: the dK/dV kernel cuts them into several work items whose
    fp32 partial sums a second kernel adds; every (query block, key tile) pair must be counted once."""
    _check(gpu_lib, N, Hl, d, kind, seed=11)


@pytest.mark.parametrize("N,Hl,d,layout", [(6000, 2, 128, 0), (7300, 3, 64, 1), (2400, 1, 128, 0)])
def test_long_block_rows_are_cut_into_several_work_items(gpu_lib, N, Hl, d, layout):
    """Block rows of up to 29 visible blocks among rows of two: the dQ kernel cuts the long ones into work items."""
    _check(gpu_lib, N, Hl, d, "global_rows", layout=layout, seed=13)


def test_head_major_and_odd_heads(gpu_lib):
    _check(gpu_lib, 1100, 3, 128, "random", layout=1, seed=3)


@pytest.mark.parametrize("d", [64, 128])
def test_full_pattern_agrees_with_the_dense_kernels(gpu_lib, d):
    N, Hl = 1024, 2                          # four block rows: none long enough to be cut into work items
    q, k, v, do = synth.attention_inputs(N, Hl, d, 9)
    tq, tk, tv, tdo = (to_gpu_bf16(a) for a in (q, k, v, do))
    pat = gpu_lib.SparsePattern(np.ones((4, 4), bool))
    o, lse = gpu_lib.ulysses_sparse_attn_fwd(tq, tk, tv, pat, 0.09)
    o2, lse2 = gpu_lib.ulysses_attn_fwd(tq, tk, tv, 0.09, True)
    if d == 64:
        assert torch.equal(o, o2) and torch.equal(lse, lse2)      # one kernel, same tiles in the same order
    else:
        # d = 128: the dense forward is a kernel of its own (other tile walk, other reference maxima), so the two
        # agree to the rounding of P and O only
        assert max_abs(f64_of(lse), f64_of(lse2)) <= 1e-5
        diff = (f64_of(o) - f64_of(o2))
        assert np.all(np.abs(diff) <= 2.0 ** -7 * np.maximum(np.abs(f64_of(o2)), 0.25))
    for a, b in zip(gpu_lib.ulysses_sparse_attn_bwd(tq, tk, tv, o, tdo, lse, pat, 0.09),
                    gpu_lib.ulysses_attn_bwd(tq, tk, tv, o, tdo, lse, 0.09, True)):
        assert rel_l2(f64_of(a), f64_of(b)) <= 5e-3               # same terms, summed in another order


def test_backward_with_cut_columns_is_deterministic(gpu_lib):
    """Partial sums of a cut block column are added in a fixed order: two runs give the same bits."""
    N, Hl, d = 6000, 2, 128
    q, k, v, do = synth.attention_inputs(N, Hl, d, 77)
    tq, tk, tv, tdo = (to_gpu_bf16(a) for a in (q, k, v, do))
    pat = gpu_lib.SparsePattern(_mask((N + B - 1) // B, "window_global", 0))
    o, lse = gpu_lib.ulysses_sparse_attn_fwd(tq, tk, tv, pat, 0.09)
    first = gpu_lib.ulysses_sparse_attn_bwd(tq, tk, tv, o, tdo, lse, pat, 0.09)
    again = gpu_lib.ulysses_sparse_attn_bwd(tq, tk, tv, o, tdo, lse, pat, 0.09)
    for a, b in zip(first, again):
        assert torch.equal(a, b)


def test_pattern_is_checked_on_the_host(gpu_lib):
    with pytest.raises(ValueError):
        gpu_lib.SparsePattern(np.array([[1, 0], [1, 0]]))
    z = torch.zeros((300, 1, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ValueError):
        gpu_lib.ulysses_sparse_attn_fwd(z, z.clone(), z.clone(), gpu_lib.SparsePattern(np.eye(3)), 0.1)
