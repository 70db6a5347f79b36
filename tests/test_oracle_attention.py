"""Pins for the oracle's attention (CPU only).

Equation 1 of the paper, Softmax(Q K^T / sqrt(d)) V per head, and its causal variant are
checked against: dense numpy softmax (a library matmul/exp route that shares no code with
the C loops), closed forms (row 0, constant V, constant K, key shift invariance), and for the
backward pass torch autograd on the forward definition, central finite differences, and the
column-sum invariants.  A dropped term, a wrong sign, a transposed operand or an off-by-one
in the mask fails at least one of these.
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as synth


def _inputs(N, Hl, d, seed=7, mult=1.0):
    q, k, v, do = synth.attention_inputs(N, Hl, d, seed, mult)
    return tuple(synth.bf16_bits_to_f64(a) for a in (q, k, v, do))


def _numpy_attn(q, k, v, scale, causal):
    """Textbook dense softmax attention via numpy matmuls; q,k,v [N,Hl,d]."""
    N = q.shape[0]
    S = scale * np.einsum("ihc,jhc->hij", q, k)
    if causal:
        S = np.where(np.tril(np.ones((N, N), bool))[None], S, -np.inf)
    m = S.max(-1, keepdims=True)
    E = np.exp(S - m)
    l = E.sum(-1, keepdims=True)
    O = np.einsum("hij,jhc->ihc", E / l, v)
    return O, (m + np.log(l))[..., 0], E / l


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("N,Hl,d", [(1, 1, 4), (5, 2, 8), (33, 3, 16), (130, 2, 64), (70, 2, 256)])
def test_forward_equals_dense_numpy(N, Hl, d, causal):
    q, k, v, _ = _inputs(N, Hl, d)
    scale = 1.0 / np.sqrt(d)
    o, lse = oracle.attn_fwd(q, k, v, scale, causal)
    o_ref, lse_ref, _ = _numpy_attn(q, k, v, scale, causal)
    np.testing.assert_allclose(o, o_ref, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, lse_ref, rtol=0, atol=1e-13)


def test_layouts_agree():
    q, k, v, do = _inputs(40, 3, 8)
    t = lambda a: np.ascontiguousarray(a.transpose(1, 0, 2))
    o0, l0 = oracle.attn_fwd(q, k, v, 0.3, True, oracle.LAYOUT_SEQ_HEAD)
    o1, l1 = oracle.attn_fwd(t(q), t(k), t(v), 0.3, True, oracle.LAYOUT_HEAD_SEQ)
    assert np.array_equal(t(o0), o1) and np.array_equal(l0, l1)
    g0 = oracle.attn_bwd(q, k, v, do, 0.3, True, oracle.LAYOUT_SEQ_HEAD)
    g1 = oracle.attn_bwd(t(q), t(k), t(v), t(do), 0.3, True, oracle.LAYOUT_HEAD_SEQ)
    for a, b in zip(g0, g1):
        assert np.array_equal(t(a), b)


def test_probabilities_sum_to_one_and_match_brute_force():
    # V = identity (N = d) makes O equal to the probability matrix itself.
    N = d = 24
    q, k, _, _ = _inputs(N, 1, d)
    v = np.eye(N).reshape(N, 1, d)
    o, lse = oracle.attn_fwd(q, k, v, 0.25, True)
    Pm = o[:, 0, :]
    np.testing.assert_allclose(Pm.sum(1), 1.0, rtol=0, atol=1e-15 * N)
    assert (np.triu(Pm, 1) == 0).all()                      # nothing above the diagonal
    assert (np.diag(Pm) > 0).all()                          # the diagonal is visible
    for i in range(N):                                      # brute force, pure python
        s = [0.25 * sum(q[i, 0, c] * k[j, 0, c] for c in range(d)) for j in range(i + 1)]
        z = sum(np.exp(x) for x in s)
        for j in range(i + 1):
            assert abs(Pm[i, j] - np.exp(s[j]) / z) < 1e-14
        assert abs(lse[0, i] - np.log(z)) < 1e-13


def test_row_zero_and_constant_v():
    q, k, v, _ = _inputs(50, 2, 16)
    o, lse = oracle.attn_fwd(q, k, v, 0.25, True)
    np.testing.assert_allclose(o[0], v[0], atol=1e-15)
    np.testing.assert_allclose(lse[:, 0], 0.25 * (q[0] * k[0]).sum(-1), atol=1e-14)
    vc = np.broadcast_to(np.array([1.5, -2.0] * 8), v.shape).copy()
    oc, _ = oracle.attn_fwd(q, k, vc, 0.25, True)
    np.testing.assert_allclose(oc, vc, atol=1e-14)


@pytest.mark.parametrize("N", [64, 4096])
def test_constant_k_closed_form(N):
    """K constant => P_ij = 1/(i+1): O is the prefix mean of V, LSE_i = S_i0 + log(i+1),
    dQ = 0 and dV_j = sum_{i>=j} dO_i/(i+1).  Valid at any N, so it also pins the row-sampled
    entry points at a size where the full oracle is not run."""
    Hl, d, s = 2, 16, 0.25
    q, _, v, do = _inputs(N, Hl, d)
    k = np.broadcast_to(np.linspace(-1, 1, d), (N, Hl, d)).copy()
    cnt = np.arange(1, N + 1, dtype=np.float64)[:, None, None]
    o_ref = np.cumsum(v, 0) / cnt
    lse_ref = (s * (q * k).sum(-1) + np.log(cnt[..., 0])).T
    rows = np.unique(np.r_[0, 1, N - 1, np.random.default_rng(0).integers(0, N, 16)])
    o_r, lse_r = oracle.attn_fwd_rows(q, k, v, rows, s, True)
    np.testing.assert_allclose(o_r, o_ref[rows], atol=1e-12)
    np.testing.assert_allclose(lse_r, lse_ref[:, rows], atol=1e-12)
    # masked-dO backward over the sampled rows
    dq_r, dk, dv = oracle.attn_bwd_rows(q, k, v, do, rows, s, True)
    np.testing.assert_allclose(dq_r, 0.0, atol=1e-12)
    w = np.zeros((N, 1, 1)); w[rows] = 1.0
    dv_ref = np.cumsum((w * do / cnt)[::-1], 0)[::-1]
    np.testing.assert_allclose(dv, dv_ref, atol=1e-12)
    # dK_j = s * sum_{i>=j} Q_i (dO_i.V_j - D_i)/(i+1)
    D = (do * o_ref).sum(-1, keepdims=True)
    A = np.cumsum(((w / cnt)[..., None] * q[:, :, :, None] * do[:, :, None, :])[::-1], 0)[::-1]   # [N,Hl,d,d]
    B = np.cumsum((w * D * q / cnt)[::-1], 0)[::-1]
    dk_ref = s * (np.einsum("jhcd,jhd->jhc", A, v) - B)
    np.testing.assert_allclose(dk, dk_ref, atol=1e-11)
    if N <= 64:
        o, lse = oracle.attn_fwd(q, k, v, s, True)
        np.testing.assert_allclose(o, o_ref, atol=1e-13)
        np.testing.assert_allclose(lse, lse_ref, atol=1e-13)


def test_key_shift_invariance():
    q, k, v, _ = _inputs(37, 2, 8)
    o0, _ = oracle.attn_fwd(q, k, v, 0.35, True)
    o1, _ = oracle.attn_fwd(q, k + np.linspace(0.5, 2, 8), v, 0.35, True)
    np.testing.assert_allclose(o0, o1, atol=1e-12)


def _torch_grads(q, k, v, do, scale, causal):
    tq, tk, tv = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (q, k, v))
    S = scale * torch.einsum("ihc,jhc->hij", tq, tk)
    if causal:
        N = q.shape[0]
        S = S.masked_fill(~torch.tril(torch.ones(N, N, dtype=torch.bool)), float("-inf"))
    O = torch.einsum("hij,jhc->ihc", torch.softmax(S, -1), tv)
    (O * torch.tensor(do)).sum().backward()
    return tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy()


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("N,Hl,d", [(1, 1, 4), (7, 2, 8), (65, 2, 32), (40, 1, 256)])
def test_backward_equals_torch_autograd(N, Hl, d, causal):
    q, k, v, do = _inputs(N, Hl, d, seed=11)
    scale = 1.0 / np.sqrt(d)
    got = oracle.attn_bwd(q, k, v, do, scale, causal)
    ref = _torch_grads(q, k, v, do, scale, causal)
    for g, r in zip(got, ref):
        np.testing.assert_allclose(g, r, rtol=0, atol=1e-12)


def test_backward_finite_differences():
    N, Hl, d, s, eps = 9, 2, 4, 0.5, 1e-6
    q, k, v, do = _inputs(N, Hl, d, seed=3)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, s, True)
    loss = lambda q_, k_, v_: (oracle.attn_fwd(q_, k_, v_, s, True)[0] * do).sum()
    rng = np.random.default_rng(0)
    for which, g in (("q", dq), ("k", dk), ("v", dv)):
        for _ in range(12):
            idx = tuple(rng.integers(0, n) for n in (N, Hl, d))
            args = {"q": q.copy(), "k": k.copy(), "v": v.copy()}
            args[which][idx] += eps
            up = loss(args["q"], args["k"], args["v"])
            args[which][idx] -= 2 * eps
            dn = loss(args["q"], args["k"], args["v"])
            fd = (up - dn) / (2 * eps)
            assert abs(fd - g[idx]) < 1e-6 * max(1.0, abs(g[idx])), (which, idx, fd, g[idx])


@pytest.mark.parametrize("causal", [True, False])
def test_backward_sum_invariants(causal):
    q, k, v, do = _inputs(200, 2, 16, seed=5, mult=2.0)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, 0.25, causal)
    np.testing.assert_allclose(dv.sum(0), do.sum(0), atol=1e-11)      # rows of P sum to one
    np.testing.assert_allclose(dk.sum(0), 0.0, atol=1e-11)            # rows of dS sum to zero


def test_row_sampled_entry_points_match_full():
    N, Hl, d, s = 150, 3, 8, 0.3
    q, k, v, do = _inputs(N, Hl, d, seed=9)
    rows = np.array([0, 1, 17, 63, 64, 65, 149])
    o, lse = oracle.attn_fwd(q, k, v, s, True)
    o_r, lse_r = oracle.attn_fwd_rows(q, k, v, rows, s, True)
    assert np.array_equal(o_r, o[rows]) and np.array_equal(lse_r, lse[:, rows])
    do_m = np.zeros_like(do); do_m[rows] = do[rows]
    dq, dk, dv = oracle.attn_bwd(q, k, v, do_m, s, True)
    dq_r, dk_r, dv_r = oracle.attn_bwd_rows(q, k, v, do, rows, s, True)
    np.testing.assert_allclose(dq_r, dq[rows], atol=1e-14)
    np.testing.assert_allclose(dk_r, dk, atol=1e-14)
    np.testing.assert_allclose(dv_r, dv, atol=1e-14)
    # dQ rows do not depend on the other rows' dO
    dq_full = oracle.attn_bwd(q, k, v, do, s, True)[0]
    np.testing.assert_allclose(dq_r, dq_full[rows], atol=1e-14)


def test_sharding_equivalence():
    """Attention on a rank's unpacked heads equals those heads of attention on the global
    tensor: sequence parallelism changes where the work runs, not its result (Section 4.5)."""
    N, H, d, P = 24, 6, 8, 3
    nl, Hl = N // P, H // P
    bits = {n: synth.normal_bf16((N, H, d), 21, tid) for n, tid in (("q", 2), ("k", 3), ("v", 4))}
    glob = {n: synth.bf16_bits_to_f64(b) for n, b in bits.items()}
    o_glob, _ = oracle.attn_fwd(glob["q"], glob["k"], glob["v"], 0.35, True)
    for r in range(P):
        loc = {}
        for n, b in bits.items():
            sent = [oracle.pack(b[qq * nl:(qq + 1) * nl], P) for qq in range(P)]
            recv = np.stack([sent[qq][r] for qq in range(P)])
            loc[n] = oracle.bf16_to_f64(oracle.unpack(recv))
        o_loc, _ = oracle.attn_fwd(loc["q"], loc["k"], loc["v"], 0.35, True)
        assert np.array_equal(o_loc, o_glob[:, r * Hl:(r + 1) * Hl])


def test_bf16_decode_is_exact():
    bits = np.arange(0, 0x7F80, 7, dtype=np.uint16)
    bits = np.concatenate([bits, bits | 0x8000])
    assert np.array_equal(oracle.bf16_to_f64(bits), synth.bf16_bits_to_f32(bits).astype(np.float64))
    assert oracle.bf16_to_f64(np.array([0x3F80, 0xC000, 0x3DCD], np.uint16)).tolist() == [1.0, -2.0, 0.10009765625]
