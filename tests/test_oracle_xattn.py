"""Pins of the oracle's cross-attention (Equation 1 with Nq queries over Nk keys, no mask; the paper
lists cross-attention among the supported forms in Section 3.4).  None of them shares code with it:
numpy matrix products, torch autograd, central finite differences, closed forms, and the case Nq = Nk
where it must equal the (separately written and pinned) non-causal self-attention oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as synth


def _inputs(Nq, Nk, Hl, d, seed=21, mult=1.0):
    q, _, _, do = synth.attention_inputs(Nq, Hl, d, seed, mult)
    _, k, v, _ = synth.attention_inputs(Nk, Hl, d, seed + 1, mult)
    return tuple(synth.bf16_bits_to_f64(a) for a in (q, k, v, do))


SHAPES = [(1, 1, 1, 4), (1, 9, 2, 8), (9, 1, 2, 8), (5, 12, 2, 8), (40, 17, 3, 16), (33, 130, 2, 64)]


@pytest.mark.parametrize("Nq,Nk,Hl,d", SHAPES)
def test_forward_equals_dense_numpy(Nq, Nk, Hl, d):
    q, k, v, _ = _inputs(Nq, Nk, Hl, d)
    scale = 1.0 / np.sqrt(d)
    S = scale * np.einsum("ihc,jhc->hij", q, k)
    m = S.max(-1, keepdims=True)
    E = np.exp(S - m)
    o_ref = np.einsum("hij,jhc->ihc", E / E.sum(-1, keepdims=True), v)
    lse_ref = (m + np.log(E.sum(-1, keepdims=True)))[..., 0]
    o, lse = oracle.xattn_fwd(q, k, v, scale)
    np.testing.assert_allclose(o, o_ref, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, lse_ref, rtol=0, atol=1e-13)


@pytest.mark.parametrize("Nq,Nk,Hl,d", SHAPES)
def test_backward_equals_torch_autograd(Nq, Nk, Hl, d):
    q, k, v, do = _inputs(Nq, Nk, Hl, d, seed=5)
    scale = 0.3
    tq, tk, tv = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (q, k, v))
    P = torch.softmax(scale * torch.einsum("ihc,jhc->hij", tq, tk), -1)
    (torch.einsum("hij,jhc->ihc", P, tv) * torch.tensor(do)).sum().backward()
    got = oracle.xattn_bwd(q, k, v, do, scale)
    for g, r in zip(got, (tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy())):
        np.testing.assert_allclose(g, r, rtol=0, atol=1e-12)


def test_backward_finite_differences():
    Nq, Nk, Hl, d, s, eps = 6, 11, 2, 4, 0.5, 1e-6
    q, k, v, do = _inputs(Nq, Nk, Hl, d, seed=3)
    grads = dict(zip("qkv", oracle.xattn_bwd(q, k, v, do, s)))
    loss = lambda a: (oracle.xattn_fwd(a["q"], a["k"], a["v"], s)[0] * do).sum()
    rng = np.random.default_rng(0)
    for which in "qkv":
        for _ in range(10):
            a = {"q": q.copy(), "k": k.copy(), "v": v.copy()}
            idx = tuple(int(rng.integers(0, n)) for n in a[which].shape)
            a[which][idx] += eps
            up = loss(a)
            a[which][idx] -= 2 * eps
            fd = (up - loss(a)) / (2 * eps)
            assert abs(fd - grads[which][idx]) < 1e-6 * max(1.0, abs(grads[which][idx])), (which, idx)


def test_square_case_equals_the_self_attention_oracle():
    q, k, v, do = _inputs(50, 50, 2, 16, seed=9)
    for layout in (0, 1):
        a = [np.ascontiguousarray(t.transpose(1, 0, 2)) if layout else t for t in (q, k, v, do)]
        o, lse = oracle.xattn_fwd(a[0], a[1], a[2], 0.25, layout)
        o2, lse2 = oracle.attn_fwd(a[0], a[1], a[2], 0.25, False, layout)
        np.testing.assert_allclose(o, o2, rtol=0, atol=1e-14)
        np.testing.assert_allclose(lse, lse2, rtol=0, atol=1e-14)
        for g, r in zip(oracle.xattn_bwd(*a, 0.25, layout), oracle.attn_bwd(*a, 0.25, False, layout)):
            np.testing.assert_allclose(g, r, rtol=0, atol=1e-13)


def test_closed_forms_and_invariants():
    Nq, Nk, Hl, d = 23, 37, 2, 8
    q, k, v, do = _inputs(Nq, Nk, Hl, d, seed=13)
    # constant K: uniform weights 1/Nk -> O_i = mean of V, LSE_i = S_i0 + log Nk, dQ = 0
    kc = np.broadcast_to(k[:1], k.shape).copy()
    o, lse = oracle.xattn_fwd(q, kc, v, 0.7)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(0), o.shape), rtol=0, atol=1e-13)
    s0 = 0.7 * np.einsum("ihc,hc->hi", q, kc[0])
    np.testing.assert_allclose(lse, s0 + np.log(Nk), rtol=0, atol=1e-13)
    dq, dk, dv = oracle.xattn_bwd(q, kc, v, do, 0.7)
    assert np.abs(dq).max() < 1e-13
    np.testing.assert_allclose(dv, np.broadcast_to(do.sum(0) / Nk, dv.shape), rtol=0, atol=1e-13)
    # any K: sum_j dV_j = sum_i dO_i and sum_j dK_j = 0 (each row of dS sums to zero)
    dq, dk, dv = oracle.xattn_bwd(q, k, v, do, 0.7)
    np.testing.assert_allclose(dv.sum(0), do.sum(0), rtol=0, atol=1e-12)
    assert np.abs(dk.sum(0)).max() < 1e-12
    # a single key: every query returns that value row
    o1, lse1 = oracle.xattn_fwd(q, k[:1], v[:1], 0.7)
    np.testing.assert_allclose(o1, np.broadcast_to(v[:1], o1.shape), rtol=0, atol=1e-14)


def test_empty_key_set_is_rejected():
    q, k, v, _ = _inputs(4, 4, 1, 8)
    with pytest.raises(ValueError):
        oracle.xattn_fwd(q, k[:0], v[:0], 1.0)
