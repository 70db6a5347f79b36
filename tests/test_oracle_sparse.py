"""Pins of the oracle's block-sparse causal attention (Sections 3.4 / 4.3 name blocked sparse attention
without fixing a pattern; the reading is stated in the oracle: causal AND a caller-given block mask).
Checked against numpy and torch with the mask expanded to token level, finite differences, and the
dense causal oracle when every lower-triangular block is set."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as synth


def _inputs(N, Hl, d, seed=31):
    return tuple(synth.bf16_bits_to_f64(a) for a in synth.attention_inputs(N, Hl, d, seed))


def _random_mask(nb, seed, density=0.5):
    rng = np.random.default_rng(seed)
    m = np.tril(rng.random((nb, nb)) < density)
    np.fill_diagonal(m, True)
    return m


def _token_mask(mask, N, B):
    t = np.kron(np.asarray(mask, bool), np.ones((B, B), bool))[:N, :N]
    return t & np.tril(np.ones((N, N), bool))


@pytest.mark.parametrize("N,B,Hl,d", [(1, 4, 1, 4), (19, 4, 2, 8), (64, 16, 2, 16), (70, 16, 3, 8)])
def test_forward_and_backward_match_dense_masked_torch(N, B, Hl, d):
    q, k, v, do = _inputs(N, Hl, d)
    mask = _random_mask((N + B - 1) // B, N)
    tm = torch.tensor(_token_mask(mask, N, B))
    tq, tk, tv = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (q, k, v))
    S = (0.4 * torch.einsum("ihc,jhc->hij", tq, tk)).masked_fill(~tm, float("-inf"))
    O = torch.einsum("hij,jhc->ihc", torch.softmax(S, -1), tv)
    (O * torch.tensor(do)).sum().backward()
    o, lse = oracle.sparse_attn_fwd(q, k, v, mask, B, 0.4)
    np.testing.assert_allclose(o, O.detach().numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, torch.logsumexp(S, -1).detach().numpy(), rtol=0, atol=1e-13)
    for g, r in zip(oracle.sparse_attn_bwd(q, k, v, do, mask, B, 0.4), (tq.grad, tk.grad, tv.grad)):
        np.testing.assert_allclose(g, r.numpy(), rtol=0, atol=1e-12)


def test_full_lower_triangle_equals_the_causal_oracle():
    N, B, Hl, d = 90, 16, 2, 16
    q, k, v, do = _inputs(N, Hl, d, seed=4)
    nb = (N + B - 1) // B
    full = np.tril(np.ones((nb, nb), bool))
    for layout in (0, 1):
        a = [np.ascontiguousarray(t.transpose(1, 0, 2)) if layout else t for t in (q, k, v, do)]
        o, lse = oracle.sparse_attn_fwd(a[0], a[1], a[2], full, B, 0.3, layout)
        o2, lse2 = oracle.attn_fwd(a[0], a[1], a[2], 0.3, True, layout)
        np.testing.assert_allclose(o, o2, rtol=0, atol=1e-14)
        np.testing.assert_allclose(lse, lse2, rtol=0, atol=1e-14)
        for g, r in zip(oracle.sparse_attn_bwd(*a, full, B, 0.3, layout), oracle.attn_bwd(*a, 0.3, True, layout)):
            np.testing.assert_allclose(g, r, rtol=0, atol=1e-13)


def test_diagonal_only_is_block_local_attention():
    """Only diagonal blocks: every block of B tokens attends within itself, i.e. independent short sequences."""
    N, B, Hl, d = 48, 16, 2, 8
    q, k, v, do = _inputs(N, Hl, d, seed=6)
    o, lse = oracle.sparse_attn_fwd(q, k, v, np.eye(3, dtype=bool), B, 0.5)
    dq, dk, dv = oracle.sparse_attn_bwd(q, k, v, do, np.eye(3, dtype=bool), B, 0.5)
    for b in range(3):
        sl = slice(b * B, (b + 1) * B)
        ob, lb = oracle.attn_fwd(q[sl], k[sl], v[sl], 0.5, True)
        np.testing.assert_allclose(o[sl], ob, rtol=0, atol=1e-14)
        np.testing.assert_allclose(lse[:, sl], lb, rtol=0, atol=1e-14)
        for g, r in zip((dq[sl], dk[sl], dv[sl]), oracle.attn_bwd(q[sl], k[sl], v[sl], do[sl], 0.5, True)):
            np.testing.assert_allclose(g, r, rtol=0, atol=1e-13)


def test_backward_finite_differences():
    N, B, Hl, d, s, eps = 14, 4, 2, 4, 0.5, 1e-6
    q, k, v, do = _inputs(N, Hl, d, seed=3)
    mask = _random_mask(4, 1)
    grads = dict(zip("qkv", oracle.sparse_attn_bwd(q, k, v, do, mask, B, s)))
    loss = lambda a: (oracle.sparse_attn_fwd(a["q"], a["k"], a["v"], mask, B, s)[0] * do).sum()
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


def test_missing_diagonal_block_is_rejected():
    q, k, v, _ = _inputs(8, 1, 4)
    with pytest.raises(ValueError):
        oracle.sparse_attn_fwd(q, k, v, np.array([[1, 0], [1, 0]]), 4, 1.0)
