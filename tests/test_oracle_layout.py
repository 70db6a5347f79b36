"""Pins for the oracle's layout transforms (CPU only).

The index loops in the oracle are checked against things they do not share code with:
numpy's reshape/transpose (a library routine), the paper's joint statement that after the
first all-to-all each device holds the full sequence for its own head subset (Section 3.1),
permutation/bijectivity, the round trip through the second all-to-all, and byte conservation
(Section 3.2: each rank's share of an all-to-all message of size M is M/P).
"""
import itertools

import numpy as np
import pytest

import oracle
import synth_inputs as synth

SHAPES = [  # nl, H, d, P
    (3, 6, 8, 1), (3, 6, 8, 2), (3, 6, 8, 3), (3, 6, 8, 6),
    (5, 7, 16, 7), (5, 7, 16, 1), (4, 56, 8, 8), (16, 8, 64, 4), (1, 4, 2, 2),
]


def _rand(shape, tid=0):
    return synth.bits_u16(shape, 1234, tid)


@pytest.mark.parametrize("nl,H,d,P", SHAPES)
def test_pack_equals_numpy_transpose(nl, H, d, P):
    x = _rand((nl, H, d))
    ref = x.reshape(nl, P, H // P, d).transpose(1, 0, 2, 3)
    assert np.array_equal(oracle.pack(x, P), ref)


@pytest.mark.parametrize("nl,H,d,P", SHAPES)
def test_unpack_equals_numpy(nl, H, d, P):
    r = _rand((P, nl, H // P, d), 1)
    assert np.array_equal(oracle.unpack(r, oracle.LAYOUT_SEQ_HEAD), r.reshape(P * nl, H // P, d))
    assert np.array_equal(oracle.unpack(r, oracle.LAYOUT_HEAD_SEQ),
                          r.reshape(P * nl, H // P, d).transpose(1, 0, 2))


def test_pack_hand_enumerated():
    # nl=2, H=4, P=2, d=1: x[n,h] = 10*n + h.  Destination rank p gets heads {2p, 2p+1}.
    x = np.array([[0, 1, 2, 3], [10, 11, 12, 13]], np.uint16).reshape(2, 4, 1)
    expect = np.array([[[0, 1], [10, 11]], [[2, 3], [12, 13]]], np.uint16).reshape(2, 2, 2, 1)
    assert np.array_equal(oracle.pack(x, 2), expect)
    # receive side: chunks from source ranks 0 and 1 (tokens 0-1 and 2-3) for 2 local heads
    r = np.array([[[0, 1], [10, 11]], [[20, 21], [30, 31]]], np.uint16).reshape(2, 2, 2, 1)
    assert oracle.unpack(r).reshape(4, 2).tolist() == [[0, 1], [10, 11], [20, 21], [30, 31]]
    assert oracle.unpack(r, oracle.LAYOUT_HEAD_SEQ).reshape(2, 4).tolist() == [[0, 10, 20, 30], [1, 11, 21, 31]]


def _exchange(chunks_by_src):
    """All-to-all by pointer routing: R_r[q] = S_q[r]."""
    P = len(chunks_by_src)
    return [np.stack([chunks_by_src[q][r] for q in range(P)]) for r in range(P)]


@pytest.mark.parametrize("N,H,d,P", [(12, 6, 4, 3), (16, 8, 8, 4), (14, 7, 2, 7), (8, 4, 4, 1)])
@pytest.mark.parametrize("layout", [oracle.LAYOUT_SEQ_HEAD, oracle.LAYOUT_HEAD_SEQ])
def test_joint_definition_and_round_trip(N, H, d, P, layout):
    """Emulated P-rank exchange: rank r ends up with the head slice of the global tensor;
    the reverse path restores every rank's sequence shard."""
    nl, Hl = N // P, H // P
    G = _rand((N, H, d))
    shards = [G[q * nl:(q + 1) * nl] for q in range(P)]
    sent = [oracle.pack(s, P) for s in shards]
    assert sum(s.nbytes for s in sent) == G.nbytes            # byte conservation
    assert all(s.nbytes == G.nbytes // P for s in sent)       # per-rank share M/P
    recv = _exchange(sent)
    ys = [oracle.unpack(recv[r], layout) for r in range(P)]
    for r in range(P):
        ref = G[:, r * Hl:(r + 1) * Hl, :]
        if layout == oracle.LAYOUT_HEAD_SEQ:
            ref = ref.transpose(1, 0, 2)
        assert np.array_equal(ys[r], ref)
    # every (token, head) pair appears on exactly one rank
    seen = np.zeros((N, H), np.int32)
    for r in range(P):
        seen[:, r * Hl:(r + 1) * Hl] += 1
    assert (seen == 1).all()
    # second all-to-all: back to [nl, H, d] on every rank
    sent2 = [oracle.pack_rev(ys[r], P, layout) for r in range(P)]
    recv2 = _exchange(sent2)
    for q in range(P):
        assert np.array_equal(oracle.unpack_rev(recv2[q]), shards[q])


@pytest.mark.parametrize("nl,H,d,P", [(7, 6, 8, 3), (3, 14, 4, 2), (64, 8, 64, 4)])
def test_pack_is_the_stated_permutation(nl, H, d, P):
    """Recover each destination element's source index from the payload (low then high 16 bits)."""
    n_el = nl * H * d
    idx = np.arange(n_el, dtype=np.int64)
    lo = oracle.pack((idx & 0xFFFF).astype(np.uint16).reshape(nl, H, d), P).reshape(-1).astype(np.int64)
    hi = oracle.pack((idx >> 16).astype(np.uint16).reshape(nl, H, d), P).reshape(-1).astype(np.int64)
    src = (hi << 16) | lo
    assert np.array_equal(np.sort(src), idx)                  # bijection
    Hl = H // P
    for (p, n, hl, c) in itertools.islice(itertools.product(range(P), range(nl), range(Hl), range(d)), 0, None, 37):
        assert src[((p * nl + n) * Hl + hl) * d + c] == (n * H + p * Hl + hl) * d + c


def test_p1_is_identity():
    x = _rand((9, 5, 8))
    assert np.array_equal(oracle.pack(x, 1).reshape(x.shape), x)
    assert np.array_equal(oracle.unpack(x.reshape(1, 9, 5, 8)), x)
    assert np.array_equal(oracle.unpack_rev(x.reshape(1, 9, 5, 8)), x)
    assert np.array_equal(oracle.pack_rev(x, 1).reshape(x.shape), x)


def test_bad_head_split_rejected():
    with pytest.raises(ValueError):
        oracle.pack(_rand((4, 6, 8)), 4)


def _golden_comm_rows():
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "comm_volume_section_3_2.txt")
    rows = []
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            rows.append(tuple(int(x) for x in line.split()))
    return rows


@pytest.mark.parametrize("N,h,P,qkv_total,out_total,per_rank", _golden_comm_rows())
def test_message_sizes_match_the_papers_communication_analysis(N, h, P, qkv_total, out_total, per_rank):
    """What the transforms hand to the two all-to-alls has the sizes Section 3.2 states: 3Nh and Nh
    elements in aggregate, 4Nh/P per rank, and every (source, destination) pair carries the same
    share of it."""
    d = 8
    H = h // d
    nl, Hl = N // P, H // P
    x = _rand((nl, H, d))
    sent_qkv = [oracle.pack(x, P) for _ in range(3)]                    # one rank's Q, K, V send buffers
    y = oracle.unpack(sent_qkv[0].reshape(P, nl, Hl, d))                 # shape of a rank's attention output
    sent_out = oracle.pack_rev(y, P)
    rank_elems = sum(s.size for s in sent_qkv) + sent_out.size
    assert rank_elems == per_rank
    assert P * sum(s.size for s in sent_qkv) == qkv_total and P * sent_out.size == out_total
    assert all(s.shape[0] == P and s[0].size * P == s.size for s in sent_qkv + [sent_out])   # equal chunks
