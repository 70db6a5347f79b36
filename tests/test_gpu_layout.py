"""GPU parity of the layout transforms against the oracle: bit-exact, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as synth
from _util import bits_of, to_gpu_u16

pytestmark = pytest.mark.gpu

# nl, H, d, P  (small enough for the index-loop oracle to finish in seconds)
SMALL = [
    (512, 8, 64, 4),        # the tiny config
    (333, 6, 128, 3),       # ragged rows, non-power-of-two groups
    (257, 56, 128, 8),      # 7 local heads
    (1000, 32, 128, 32),    # one local head
    (77, 4, 8, 2),          # 16-byte runs
    (5, 6, 4, 3),           # run of 16 bytes with 2 heads
    (129, 3, 2, 3),         # 4-byte runs: narrow-vector path
    (64, 5, 1, 5),          # 2-byte runs
    (1, 1, 64, 1), (3, 16, 64, 1),
]


@pytest.mark.parametrize("nl,H,d,P", SMALL)
def test_pack_and_unpack_rev_bit_exact(gpu_lib, nl, H, d, P):
    x = synth.bits_u16((nl, H, d), 99, synth.TID_X)
    ref = oracle.pack(x, P)
    got = gpu_lib.ulysses_pack(to_gpu_u16(x), P)
    assert np.array_equal(bits_of(got), ref)
    back = gpu_lib.ulysses_unpack_rev(got)
    assert np.array_equal(bits_of(back), x)
    assert np.array_equal(bits_of(back), oracle.unpack_rev(ref))


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("nl,H,d,P", SMALL)
def test_unpack_and_pack_rev_bit_exact(gpu_lib, nl, H, d, P, layout):
    r = synth.bits_u16((P, nl, H // P, d), 99, synth.TID_R)
    ref = oracle.unpack(r, layout)
    got = gpu_lib.ulysses_unpack(to_gpu_u16(r), layout)
    assert np.array_equal(bits_of(got), ref)
    back = gpu_lib.ulysses_pack_rev(got, P, layout)
    assert np.array_equal(bits_of(back), r)
    assert np.array_equal(bits_of(back), oracle.pack_rev(ref, P, layout))


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("nl,H,d,P", SMALL[:5])
def test_qkv_in_one_launch_bit_exact(gpu_lib, nl, H, d, P, layout):
    """Q, K, V transformed by one launch equal the oracle applied to each tensor."""
    xs = [synth.bits_u16((nl, H, d), 7, synth.TID_X + 10 * t) for t in range(3)]
    sends = gpu_lib.ulysses_pack_qkv([to_gpu_u16(x) for x in xs], P)
    for x, s_ in zip(xs, sends):
        assert np.array_equal(bits_of(s_), oracle.pack(x, P))
    rs = [synth.bits_u16((P, nl, H // P, d), 7, synth.TID_R + 10 * t) for t in range(3)]
    ys = gpu_lib.ulysses_unpack_qkv([to_gpu_u16(r) for r in rs], layout)
    for r, y in zip(rs, ys):
        assert np.array_equal(bits_of(y), oracle.unpack(r, layout))


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("nl,H,d,P", SMALL[:5])
def test_reverse_transforms_of_three_tensors_in_one_launch(gpu_lib, nl, H, d, P, layout):
    """dQ, dK, dV back to sequence-parallel form: each tensor equals the oracle's reverse transform."""
    Hl, N = H // P, nl * P
    shape = (Hl, N, d) if layout == 1 else (N, Hl, d)
    gs = [synth.bits_u16(shape, 8, synth.TID_X + 10 * t) for t in range(3)]
    sends = gpu_lib.ulysses_pack_rev_qkv([to_gpu_u16(g) for g in gs], P, layout)
    for g, s_ in zip(gs, sends):
        assert np.array_equal(bits_of(s_), oracle.pack_rev(g, P, layout))
    rs = [synth.bits_u16((P, nl, Hl, d), 8, synth.TID_R + 10 * t) for t in range(3)]
    ys = gpu_lib.ulysses_unpack_rev_qkv([to_gpu_u16(r) for r in rs])
    for r, y in zip(rs, ys):
        assert np.array_equal(bits_of(y), oracle.unpack_rev(r))


@pytest.mark.parametrize("elem", [torch.uint8, torch.int32])
def test_other_element_sizes(gpu_lib, elem):
    nl, H, d, P = 37, 6, 24, 3
    g = torch.Generator().manual_seed(5)
    x = torch.randint(0, 127, (nl, H, d), generator=g, dtype=torch.int32).to(elem)
    got = gpu_lib.ulysses_pack(x.cuda(), P).cpu()
    ref = x.reshape(nl, P, H // P, d).permute(1, 0, 2, 3)
    assert torch.equal(got, ref)
    assert torch.equal(gpu_lib.ulysses_unpack_rev(got.cuda()).cpu(), x)


# nl, H, d, P: shapes whose contiguous run is one element of 2 / 4 / 8 bytes (bf16-sized payloads), which go
# through the LDS-staged transpose; several row tiles, ragged ends, more than 64 groups
SHORT_RUNS = [(5000, 8, 1, 8), (333, 130, 1, 130), (4097, 6, 2, 6), (1300, 12, 4, 12), (70, 2, 1, 2), (9000, 70, 1, 70)]


@pytest.mark.parametrize("nl,H,d,P", SHORT_RUNS)
def test_short_runs_bit_exact(gpu_lib, nl, H, d, P):
    x = synth.bits_u16((nl, H, d), 5, synth.TID_X)
    ref = oracle.pack(x, P)
    got = gpu_lib.ulysses_pack(to_gpu_u16(x), P)
    assert np.array_equal(bits_of(got), ref)
    assert np.array_equal(bits_of(gpu_lib.ulysses_unpack_rev(got)), x)


@pytest.mark.parametrize("N,Hl,d", [(3000, 5, 1), (1025, 80, 2), (513, 3, 4), (100, 2, 1)])
def test_head_major_short_runs_bit_exact(gpu_lib, N, Hl, d):
    """[N, Hl, d] <-> [Hl, N, d] with d of 1, 2 or 4 elements: runs of 2 to 8 bytes."""
    r = synth.bits_u16((1, N, Hl, d), 6, synth.TID_R)
    ref = oracle.unpack(r, 1)
    got = gpu_lib.ulysses_unpack(to_gpu_u16(r), 1)
    assert np.array_equal(bits_of(got), ref)
    assert np.array_equal(bits_of(gpu_lib.ulysses_pack_rev(got, 1, 1)), r)


def test_single_byte_runs(gpu_lib):
    g = torch.Generator().manual_seed(9)
    x = torch.randint(0, 255, (7001, 9, 1), generator=g, dtype=torch.int32).to(torch.uint8)
    got = gpu_lib.ulysses_pack(x.cuda(), 9).cpu()
    assert torch.equal(got, x.reshape(7001, 9, 1, 1).permute(1, 0, 2, 3))
    assert torch.equal(gpu_lib.ulysses_unpack_rev(got.cuda()).cpu(), x)


def test_empty_input_is_a_no_op(gpu_lib):
    x = torch.empty((0, 8, 64), dtype=torch.int16, device="cuda")
    assert gpu_lib.ulysses_pack(x, 4).shape == (4, 0, 2, 64)


@pytest.mark.parametrize("name", ["gpt1.3b", "gpt7b", "gpt30b", "1m"])
def test_full_size_configs_bit_exact(gpu_lib, name):
    """Full BASELINE shapes in the launch configuration the benchmark times, whole-tensor compare."""
    c = synth.CONFIGS[name]
    nl, H, d, P = c["N"] // c["P"], c["H"], c["d"], c["P"]
    x = synth.bits_u16((nl, H, d), synth.config_seed(name), synth.TID_X)
    got = gpu_lib.ulysses_pack(to_gpu_u16(x), P)
    assert np.array_equal(bits_of(got), oracle.pack(x, P))
    del got
    r = synth.bits_u16((P, nl, H // P, d), synth.config_seed(name), synth.TID_R)
    for layout in (0, 1):
        got = gpu_lib.ulysses_unpack(to_gpu_u16(r), layout)
        assert np.array_equal(bits_of(got), oracle.unpack(r, layout))
        del got


def test_tensors_beyond_four_gib(gpu_lib):
    """4.9 GB per tensor (2.46e9 elements): element offsets pass 2^31 and byte offsets 2^32 on both sides of every
    transform.  The oracle's index loops run on sampled row ranges (start, both places where an offset crosses
    2^31 elements, end): for a set R of local rows, pack(x[R]) = pack(x)[:, R], and likewise for the others."""
    nl, H, d, P = 1200003, 32, 64, 8
    Hl = H // P
    g = torch.Generator(device="cuda").manual_seed(2309)
    x = torch.randint(-32768, 32767, (nl, H, d), generator=g, dtype=torch.int16, device="cuda")
    assert x.numel() > (1 << 31)
    src_cross = (1 << 31) // (H * d)                       # row of x where the element offset passes 2^31
    dst_cross = ((1 << 31) // (Hl * d)) % nl               # local row where the offset inside send passes 2^31
    R = np.unique(np.concatenate([np.arange(0, 300), np.arange(src_cross - 300, src_cross + 300),
                                  np.arange(dst_cross - 300, dst_cross + 300), np.arange(nl - 300, nl)]))
    Rt = torch.from_numpy(R).cuda()

    send = gpu_lib.ulysses_pack(x, P)                       # [P, nl, Hl, d]
    assert np.array_equal(bits_of(send[:, Rt]), oracle.pack(bits_of(x[Rt]), P))
    back = gpu_lib.ulysses_unpack_rev(send)                 # [nl, H, d]
    assert np.array_equal(bits_of(back[Rt]), oracle.unpack_rev(bits_of(send[:, Rt])))
    assert torch.equal(back, x)
    del back
    y = gpu_lib.ulysses_unpack(send, 1)                     # [Hl, P*nl, d]
    ref = oracle.unpack(bits_of(send[:, Rt]), 1)            # [Hl, P*|R|, d]
    assert np.array_equal(bits_of(y.view(Hl, P, nl, d)[:, :, Rt]), ref.reshape(Hl, P, R.size, d))
    again = gpu_lib.ulysses_pack_rev(y, P, 1)               # [P, nl, Hl, d]
    assert np.array_equal(bits_of(again[:, Rt]), oracle.pack_rev(ref, P, 1))
    assert torch.equal(again, send)
