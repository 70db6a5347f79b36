"""GPU parity of attention forward/backward against the fp64 oracle, through the C ABI.

Tolerances (bf16 inputs, stated by the target): max-abs 1e-2 on O, relative L2 2e-2 on each of
dQ, dK, dV.  P goes through the bf16 matrix product and O is stored in bf16, so for large |O| the
rounding the arithmetic implies already exceeds 1e-2; there the bound is the one derived in
_util.o_tolerance from the oracle's own sum_j P_ij |V_jc|.  LSE is fp32 on the GPU: max-abs 2e-3.
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as synth
from _util import f64_of, max_abs, o_within_tolerance, rel_l2, sample_rows, to_gpu_bf16

pytestmark = pytest.mark.gpu

TOL_O, TOL_G, TOL_LSE = 1e-2, 2e-2, 2e-3


def _run_gpu(uly, q, k, v, do, scale, causal, layout):
    tq, tk, tv, tdo = (to_gpu_bf16(a) for a in (q, k, v, do))
    o, lse = uly.ulysses_attn_fwd(tq, tk, tv, scale, causal, layout)
    dq, dk, dv = uly.ulysses_attn_bwd(tq, tk, tv, o, tdo, lse, scale, causal, layout)
    torch.cuda.synchronize()
    return o, lse, dq, dk, dv


def _full_parity(uly, N, Hl, d, causal=True, layout=0, seed=1, mult=1.0, scale=None):
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    q, k, v, do = synth.attention_inputs(N, Hl, d, seed, mult)           # [N,Hl,d]
    if layout == 1:
        q, k, v, do = (np.ascontiguousarray(a.transpose(1, 0, 2)) for a in (q, k, v, do))
    o, lse, dq, dk, dv = _run_gpu(uly, q, k, v, do, scale, causal, layout)
    fq, fk, fv, fdo = (oracle.bf16_to_f64(a) for a in (q, k, v, do))
    o_ref, lse_ref = oracle.attn_fwd(fq, fk, fv, scale, causal, layout)
    o_abs, _ = oracle.attn_fwd(fq, fk, np.abs(fv), scale, causal, layout)     # sum_j P_ij |V_jc|
    dq_ref, dk_ref, dv_ref = oracle.attn_bwd(fq, fk, fv, fdo, scale, causal, layout)
    ok, worst, n_bad = o_within_tolerance(f64_of(o), o_ref, o_abs, TOL_O)
    assert ok, (worst, n_bad)
    assert max_abs(f64_of(lse), lse_ref) <= TOL_LSE
    for name, got, ref in (("dq", dq, dq_ref), ("dk", dk, dk_ref), ("dv", dv, dv_ref)):
        err = rel_l2(f64_of(got), ref)
        assert err <= TOL_G, (name, err)


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("N", [1, 31, 33, 128, 129, 200, 257, 700, 1300])
def test_head_dimension_256(gpu_lib, N, causal):
    """d = 256 runs its own (simpler) kernels: ragged sizes, several tiles per head, both masks."""
    _full_parity(gpu_lib, N, 2, 256, causal=causal, seed=N + 256)


def test_head_dimension_256_head_major_and_odd_heads(gpu_lib):
    _full_parity(gpu_lib, 900, 3, 256, layout=1, seed=11)
    _full_parity(gpu_lib, 515, 5, 256, causal=False, layout=1, seed=12)


@pytest.mark.parametrize("N,Hl,d,layout", [(2177, 2, 128, 0), (5000, 1, 64, 0), (4100, 3, 128, 1), (9000, 1, 128, 0)])
def test_forward_with_workspace_cuts_long_rows(gpu_lib, N, Hl, d, layout):
    """Short sequences: with a workspace the causal forward cuts the keys of long rows into work items and merges
    them; O and LSE must meet the oracle like the plain forward's, and agree with it closely."""
    scale = 1.0 / np.sqrt(d)
    q, k, v, _ = synth.attention_inputs(N, Hl, d, 31 + N)
    if layout == 1:
        q, k, v = (np.ascontiguousarray(a.transpose(1, 0, 2)) for a in (q, k, v))
    tq, tk, tv = (to_gpu_bf16(a) for a in (q, k, v))
    need = gpu_lib.ulysses_attn_fwd_workspace_bytes(N, Hl, d, True)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    o, lse = gpu_lib.ulysses_attn_fwd(tq, tk, tv, scale, True, layout, workspace=ws)
    o2, lse2 = gpu_lib.ulysses_attn_fwd(tq, tk, tv, scale, True, layout, workspace=ws)
    o_plain, lse_plain = gpu_lib.ulysses_attn_fwd(tq, tk, tv, scale, True, layout)
    torch.cuda.synchronize()
    assert torch.equal(o, o2) and torch.equal(lse, lse2)                   # pieces are merged in a fixed order
    fq, fk, fv = (oracle.bf16_to_f64(a) for a in (q, k, v))
    o_ref, lse_ref = oracle.attn_fwd(fq, fk, fv, scale, True, layout)
    o_abs, _ = oracle.attn_fwd(fq, fk, np.abs(fv), scale, True, layout)
    ok, worst, n_bad = o_within_tolerance(f64_of(o), o_ref, o_abs, TOL_O)
    assert ok, (worst, n_bad)
    assert max_abs(f64_of(lse), lse_ref) <= TOL_LSE
    assert max_abs(f64_of(lse), f64_of(lse_plain)) <= 1e-4 and rel_l2(f64_of(o), f64_of(o_plain)) <= 5e-3


def test_tiny_config_full(gpu_lib):
    c = synth.CONFIGS["tiny"]
    _full_parity(gpu_lib, c["N"], c["H"] // c["P"], c["d"], seed=synth.config_seed("tiny"))


@pytest.mark.parametrize("N", [1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 200, 257, 333, 700])
@pytest.mark.parametrize("d", [64, 128])
def test_ragged_sizes(gpu_lib, N, d):
    _full_parity(gpu_lib, N, 3, d, seed=N)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("N", [65, 384, 777])
def test_non_causal(gpu_lib, N, d):
    _full_parity(gpu_lib, N, 2, d, causal=False, seed=N + 1)


@pytest.mark.parametrize("causal", [True, False])
def test_head_major_layout(gpu_lib, causal):
    _full_parity(gpu_lib, 300, 3, 128, causal=causal, layout=1, seed=4)


def test_wide_logit_range(gpu_lib):
    """Q, K scaled by 3 (logit sigma about 9): near one-hot rows, exercises the running max."""
    _full_parity(gpu_lib, 1024, 2, 128, seed=8, mult=3.0)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("causal", [True, False])
def test_row_maximum_climbs_block_after_block(gpu_lib, causal, d):
    """Keys whose scores grow by about 7 nats (10 in the exponent of 2) from one 32-key block to the next, in
    steps or not at all for a stretch: every kernel's running reference maximum has to move again and again,
    also by more than any lazy threshold, and everything accumulated so far has to be rescaled each time
    (ordinary inputs do that in the first few blocks only)."""
    N, Hl = 1500, 2
    scale = 1.0 / np.sqrt(d)
    q, k, v, _ = synth.attention_inputs(N, Hl, d, 41 + d)
    fq, fk = synth.bf16_bits_to_f32(q), synth.bf16_bits_to_f32(k)
    u = np.zeros(d, np.float32)
    u[: d // 8] = 1.0                                   # q.k gets a term a_j |u|^2, |u|^2 = d / 8
    step = np.floor(np.arange(N) / 32.0)
    step = np.where((step % 7) < 3, step - (step % 7), step)        # plateaus: blocks whose maximum does not move
    a = (7.0 / scale / (d // 8)) * step                               # so that scale * a_j |u|^2 = 7 * step
    fq = 0.25 * fq + u                                   # every query: u plus a little noise
    fk = 0.25 * fk + (a[:, None, None] * u).astype(np.float32)
    q, k = synth.f32_to_bf16_bits(fq), synth.f32_to_bf16_bits(fk)
    tq, tk, tv = (to_gpu_bf16(x) for x in (q, k, v))
    o, lse = gpu_lib.ulysses_attn_fwd(tq, tk, tv, scale, causal, 0)
    torch.cuda.synchronize()
    f64 = [oracle.bf16_to_f64(x) for x in (q, k, v)]
    o_ref, lse_ref = oracle.attn_fwd(*f64, scale, causal, 0)
    o_abs, _ = oracle.attn_fwd(f64[0], f64[1], np.abs(f64[2]), scale, causal, 0)
    ok, worst, n_bad = o_within_tolerance(f64_of(o), o_ref, o_abs, TOL_O)
    assert ok, (worst, n_bad)
    # LSE is of the order of 300 here; fp32 carries it to about 3e-5, the kernels' own arithmetic adds a little
    assert max_abs(f64_of(lse), lse_ref) <= 2e-3 + 4e-7 * np.abs(lse_ref).max()
    # (Forward only: with rows this close to one-hot, dS = P (dP - delta) is the difference of two nearly equal
    # numbers, delta comes from the bf16-rounded O, and no bf16 backward meets a relative bound on dQ.)


def test_multi_tile_medium(gpu_lib):
    _full_parity(gpu_lib, 1536, 7, 128, seed=12)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("N", [1021, 2177, 3200])
def test_paired_tile_walks(gpu_lib, N, d):
    """Several key/query tiles per head: the backward kernels give each workgroup a tile and its mirror
    image and walk them in opposite directions (odd tile counts leave the middle tile on its own;
    N not a multiple of 128 adds blocks past the end of the sequence)."""
    _full_parity(gpu_lib, N, 1, d, seed=N + d)


@pytest.mark.parametrize("N", [1021, 2177])
def test_paired_tile_walks_head_major(gpu_lib, N):
    _full_parity(gpu_lib, N, 2, 128, layout=1, seed=N)


def _sweep_cases():
    rng = np.random.default_rng(20230925)
    cases = []
    for _ in range(36):
        N = int(rng.integers(1, 1400))
        cases.append((N, int(rng.choice([64, 128])), bool(rng.integers(0, 2)), int(rng.integers(0, 2)),
                      int(rng.choice([1, 2, 3, 5]))))
    return cases


@pytest.mark.parametrize("N,d,causal,layout,Hl", _sweep_cases())
def test_shape_sweep(gpu_lib, N, d, causal, layout, Hl):
    """Seeded sweep over sequence length, head dim, mask, layout and head count."""
    _full_parity(gpu_lib, N, Hl, d, causal=causal, layout=layout, seed=N)


def _parity_on(gpu_lib, q, k, v, do, scale, causal=True):
    o, lse, dq, dk, dv = _run_gpu(gpu_lib, q, k, v, do, scale, causal, 0)
    fq, fk, fv, fdo = (oracle.bf16_to_f64(a) for a in (q, k, v, do))
    o_ref, lse_ref = oracle.attn_fwd(fq, fk, fv, scale, causal)
    o_abs, _ = oracle.attn_fwd(fq, fk, np.abs(fv), scale, causal)
    ok, worst, n_bad = o_within_tolerance(f64_of(o), o_ref, o_abs, TOL_O)
    assert ok, (worst, n_bad)
    assert max_abs(f64_of(lse), lse_ref) <= TOL_LSE
    for name, got, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), oracle.attn_bwd(fq, fk, fv, fdo, scale, causal)):
        denom = np.sqrt((ref ** 2).sum())
        if denom < 1e-6:                      # an exactly-zero gradient (e.g. dQ for constant K)
            assert np.abs(f64_of(got)).max() <= 2e-2, name
        else:
            assert rel_l2(f64_of(got), ref) <= TOL_G, name


@pytest.mark.parametrize("case", ["constant_k", "zero_q", "one_hot", "huge_logits"])
def test_degenerate_inputs(gpu_lib, case):
    """The degenerate cases of softmax: uniform rows (constant K, zero Q), one-hot rows, saturating logits."""
    N, Hl, d = 1500, 2, 128
    q, k, v, do = synth.attention_inputs(N, Hl, d, 77)
    scale = 1.0 / np.sqrt(d)
    if case == "constant_k":
        k = np.broadcast_to(k[:1], k.shape).copy()
    elif case == "zero_q":
        q = np.zeros_like(q)
    elif case == "one_hot":
        scale = 4.0                                   # logit sigma about 45: one key takes all the weight
    elif case == "huge_logits":
        q, k, _, _ = synth.attention_inputs(N, Hl, d, 78, 8.0)   # |logit| up to several thousand before scaling
        scale = 1.0
    _parity_on(gpu_lib, q, k, v, do, scale)


def test_backward_is_deterministic(gpu_lib):
    q, k, v, do = synth.attention_inputs(777, 2, 128, 3)
    a = _run_gpu(gpu_lib, q, k, v, do, 0.088, True, 0)
    b = _run_gpu(gpu_lib, q, k, v, do, 0.088, True, 0)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_empty_sequence(gpu_lib):
    z = torch.empty((0, 2, 64), dtype=torch.bfloat16, device="cuda")
    o, lse = gpu_lib.ulysses_attn_fwd(z, z.clone(), z.clone(), 0.125)
    assert o.shape == (0, 2, 64) and lse.shape == (2, 0)


@pytest.mark.parametrize("name", ["gpt1.3b", "gpt7b", "gpt30b", "1m"])
def test_full_size_configs_sampled_rows(gpu_lib, name):
    """BASELINE shapes at full size, in the launch configuration the benchmark times.

    (A) dense dO: O, LSE and dQ of 64 sampled query rows are exact per-row quantities the oracle
        computes one by one; the column-sum invariants sum_j dV_j = sum_i dO_i and sum_j dK_j = 0
        cover every row.
    (B) dO zeroed outside the sampled rows: the whole dK and dV equal the oracle's row-sampled
        backward (backward is linear in dO and rows are independent).
    """
    c = synth.CONFIGS[name]
    N, P, d = c["N"], c["P"], c["d"]
    Hl = c["H"] // P
    scale = 1.0 / np.sqrt(d)
    seed = synth.config_seed(name)
    q, k, v, do = synth.attention_inputs(N, Hl, d, seed, c["qk_mult"])
    rows = sample_rows(N, 64, P, seed)
    tq, tk, tv, tdo = (to_gpu_bf16(a) for a in (q, k, v, do))
    print(f"[{name}] N={N} Hl={Hl} d={d}: forward", flush=True)
    o, lse = gpu_lib.ulysses_attn_fwd(tq, tk, tv, scale, True)
    torch.cuda.synchronize()
    print(f"[{name}] backward (dense dO)", flush=True)
    dq, dk, dv = gpu_lib.ulysses_attn_bwd(tq, tk, tv, o, tdo, lse, scale, True)
    torch.cuda.synchronize()
    idx = torch.from_numpy(rows).cuda()
    o_s, lse_s, dq_s = f64_of(o[idx]), f64_of(lse[:, idx]), f64_of(dq[idx])
    sum_dv = dv.double().sum(0).cpu().numpy(); sum_dk = dk.double().sum(0).cpu().numpy()
    sum_do = tdo.double().sum(0).cpu().numpy()
    dk_rms = float(dk.double().pow(2).mean().sqrt())
    # (B) masked dO
    tdo_m = torch.zeros_like(tdo); tdo_m[idx] = tdo[idx]
    print(f"[{name}] backward (masked dO)", flush=True)
    _, dk_m, dv_m = gpu_lib.ulysses_attn_bwd(tq, tk, tv, o, tdo_m, lse, scale, True)
    torch.cuda.synchronize()
    dk_m, dv_m = f64_of(dk_m), f64_of(dv_m)
    del tq, tk, tv, tdo, tdo_m, o, lse, dq, dk, dv
    torch.cuda.empty_cache()

    print(f"[{name}] oracle on {rows.size} rows", flush=True)
    fq, fk, fv, fdo = (oracle.bf16_to_f64(a) for a in (q, k, v, do))
    o_ref, lse_ref = oracle.attn_fwd_rows(fq, fk, fv, rows, scale, True)
    o_abs, _ = oracle.attn_fwd_rows(fq, fk, np.abs(fv), rows, scale, True)    # sum_j P_ij |V_jc|
    dq_ref, dk_ref, dv_ref = oracle.attn_bwd_rows(fq, fk, fv, fdo, rows, scale, True)
    ok, worst, n_bad = o_within_tolerance(o_s, o_ref, o_abs, TOL_O)
    assert ok, (worst, n_bad)
    assert max_abs(lse_s, lse_ref) <= TOL_LSE
    assert rel_l2(dq_s, dq_ref) <= TOL_G
    assert rel_l2(dk_m, dk_ref) <= TOL_G
    assert rel_l2(dv_m, dv_ref) <= TOL_G
    # invariants over all rows (bf16 output rounding: N independent errors of relative size 2^-9)
    assert rel_l2(sum_dv, sum_do) <= 1e-2
    assert np.abs(sum_dk).max() <= 0.05 * dk_rms * np.sqrt(N)


@pytest.mark.parametrize("layout", [0, 1])
def test_tensors_beyond_four_gib(gpu_lib, layout):
    """520 heads of 32768 tokens: every tensor is 4.36 GB, so element offsets pass 2^31 and byte offsets 2^32.
    Three heads (first, middle, last) carry data and are checked on sampled rows as in the full-size test; the
    other heads are zero and must give exactly zero O and gradients (nothing leaks between heads)."""
    N, Hl, d, sel = 32768, 520, 128, [0, 259, 519]
    scale = 1.0 / np.sqrt(d)
    q, k, v, do = synth.attention_inputs(N, len(sel), d, 4321)
    rows = sample_rows(N, 48, 1, 4321)
    shape = (Hl, N, d) if layout == 1 else (N, Hl, d)

    def place(bits):
        big = torch.zeros(shape, dtype=torch.bfloat16, device="cuda")
        small = to_gpu_bf16(bits)
        if layout == 1:
            big[sel] = small.permute(1, 0, 2)
        else:
            big[:, sel] = small
        return big

    def take(t):                     # -> [N, 3, d]
        return t[sel].permute(1, 0, 2) if layout == 1 else t[:, sel]

    tq, tk, tv, tdo = (place(a) for a in (q, k, v, do))
    assert tq.numel() * 2 > (1 << 32)
    print("[>4GiB] forward", flush=True)
    o, lse = gpu_lib.ulysses_attn_fwd(tq, tk, tv, scale, True, layout)
    print("[>4GiB] backward (dense dO)", flush=True)
    dq, dk, dv = gpu_lib.ulysses_attn_bwd(tq, tk, tv, o, tdo, lse, scale, True, layout)
    torch.cuda.synchronize()
    idx = torch.from_numpy(rows).cuda()
    o_s, dq_s = f64_of(take(o)[idx]), f64_of(take(dq)[idx])
    lse_s = f64_of(lse[sel][:, idx])
    others = [h for h in range(Hl) if h not in sel]
    for t in (o, dq, dk, dv):
        rest = t[others] if layout == 1 else t[:, others]
        assert not bool(rest.any())
    tdo_m = torch.zeros_like(tdo)
    if layout == 1:
        tdo_m[:, idx] = tdo[:, idx]
    else:
        tdo_m[idx] = tdo[idx]
    del dq, dk, dv
    print("[>4GiB] backward (masked dO)", flush=True)
    _, dk_m, dv_m = gpu_lib.ulysses_attn_bwd(tq, tk, tv, o, tdo_m, lse, scale, True, layout)
    torch.cuda.synchronize()
    dk_m, dv_m = f64_of(take(dk_m)), f64_of(take(dv_m))
    del tq, tk, tv, tdo, tdo_m, o, lse
    torch.cuda.empty_cache()

    print(f"[>4GiB] oracle on {rows.size} rows", flush=True)
    fq, fk, fv, fdo = (oracle.bf16_to_f64(a) for a in (q, k, v, do))
    o_ref, lse_ref = oracle.attn_fwd_rows(fq, fk, fv, rows, scale, True)
    o_abs, _ = oracle.attn_fwd_rows(fq, fk, np.abs(fv), rows, scale, True)
    dq_ref, dk_ref, dv_ref = oracle.attn_bwd_rows(fq, fk, fv, fdo, rows, scale, True)
    ok, worst, n_bad = o_within_tolerance(o_s, o_ref, o_abs, TOL_O)
    assert ok, (worst, n_bad)
    assert max_abs(lse_s, lse_ref) <= TOL_LSE
    assert rel_l2(dq_s, dq_ref) <= TOL_G
    assert rel_l2(dk_m, dk_ref) <= TOL_G
    assert rel_l2(dv_m, dv_ref) <= TOL_G
