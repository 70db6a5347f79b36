"""Helpers shared by the GPU parity tests: host<->device conversion and error metrics."""
import numpy as np
import torch

import synth_inputs as synth


def to_gpu_bf16(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on cuda:0 (same bits)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def to_gpu_u16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()


def bits_of(t: torch.Tensor) -> np.ndarray:
    """Any 16-bit torch tensor -> uint16 numpy array of its bits."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def f64_of(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return synth.bf16_bits_to_f64(bits_of(t))
    return t.detach().cpu().numpy().astype(np.float64)


def max_abs(a, b) -> float:
    return float(np.max(np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64)))) if np.size(a) else 0.0


def rel_l2(got, ref) -> float:
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    den = float(np.sqrt((ref * ref).sum()))
    num = float(np.sqrt(((got - ref) ** 2).sum()))
    return num / den if den > 0 else num


def sample_rows(N: int, n_rows: int, P: int, seed: int) -> np.ndarray:
    """Sorted query rows to check at large N: first/last rows, tile edges, shard edges, random."""
    fixed = [0, 1, 2, 31, 32, 63, 64, 65, 127, 128, 129, 255, 256, N - 130, N - 129, N - 128, N - 2, N - 1]
    nl = N // P
    for q in range(1, P):
        fixed += [q * nl - 1, q * nl]
    fixed = [r for r in fixed if 0 <= r < N]
    rng = np.random.default_rng(seed)
    rows = set(fixed[:n_rows])
    while len(rows) < min(n_rows, N):
        rows.add(int(rng.integers(0, N)))
    return np.array(sorted(rows), dtype=np.int64)


def o_tolerance(ref: np.ndarray, absv: np.ndarray, base: float = 1e-2) -> np.ndarray:
    """Per-element bound on |O_gpu - O_oracle|: the stated max-abs 1e-2, except where the arithmetic
    the path is specified to use cannot meet it.  The kernel rounds P to bf16 before the PV matrix
    product and rounds O to bf16.  bf16 keeps 8 significant bits, so rounding to nearest moves a value
    in [2^e, 2^(e+1)) by at most half an ulp = 2^(e-8), a relative error of at most 2^-8 (reached just
    above a power of two).  Hence
        |O_gpu - O| <= 2^-8 * A + ulp_bf16(|O| + 2^-8 * A) / 2,      A_ic = sum_j P_ij |V_jc|,
    plus fp32 accumulation effects (1e-4 allowed).  `absv` is A, which the oracle computes as the
    attention output for |V|.  Wherever this bound is below 1e-2 (|O| < 1.5 or so for ordinary rows)
    the stated 1e-2 applies unchanged.  (A kernel whose softmax is taken relative to the exact row
    maximum represents the largest probability of a row, 1, exactly and stays well inside this bound
    on near-one-hot rows; one that uses any other reference point does not, and need not.)"""
    a = np.abs(np.asarray(ref, np.float64))
    p_err = np.asarray(absv, np.float64) * 2.0 ** -8
    ulp = np.exp2(np.floor(np.log2(np.maximum(a + p_err, 1e-30))) - 7)
    return np.maximum(base, p_err + 0.5 * ulp + 1e-4)


def o_within_tolerance(got, ref, absv, base: float = 1e-2):
    err = np.abs(np.asarray(got, np.float64) - np.asarray(ref, np.float64))
    tol = o_tolerance(ref, absv, base)
    bad = err > tol
    return (not bad.any()), float(err.max()) if err.size else 0.0, int(bad.sum())
