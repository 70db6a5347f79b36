"""Seeded synthetic inputs shared by the oracle tests, the GPU parity tests and the benchmark.

This module draws numbers and converts number formats; it contains none of the
method's arithmetic (no layout maps, no attention).  The generator itself is the
small C file next to this one, compiled on first use (or by ``build()``).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.c")
_LIB = os.path.join(_HERE, "libsynth_gen.so")
_lib = None

# tensor ids (fixed so every consumer regenerates the same bytes)
TID_X, TID_R, TID_Q, TID_K, TID_V, TID_DO = 0, 1, 2, 3, 4, 5
BASE_SEED = 0xC0FFEE00


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.synth_normal_bf16.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_uint64, ctypes.c_uint32, ctypes.c_float]
        lib.synth_normal_bf16.restype = None
        lib.synth_bits_u16.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                       ctypes.c_uint64, ctypes.c_uint32]
        lib.synth_bits_u16.restype = None
        _lib = lib
    return _lib


def normal_bf16(shape, seed: int, tensor_id: int, mult: float = 1.0, start: int = 0) -> np.ndarray:
    """bf16 bit patterns (uint16) of N(0,1)*mult samples, shape ``shape``, C order."""
    out = np.empty(shape, dtype=np.uint16)
    _load().synth_normal_bf16(out.ctypes.data, out.size, start, seed, tensor_id, mult)
    return out


def bits_u16(shape, seed: int, tensor_id: int, start: int = 0) -> np.ndarray:
    """Uniform random 16-bit payloads."""
    out = np.empty(shape, dtype=np.uint16)
    _load().synth_bits_u16(out.ctypes.data, out.size, start, seed, tensor_id)
    return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact decode of bf16 bit patterns to float32."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(bits).astype(np.float64)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


# ---- the workload table: shapes of one GPU's share -------------------------------------------
# name: N (global tokens), P (emulated sequence-parallel degree), H (total heads), d (head dim),
#       qk_mult (Q and K are multiplied by this in fp32 before rounding to bf16)
CONFIGS = {
    "tiny":     dict(idx=1, N=2048,    P=4,  H=8,  d=64,  qk_mult=1.0),
    "gpt1.3b":  dict(idx=2, N=32768,   P=8,  H=16, d=128, qk_mult=1.0),
    "gpt7b":    dict(idx=3, N=131072,  P=8,  H=32, d=128, qk_mult=1.0),
    "gpt30b":   dict(idx=4, N=262144,  P=8,  H=56, d=128, qk_mult=3.0),
    "1m":       dict(idx=5, N=1048576, P=32, H=32, d=128, qk_mult=1.0),
}


def config_seed(name: str) -> int:
    return BASE_SEED + CONFIGS[name]["idx"]


def attention_inputs(N: int, Hl: int, d: int, seed: int, qk_mult: float = 1.0):
    """Q, K, V, dO as bf16 bit patterns, each [N, Hl, d]."""
    shp = (N, Hl, d)
    return (normal_bf16(shp, seed, TID_Q, qk_mult), normal_bf16(shp, seed, TID_K, qk_mult),
            normal_bf16(shp, seed, TID_V, 1.0), normal_bf16(shp, seed, TID_DO, 1.0))
