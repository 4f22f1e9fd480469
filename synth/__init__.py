"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path's tests.

This package is harness code. It contains no arithmetic of the decode method:
only a counter-based integer hash, a table of normal quantiles rounded once to
bf16, the model shapes of the benchmark configurations, and the random draws
(batch sizes, KV lengths, page tables) that describe one decode step.

value(seed, tensor_id, i) = table[hash(seed, tensor_id, i) & 0xFFFF]

where ``table`` holds bf16(mean + sigma * Phi^-1((j + 0.5) / 65536)).  The host
side evaluates the hash in C (``synth.c``); the device side evaluates the very
same integer expression with torch ops (``synth.gpu``).
"""
from __future__ import annotations

import ctypes
import functools
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsynth.so")
_M32 = 0xFFFFFFFF


def build(force: bool = False) -> str:
    """Compile synth.c into libsynth.so (gcc, OpenMP)."""
    src = os.path.join(_HERE, "synth.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, src])
    return _LIB_PATH


@functools.lru_cache(maxsize=1)
def _lib():
    build()
    lib = ctypes.CDLL(_LIB_PATH)
    lib.synth_hash.restype = ctypes.c_uint32
    lib.synth_hash.argtypes = [ctypes.c_uint32] * 3
    for name in ("synth_fill_bf16", "synth_fill_f32"):
        f = getattr(lib, name)
        f.restype = None
        f.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_uint32,
                      ctypes.c_uint32, ctypes.c_void_p]
    lib.synth_fill_f32_blocks.restype = None
    lib.synth_fill_f32_blocks.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p]
    return lib


def _fmix32(h: int) -> int:
    h &= _M32
    h ^= h >> 16
    h = (h * 0x85EBCA6B) & _M32
    h ^= h >> 13
    h = (h * 0xC2B2AE35) & _M32
    h ^= h >> 16
    return h


def keys(seed: int, tensor_id: int) -> tuple[int, int]:
    """Two 32-bit hash keys for one tensor of one seeded workload."""
    k1 = _fmix32((seed * 0x9E3779B1 + 0x7F4A7C15) & _M32 ^ _fmix32(tensor_id + 0x165667B1))
    k2 = _fmix32(k1 ^ (tensor_id * 0x27D4EB2F + seed) & _M32)
    return k1, k2


def hash_py(k1: int, k2: int, idx: int) -> int:
    """Reference evaluation of the element hash in Python integers."""
    return _fmix32((_fmix32((idx ^ k1) & _M32) + k2) & _M32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


@functools.lru_cache(maxsize=16)
def normal_table(mean: float, sigma: float) -> np.ndarray:
    """65 536 normal quantiles, scaled, rounded once to bf16 (bit patterns)."""
    from scipy.special import ndtri
    q = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
    t = f32_to_bf16_bits((mean + sigma * q).astype(np.float32))
    t.setflags(write=False)
    return t


def tensor_bits(seed: int, tensor_id: int, n: int, mean: float, sigma: float, i0: int = 0) -> np.ndarray:
    """bf16 bit patterns (uint16) of elements [i0, i0+n) of a synthetic tensor."""
    assert 0 <= i0 and i0 + n <= 1 << 32
    k1, k2 = keys(seed, tensor_id)
    out = np.empty(n, dtype=np.uint16)
    tab = normal_table(mean, sigma)
    _lib().synth_fill_bf16(out.ctypes.data, n, i0, k1, k2, tab.ctypes.data)
    return out


def tensor_f32(seed: int, tensor_id: int, n: int, mean: float, sigma: float, i0: int = 0) -> np.ndarray:
    """The same elements widened exactly to fp32."""
    assert 0 <= i0 and i0 + n <= 1 << 32
    k1, k2 = keys(seed, tensor_id)
    out = np.empty(n, dtype=np.float32)
    tab = normal_table(mean, sigma)
    _lib().synth_fill_f32(out.ctypes.data, n, i0, k1, k2, tab.ctypes.data)
    return out


def fill_blocks_f32(out: np.ndarray, seed: int, tensor_id: int, blocks, block_elems: int, mean: float,
                    sigma: float) -> None:
    """Writes the blocks `blocks` (block b = elements [b*block_elems, (b+1)*block_elems)) of a synthetic
    tensor into `out`, which holds the tensor in full; everything else in `out` is left as it is."""
    assert out.dtype == np.float32 and out.flags.c_contiguous
    blocks = np.ascontiguousarray(blocks, dtype=np.int32)
    assert blocks.size == 0 or (blocks.min() >= 0 and (int(blocks.max()) + 1) * block_elems <= min(out.size, 1 << 32))
    k1, k2 = keys(seed, tensor_id)
    tab = normal_table(mean, sigma)
    _lib().synth_fill_f32_blocks(out.ctypes.data, blocks.ctypes.data, blocks.size, block_elems, k1, k2,
                                 tab.ctypes.data)


from .workloads import *  # noqa: E402,F401,F403
