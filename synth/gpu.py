"""Device-side evaluation of the synthetic-input generator (harness code).

Evaluates the same integer hash as synth.c with torch int64 ops (every
intermediate is masked to 32 bits, so signed 64-bit wrap-around and arithmetic
right shifts cannot change the result) and looks the value up in the same
bf16 table.  Works chunk by chunk so temporaries stay small even for the
70B-shaped model.
"""
from __future__ import annotations

import numpy as np
import torch

from . import keys, normal_table
from .workloads import KIND, HIDDEN_TID0, LM_TID, ModelShape, kv_pool_shape, lm_specs, weight_specs

_M32 = 0xFFFFFFFF
_CHUNK = 1 << 25


def _fmix32(h: torch.Tensor) -> torch.Tensor:
    h = h ^ (h >> 16)
    h = (h * 0x85EBCA6B) & _M32
    h = h ^ (h >> 13)
    h = (h * 0xC2B2AE35) & _M32
    h = h ^ (h >> 16)
    return h


_tables: dict = {}


def _table(mean: float, sigma: float, device) -> torch.Tensor:
    key = (mean, sigma, str(device))
    if key not in _tables:
        bits = np.array(normal_table(mean, sigma)).view(np.int16)
        _tables[key] = torch.from_numpy(bits.copy()).view(torch.bfloat16).to(device)
    return _tables[key]


def tensor_gpu(seed: int, tensor_id: int, n: int, mean: float, sigma: float, device="cuda",
               i0: int = 0, out: torch.Tensor | None = None) -> torch.Tensor:
    """bf16 tensor [n] holding elements [i0, i0+n) of a synthetic tensor."""
    assert 0 <= i0 and i0 + n <= 1 << 32
    k1, k2 = keys(seed, tensor_id)
    tab = _table(mean, sigma, device)
    if out is None:
        out = torch.empty(n, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    for c0 in range(0, n, _CHUNK):
        c1 = min(n, c0 + _CHUNK)
        idx = torch.arange(i0 + c0, i0 + c1, dtype=torch.int64, device=device)
        h = _fmix32((_fmix32((idx ^ k1) & _M32) + k2) & _M32)
        flat[c0:c1] = tab[h & 0xFFFF]
    return out


def layer_weights_gpu(s: ModelShape, seed: int, layer: int, device="cuda") -> dict[str, torch.Tensor]:
    return {name: tensor_gpu(seed, layer * 64 + KIND[name], int(np.prod(shape)), mean, sigma,
                             device).view(*shape)
            for name, shape, mean, sigma in weight_specs(s)}


def lm_weights_gpu(s: ModelShape, seed: int, device="cuda") -> dict[str, torch.Tensor]:
    return {name: tensor_gpu(seed, LM_TID[name], int(np.prod(shape)), mean, sigma, device).view(*shape)
            for name, shape, mean, sigma in lm_specs(s)}


def kv_pool_gpu(s: ModelShape, seed: int, layer: int, n_pages: int, device="cuda"):
    shape = kv_pool_shape(s, n_pages)
    n = int(np.prod(shape))
    k = tensor_gpu(seed, layer * 64 + KIND["kpool"], n, 0.0, 1.0, device).view(*shape)
    v = tensor_gpu(seed, layer * 64 + KIND["vpool"], n, 0.0, 1.0, device).view(*shape)
    return k, v


def hidden_gpu(s: ModelShape, seed: int, step: int, batch: int, device="cuda") -> torch.Tensor:
    return tensor_gpu(seed, HIDDEN_TID0 + step, batch * s.H, 0.0, 1.0, device).view(batch, s.H)
