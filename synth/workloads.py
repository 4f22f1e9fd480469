"""Model shapes and seeded step draws of the benchmark configurations (harness code).

Shapes follow the five benchmark configurations: a tiny 2-layer decoder, a
Llama-3-8B-shaped dense decoder, a Qwen3-30B-A3B-like MoE decoder and a
Llama-3-70B-shaped dense decoder.  Weights ~ N(0, 0.02) (RMSNorm gains
1 + N(0, 0.02)), KV cache and input hidden state ~ N(0, 1), all bf16.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    H: int
    nq: int
    nkv: int
    d: int
    F: int = 0            # dense SwiGLU width (0 for MoE models)
    eps: float = 1e-5
    theta: float = 10000.0
    page: int = 16
    n_experts: int = 0
    top_k: int = 0
    moe_F: int = 0        # per-expert SwiGLU width
    qk_norm: bool = False # per-head RMSNorm of q and k before RoPE (Qwen3-style)
    vocab: int = 0        # > 0: token embedding, final norm and vocabulary projection exist

    @property
    def is_moe(self) -> bool:
        return self.n_experts > 0


TINY = ModelShape("tiny", 2, 256, 4, 2, 64, 1024)
TINY_MOE = ModelShape("tiny-moe", 2, 256, 4, 2, 64, 0, n_experts=16, top_k=2, moe_F=256)
LLAMA3_8B = ModelShape("llama3-8b", 32, 4096, 32, 8, 128, 14336)
QWEN3_30B_A3B = ModelShape("qwen3-30b-a3b", 48, 2048, 32, 4, 128, 0, n_experts=128, top_k=8, moe_F=768)
LLAMA3_70B = ModelShape("llama3-70b", 80, 8192, 64, 8, 128, 28672)
# the paper's end-to-end models (Sec. 4.3): Qwen3-32B-shaped dense decoder with per-head Q / K norm, and small
# decoders with a vocabulary for chained decode iterations
QWEN3_32B = ModelShape("qwen3-32b", 64, 5120, 64, 8, 128, 25600, eps=1e-6, theta=1000000.0, qk_norm=True)
TINY_QK = ModelShape("tiny-qk", 2, 256, 4, 2, 64, 1024, qk_norm=True)
TINY_LM = ModelShape("tiny-lm", 2, 256, 4, 2, 64, 1024, qk_norm=True, vocab=1024)
TINY_MOE_LM = ModelShape("tiny-moe-lm", 2, 256, 4, 2, 64, 0, n_experts=16, top_k=2, moe_F=256, qk_norm=True, vocab=1024)

SHAPES = {s.name: s for s in (TINY, TINY_MOE, LLAMA3_8B, QWEN3_30B_A3B, LLAMA3_70B, QWEN3_32B, TINY_QK, TINY_LM,
                              TINY_MOE_LM)}

# tensor kinds inside one layer; tensor id = layer * 64 + kind
KIND = {"g1": 0, "wq": 1, "wk": 2, "wv": 3, "wo": 4, "g2": 5, "wg": 6, "wu": 7, "wd": 8,
        "wr": 9, "eg": 10, "eu": 11, "ed": 12, "kpool": 13, "vpool": 14, "gq": 15, "gk": 16}
HIDDEN_TID0 = 0x7F000000
LM_TID = {"embed": 0x7E000001, "gf": 0x7E000002, "wlm": 0x7E000003}     # model-level tensors of a model with a vocabulary


def weight_specs(s: ModelShape) -> list[tuple[str, tuple[int, ...], float, float]]:
    """(name, shape, mean, sigma) of every weight tensor of one layer, row-major [out, in]."""
    specs = [("g1", (s.H,), 1.0, 0.02),
             ("wq", (s.nq * s.d, s.H), 0.0, 0.02),
             ("wk", (s.nkv * s.d, s.H), 0.0, 0.02),
             ("wv", (s.nkv * s.d, s.H), 0.0, 0.02),
             ("wo", (s.H, s.nq * s.d), 0.0, 0.02),
             ("g2", (s.H,), 1.0, 0.02)]
    if s.qk_norm:
        specs += [("gq", (s.d,), 1.0, 0.25), ("gk", (s.d,), 1.0, 0.25)]      # wide, so that a misplaced gain shows in the output
    if s.is_moe:
        specs += [("wr", (s.n_experts, s.H), 0.0, 0.02),
                  ("eg", (s.n_experts, s.moe_F, s.H), 0.0, 0.02),
                  ("eu", (s.n_experts, s.moe_F, s.H), 0.0, 0.02),
                  ("ed", (s.n_experts, s.H, s.moe_F), 0.0, 0.02)]
    else:
        specs += [("wg", (s.F, s.H), 0.0, 0.02),
                  ("wu", (s.F, s.H), 0.0, 0.02),
                  ("wd", (s.H, s.F), 0.0, 0.02)]
    return specs


def layer_weight_elems(s: ModelShape) -> int:
    return sum(int(np.prod(shape)) for _, shape, _, _ in weight_specs(s))


def layer_weights_f32(s: ModelShape, seed: int, layer: int) -> dict[str, np.ndarray]:
    """One layer's weights on the host, bf16 values widened exactly to fp32."""
    from . import tensor_f32
    return {name: tensor_f32(seed, layer * 64 + KIND[name], int(np.prod(shape)), mean, sigma).reshape(shape)
            for name, shape, mean, sigma in weight_specs(s)}


def lm_specs(s: ModelShape) -> list[tuple[str, tuple[int, ...], float, float]]:
    """(name, shape, mean, sigma) of the model-level tensors: token embedding (unit variance, like the synthetic
    hidden states), final RMSNorm gain, vocabulary projection."""
    return [("embed", (s.vocab, s.H), 0.0, 1.0), ("gf", (s.H,), 1.0, 0.02), ("wlm", (s.vocab, s.H), 0.0, 0.02)]


def lm_weights_f32(s: ModelShape, seed: int) -> dict[str, np.ndarray]:
    from . import tensor_f32
    return {name: tensor_f32(seed, LM_TID[name], int(np.prod(shape)), mean, sigma).reshape(shape)
            for name, shape, mean, sigma in lm_specs(s)}


def kv_pool_shape(s: ModelShape, n_pages: int) -> tuple[int, int, int, int]:
    """One layer's K (or V) pool: [physical page][slot][kv head][head dim]."""
    return (n_pages, s.page, s.nkv, s.d)


def kv_pool_f32(s: ModelShape, seed: int, layer: int, n_pages: int) -> tuple[np.ndarray, np.ndarray]:
    from . import tensor_f32
    shape = kv_pool_shape(s, n_pages)
    n = int(np.prod(shape))
    k = tensor_f32(seed, layer * 64 + KIND["kpool"], n, 0.0, 1.0).reshape(shape)
    v = tensor_f32(seed, layer * 64 + KIND["vpool"], n, 0.0, 1.0).reshape(shape)
    return k, v


def kv_pool_pages_f32(s: ModelShape, seed: int, layer: int, kbuf: np.ndarray, vbuf: np.ndarray, page_ids) -> None:
    """Fills only the listed physical pages of one layer's K and V pools (full-size fp32 buffers of
    kv_pool_shape): what an oracle run over a few sequences reads, without generating the whole pool."""
    from . import fill_blocks_f32
    page_elems = s.page * s.nkv * s.d
    fill_blocks_f32(kbuf.reshape(-1), seed, layer * 64 + KIND["kpool"], page_ids, page_elems, 0.0, 1.0)
    fill_blocks_f32(vbuf.reshape(-1), seed, layer * 64 + KIND["vpool"], page_ids, page_elems, 0.0, 1.0)


def hidden_f32(s: ModelShape, seed: int, step: int, batch: int) -> np.ndarray:
    from . import tensor_f32
    return tensor_f32(seed, HIDDEN_TID0 + step, batch * s.H, 0.0, 1.0).reshape(batch, s.H)


@dataclass
class Step:
    """Dynamic shape parameters of one decode step.

    kv_len[b] counts the tokens already cached for sequence b; the new token sits
    at position kv_len[b], is appended there, and attention covers kv_len[b] + 1
    keys.  Sequence b owns pages page_ids[page_indptr[b]:page_indptr[b+1]], that is
    ceil((kv_len[b] + 1) / page) physical pages.
    """
    batch: int
    kv_len: np.ndarray       # int32 [B]
    page_indptr: np.ndarray  # int32 [B+1]
    page_ids: np.ndarray     # int32 [page_indptr[B]]


def pages_needed(kv_len: int, page: int) -> int:
    return (kv_len + 1 + page - 1) // page


def draw_step(rng: np.random.Generator, s: ModelShape, batch_choices, len_lo: int, len_hi: int,
              n_pool_pages: int) -> Step:
    """Draw one step: batch size, ragged KV lengths, a random permuted page table."""
    batch = int(rng.choice(np.asarray(batch_choices)))
    kv_len = rng.integers(len_lo, len_hi + 1, size=batch).astype(np.int32)
    npg = np.array([pages_needed(int(l), s.page) for l in kv_len], dtype=np.int64)
    indptr = np.zeros(batch + 1, dtype=np.int32)
    indptr[1:] = np.cumsum(npg)
    assert indptr[-1] <= n_pool_pages, "page pool too small for this draw"
    page_ids = rng.permutation(n_pool_pages)[: indptr[-1]].astype(np.int32)
    return Step(batch, kv_len, indptr, page_ids)


def pool_pages_for(s: ModelShape, max_batch: int, max_len: int) -> int:
    return max_batch * pages_needed(max_len, s.page)
