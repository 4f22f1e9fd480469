"""Test harness: puts one seeded synthetic workload on the GPU (through the C ABI binding) and on the
CPU oracle, so the two can be compared.  The two sides share only the seeded generators of `synth`."""
from __future__ import annotations

import numpy as np

import synth


def bf16_to_f32_np(t):
    """torch bf16 (any device) -> numpy fp32, exact."""
    import torch
    return t.detach().to(torch.float32).cpu().numpy()


class GpuModel:
    """Weights and KV pools of one seeded model resident on the GPU, bound to a Decoder."""

    def __init__(self, shape, seed: int, n_pool_pages: int, device="cuda"):
        import torch
        from synth import gpu as sgpu
        self.shape, self.seed, self.n_pool_pages, self.device = shape, seed, n_pool_pages, device
        self.weights = [sgpu.layer_weights_gpu(shape, seed, l, device) for l in range(shape.n_layers)]
        pshape = (shape.n_layers,) + synth.kv_pool_shape(shape, n_pool_pages)
        self.kpool = torch.empty(pshape, dtype=torch.bfloat16, device=device)
        self.vpool = torch.empty(pshape, dtype=torch.bfloat16, device=device)
        self.reset_pools()

    def reset_pools(self):
        from synth import gpu as sgpu
        n = int(np.prod(self.kpool.shape[1:]))
        for l in range(self.shape.n_layers):
            sgpu.tensor_gpu(self.seed, l * 64 + synth.KIND["kpool"], n, 0.0, 1.0, self.device, out=self.kpool[l])
            sgpu.tensor_gpu(self.seed, l * 64 + synth.KIND["vpool"], n, 0.0, 1.0, self.device, out=self.vpool[l])

    def bind(self, dec):
        for l, w in enumerate(self.weights):
            dec.bind_layer_weights(l, w)
        dec.bind_kv_pool(self.kpool, self.vpool)

    def hidden(self, step_index: int, batch: int):
        from synth import gpu as sgpu
        return sgpu.hidden_gpu(self.shape, self.seed, step_index, batch, self.device)


def oracle_step(shape, seed: int, n_pool_pages: int, step, step_index: int, n_layers=None, forced_topk_of=None,
                tile_m: int = 16, x0=None, first_layer: int = 0):
    """The CPU oracle on the same seeded inputs, generated layer by layer."""
    import oracle
    n_layers = shape.n_layers if n_layers is None else n_layers
    if x0 is None:
        x0 = synth.hidden_f32(shape, seed, step_index, step.batch)
    pools = {}

    def pools_of(l):
        pools.clear()                               # one layer resident at a time
        pools[l] = synth.kv_pool_f32(shape, seed, first_layer + l, n_pool_pages)
        return pools[l]

    return oracle.decode_step(shape, n_layers, x0, lambda l: synth.layer_weights_f32(shape, seed, first_layer + l),
                              pools_of, step, forced_topk_of=forced_topk_of, tile_m=tile_m)


def rel_err(gpu: np.ndarray, ref: np.ndarray) -> float:
    """max |err| / RMS(reference): the quantity the floating-point bar bounds by 2e-2."""
    ref = ref.astype(np.float64)
    return float(np.abs(gpu.astype(np.float64) - ref).max() / np.sqrt(np.mean(ref ** 2)))


def fixed_step(shape, batch: int, kv_len, n_pool_pages: int, seed: int):
    rng = np.random.default_rng(seed)
    kv_len = np.asarray(kv_len, np.int32)
    assert len(kv_len) == batch
    npg = np.array([synth.pages_needed(int(l), shape.page) for l in kv_len], dtype=np.int64)
    indptr = np.zeros(batch + 1, dtype=np.int32)
    indptr[1:] = np.cumsum(npg)
    page_ids = rng.permutation(n_pool_pages)[: indptr[-1]].astype(np.int32)
    return synth.Step(batch, kv_len, indptr, page_ids)


def sub_step(step, sel):
    """The step restricted to the sequences `sel` (same physical pages): sequences of a dense decoder do
    not interact, so the oracle can check a few of them without computing the whole batch."""
    sel = [int(b) for b in sel]
    pages = [step.page_ids[step.page_indptr[b]:step.page_indptr[b + 1]] for b in sel]
    indptr = np.zeros(len(sel) + 1, dtype=np.int32)
    indptr[1:] = np.cumsum([len(p) for p in pages])
    return synth.Step(len(sel), step.kv_len[sel].astype(np.int32), indptr, np.concatenate(pages).astype(np.int32))


class SparsePools:
    """Full-size fp32 K/V pool buffers of one layer in which only the pages a step reads are generated."""

    def __init__(self, shape, seed: int, n_pool_pages: int):
        self.shape, self.seed = shape, seed
        self.k = np.zeros(synth.kv_pool_shape(shape, n_pool_pages), dtype=np.float32)
        self.v = np.zeros_like(self.k)

    def of(self, layer: int, page_ids):
        synth.kv_pool_pages_f32(self.shape, self.seed, layer, self.k, self.v, page_ids)
        return self.k, self.v


def oracle_on_sequences(shape, seed: int, step, sel, step_index: int, weights_of, pools: SparsePools):
    """CPU oracle over the sequences `sel` of a step; returns its dict (final, layers)."""
    import oracle
    sub = sub_step(step, sel)
    x0 = synth.hidden_f32(shape, seed, step_index, step.batch)[[int(b) for b in sel]]
    return oracle.decode_step(shape, shape.n_layers, x0, weights_of, lambda l: pools.of(l, sub.page_ids), sub)
