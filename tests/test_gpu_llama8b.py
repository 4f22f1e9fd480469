"""Config 2 at full size, in the launch configuration bench.py times: Llama-3-8B-shaped decoder, batch 1,
1024 cached tokens, random permuted page table.  The whole 32-layer chain is compared with the CPU
oracle layer by layer (the oracle regenerates one layer's inputs at a time)."""
import numpy as np
import pytest

import synth
from harness import GpuModel, bf16_to_f32_np, fixed_step, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-2


def test_llama8b_bs1_full_chain_matches_oracle_per_layer():
    import torch
    import oracle
    import paper_2604_13327_amd as etc
    s = synth.LLAMA3_8B
    seed, L = 2024, 1024
    n_pool = synth.pages_needed(L, s.page) + 16
    model = GpuModel(s, seed, n_pool)
    dec = etc.Decoder(s, kv_chunk_tokens=128, sampled_batches=[1], max_kv_len=L + 1,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN, spin_budget=2000000)
    model.bind(dec)
    step = fixed_step(s, 1, [L], n_pool, seed=7)
    dec.bind_step(step)
    x = model.hidden(0, 1)
    out = torch.empty_like(x)
    dec.launch(x, out)
    torch.cuda.synchronize()
    assert (dec.error_word() == 0).all()
    assert (dec.event_counters() == 0).all()
    assert (dec.exec_counts() == 1).all()
    info = dec.step_info()
    assert info.n_queues == 256 and info.algorithmic_bytes > 14.0e9
    gpu_layers = [dec.layer_hidden(l) for l in range(s.n_layers)]
    got = bf16_to_f32_np(out)
    dec.close()

    # the dynamic scheduler (Alg. 2) on the same step: same task bodies, so the same bits in every layer
    model.reset_pools()
    dyn = etc.Decoder(s, kv_chunk_tokens=128, sampled_batches=[1], max_kv_len=L + 1, kind=etc.SCHED_DYNAMIC,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN, spin_budget=2000000)
    model.bind(dyn)
    dyn.bind_step(step)
    out_dyn = torch.empty_like(x)
    for rep in range(2):                    # the second launch runs on the re-armed events and queue words
        model.reset_pools()
        out_dyn.zero_()
        dyn.launch(x, out_dyn)
        torch.cuda.synchronize()
        assert (dyn.error_word() == 0).all()
        assert (dyn.event_counters() == 0).all()
        assert (dyn.exec_counts() == rep + 1).all()
        np.testing.assert_array_equal(bf16_to_f32_np(out_dyn), got)
    for l in range(s.n_layers):
        np.testing.assert_array_equal(dyn.layer_hidden(l), gpu_layers[l])
    dyn.close()
    del model
    torch.cuda.empty_cache()

    xo = synth.hidden_f32(s, seed, 0, 1)
    oshape = oracle.shape_of(s)
    worst = 0.0
    for l in range(s.n_layers):
        w = synth.layer_weights_f32(s, seed, l)
        kp, vp = synth.kv_pool_f32(s, seed, l, n_pool)
        oracle.layer(oshape, xo, w, kp, vp, step.kv_len, step.page_indptr, step.page_ids)
        e = rel_err(gpu_layers[l], xo)
        worst = max(worst, e)
        assert e <= TOL, f"layer {l}: {e}"
    assert rel_err(got, xo) <= TOL
    print(f"llama8b worst per-layer max|err|/rms = {worst:.3e}")
