"""Config 5: Llama-3-70B-shaped decoder on ONE GPU (about 137 GB of weights and up to 86 GB of KV pool
resident in the 288 GB of HBM), batch 32, KV lengths from U[2048, 8192], random permuted page table.
The whole 80-layer chain runs in one launch; the oracle runs all 32 sequences through all 80 layers and
is compared per layer and at the end, every row."""
import numpy as np
import pytest

import synth
from harness import GpuModel, SparsePools, bf16_to_f32_np, oracle_on_sequences, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-2
MAX_LEN = 8192
BATCH = 32


def test_llama70b_b32_full_chain_matches_oracle_on_every_sequence():
    import torch
    import paper_2604_13327_amd as etc
    s = synth.LLAMA3_70B
    seed = 7070
    free, total = torch.cuda.mem_get_info()
    if total < 250e9:
        pytest.skip("needs the 288 GB of an MI355X")
    n_pool = BATCH * synth.pages_needed(MAX_LEN, s.page) + 16
    model = GpuModel(s, seed, n_pool)
    print("70B weights and KV pool resident", flush=True)
    dec = etc.Decoder(s, kv_chunk_tokens=128, sampled_batches=[BATCH], max_kv_len=MAX_LEN + 1,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN, spin_budget=4000000)
    model.bind(dec)
    rng = np.random.default_rng(seed)
    step = synth.draw_step(rng, s, [BATCH], 2048, MAX_LEN, n_pool)
    dec.bind_step(step)
    x = model.hidden(0, BATCH)
    out = torch.empty_like(x)
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    dec.launch(x, out)
    t1.record()
    torch.cuda.synchronize()
    info = dec.step_info()
    ms = t0.elapsed_time(t1)
    print(f"70B B={BATCH}: {info.n_tasks} tasks, {info.algorithmic_bytes / 1e9:.1f} GB algorithmic, first launch {ms:.1f} ms "
          f"({info.algorithmic_bytes / ms / 1e6:.0f} GB/s)", flush=True)
    assert (dec.error_word() == 0).all(), dec.error_word()
    assert (dec.event_counters() == 0).all()
    assert (dec.exec_counts() == 1).all()
    got = bf16_to_f32_np(out)
    gpu_layers = [None] * s.n_layers
    sel = list(range(BATCH))
    for l in range(s.n_layers):
        gpu_layers[l] = dec.layer_hidden(l)[sel]
    dec.close()

    pools = SparsePools(s, seed, n_pool)
    done = [0]

    def weights_of(l):
        if l % 10 == 0:
            print(f"oracle layer {l}/{s.n_layers}", flush=True)
        done[0] = l
        return synth.layer_weights_f32(s, seed, l)

    ref = oracle_on_sequences(s, seed, step, sel, 0, weights_of, pools)
    errs = np.array([[rel_err(gpu_layers[l][j], ref["layers"][l][j]) for j in range(len(sel))] for l in range(s.n_layers)])
    print("kv_len of the sequences:", step.kv_len[sel].tolist())
    for l in range(0, s.n_layers, 8):
        print(f"layer {l}: max|err|/rms over the sequences: worst {errs[l].max():.3e} (sequence {int(errs[l].argmax())}), "
              f"median {np.median(errs[l]):.3e}", flush=True)
    worst = float(errs.max())
    assert worst <= TOL, f"layer {int(errs.max(axis=1).argmax())}: {worst}"
    assert rel_err(got[sel], ref["final"]) <= TOL
    print(f"llama70b B={BATCH}: all {len(sel)} sequences, worst per-layer max|err|/rms = {worst:.3e}")
