"""Config 3: Llama-3-8B-shaped decoder under dynamic shapes.  100 consecutive steps on ONE context (no
re-create): batch size drawn from {1, 4, 16, 64}, KV lengths from U[128, 4096], a fresh random page table
per step.  Every step checks the scheduling invariants (event counters drained, every task ran once).
On the first step of every sampled batch size (1, 4, 16, 64) the oracle runs ALL sequences of the step, every
layer: every column block and every K-slice partial of the large-batch projection paths is compared at full
size.  On the other steps it follows one sequence out of every block of 16 columns plus the last one
(sequences of a dense decoder do not interact, so a subset of the batch is an exact check of those rows)."""
import numpy as np
import pytest

import synth
from harness import GpuModel, SparsePools, bf16_to_f32_np, oracle_on_sequences, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-2
N_STEPS = 100
MAX_LEN = 4096


N_SEGMENTS = 5       # the 100 steps run as five tests on the one context, so that none is silent for minutes


@pytest.fixture(scope="module")
def run100():
    """The one context of the 100 steps, the model on both sides and the drawn steps."""
    import paper_2604_13327_amd as etc
    s = synth.LLAMA3_8B
    seed = 3030
    n_pool = 64 * synth.pages_needed(MAX_LEN, s.page) + 16
    model = GpuModel(s, seed, n_pool)
    dec = etc.Decoder(s, kv_chunk_tokens=64, sampled_batches=[1, 4, 16, 64], max_kv_len=MAX_LEN + 1,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN, spin_budget=2000000)
    model.bind(dec)
    rng = np.random.default_rng(seed)
    state = {"s": s, "seed": seed, "n_pool": n_pool, "model": model, "dec": dec,
             "weights": [synth.layer_weights_f32(s, seed, l) for l in range(s.n_layers)],     # ~28 GB of host memory
             "pools": SparsePools(s, seed, n_pool),
             "steps": [synth.draw_step(rng, s, [1, 4, 16, 64], 128, MAX_LEN, n_pool) for _ in range(N_STEPS)],
             "seen": {}, "worst": 0.0, "bytes": [], "done": 0}
    yield state
    dec.close()


@pytest.mark.parametrize("segment", range(N_SEGMENTS))
def test_llama8b_100_steps_of_changing_shape_without_recreate(run100, segment):
    import torch
    st = run100
    s, seed, model, dec, seen = st["s"], st["seed"], st["model"], st["dec"], st["seen"]
    per = N_STEPS // N_SEGMENTS
    assert st["done"] == segment * per, "the segments are consecutive steps of one context"
    for i in range(segment * per, (segment + 1) * per):
        step = st["steps"][i]
        B = step.batch
        # the step appends one row per sequence and layer; put the seeded rows back afterwards so that the
        # steps stay independent draws (a later step may own the same physical page)
        pg = torch.as_tensor(step.page_ids[step.page_indptr[:-1] + step.kv_len // s.page].astype(np.int64), device="cuda")
        sl = torch.as_tensor((step.kv_len % s.page).astype(np.int64), device="cuda")
        keep_k, keep_v = model.kpool[:, pg, sl].clone(), model.vpool[:, pg, sl].clone()
        dec.bind_step(step)
        x = model.hidden(i, B)
        out = torch.empty_like(x)
        dec.launch(x, out)
        torch.cuda.synchronize()
        assert (dec.error_word() == 0).all(), (i, dec.error_word())
        assert (dec.event_counters() == 0).all(), f"step {i}: an event counter did not drain"
        assert (dec.exec_counts() == 1).all(), f"step {i}: a task did not run exactly once"
        info = dec.step_info()
        assert info.sampled_batch == B
        got = bf16_to_f32_np(out)
        if B not in seen:                     # first step of this batch size: every row
            sel = list(range(B))
        else:                                 # one column of every 16-column block of the tiles, and the last column
            sel = sorted({min(B - 1, 3 + 16 * k) for k in range((B + 15) // 16)} | {B - 1})
        ref = oracle_on_sequences(s, seed, step, sel, i, lambda l: st["weights"][l], st["pools"])
        for l in range(s.n_layers):
            e = rel_err(dec.layer_hidden(l)[sel], ref["layers"][l])
            st["worst"] = max(st["worst"], e)
            assert e <= TOL, f"step {i} (batch {B}) layer {l}: {e}"
        assert rel_err(got[sel], ref["final"]) <= TOL, f"step {i} (batch {B}) final"
        model.kpool[:, pg, sl] = keep_k
        model.vpool[:, pg, sl] = keep_v
        seen[B] = seen.get(B, 0) + 1
        st["bytes"].append(int(info.algorithmic_bytes))
        st["done"] = i + 1
    print(f"steps {segment * per}..{(segment + 1) * per - 1}: batches so far {dict(sorted(seen.items()))}, worst per-layer "
          f"max|err|/rms {st['worst']:.3e}", flush=True)
    if segment == N_SEGMENTS - 1:
        assert set(seen) == {1, 4, 16, 64}
        print(f"llama8b dynamic shapes: {N_STEPS} steps, worst per-layer max|err|/rms = {st['worst']:.3e}, "
              f"algorithmic bytes per step {min(st['bytes']) / 1e9:.1f}..{max(st['bytes']) / 1e9:.1f} GB")


def test_llama8b_changing_shapes_under_the_dynamic_scheduler():
    """The same kind of step sequence (batch from {1, 4, 16, 64}, lengths U[128, 4096], one context each) under
    the dynamic scheduler: every step drains its events, runs every task once and gives the same bits as the
    static scheduler on the same step."""
    import torch
    import paper_2604_13327_amd as etc
    s = synth.LLAMA3_8B
    seed = 3031
    n_pool = 64 * synth.pages_needed(MAX_LEN, s.page) + 16
    model = GpuModel(s, seed, n_pool)
    rng = np.random.default_rng(seed)
    steps = [synth.draw_step(rng, s, [b], 128, MAX_LEN, n_pool) for b in (4, 1, 64, 16, 1, 64, 4, 16)]
    outs = {}
    for kind in (etc.SCHED_STATIC, etc.SCHED_DYNAMIC):
        dec = etc.Decoder(s, kv_chunk_tokens=64, sampled_batches=[1, 4, 16, 64], max_kv_len=MAX_LEN + 1, kind=kind,
                          debug_flags=etc.DEBUG_EXEC_COUNT, spin_budget=2000000)
        model.bind(dec)
        for i, step in enumerate(steps):
            model.reset_pools()
            dec.bind_step(step)
            x = model.hidden(i, step.batch)
            out = torch.empty_like(x)
            dec.launch(x, out)
            torch.cuda.synchronize()
            assert (dec.error_word() == 0).all(), (kind, i, dec.error_word())
            assert (dec.event_counters() == 0).all(), f"kind {kind} step {i}: an event counter did not drain"
            assert (dec.exec_counts() == 1).all(), f"kind {kind} step {i}: a task did not run exactly once"
            outs[(kind, i)] = bf16_to_f32_np(out)
            print(f"kind {kind} step {i} (batch {step.batch}) done", flush=True)
        dec.close()
    for i in range(len(steps)):
        np.testing.assert_array_equal(outs[(etc.SCHED_DYNAMIC, i)], outs[(etc.SCHED_STATIC, i)])
