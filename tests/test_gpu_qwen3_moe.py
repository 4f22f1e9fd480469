"""Config 4 at full size: Qwen3-30B-A3B-shaped MoE decoder (48 layers, 128 experts, top-8, expert width
768), ragged KV lengths drawn from U[256, 2048], random permuted page table.  Same checks as the tiny
MoE tests: integer routing data bit-exact on the GPU's own logits, floats against the oracle that follows
the GPU's routing, per layer and final; the free-running oracle may differ only on near ties."""
import numpy as np
import pytest

import synth
from harness import GpuModel, fixed_step
from test_gpu_moe import check_moe_step, expected_exec_counts, free_running_mismatches

pytestmark = pytest.mark.gpu
SPIN = 2000000
MAX_LEN = 2048


@pytest.fixture(scope="module")
def qwen_model():
    s = synth.QWEN3_30B_A3B
    return GpuModel(s, seed=4242, n_pool_pages=64 * synth.pages_needed(MAX_LEN, s.page) + 16)


def test_qwen3_moe_all_batches_match_oracle(qwen_model):
    """One context serves B = 1, 8, 32 and 64 (the sampled sizes) and an unsampled B = 5, without re-create."""
    import paper_2604_13327_amd as etc
    s, m = synth.QWEN3_30B_A3B, qwen_model
    dec = etc.Decoder(s, kv_chunk_tokens=64, sampled_batches=[1, 8, 32, 64], max_kv_len=MAX_LEN + 1, moe_tile_m=16,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN | etc.DEBUG_ROUTING, spin_budget=SPIN)
    m.bind(dec)
    rng = np.random.default_rng(77)
    for i, B in enumerate((1, 8, 5, 32, 64)):
        kv_len = rng.integers(256, MAX_LEN + 1, size=B)
        step = fixed_step(s, B, kv_len, m.n_pool_pages, seed=900 + i)
        m.reset_pools()
        dec.bind_step(step)
        info = dec.step_info()
        assert info.sampled_batch == {1: 1, 8: 8, 5: 8, 32: 32, 64: 64}[B]
        worst, routes, _ = check_moe_step(dec, m, s, step, 16, step_index=i, kv_chunk=64, max_kv_len=MAX_LEN + 1)
        distinct = [len(np.unique(r["ids"])) for r in routes]
        print(f"qwen3-moe B={B}: tasks {info.n_tasks}, worst per-layer max|err|/rms = {worst:.3e}, "
              f"distinct experts per layer {min(distinct)}..{max(distinct)}", flush=True)
        if B in (1, 64):
            n = free_running_mismatches(s, m, step, routes, step_index=i)
            print(f"qwen3-moe B={B}: free-running oracle picks a different expert set for {n} of {B * s.n_layers} "
                  f"(token, layer) pairs, all near ties", flush=True)
    dec.close()


def test_qwen3_moe_dynamic_scheduler_agrees_bitwise_with_static(qwen_model):
    """The dynamic scheduler (Alg. 2: ready queue, early push; expert events armed at run time release each
    expert's GroupGEMM row tiles, Sec. 2.4) runs the same task bodies, so a sampled batch (8), an unsampled one
    (5) and a large one (64) give the same bits as the static queues; every released task runs once, the
    surplus row-tile slots not at all, and every event ends at zero, also on the second launch."""
    import paper_2604_13327_amd as etc
    from test_gpu_moe import _launch
    s, m = synth.QWEN3_30B_A3B, qwen_model
    rng = np.random.default_rng(78)
    steps = [fixed_step(s, B, rng.integers(256, MAX_LEN + 1, size=B), m.n_pool_pages, seed=950 + i)
             for i, B in enumerate((8, 5, 64))]
    outs = {}
    for kind in (etc.SCHED_STATIC, etc.SCHED_DYNAMIC):
        dec = etc.Decoder(s, kv_chunk_tokens=64, sampled_batches=[8, 64], max_kv_len=MAX_LEN + 1, moe_tile_m=16,
                          kind=kind, debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_ROUTING, spin_budget=SPIN)
        m.bind(dec)
        for i, step in enumerate(steps):
            dec.bind_step(step)
            for rep in range(2):
                m.reset_pools()
                o = _launch(dec, m, step, step_index=i)
                assert (dec.error_word() == 0).all(), dec.error_word()
                assert (dec.event_counters() == 0).all()
                np.testing.assert_array_equal(dec.exec_counts(), expected_exec_counts(dec, s, 64, MAX_LEN + 1, 16, rep + 1))
                outs.setdefault((kind, i), []).append(o)
            print(f"qwen3-moe kind {kind} B={step.batch}: done", flush=True)
        dec.close()
    for i in range(len(steps)):
        ref = outs[(etc.SCHED_STATIC, i)][0]
        for o in outs[(etc.SCHED_STATIC, i)][1:] + outs[(etc.SCHED_DYNAMIC, i)]:
            np.testing.assert_array_equal(o, ref)
