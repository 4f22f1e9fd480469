"""GPU parity of the dense Qwen3-style path: per-head RMSNorm of q and k before RoPE (the Q-Norm / K-Norm tasks of
paper Sec. 4.3), against the CPU oracle on the same seeded inputs, through the C ABI.  Bar: max|err| <= 2e-2 *
RMS(oracle), per layer and final; task counts and event counters exact."""
import dataclasses

import numpy as np
import pytest

import synth
from harness import GpuModel, bf16_to_f32_np, fixed_step, oracle_step, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-2
SPIN = 400000


def _etc():
    import paper_2604_13327_amd as etc
    return etc


def _run(dec, model, step, step_index=0):
    import torch
    x = model.hidden(step_index, step.batch)
    out = torch.empty_like(x)
    dec.bind_step(step)
    dec.launch(x, out)
    torch.cuda.synchronize()
    return bf16_to_f32_np(out)


def _check_invariants(dec):
    assert (dec.error_word() == 0).all(), dec.error_word()
    assert (dec.event_counters() == 0).all()
    assert (dec.exec_counts() == 1).all()


@pytest.fixture(scope="module")
def qk_model():
    return GpuModel(synth.TINY_QK, seed=21, n_pool_pages=160)


@pytest.mark.parametrize("kind", [0, 1, 2])
def test_tiny_qk_norm_decoder_matches_oracle_per_layer(qk_model, kind):
    etc = _etc()
    s = synth.TINY_QK
    qk_model.reset_pools()
    step = fixed_step(s, 3, [100, 7, 64], qk_model.n_pool_pages, seed=4)
    dec = etc.Decoder(s, kv_chunk_tokens=32, sampled_batches=[4], max_kv_len=129, kind=kind,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN, spin_budget=SPIN)
    qk_model.bind(dec)
    out = _run(dec, qk_model, step)
    _check_invariants(dec)
    ref = oracle_step(s, qk_model.seed, qk_model.n_pool_pages, step, 0)
    for l in range(s.n_layers):
        assert rel_err(dec.layer_hidden(l), ref["layers"][l]) <= TOL, f"layer {l}"
    assert rel_err(out, ref["final"]) <= TOL
    dec.close()


def test_tiny_qk_norm_appends_the_normalised_key(qk_model):
    """The cache row of the new token is the normalised, gain-scaled, rotated key; exactly one slot per layer changes."""
    import torch
    import oracle
    etc = _etc()
    s = synth.TINY_QK
    qk_model.reset_pools()
    before_k, before_v = qk_model.kpool.clone(), qk_model.vpool.clone()
    step = fixed_step(s, 2, [37, 16], qk_model.n_pool_pages, seed=5)
    dec = etc.Decoder(s, kv_chunk_tokens=16, sampled_batches=[2], max_kv_len=129, spin_budget=SPIN)
    qk_model.bind(dec)
    _run(dec, qk_model, step)
    exp = torch.zeros(qk_model.kpool.shape[:3], dtype=torch.bool, device="cuda")
    where = []
    for b, L in enumerate((37, 16)):
        page, slot = int(step.page_ids[step.page_indptr[b] + L // s.page]), L % s.page
        exp[:, page, slot] = True
        where.append((page, slot))
    assert torch.equal((qk_model.kpool != before_k).any(dim=-1).any(dim=-1), exp)
    assert torch.equal((qk_model.vpool != before_v).any(dim=-1).any(dim=-1), exp)
    w = synth.layer_weights_f32(s, qk_model.seed, 0)
    kp, vp = synth.kv_pool_f32(s, qk_model.seed, 0, qk_model.n_pool_pages)
    x = synth.hidden_f32(s, qk_model.seed, 0, 2)
    _, dbg = oracle.layer(oracle.shape_of(s), x.copy(), w, kp, vp, step.kv_len, step.page_indptr, step.page_ids, debug=True)
    for b, (page, slot) in enumerate(where):
        got = bf16_to_f32_np(qk_model.kpool[0, page, slot]).ravel()
        assert rel_err(got, dbg["k_rot"][b]) <= TOL
        # a normalised head with gains near one has a root mean square near one: an un-normalised key would not
        assert 0.5 < float(np.sqrt(np.mean(got ** 2))) < 1.5
        gotv = bf16_to_f32_np(qk_model.vpool[0, page, slot]).ravel()
        assert rel_err(gotv, dbg["v_new"][b]) <= TOL
    dec.close()


def test_tiny_qk_norm_three_chained_steps(qk_model):
    """Steps 2 and 3 read the normalised keys the earlier steps appended (nothing reset in between)."""
    import torch
    import oracle
    etc = _etc()
    s = synth.TINY_QK
    qk_model.reset_pools()
    dec = etc.Decoder(s, kv_chunk_tokens=16, sampled_batches=[2], max_kv_len=129,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN, spin_budget=SPIN)
    qk_model.bind(dec)
    L0 = np.array([30, 14], np.int32)
    npg = [synth.pages_needed(int(l) + 2, s.page) for l in L0]
    owned = np.random.default_rng(8).permutation(qk_model.n_pool_pages)[: sum(npg)].astype(np.int32)
    own = [owned[: npg[0]], owned[npg[0]:]]
    pools = [list(synth.kv_pool_f32(s, qk_model.seed, l, qk_model.n_pool_pages)) for l in range(s.n_layers)]
    bf16 = lambda a: torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()      # noqa: E731
    for t in range(3):
        kv = L0 + t
        cnt = [synth.pages_needed(int(l), s.page) for l in kv]
        indptr = np.concatenate([[0], np.cumsum(cnt)]).astype(np.int32)
        step = synth.Step(2, kv.astype(np.int32), indptr, np.concatenate([own[b][: cnt[b]] for b in range(2)]).astype(np.int32))
        out = _run(dec, qk_model, step, step_index=t)
        _check_invariants(dec)
        ref = oracle.decode_step(s, s.n_layers, synth.hidden_f32(s, qk_model.seed, t, 2),
                                 lambda l: synth.layer_weights_f32(s, qk_model.seed, l), lambda l: pools[l], step)
        for l in range(s.n_layers):
            assert rel_err(dec.layer_hidden(l), ref["layers"][l]) <= TOL, f"step {t} layer {l}"
            for b in range(2):
                pg, sl = int(own[b][kv[b] // s.page]), int(kv[b] % s.page)
                for pool in pools[l]:
                    pool[pg, sl] = bf16(pool[pg, sl])
        assert rel_err(out, ref["final"]) <= TOL, f"step {t}"
    dec.close()


def test_qwen3_32b_widths_four_layers_match_oracle():
    """The real Qwen3-32B layer (hidden 5120, 64 / 8 heads of 128, ffn 25600, eps 1e-6, theta 1e6, per-head norms),
    four layers deep so that the oracle finishes in seconds; batch 8 with ragged lengths across several KV chunks."""
    etc = _etc()
    s = dataclasses.replace(synth.QWEN3_32B, name="qwen3-32b-4l", n_layers=4)
    model = GpuModel(s, seed=31, n_pool_pages=600)
    rng = np.random.default_rng(2)
    kv = rng.integers(1, 1024, size=8).astype(np.int32)
    kv[0], kv[1] = 1023, 1
    step = fixed_step(s, 8, kv, model.n_pool_pages, seed=6)
    outs = []
    for kind in (0, 1):
        model.reset_pools()
        dec = etc.Decoder(s, kv_chunk_tokens=256, sampled_batches=[8], max_kv_len=1025, kind=kind,
                          debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN, spin_budget=SPIN)
        model.bind(dec)
        outs.append(_run(dec, model, step))
        _check_invariants(dec)
        if kind == 0:
            layers = [dec.layer_hidden(l).copy() for l in range(s.n_layers)]
        dec.close()
    np.testing.assert_array_equal(outs[0], outs[1])
    ref = oracle_step(s, model.seed, model.n_pool_pages, step, 0)
    for l in range(s.n_layers):
        assert rel_err(layers[l], ref["layers"][l]) <= TOL, f"layer {l}"
    assert rel_err(outs[0], ref["final"]) <= TOL
