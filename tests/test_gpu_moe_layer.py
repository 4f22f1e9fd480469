"""GPU parity of the MoE layer on its own over a block of tokens (paper Sec. 2.4; the token sweep of Sec. 4.2 / 4.5),
through the C ABI, against the CPU oracle.

Integer work is compared on identical inputs, bit for bit: the oracle's top-k applied to the logits the GPU dumped
gives the GPU's ids; the oracle's grouping of those ids gives the GPU's permutation and both indptr arrays.  Floats
(routing weights, y) are compared with the oracle following the GPU's routing (a flip between the k-th and (k+1)-th
expert by rounding noise would otherwise look like an error): max|err| <= 2e-2 * RMS(oracle y).  All three schedulers
and the kernel-by-kernel comparator must give the same bits."""
import numpy as np
import pytest

import synth
from harness import bf16_to_f32_np, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-2
SPIN = 2000000


def _etc():
    import paper_2604_13327_amd as etc
    return etc


def _weights(s, seed):
    from synth import gpu as sgpu
    return sgpu.layer_weights_gpu(s, seed, 0)


def _routing(layer, s, T):
    from paper_2604_13327_amd import binding as b
    E, K = s.n_experts, s.top_k
    return {"logits": layer.routing_debug(b.DBG_ROUTER_LOGITS, 0, (T, E), np.float32),
            "ids": layer.routing_debug(b.DBG_TOPK_IDS, 0, (T, K), np.int32),
            "w": layer.routing_debug(b.DBG_TOPK_W, 0, (T, K), np.float32),
            "perm": layer.routing_debug(b.DBG_PERMUTATION, 0, (T * K,), np.int32),
            "tok_indptr": layer.routing_debug(b.DBG_TOK_INDPTR, 0, (E + 1,), np.int32),
            "exp_indptr": layer.routing_debug(b.DBG_EXP_INDPTR, 0, (E + 1,), np.int32)}


def _check_against_oracle(s, seed, x, y, r, tile_m, forced=None):
    import oracle
    T = x.shape[0]
    if forced is None:
        for b in range(T):
            np.testing.assert_array_equal(r["ids"][b], oracle.topk(r["logits"][b], s.top_k), err_msg=f"token {b}")
    else:
        np.testing.assert_array_equal(r["ids"], forced)
    count, tok_indptr, perm, exp_indptr = oracle.group(r["ids"], s.n_experts, tile_m)
    np.testing.assert_array_equal(r["perm"], perm)
    np.testing.assert_array_equal(r["tok_indptr"], tok_indptr)
    np.testing.assert_array_equal(r["exp_indptr"], exp_indptr)
    assert int(count.sum()) == T * s.top_k
    w = synth.layer_weights_f32(s, seed, 0)
    ref, _, ref_logits, ref_w = oracle.moe_layer(oracle.shape_of(s, tile_m), bf16_to_f32_np(x), w, forced_topk=r["ids"])
    assert rel_err(r["logits"], ref_logits) <= TOL
    np.testing.assert_allclose(r["w"], ref_w, rtol=5e-2, atol=2e-3)       # softmax of logits that carry the logit error
    for b in range(T):                                                   # and exactly the softmax of the GPU's own logits
        np.testing.assert_allclose(r["w"][b], oracle.route_weights(r["logits"][b], r["ids"][b]), rtol=2e-5, atol=1e-7)
    e = rel_err(y, ref)
    assert e <= TOL, e
    return e


def _run(layer, x, kbk=False):
    import torch
    y = torch.full_like(x, float("nan"))
    (layer.launch_kernel_by_kernel if kbk else layer.launch)(x, y)
    torch.cuda.synchronize()
    return bf16_to_f32_np(y)


@pytest.mark.parametrize("tokens,tile_m", [(1, 16), (70, 4), (128, 16), (300, 64), (64, 1)])
def test_tiny_moe_layer_matches_oracle_and_schedulers_agree(tokens, tile_m):
    from synth import gpu as sgpu
    etc = _etc()
    s, seed = synth.TINY_MOE, 51
    w = _weights(s, seed)
    x = sgpu.hidden_gpu(s, seed, tokens, tokens)
    outs = []
    for kind, kbk in ((0, False), (0, True), (1, False), (2, False)):
        layer = etc.MoeLayer(s, [tokens], kind=kind, moe_tile_m=tile_m,
                             debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_ROUTING, spin_budget=SPIN)
        layer.bind_weights(w)
        layer.bind_tokens(tokens)
        for rep in range(2):                       # the second launch runs on the re-armed event tensors
            y = _run(layer, x, kbk)
            assert (layer.error_word() == 0).all(), layer.error_word()
            if not kbk:
                assert (layer.event_counters() == 0).all()
        r = _routing(layer, s, tokens)
        if kind != 1 and not kbk:
            assert (layer.exec_counts() == 2).all()
        if kind == 1:                              # surplus row-tile slots never run under the dynamic scheduler
            plan = etc.moe_layer_plan_build(s, tokens, layer.step_info().n_queues, kind=1, moe_tile_m=tile_m)
            t = plan["tasks"]
            want = np.full(len(t), 2, np.int32)
            want[t["id"][((t["fn"] == 12) | (t["fn"] == 13)) & (t["c0"] >= int(r["exp_indptr"][-1]))]] = 0
            np.testing.assert_array_equal(layer.exec_counts(), want)
        outs.append((y, r))
        layer.close()
    for y, r in outs[1:]:
        np.testing.assert_array_equal(y, outs[0][0])
        for k in r:
            np.testing.assert_array_equal(r[k], outs[0][1][k], err_msg=k)
    _check_against_oracle(s, seed, x, outs[0][0], outs[0][1], tile_m)


def test_tiny_moe_layer_token_count_changes_without_recreate_and_forced_skew():
    """One context, several token counts (each runs the next larger sampled plan); then every token forced onto the
    same two experts: one expert's rows span many row tiles, all other experts are empty."""
    from synth import gpu as sgpu
    etc = _etc()
    s, seed, tile_m = synth.TINY_MOE, 52, 16
    w = _weights(s, seed)
    for kind in (0, 1):
        layer = etc.MoeLayer(s, [16, 200], kind=kind, moe_tile_m=tile_m, debug_flags=etc.DEBUG_ROUTING, spin_budget=SPIN)
        layer.bind_weights(w)
        for tokens in (200, 5, 16, 17, 130):
            x = sgpu.hidden_gpu(s, seed, tokens, tokens)
            layer.bind_tokens(tokens)
            assert layer.step_info().sampled_batch == (16 if tokens <= 16 else 200)
            y = _run(layer, x)
            assert (layer.error_word() == 0).all() and (layer.event_counters() == 0).all()
            _check_against_oracle(s, seed, x, y, _routing(layer, s, tokens), tile_m)
        tokens = 130
        forced = np.tile(np.array([[3, 9]], np.int32), (tokens, 1))
        layer.force_routing(0, forced)
        y = _run(layer, x)
        assert (layer.error_word() == 0).all() and (layer.event_counters() == 0).all()
        r = _routing(layer, s, tokens)
        assert r["exp_indptr"][-1] == 2 * -(-tokens // tile_m)
        _check_against_oracle(s, seed, x, y, r, tile_m, forced=forced)
        layer.force_routing(0, None)
        with pytest.raises(etc.EtcError):
            layer.bind_tokens(201)
        layer.close()


@pytest.mark.parametrize("tokens", [128, 1024])
def test_qwen3_moe_layer_matches_oracle(tokens):
    """The Qwen3-30B-A3B layer shape (128 experts, top-8, hidden 2048, expert FFN 768), row tiles of 64 tokens."""
    from synth import gpu as sgpu
    etc = _etc()
    s, seed, tile_m = synth.QWEN3_30B_A3B, 53, 64
    from synth.workloads import weight_specs, KIND
    w = {name: sgpu.tensor_gpu(seed, KIND[name], int(np.prod(shape)), mean, sigma, "cuda").view(*shape)
         for name, shape, mean, sigma in weight_specs(s) if name in ("g2", "wr", "eg", "eu", "ed")}
    x = sgpu.hidden_gpu(s, seed, tokens, tokens)
    outs = []
    for kind in (0, 1):
        layer = etc.MoeLayer(s, [tokens], kind=kind, moe_tile_m=tile_m, debug_flags=etc.DEBUG_ROUTING, spin_budget=SPIN)
        layer.bind_weights(w)
        layer.bind_tokens(tokens)
        y = _run(layer, x)
        assert (layer.error_word() == 0).all(), layer.error_word()
        assert (layer.event_counters() == 0).all()
        outs.append((y, _routing(layer, s, tokens)))
        layer.close()
    np.testing.assert_array_equal(outs[0][0], outs[1][0])
    e = _check_against_oracle(s, seed, x, outs[0][0], outs[0][1], tile_m)
    print(f"qwen3 MoE layer, {tokens} tokens: max|err|/rms = {e:.3e}, row tiles {int(outs[0][1]['exp_indptr'][-1])}")
