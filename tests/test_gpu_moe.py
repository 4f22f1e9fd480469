"""GPU parity of the MoE path (router, top-k, token grouping, GroupGEMM, combine) against the CPU oracle.

Integer work is compared on identical inputs: the oracle's top-k and grouping applied to the logits the
GPU dumped must give the GPU's ids, permutation and both indptr arrays bit for bit.  Floating point
downstream is compared with the oracle following the GPU's routing (a legitimate flip of the k-th and
(k+1)-th expert by accumulated rounding noise would otherwise look like an error); the free-running
oracle is compared as well, and every selection it disagrees on must sit on a near tie."""
import numpy as np
import pytest

import synth
from harness import GpuModel, bf16_to_f32_np, fixed_step, oracle_step, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-2
SPIN = 400000
FN_MOE_GATEUP, FN_MOE_DOWN = 12, 13


def _etc():
    import paper_2604_13327_amd as etc
    return etc


def _b():
    from paper_2604_13327_amd import binding
    return binding


def _launch(dec, model, step, step_index=0, kbk=False):
    import torch
    x = model.hidden(step_index, step.batch)
    out = torch.empty_like(x)
    (dec.launch_kernel_by_kernel if kbk else dec.launch)(x, out)
    torch.cuda.synchronize()
    return bf16_to_f32_np(out)


def _routing(dec, s, B, layer):
    from paper_2604_13327_amd import binding as b
    E, K = s.n_experts, s.top_k
    return {"logits": dec.routing_debug(b.DBG_ROUTER_LOGITS, layer, (B, E), np.float32),
            "ids": dec.routing_debug(b.DBG_TOPK_IDS, layer, (B, K), np.int32),
            "w": dec.routing_debug(b.DBG_TOPK_W, layer, (B, K), np.float32),
            "perm": dec.routing_debug(b.DBG_PERMUTATION, layer, (B * K,), np.int32),
            "tok_indptr": dec.routing_debug(b.DBG_TOK_INDPTR, layer, (E + 1,), np.int32),
            "exp_indptr": dec.routing_debug(b.DBG_EXP_INDPTR, layer, (E + 1,), np.int32)}


def expected_exec_counts(dec, s, kv_chunk, max_kv_len, tile_m, launches=1):
    """Executions per task after `launches` launches of the bound step.  Static queues run every task of
    the sampled grid (surplus row-tile slots are no-ops that still notify).  Under the dynamic scheduler an
    expert's event releases only that expert's row tiles (Sec. 2.4), so the GroupGEMM tasks of slots beyond
    exp_indptr[E] never run.  Needs DEBUG_ROUTING for the dynamic case."""
    import paper_2604_13327_amd as etc
    from paper_2604_13327_amd import binding as b
    info = dec.step_info()
    want = np.full(info.n_tasks, launches, np.int32)
    if dec.kind != etc.SCHED_DYNAMIC:
        return want
    plan = etc.plan_build(s, kv_chunk, info.sampled_batch, info.n_queues, max_kv_len=max_kv_len, kind=dec.kind,
                          moe_tile_m=tile_m)
    t = plan["tasks"]
    assert len(t) == info.n_tasks
    for layer in range(s.n_layers):
        live = int(dec.routing_debug(b.DBG_EXP_INDPTR, layer, (s.n_experts + 1,), np.int32)[-1])
        dead = (t["layer"] == layer) & ((t["fn"] == FN_MOE_GATEUP) | (t["fn"] == FN_MOE_DOWN)) & (t["c0"] >= live)
        want[t["id"][dead]] = 0
    return want


def check_moe_step(dec, model, s, step, tile_m, step_index=0, forced=None, layers=None, first_layer=0,
                   kv_chunk=32, max_kv_len=129):
    """One launch, then every check of the module docstring.  Returns the worst per-layer error."""
    import oracle
    B = step.batch
    n_layers = s.n_layers if layers is None else layers
    out = _launch(dec, model, step, step_index)
    assert (dec.error_word() == 0).all(), dec.error_word()
    assert (dec.event_counters() == 0).all(), "an event counter did not drain to zero"
    np.testing.assert_array_equal(dec.exec_counts(), expected_exec_counts(dec, s, kv_chunk, max_kv_len, tile_m),
                                  err_msg="a task did not run exactly once (surplus row-tile slots under the "
                                          "dynamic scheduler: not at all)")
    routes = [_routing(dec, s, B, l) for l in range(n_layers)]
    for l, r in enumerate(routes):
        # integers on identical inputs
        if forced is None:
            for b in range(B):
                np.testing.assert_array_equal(r["ids"][b], oracle.topk(r["logits"][b], s.top_k), err_msg=f"layer {l} token {b}")
        else:
            np.testing.assert_array_equal(r["ids"], forced[l])
        count, tok_indptr, perm, exp_indptr = oracle.group(r["ids"], s.n_experts, tile_m)
        np.testing.assert_array_equal(r["perm"], perm)
        np.testing.assert_array_equal(r["tok_indptr"], tok_indptr)
        np.testing.assert_array_equal(r["exp_indptr"], exp_indptr)
        assert int(count.sum()) == B * s.top_k
        for b in range(B):
            np.testing.assert_allclose(r["w"][b], oracle.route_weights(r["logits"][b], r["ids"][b]), rtol=2e-5, atol=1e-7)
    # floats, oracle following the GPU's routing
    ref = oracle_step(s, model.seed, model.n_pool_pages, step, step_index, n_layers=n_layers,
                      forced_topk_of=lambda l: routes[l]["ids"], tile_m=tile_m, first_layer=first_layer)
    worst = 0.0
    for l in range(n_layers):
        e = rel_err(dec.layer_hidden(l), ref["layers"][l])
        worst = max(worst, e)
        assert e <= TOL, f"layer {l}: {e}"
    if n_layers == s.n_layers:
        assert rel_err(out, ref["final"]) <= TOL
    return worst, routes, out


def free_running_mismatches(s, model, step, routes, step_index=0, n_layers=None):
    """Free-running oracle vs GPU.  Tokens of a decoder step do not interact, so a token is followed until its
    routing first differs (from then on the two sides legitimately compute different things for it).  Up to that
    point the GPU's router logits of the token differ from the oracle's by rounding noise only, which is measured
    here; a differing selection is accepted only as a near tie within that noise: every expert chosen by one side
    alone is within 4 x max|logit_gpu - logit_oracle| (of this token, this layer) of every expert chosen by the
    other side alone, and that noise itself is small against the logits.  Returns the number of differing sets."""
    import oracle
    n_layers = s.n_layers if n_layers is None else n_layers
    x = synth.hidden_f32(s, model.seed, step_index, step.batch)
    oshape = oracle.shape_of(s)
    n_diff = 0
    diverged = np.zeros(step.batch, bool)
    for l in range(n_layers):
        w = synth.layer_weights_f32(s, model.seed, l)
        kp, vp = synth.kv_pool_f32(s, model.seed, l, model.n_pool_pages)
        ids, dbg = oracle.layer(oshape, x, w, kp, vp, step.kv_len, step.page_indptr, step.page_ids, debug=True)
        for b in range(step.batch):
            if diverged[b]:
                continue
            lg = dbg["router_logits"][b].astype(np.float64)
            noise = float(np.abs(routes[l]["logits"][b].astype(np.float64) - lg).max())
            assert noise <= 2e-2 * float(np.sqrt(np.mean(lg ** 2))), f"layer {l} token {b}: router logits off by {noise}"
            a, g = set(ids[b].tolist()), set(routes[l]["ids"][b].tolist())
            if a != g:
                n_diff += 1
                diverged[b] = True
                only_a, only_g = sorted(a - g), sorted(g - a)
                gap = max(abs(float(lg[i]) - float(lg[j])) for i in only_a for j in only_g)
                assert gap <= 4 * noise, (f"layer {l} token {b}: routing differs beyond a near tie "
                                          f"(gap {gap:.3e}, measured logit noise {noise:.3e})")
    return n_diff


# ---------------------------------------------------------------- tiny MoE decoder
@pytest.fixture(scope="module")
def tiny_moe_model():
    return GpuModel(synth.TINY_MOE, seed=21, n_pool_pages=96)


@pytest.mark.parametrize("batch,tile_m", [(1, 16), (3, 16), (5, 2), (7, 1), (16, 4)])
def test_tiny_moe_matches_oracle(tiny_moe_model, batch, tile_m):
    etc = _etc()
    s, m = synth.TINY_MOE, tiny_moe_model
    m.reset_pools()
    rng = np.random.default_rng(100 + batch)
    step = fixed_step(s, batch, rng.integers(0, 80, size=batch), m.n_pool_pages, seed=batch)
    dec = etc.Decoder(s, kv_chunk_tokens=32, sampled_batches=[batch], max_kv_len=129, moe_tile_m=tile_m,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN | etc.DEBUG_ROUTING, spin_budget=SPIN)
    m.bind(dec)
    dec.bind_step(step)
    worst, routes, _ = check_moe_step(dec, m, s, step, tile_m)
    m.reset_pools()
    free_running_mismatches(s, m, step, routes)
    print(f"tiny-moe B={batch} tile_m={tile_m}: worst per-layer max|err|/rms = {worst:.3e}")
    dec.close()


@pytest.mark.parametrize("kind", [0, 1])          # static queues; ready queue with run-time armed expert events
def test_tiny_moe_forced_routing_and_skewed_load(tiny_moe_model, kind):
    """etc_force_routing: every token to the same two experts (one long expert range spanning several row
    tiles, fourteen empty experts), then a token that names one expert twice."""
    etc = _etc()
    s, m = synth.TINY_MOE, tiny_moe_model
    B, tile_m = 6, 4
    m.reset_pools()
    step = fixed_step(s, B, [5, 17, 0, 33, 64, 9], m.n_pool_pages, seed=4)
    dec = etc.Decoder(s, kv_chunk_tokens=32, sampled_batches=[8], max_kv_len=129, moe_tile_m=tile_m, kind=kind,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN | etc.DEBUG_ROUTING, spin_budget=SPIN)
    m.bind(dec)
    dec.bind_step(step)
    forced = [np.tile(np.array([[11, 3]], np.int32), (B, 1)), np.tile(np.array([[0, 15]], np.int32), (B, 1))]
    forced[1][2] = [7, 7]
    for l in range(s.n_layers):
        dec.force_routing(l, forced[l])
    check_moe_step(dec, m, s, step, tile_m, forced=forced)
    # forced routing weights: the last layer's output is affine in them (x_mid + sum_k w_k y_k), so the output for
    # the mean of two weight vectors is the mean of the two outputs; and forcing the weights the device computed
    # itself changes nothing, bit for bit
    last = s.n_layers - 1
    w_dev = dec.routing_debug(_b().DBG_TOPK_W, last, (B, s.top_k), np.float32).copy()
    base = dec.layer_hidden(last).copy()
    outs = []
    rng = np.random.default_rng(3)
    wa, wb = rng.random((B, s.top_k), dtype=np.float32), rng.random((B, s.top_k), dtype=np.float32)
    for wts in (w_dev, wa, wb, (0.5 * (wa.astype(np.float64) + wb)).astype(np.float32)):
        dec.force_routing(last, forced[last], wts)
        m.reset_pools()
        dec.bind_step(step)
        _launch(dec, m, step)
        np.testing.assert_array_equal(dec.routing_debug(_b().DBG_TOPK_W, last, (B, s.top_k), np.float32), wts)
        outs.append(dec.layer_hidden(last).copy())
    np.testing.assert_array_equal(outs[0], base)
    mean = 0.5 * (outs[1].astype(np.float64) + outs[2])
    assert np.abs(outs[3] - mean).max() <= 1e-5 * np.sqrt(np.mean(mean ** 2)) + 1e-6
    assert np.abs(outs[1] - outs[2]).max() > 1e-3           # the weights do reach the combine
    # removing the override restores the device top-k
    for l in range(s.n_layers):
        dec.force_routing(l, None)
    m.reset_pools()
    dec.bind_step(step)              # re-arms the execution counters
    check_moe_step(dec, m, s, step, tile_m)
    dec.close()


def test_tiny_moe_schedulers_and_kernel_by_kernel_agree_bitwise(tiny_moe_model):
    etc = _etc()
    s, m = synth.TINY_MOE, tiny_moe_model
    step = fixed_step(s, 4, [40, 3, 77, 12], m.n_pool_pages, seed=2)
    outs = []
    for kind in (etc.SCHED_STATIC, etc.SCHED_DYNAMIC, etc.SCHED_UNFUSED):
        dec = etc.Decoder(s, kv_chunk_tokens=32, sampled_batches=[1, 4], max_kv_len=129, kind=kind, moe_tile_m=2,
                          debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_ROUTING, spin_budget=SPIN)
        m.bind(dec)
        dec.bind_step(step)
        for launches in (1, 2):                     # the second launch runs on the re-armed events
            m.reset_pools()
            outs.append(_launch(dec, m, step))
            assert (dec.error_word() == 0).all(), dec.error_word()
            assert (dec.event_counters() == 0).all()
            want = expected_exec_counts(dec, s, 32, 129, 2, launches)
            np.testing.assert_array_equal(dec.exec_counts(), want)
            if kind == etc.SCHED_DYNAMIC:
                print(f"dynamic: {int((want == 0).sum())} tasks of surplus row-tile slots were never released")
        if kind != etc.SCHED_UNFUSED:               # one launch per operator stage, also from a context built for the
            m.reset_pools()                         # ready queue (no events there: every slot task runs)
            outs.append(_launch(dec, m, step, kbk=True))
            m.reset_pools()
            outs.append(_launch(dec, m, step))      # and the scheduler's own state is untouched by it
            assert (dec.error_word() == 0).all() and (dec.event_counters() == 0).all()
        dec.close()
    for o in outs[1:]:
        np.testing.assert_array_equal(o, outs[0])


@pytest.mark.parametrize("kind", [0, 1])
def test_tiny_moe_smaller_batch_reuses_the_sampled_queue(tiny_moe_model, kind):
    """A batch below the sampled size runs on the larger queue: surplus router, row-tile and combine
    slots are no-ops that still notify (Sec. 3.1; under the dynamic scheduler the surplus row-tile slots are
    never released instead), and nothing is re-created between the steps."""
    etc = _etc()
    s, m = synth.TINY_MOE, tiny_moe_model
    dec = etc.Decoder(s, kv_chunk_tokens=32, sampled_batches=[8], max_kv_len=129, moe_tile_m=2, kind=kind,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN | etc.DEBUG_ROUTING, spin_budget=SPIN)
    m.bind(dec)
    for i, B in enumerate((8, 3, 1, 6)):
        rng = np.random.default_rng(B)
        step = fixed_step(s, B, rng.integers(0, 100, size=B), m.n_pool_pages, seed=50 + i)
        m.reset_pools()
        dec.bind_step(step)
        check_moe_step(dec, m, s, step, 2, step_index=i)
    dec.close()
