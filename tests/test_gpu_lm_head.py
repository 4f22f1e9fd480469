"""GPU parity of a whole decode iteration (paper Sec. 4.2: token in, all layers, sampling, token out): embedding
look-up, final RMSNorm, vocabulary projection and greedy token as tasks of the same event-gated megakernel,
against the CPU oracle, through the C ABI.

Floating point: logits within 2e-2 * RMS(oracle logits).  The token is an integer decided by floating point, so
both sides decide in the same precision: the GPU's token must be the arg-max (ties: lower id) of the GPU's own
fp32 logits, bit for bit; and it must equal the oracle's token whenever the oracle's two best logits are further
apart than twice the largest logit error measured on that row."""
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


def _lm(shape, seed):
    from synth import gpu as sgpu
    return sgpu.lm_weights_gpu(shape, seed)


def _check_invariants(dec):
    assert (dec.error_word() == 0).all(), dec.error_word()
    assert (dec.event_counters() == 0).all()
    assert (dec.exec_counts() == 1).all()


def _check_tokens(tok, logits, ref_logits, ref_tok):
    np.testing.assert_array_equal(tok, np.argmax(logits, axis=1).astype(np.int32))      # first maximum = lower id
    assert rel_err(logits, ref_logits) <= TOL
    for b in range(len(tok)):
        top2 = np.sort(ref_logits[b].astype(np.float64))[-2:]
        if top2[1] - top2[0] > 2.0 * float(np.abs(logits[b].astype(np.float64) - ref_logits[b]).max()):
            assert tok[b] == ref_tok[b], f"sequence {b}"


@pytest.fixture(scope="module")
def lm_model():
    m = GpuModel(synth.TINY_LM, seed=41, n_pool_pages=160)
    m.lm = _lm(synth.TINY_LM, 41)
    return m


def _decoder(etc, s, model, kind=0, sampled=(4,), chunk=32):
    dec = etc.Decoder(s, kv_chunk_tokens=chunk, sampled_batches=list(sampled), max_kv_len=129, kind=kind,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN, spin_budget=SPIN)
    model.bind(dec)
    dec.bind_lm_head(model.lm["embed"], model.lm["gf"], model.lm["wlm"])
    return dec


def test_tiny_iteration_from_hidden_states_matches_oracle_and_all_schedulers_agree(lm_model):
    import torch
    import oracle
    etc = _etc()
    s = synth.TINY_LM
    step = fixed_step(s, 3, [100, 7, 64], lm_model.n_pool_pages, seed=4)
    x = lm_model.hidden(0, 3)
    got = []
    for kind, kbk in ((0, False), (0, True), (1, False), (2, False)):
        lm_model.reset_pools()
        dec = _decoder(etc, s, lm_model, kind)
        tok = torch.full((3,), -1, dtype=torch.int32, device="cuda")
        logits = torch.full((3, s.vocab), float("nan"), device="cuda")
        hid = torch.empty_like(x)
        dec.bind_step(step)
        dec.launch_tokens(tok, hidden_in=x, logits_out=logits, hidden_out=hid, kernel_by_kernel=kbk)
        torch.cuda.synchronize()
        if not kbk:
            _check_invariants(dec)
        got.append((tok.cpu().numpy(), logits.cpu().numpy(), bf16_to_f32_np(hid)))
        # a model with a vocabulary is not launched without its token buffers
        with pytest.raises(etc.EtcError):
            dec.launch(x, hid)
        dec.close()
    for g in got[1:]:
        for a, b in zip(g, got[0]):
            np.testing.assert_array_equal(a, b)
    lm_model.reset_pools()
    ref = oracle_step(s, lm_model.seed, lm_model.n_pool_pages, step, 0)
    w = synth.lm_weights_f32(s, lm_model.seed)
    ref_logits, ref_tok = oracle.lm_head(oracle.shape_of(s), ref["final"], w["gf"], w["wlm"])
    tok, logits, hid = got[0]
    assert rel_err(hid, ref["final"]) <= TOL
    _check_tokens(tok, logits, ref_logits, ref_tok)


def test_token_input_reads_the_embedding_row_and_a_bad_id_is_an_error(lm_model):
    import torch
    etc = _etc()
    s = synth.TINY_LM
    lm_model.reset_pools()
    step = fixed_step(s, 2, [20, 33], lm_model.n_pool_pages, seed=5)
    dec = _decoder(etc, s, lm_model, sampled=(2,))
    ids = torch.tensor([s.vocab - 1, 17], dtype=torch.int32, device="cuda")
    outs = []
    for use_tokens in (True, False):
        lm_model.reset_pools()
        tok = torch.full((2,), -1, dtype=torch.int32, device="cuda")
        logits = torch.empty((2, s.vocab), device="cuda")
        dec.bind_step(step)
        if use_tokens:
            dec.launch_tokens(tok, token_in=ids, logits_out=logits)
        else:
            dec.launch_tokens(tok, hidden_in=lm_model.lm["embed"][ids.long()].contiguous(), logits_out=logits)
        torch.cuda.synchronize()
        _check_invariants(dec)
        outs.append((tok.cpu().numpy(), logits.cpu().numpy()))
    np.testing.assert_array_equal(outs[0][0], outs[1][0])
    np.testing.assert_array_equal(outs[0][1], outs[1][1])
    # both inputs, or neither, are refused on the host
    tok = torch.zeros(2, dtype=torch.int32, device="cuda")
    with pytest.raises(etc.EtcError):
        dec.launch_tokens(tok, token_in=ids, hidden_in=lm_model.hidden(0, 2))
    with pytest.raises(etc.EtcError):
        dec.launch_tokens(tok)
    # an id outside the table: error word, row 0 is read instead (the kernel drains normally), the context is dead
    bad = torch.tensor([3, s.vocab], dtype=torch.int32, device="cuda")
    dec.launch_tokens(tok, token_in=bad)
    torch.cuda.synchronize()
    assert dec.error_word()[0] == 4                 # ERR_BAD_TABLE
    with pytest.raises(etc.EtcError):
        dec.launch_tokens(tok, token_in=ids)
    dec.close()


def test_equal_logits_give_the_lower_id(lm_model):
    """Rows of the projection that are copies of each other give bitwise equal logits (same operations in the same
    order), across tiles and across tasks: the token is the lowest id among the maxima."""
    import torch
    etc = _etc()
    s = synth.TINY_LM
    lm_model.reset_pools()
    step = fixed_step(s, 2, [9, 40], lm_model.n_pool_pages, seed=6)
    x = lm_model.hidden(3, 2)
    w = lm_model.lm["wlm"]
    for first_max in (0, 5, 700, s.vocab - 1):
        # one run with the row itself everywhere tells the sign of its logit per sequence; then the rows below
        # first_max get the opposite sign
        wl = w[3:4].repeat(s.vocab, 1).contiguous()
        dec = etc.Decoder(s, kv_chunk_tokens=32, sampled_batches=[2], max_kv_len=129, spin_budget=SPIN)
        lm_model.bind(dec)
        dec.bind_lm_head(None, lm_model.lm["gf"], wl)
        tok = torch.full((2,), -1, dtype=torch.int32, device="cuda")
        logits = torch.empty((2, s.vocab), device="cuda")
        dec.bind_step(step)
        dec.launch_tokens(tok, hidden_in=x, logits_out=logits)
        torch.cuda.synchronize()
        lg = logits.cpu().numpy()
        assert (lg == lg[:, :1]).all()
        np.testing.assert_array_equal(tok.cpu().numpy(), [0, 0])
        dec.close()
        if first_max == 0:
            continue
        wl2 = wl.clone()
        wl2[:first_max] = -wl2[:first_max]
        dec = etc.Decoder(s, kv_chunk_tokens=32, sampled_batches=[2], max_kv_len=129, spin_budget=SPIN)
        lm_model.reset_pools()
        lm_model.bind(dec)
        dec.bind_lm_head(None, lm_model.lm["gf"], wl2)
        dec.bind_step(step)
        dec.launch_tokens(tok, hidden_in=x, logits_out=logits)
        torch.cuda.synchronize()
        want = [first_max if lg[b, 0] > 0 else 0 for b in range(2)]
        np.testing.assert_array_equal(tok.cpu().numpy(), want)
        dec.close()
        lm_model.reset_pools()


def test_chained_iterations_without_a_host_round_trip(lm_model):
    """Five iterations queued back to back: each launch reads the token the previous one sampled, the host only
    binds the next step's shapes in between (no synchronisation) and waits once at the end.  The oracle follows
    the GPU's tokens (so that a near tie cannot fork the two chains) on its own KV pools."""
    import torch
    import oracle
    etc = _etc()
    s = synth.TINY_LM
    lm_model.reset_pools()
    dec = _decoder(etc, s, lm_model, sampled=(2,), chunk=16)
    N, B = 5, 2
    L0 = np.array([30, 13], np.int32)
    npg = [synth.pages_needed(int(l) + N, s.page) for l in L0]
    owned = np.random.default_rng(9).permutation(lm_model.n_pool_pages)[: sum(npg)].astype(np.int32)
    own = [owned[: npg[0]], owned[npg[0]:]]
    toks = torch.full((N + 1, B), -1, dtype=torch.int32, device="cuda")
    toks[0] = torch.tensor([11, 1000], dtype=torch.int32)
    logits = torch.empty((N, B, s.vocab), device="cuda")
    steps = []
    for t in range(N):
        kv = L0 + t
        cnt = [synth.pages_needed(int(l), s.page) for l in kv]
        indptr = np.concatenate([[0], np.cumsum(cnt)]).astype(np.int32)
        steps.append(synth.Step(B, kv.astype(np.int32), indptr,
                                np.concatenate([own[b][: cnt[b]] for b in range(B)]).astype(np.int32)))
        dec.bind_step(steps[-1])
        dec.launch_tokens(toks[t + 1], token_in=toks[t], logits_out=logits[t])
    torch.cuda.synchronize()
    assert (dec.error_word() == 0).all()
    assert (dec.event_counters() == 0).all()
    assert (dec.exec_counts() == 1).all()          # counted per bound step
    toks_h, logits_h = toks.cpu().numpy(), logits.cpu().numpy()
    w = synth.lm_weights_f32(s, lm_model.seed)
    pools = [list(synth.kv_pool_f32(s, lm_model.seed, l, lm_model.n_pool_pages)) for l in range(s.n_layers)]
    bf16 = lambda a: torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()      # noqa: E731
    for t in range(N):
        ref = oracle.decode_step(s, s.n_layers, oracle.embed(w["embed"], toks_h[t]),
                                 lambda l: synth.layer_weights_f32(s, lm_model.seed, l), lambda l: pools[l], steps[t])
        ref_logits, ref_tok = oracle.lm_head(oracle.shape_of(s), ref["final"], w["gf"], w["wlm"])
        _check_tokens(toks_h[t + 1], logits_h[t], ref_logits, ref_tok)
        for l in range(s.n_layers):
            for b in range(B):                           # the cache holds bf16
                kv = steps[t].kv_len
                pg, sl = int(own[b][kv[b] // s.page]), int(kv[b] % s.page)
                for pool in pools[l]:
                    pool[pg, sl] = bf16(pool[pg, sl])
    dec.close()


def test_tiny_moe_iteration_matches_oracle():
    """The MoE decoder's last combine prepares the operand of the vocabulary projection."""
    import torch
    import oracle
    from paper_2604_13327_amd import binding as b
    etc = _etc()
    s = synth.TINY_MOE_LM
    model = GpuModel(s, seed=43, n_pool_pages=160)
    lm = _lm(s, 43)
    step = fixed_step(s, 3, [50, 3, 77], model.n_pool_pages, seed=7)
    x = model.hidden(0, 3)
    got = []
    for kind in (0, 1):
        model.reset_pools()
        dec = etc.Decoder(s, kv_chunk_tokens=32, sampled_batches=[4], max_kv_len=129, kind=kind, moe_tile_m=4,
                          debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_ROUTING, spin_budget=SPIN)
        model.bind(dec)
        dec.bind_lm_head(lm["embed"], lm["gf"], lm["wlm"])
        tok = torch.full((3,), -1, dtype=torch.int32, device="cuda")
        logits = torch.empty((3, s.vocab), device="cuda")
        dec.bind_step(step)
        dec.launch_tokens(tok, hidden_in=x, logits_out=logits)
        torch.cuda.synchronize()
        assert (dec.error_word() == 0).all() and (dec.event_counters() == 0).all()
        routes = [dec.routing_debug(b.DBG_TOPK_IDS, l, (3, s.top_k), np.int32) for l in range(s.n_layers)]
        got.append((tok.cpu().numpy(), logits.cpu().numpy()))
        dec.close()
    np.testing.assert_array_equal(got[0][0], got[1][0])
    np.testing.assert_array_equal(got[0][1], got[1][1])
    model.reset_pools()
    ref = oracle_step(s, model.seed, model.n_pool_pages, step, 0, forced_topk_of=lambda l: routes[l], tile_m=4)
    w = synth.lm_weights_f32(s, model.seed)
    ref_logits, ref_tok = oracle.lm_head(oracle.shape_of(s, 4), ref["final"], w["gf"], w["wlm"])
    _check_tokens(got[0][0], got[0][1], ref_logits, ref_tok)


@pytest.mark.parametrize("batch", [17, 64])
def test_large_batches_take_the_chunked_projection(lm_model, batch):
    """Above 16 columns the vocabulary projection runs on the chunked path (several passes of row tiles per task)."""
    import torch
    import oracle
    etc = _etc()
    s = synth.TINY_LM
    lm_model.reset_pools()
    rng = np.random.default_rng(batch)
    kv = rng.integers(1, 20, size=batch).astype(np.int32)
    step = fixed_step(s, batch, kv, lm_model.n_pool_pages, seed=8)
    dec = _decoder(etc, s, lm_model, sampled=(batch,))
    x = lm_model.hidden(1, batch)
    tok = torch.full((batch,), -1, dtype=torch.int32, device="cuda")
    logits = torch.empty((batch, s.vocab), device="cuda")
    dec.bind_step(step)
    dec.launch_tokens(tok, hidden_in=x, logits_out=logits)
    torch.cuda.synchronize()
    _check_invariants(dec)
    ref = oracle_step(s, lm_model.seed, lm_model.n_pool_pages, step, 1)
    w = synth.lm_weights_f32(s, lm_model.seed)
    ref_logits, ref_tok = oracle.lm_head(oracle.shape_of(s), ref["final"], w["gf"], w["wlm"])
    _check_tokens(tok.cpu().numpy(), logits.cpu().numpy(), ref_logits, ref_tok)
    dec.close()


@pytest.mark.parametrize("batch", [1, 8])
def test_llama3_vocabulary_at_full_width(batch):
    """Hidden 4096 and the 128256-row vocabulary of Llama-3 (8016 row tiles over 256 queues: the last task is
    ragged), two layers deep so that the oracle finishes in seconds."""
    import dataclasses
    import torch
    import oracle
    etc = _etc()
    s = dataclasses.replace(synth.LLAMA3_8B, name="llama3-8b-2l-lm", n_layers=2, vocab=128256)
    model = GpuModel(s, seed=47, n_pool_pages=300)
    lm = _lm(s, 47)
    kv = np.random.default_rng(batch).integers(1, 500, size=batch).astype(np.int32)
    step = fixed_step(s, batch, kv, model.n_pool_pages, seed=3)
    dec = etc.Decoder(s, kv_chunk_tokens=128, sampled_batches=[batch], max_kv_len=513,
                      debug_flags=etc.DEBUG_EXEC_COUNT, spin_budget=SPIN)
    model.bind(dec)
    dec.bind_lm_head(lm["embed"], lm["gf"], lm["wlm"])
    ids = torch.from_numpy(np.random.default_rng(5).integers(0, s.vocab, size=batch).astype(np.int32)).cuda()
    tok = torch.full((batch,), -1, dtype=torch.int32, device="cuda")
    logits = torch.full((batch, s.vocab), float("nan"), device="cuda")
    dec.bind_step(step)
    dec.launch_tokens(tok, token_in=ids, logits_out=logits)
    torch.cuda.synchronize()
    _check_invariants(dec)
    w = synth.lm_weights_f32(s, model.seed)
    x0 = oracle.embed(w["embed"], ids.cpu().numpy())
    ref = oracle.decode_step(s, s.n_layers, x0, lambda l: synth.layer_weights_f32(s, model.seed, l),
                             lambda l: synth.kv_pool_f32(s, model.seed, l, model.n_pool_pages), step)
    ref_logits, ref_tok = oracle.lm_head(oracle.shape_of(s), ref["final"], w["gf"], w["wlm"])
    _check_tokens(tok.cpu().numpy(), logits.cpu().numpy(), ref_logits, ref_tok)
    dec.close()
