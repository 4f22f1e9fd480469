"""GPU parity tests: the HIP megakernel, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Floating point bar: max|err| <= 2e-2 * RMS(oracle output), per layer and final.
Integer work (task execution counts, event counters) is bit-exact."""
import numpy as np
import pytest

import synth
from harness import GpuModel, bf16_to_f32_np, fixed_step, oracle_step, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-2
SPIN = 400000      # polls before a device wait gives up: a scheduling bug shows as ETC_ETIMEOUT, not as a hang


def _etc():
    import paper_2604_13327_amd as etc
    return etc


def _run(dec, model, step, step_index=0, kbk=False):
    import torch
    x = model.hidden(step_index, step.batch)
    out = torch.empty_like(x)
    dec.bind_step(step)
    (dec.launch_kernel_by_kernel if kbk else dec.launch)(x, out)
    torch.cuda.synchronize()
    return bf16_to_f32_np(out)


def _check_invariants(dec):
    assert (dec.error_word() == 0).all(), dec.error_word()
    assert (dec.event_counters() == 0).all(), "an event counter did not drain to zero"
    assert (dec.exec_counts() == 1).all(), "a task did not run exactly once"


# ---------------------------------------------------------------- row-sum example (paper Sec. 2.2)
def _rowsum_graph(etc, kind):
    from paper_2604_13327_amd import binding as b
    g = etc.EventGraph(kind=kind, debug_flags=etc.DEBUG_EXEC_COUNT, spin_budget=SPIN)
    n = g.dim(sym=0, mul=1, add=0)
    ev = g.add_event([n])                                                     # E[i], i < n (symbolic)
    g.add_call(b.FN_ROWSUM_PARTIAL, [n, g.dim(add=4)], out_edges=[g.edge(ev, [(b.MAP_DIM, 0, 1)])])
    g.add_call(b.FN_ROWSUM_FINAL, [n], in_edges=[g.edge(ev, [(b.MAP_DIM, 0, 1)])])
    return g


KINDS = [0, 1, 2]                              # static, dynamic, unfused


@pytest.mark.parametrize("kind", KINDS)
def test_rowsum_graph_symbolic_n(kind):
    import torch
    etc = _etc()
    g = _rowsum_graph(etc, kind)
    rng = np.random.default_rng(0)
    for n in (1, 2, 37):                       # one template, three instantiations, no rebuild of the context
        A = rng.integers(-8, 9, size=(n * 32, 128)).astype(np.float32)
        dA = torch.from_numpy(A).cuda()
        dB = torch.full((n * 32, 4), float("nan"), device="cuda")
        dC = torch.full((n * 32,), float("nan"), device="cuda")
        for slot, t in enumerate((dA, dB, dC)):
            g.bind_buffer(slot, t)
        g.bind_shape([n])
        for rep in range(2):                   # second launch runs on the re-armed event tensor
            dC.fill_(float("nan"))
            g.launch()
            torch.cuda.synchronize()
            np.testing.assert_array_equal(dC.cpu().numpy(), A.astype(np.float64).sum(1))
            assert (g.event_counters() == 0).all()
        info = g.step_info()
        assert info.n_tasks == 5 * n and info.n_events == (n if kind != 2 else 2)
        assert (g.exec_counts() == 2).all()
    # undersized buffer is refused on the host
    g.bind_shape([64])
    with pytest.raises(etc.EtcError):
        g.launch()
    g.close()


# ---------------------------------------------------------------- config 1: tiny 2-layer decoder
@pytest.fixture(scope="module")
def tiny_model():
    return GpuModel(synth.TINY, seed=11, n_pool_pages=160)


@pytest.mark.parametrize("kind", KINDS)
def test_tiny_decoder_matches_oracle_per_layer(tiny_model, kind):
    etc = _etc()
    s = synth.TINY
    tiny_model.reset_pools()
    step = fixed_step(s, 1, [128], tiny_model.n_pool_pages, seed=3)
    dec = etc.Decoder(s, kv_chunk_tokens=32, sampled_batches=[1], max_kv_len=129, kind=kind,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN, spin_budget=SPIN)
    tiny_model.bind(dec)
    out = _run(dec, tiny_model, step)
    _check_invariants(dec)
    ref = oracle_step(s, tiny_model.seed, tiny_model.n_pool_pages, step, 0)
    for l in range(s.n_layers):
        assert rel_err(dec.layer_hidden(l), ref["layers"][l]) <= TOL, f"layer {l}"
    assert rel_err(out, ref["final"]) <= TOL
    dec.close()


def test_tiny_kv_append_lands_in_the_right_slot(tiny_model):
    import torch
    etc = _etc()
    s = synth.TINY
    tiny_model.reset_pools()
    before_k = tiny_model.kpool.clone()
    step = fixed_step(s, 1, [37], tiny_model.n_pool_pages, seed=5)
    dec = etc.Decoder(s, kv_chunk_tokens=16, sampled_batches=[1], max_kv_len=129)
    tiny_model.bind(dec)
    _run(dec, tiny_model, step)
    changed = (tiny_model.kpool != before_k).any(dim=-1).any(dim=-1)          # [layer, page, slot]
    page, slot = int(step.page_ids[37 // s.page]), 37 % s.page
    exp = torch.zeros_like(changed)
    exp[:, page, slot] = True
    assert torch.equal(changed, exp)
    # appended K row equals the oracle's rotated key (bf16 rounding only)
    import oracle
    w = synth.layer_weights_f32(s, tiny_model.seed, 0)
    kp, vp = synth.kv_pool_f32(s, tiny_model.seed, 0, tiny_model.n_pool_pages)
    x = synth.hidden_f32(s, tiny_model.seed, 0, 1)
    _, dbg = oracle.layer(oracle.shape_of(s), x.copy(), w, kp, vp, step.kv_len, step.page_indptr, step.page_ids, debug=True)
    got = bf16_to_f32_np(tiny_model.kpool[0, page, slot]).ravel()
    assert rel_err(got, dbg["k_rot"][0]) <= TOL
    gotv = bf16_to_f32_np(tiny_model.vpool[0, page, slot]).ravel()
    assert rel_err(gotv, dbg["v_new"][0]) <= TOL
    dec.close()


def test_tiny_three_steps_in_a_row_read_back_their_own_rows(tiny_model):
    """Chained decode steps on one context, nothing reset in between: kv_len grows by one per step, so steps 2
    and 3 read the bf16 rows the earlier steps appended to the cache (step 3 also opens a new page).  The oracle
    runs the same three steps on its own pools, where it appended its own rows (rounded to the cache's bf16
    here, in the test: the storage format, not arithmetic).  Binding a step between launches neither
    synchronises nor re-creates anything."""
    import torch
    import oracle
    etc = _etc()
    s = synth.TINY
    tiny_model.reset_pools()
    dec = etc.Decoder(s, kv_chunk_tokens=16, sampled_batches=[2], max_kv_len=129,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN, spin_budget=SPIN)
    tiny_model.bind(dec)
    L0 = np.array([30, 14], np.int32)                     # 14 -> 15 -> 16: the third step starts a new page
    npg = [synth.pages_needed(int(l) + 2, s.page) for l in L0]
    rng = np.random.default_rng(8)
    owned = rng.permutation(tiny_model.n_pool_pages)[: sum(npg)].astype(np.int32)
    own = [owned[: npg[0]], owned[npg[0]:]]
    pools = [list(synth.kv_pool_f32(s, tiny_model.seed, l, tiny_model.n_pool_pages)) for l in range(s.n_layers)]
    bf16 = lambda a: torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()      # noqa: E731
    for t in range(3):
        kv = L0 + t
        cnt = [synth.pages_needed(int(l), s.page) for l in kv]
        indptr = np.concatenate([[0], np.cumsum(cnt)]).astype(np.int32)
        step = synth.Step(2, kv.astype(np.int32), indptr, np.concatenate([own[b][: cnt[b]] for b in range(2)]).astype(np.int32))
        out = _run(dec, tiny_model, step, step_index=t)
        _check_invariants(dec)
        ref = oracle.decode_step(s, s.n_layers, synth.hidden_f32(s, tiny_model.seed, t, 2), lambda l: synth.layer_weights_f32(s, tiny_model.seed, l),
                                 lambda l: pools[l], step)
        for l in range(s.n_layers):
            assert rel_err(dec.layer_hidden(l), ref["layers"][l]) <= TOL, f"step {t} layer {l}"
            for b in range(2):                            # the cache holds bf16: round the rows the oracle appended
                pg, sl = int(own[b][kv[b] // s.page]), int(kv[b] % s.page)
                for pool in pools[l]:
                    pool[pg, sl] = bf16(pool[pg, sl])
        assert rel_err(out, ref["final"]) <= TOL, f"step {t}"
    dec.close()


def test_tiny_all_schedulers_and_kernel_by_kernel_agree_bitwise(tiny_model):
    """Identical task bodies, different scheduling: the results must be identical (paper Sec. 4.5)."""
    etc = _etc()
    s = synth.TINY
    step = fixed_step(s, 3, [100, 7, 64], tiny_model.n_pool_pages, seed=9)
    outs = []
    for kind in (0, 1, 2):                 # static, dynamic, unfused
        tiny_model.reset_pools()
        dec = etc.Decoder(s, kv_chunk_tokens=32, sampled_batches=[1, 4], max_kv_len=129, kind=kind,
                          debug_flags=etc.DEBUG_EXEC_COUNT, spin_budget=SPIN)
        tiny_model.bind(dec)
        outs.append(_run(dec, tiny_model, step))
        _check_invariants(dec)
        assert dec.step_info().sampled_batch == 4          # B = 3 runs on the queues sampled for B = 4
        if kind == 0:
            tiny_model.reset_pools()
            outs.append(_run(dec, tiny_model, step, kbk=True))
        dec.close()
    for o in outs[1:]:
        np.testing.assert_array_equal(o, outs[0])
    tiny_model.reset_pools()
    ref = oracle_step(s, tiny_model.seed, tiny_model.n_pool_pages, step, 0)
    assert rel_err(outs[0], ref["final"]) <= TOL


def test_tiny_shape_dynamism_without_recreate(tiny_model):
    """One context, steps with different batch sizes and ragged lengths (Sec. 2.3), launched repeatedly."""
    etc = _etc()
    s = synth.TINY
    dec = etc.Decoder(s, kv_chunk_tokens=16, sampled_batches=[1, 4, 16], max_kv_len=129,
                      debug_flags=etc.DEBUG_EXEC_COUNT, spin_budget=SPIN)
    tiny_model.bind(dec)
    rng = np.random.default_rng(21)
    for i in range(6):
        tiny_model.reset_pools()
        step = synth.draw_step(rng, s, [1, 2, 4, 9, 16], 0, 128, tiny_model.n_pool_pages)
        out = _run(dec, tiny_model, step, step_index=i)
        _check_invariants(dec)
        tiny_model.reset_pools()
        ref = oracle_step(s, tiny_model.seed, tiny_model.n_pool_pages, step, i)
        assert rel_err(out, ref["final"]) <= TOL, f"step {i} batch {step.batch}"
    dec.close()


def test_edge_cases_and_error_paths(tiny_model):
    etc = _etc()
    s = synth.TINY
    dec = etc.Decoder(s, kv_chunk_tokens=32, sampled_batches=[2], max_kv_len=129)
    tiny_model.bind(dec)
    tiny_model.reset_pools()
    # empty cache (kv_len 0: attention over the new token only) and the maximum length
    step = fixed_step(s, 2, [0, 128], tiny_model.n_pool_pages, seed=1)
    out = _run(dec, tiny_model, step)
    tiny_model.reset_pools()
    ref = oracle_step(s, tiny_model.seed, tiny_model.n_pool_pages, step, 0)
    assert rel_err(out, ref["final"]) <= TOL
    # invalid binds are refused on the host, never reach the device
    bad = fixed_step(s, 2, [0, 128], tiny_model.n_pool_pages, seed=1)
    bad.page_ids = bad.page_ids.copy()
    bad.page_ids[0] = tiny_model.n_pool_pages            # outside the pool
    with pytest.raises(etc.EtcError):
        dec.bind_step(bad)
    with pytest.raises(etc.EtcError):
        dec.bind_step(fixed_step(s, 1, [129], tiny_model.n_pool_pages, seed=1))   # longer than max_kv_len
    with pytest.raises(etc.EtcError):
        dec.bind_step(fixed_step(s, 3, [1, 1, 1], tiny_model.n_pool_pages, seed=1))  # batch above max_batch
    dec.close()


def test_watchdog_turns_a_stuck_wait_into_an_error():
    """A wait that can never be satisfied must drain with ETC_ETIMEOUT instead of hanging.  Forced from
    the host: with a single queue the consumer launch is listed ahead of its producers, so the head task
    waits on an event that cannot fire before it gives up; the spin budget is tiny, so it gives up at once."""
    import torch
    etc = _etc()
    from paper_2604_13327_amd import binding as b
    g = etc.EventGraph(kind=0, spin_budget=2000, n_queues=1)
    n = g.dim(sym=0, mul=1, add=0)
    ev = g.add_event([g.dim(add=1)])
    g.add_call(b.FN_ROWSUM_FINAL, [n], in_edges=[g.edge(ev, [(b.MAP_CONST, 0, 0)])])
    g.add_call(b.FN_ROWSUM_PARTIAL, [n, g.dim(add=4)], out_edges=[g.edge(ev, [(b.MAP_CONST, 0, 0)])])
    A = torch.zeros(32, 128, device="cuda")
    Bm = torch.zeros(32, 4, device="cuda")
    Cm = torch.zeros(32, device="cuda")
    for slot, t in enumerate((A, Bm, Cm)):
        g.bind_buffer(slot, t)
    g.bind_shape([1])
    g.launch()
    torch.cuda.synchronize()                   # returns: the kernel drained
    with pytest.raises(etc.EtcError) as ei:
        g.event_counters()
    assert ei.value.status == -5
    assert g.error_word()[0] == 1              # the error word itself stays readable: a wait ran out of its budget
    # the context is dead now: a launch is refused on the host instead of running on inconsistent counters
    with pytest.raises(etc.EtcError) as ei:
        g.launch()
    assert ei.value.status == -3
    # binding a shape rebuilds all launch state and revives a generic-graph context; the same stuck graph times
    # out again, and this time the launch after it is the first call to notice (through the host-side mirror)
    g.bind_shape([1])
    g.launch()
    torch.cuda.synchronize()
    with pytest.raises(etc.EtcError) as ei:
        g.launch()
    assert ei.value.status == -5
    with pytest.raises(etc.EtcError) as ei:
        g.launch()
    assert ei.value.status == -3
    g.close()


def test_dynamic_scheduler_is_independent_of_listing_order_and_times_out_on_a_cycle():
    """The graph of the watchdog test (consumer launch listed ahead of its producers, one workgroup) is no
    problem for the ready queue: tasks run when they are pushed, whatever the listing order.  Two launches
    that wait for each other are never pushed; the idle popper then gives up after its (tiny) spin budget and
    the launch ends with ETC_ETIMEOUT instead of hanging."""
    import torch
    etc = _etc()
    from paper_2604_13327_amd import binding as b
    rng = np.random.default_rng(5)
    A = rng.integers(-8, 9, size=(64, 128)).astype(np.float32)
    dA = torch.from_numpy(A).cuda()
    dB = torch.full((64, 4), float("nan"), device="cuda")
    dC = torch.full((64,), float("nan"), device="cuda")
    g = etc.EventGraph(kind=1, spin_budget=SPIN, n_queues=1, debug_flags=etc.DEBUG_EXEC_COUNT)
    n = g.dim(sym=0, mul=1, add=0)
    ev = g.add_event([n])
    g.add_call(b.FN_ROWSUM_FINAL, [n], in_edges=[g.edge(ev, [(b.MAP_DIM, 0, 1)])])
    g.add_call(b.FN_ROWSUM_PARTIAL, [n, g.dim(add=4)], out_edges=[g.edge(ev, [(b.MAP_DIM, 0, 1)])])
    for slot, t in enumerate((dA, dB, dC)):
        g.bind_buffer(slot, t)
    g.bind_shape([2])
    for rep in range(2):
        dC.fill_(float("nan"))
        g.launch()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(dC.cpu().numpy(), A.astype(np.float64).sum(1))
        assert (g.event_counters() == 0).all() and (g.exec_counts() == rep + 1).all()
    g.close()

    g = etc.EventGraph(kind=1, spin_budget=2000, n_queues=2)
    n = g.dim(sym=0, mul=1, add=0)
    e1, e2 = g.add_event([g.dim(add=1)]), g.add_event([g.dim(add=1)])
    g.add_call(b.FN_ROWSUM_FINAL, [n], in_edges=[g.edge(e1, [(b.MAP_CONST, 0, 0)])],
               out_edges=[g.edge(e2, [(b.MAP_CONST, 0, 0)])])
    g.add_call(b.FN_ROWSUM_PARTIAL, [n, g.dim(add=4)], in_edges=[g.edge(e2, [(b.MAP_CONST, 0, 0)])],
               out_edges=[g.edge(e1, [(b.MAP_CONST, 0, 0)])])
    for slot, t in enumerate((dA, dB, dC)):
        g.bind_buffer(slot, t)
    g.bind_shape([1])
    g.launch()
    torch.cuda.synchronize()                   # returns: the poppers gave up
    with pytest.raises(etc.EtcError) as ei:
        g.event_counters()
    assert ei.value.status == -5
    g.close()


@pytest.mark.parametrize("kind", KINDS)
def test_generic_graph_with_data_dependent_edges(kind):
    """The two data-dependent mechanisms of Sec. 2.4 on a generic graph.  n row blocks are routed to m groups by
    a run-time table; partial-sum task (i, j) notifies the event of group route[i] (INDIRECT update; the count of
    an event is known at run time only); the final-sum grid is laid out group by group, and event g releases
    exactly the tasks [indptr[g], indptr[g+1]) (INDPTR trigger), task t summing row block perm[t].  The grid is
    sized for more row blocks than are routed, so it has surplus tasks: no-ops under the static rule (one coarse
    event), never released by the ready queue.  Whatever the routing, C is the plain row sum of A."""
    import torch
    etc = _etc()
    from paper_2604_13327_amd import binding as b
    n_max, m = 24, 5
    g = etc.EventGraph(kind=kind, debug_flags=etc.DEBUG_EXEC_COUNT, spin_budget=SPIN)
    n = g.dim(sym=0, mul=1, add=0)
    ev = g.add_event([g.dim(add=m)])
    g.add_call(b.FN_ROWSUM_PARTIAL, [n, g.dim(add=4)], out_edges=[g.edge(ev, [(b.MAP_INDIRECT, 0, 1)])])
    g.add_call(b.FN_ROWSUM_FINAL_PERM, [g.dim(add=n_max)], in_edges=[g.edge(ev, [(b.MAP_INDPTR, 0, 1)])])
    rng = np.random.default_rng(11)
    for rep, n_rows in enumerate((24, 7, 1, 19)):          # one template, several routings, no rebuild
        A = rng.integers(-8, 9, size=(n_rows * 32, 128)).astype(np.float32)
        route = rng.integers(0, m, size=n_rows).astype(np.int32)
        if rep == 1:
            route[:] = 3                                   # everything to one group, four groups empty
        perm = np.argsort(route, kind="stable").astype(np.int32)
        per_group = np.bincount(route, minlength=m)
        indptr = np.concatenate([[0], np.cumsum(per_group)]).astype(np.int32)
        count = (4 * per_group).astype(np.int32)           # four partial sums per row block notify its group's event
        perm_full = np.concatenate([perm, np.zeros(n_max - n_rows, np.int32)])
        dA = torch.from_numpy(A).cuda()
        dB = torch.full((n_rows * 32, 4), float("nan"), device="cuda")
        dC = torch.full((n_max * 32,), float("nan"), device="cuda")
        tabs = [torch.from_numpy(x).cuda() for x in (route, indptr, count, perm_full)]
        for slot, t in enumerate([dA, dB, dC] + tabs):
            g.bind_buffer(slot, t)
        g.bind_shape([n_rows])
        for launches in (1, 2):                            # the second launch runs on re-armed events
            dC.fill_(float("nan"))
            g.launch()
            torch.cuda.synchronize()
            got = dC.cpu().numpy()
            np.testing.assert_array_equal(got[: n_rows * 32], A.astype(np.float64).sum(1))
            assert np.isnan(got[n_rows * 32:]).all()       # surplus tasks wrote nothing
            assert (g.event_counters() == 0).all()
            want = np.full(4 * n_rows + n_max, launches, np.int32)
            if kind == 1:
                want[4 * n_rows + n_rows:] = 0             # the ready queue never released the surplus tasks
            np.testing.assert_array_equal(g.exec_counts(), want)
    # a table entry outside the event tensor ends the launch with an error instead of a wild access
    if kind == 1:
        bad = torch.from_numpy(np.full(n_rows, m + 3, np.int32)).cuda()
        g.bind_buffer(3, bad)
        g.bind_shape([n_rows])
        g.launch()
        torch.cuda.synchronize()
        with pytest.raises(etc.EtcError) as ei:
            g.event_counters()
        assert ei.value.status == -5
    g.close()


@pytest.mark.parametrize("batch", [17, 40, 64])
def test_tiny_large_batches_take_the_chunked_path(batch):
    """Batches above 16 columns: operand walked in double-buffered LDS chunks, 2 and 4 MFMA column blocks,
    several row tiles per task; ragged lengths including an empty cache."""
    etc = _etc()
    s = synth.TINY
    n_pool = batch * synth.pages_needed(128, s.page) + 8
    model = GpuModel(s, seed=13, n_pool_pages=n_pool)
    rng = np.random.default_rng(batch)
    kv = rng.integers(0, 129, size=batch)
    kv[0], kv[-1] = 0, 128
    step = fixed_step(s, batch, kv, n_pool, seed=batch)
    dec = etc.Decoder(s, kv_chunk_tokens=32, sampled_batches=[batch], max_kv_len=129,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN, spin_budget=SPIN)
    model.bind(dec)
    out = _run(dec, model, step)
    _check_invariants(dec)
    ref = oracle_step(s, model.seed, n_pool, step, 0)
    for l in range(s.n_layers):
        assert rel_err(dec.layer_hidden(l), ref["layers"][l]) <= TOL, f"layer {l}"
    assert rel_err(out, ref["final"]) <= TOL
    model.reset_pools()
    out2 = _run(dec, model, step, kbk=True)
    np.testing.assert_array_equal(out2, out)
    dec.close()
    # the K-slice stages under one coarse event per stage, and pushed by the dynamic scheduler
    for kind in (etc.SCHED_UNFUSED, etc.SCHED_DYNAMIC):
        dec = etc.Decoder(s, kv_chunk_tokens=32, sampled_batches=[batch], max_kv_len=129, kind=kind,
                          debug_flags=etc.DEBUG_EXEC_COUNT, spin_budget=SPIN)
        model.bind(dec)
        model.reset_pools()
        out3 = _run(dec, model, step)
        _check_invariants(dec)
        np.testing.assert_array_equal(out3, out)
        dec.close()


# ---------------------------------------------------------------- long attention chunks at head dim 128
@pytest.mark.parametrize("kind", [0, 1])
@pytest.mark.parametrize("grp,qk_norm", [(8, False), (8, True), (4, False)])
def test_long_chunks_head_dim_128(grp, qk_norm, kind):
    """Chunks longer than one batch of keys at head dim 128: 8 query heads per KV head run on the matrix cores
    (32 keys per wavefront step), 4 on the vector path.  Lengths sit on and around the 32-key steps, the 16-token pages
    and the chunk boundary: sequences of one chunk (written directly) and of two and three chunks (partial results,
    merged by the chunk task that arrives last), one key, and a last chunk that holds the step's own token alone."""
    etc = _etc()
    s = synth.ModelShape(f"d128-g{grp}", 2, 256, grp, 1, 128, 512, qk_norm=qk_norm)
    lens = [0, 31, 32, 33, 255, 256, 257, 511, 512, 700, 767]        # kv_len: keys before this step's token
    model = GpuModel(s, seed=21, n_pool_pages=len(lens) * 49 + 8)
    step = fixed_step(s, len(lens), lens, model.n_pool_pages, seed=9)
    dec = etc.Decoder(s, kv_chunk_tokens=256, sampled_batches=[len(lens)], max_kv_len=769, kind=kind,
                      debug_flags=etc.DEBUG_EXEC_COUNT | etc.DEBUG_LAYER_HIDDEN, spin_budget=SPIN)
    model.bind(dec)
    out = _run(dec, model, step)
    _check_invariants(dec)
    ref = oracle_step(s, model.seed, model.n_pool_pages, step, 0)
    for l in range(s.n_layers):
        got, want = dec.layer_hidden(l), ref["layers"][l]
        for b in range(len(lens)):
            assert rel_err(got[b], want[b]) <= TOL, f"layer {l}, sequence {b} (kv_len {lens[b]})"
    assert rel_err(out, ref["final"]) <= TOL
    dec.close()
