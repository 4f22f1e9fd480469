"""Pins of the task-level oracle (event-tensor semantics): the paper's worked traces,
the closed form of the row-sum example, brute force over every topological order of
tiny graphs, the drained-counter / exactly-once invariants, and agreement of the tiled
decoder-layer graph with the operator-level oracle.
"""
import os

import numpy as np
import pytest

import oracle
from oracle import task_sim as ts
from synth import ModelShape, Step, pages_needed

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold_lines(name):
    return [l.strip() for l in open(os.path.join(GOLD, name)) if l.strip() and not l.startswith("#")]


# ------------------------------------------------------------- paper traces
def test_notify_wait_trace_of_the_static_walkthrough():
    """Sec. 3.1: counter starts at 2, the RS task spins at 1, is released at 0."""
    gold = [int(v) for v in _gold_lines("notify_wait_trace.txt")[0].split()]
    g = ts.mm_rs_graph(1)
    st = {"in": np.array([1.0, 2.0]), "mm": np.zeros(2), "rs": np.zeros(1)}
    sim = ts.Sim(g, st)
    seen = [int(sim.count["E"][0])]
    rs_task = (1, (0,))
    assert not sim.ready(rs_task)
    sim.execute((0, (0,)))
    seen.append(int(sim.count["E"][0]))
    assert not sim.ready(rs_task)             # still spinning
    sim.execute((0, (1,)))
    seen.append(int(sim.count["E"][0]))
    assert sim.ready(rs_task)
    sim.execute(rs_task)
    sim.check_final()
    assert seen == gold
    assert st["rs"][0] == 6.0


def test_push_pop_trace_of_the_dynamic_walkthrough():
    """Sec. 3.2: RS is pushed only when the counter reaches zero, then popped by an idle CU."""
    gold = _gold_lines("push_pop_trace.txt")
    g = ts.mm_rs_graph(1)
    st = {"in": np.array([1.0, 2.0]), "mm": np.zeros(2), "rs": np.zeros(1)}
    sim = ts.run_dynamic(g, st, n_workers=2, rng=np.random.default_rng(0))
    lines = []
    for ev in sim.trace:
        if ev[0] == "push":
            lines.append(f"push {ev[1]} {ev[2][0]}")
        elif ev[0] == "notify":
            lines.append(f"notify {ev[5]}")
        elif ev[0] == "pop" and ev[2] == "RS":
            lines.append(f"pop RS {ev[3][0]}")
    assert lines == gold


# ------------------------------------------------------------- row-sum example (Sec. 2.2)
@pytest.mark.parametrize("n", [1, 2, 5])
def test_rowsum_closed_form_for_symbolic_n(n):
    rng = np.random.default_rng(n)
    A = rng.integers(-8, 9, size=(n * 32, 128)).astype(np.float32)   # integers: every order is exact
    g = ts.rowsum_graph(n)
    assert g.events["E"] == (n,)
    sim = ts.run_order(g, ts.rowsum_state(A), lambda ready: ready[int(rng.integers(len(ready)))])
    np.testing.assert_array_equal(sim.state["C"], A.astype(np.float64).sum(1))
    assert len(sim.tasks) == 5 * n
    # the template instantiates to 4 producers per event whatever n is
    assert (ts.Sim(g, ts.rowsum_state(A)).count["E"] == 4).all()


def test_rowsum_every_topological_order_is_bit_identical():
    rng = np.random.default_rng(7)
    A = rng.standard_normal((32, 128)).astype(np.float32)           # non-integers: order would show
    outs = [sim.state["C"].copy() for sim in ts.all_orders(ts.rowsum_graph(1), ts.rowsum_state(A))]
    assert len(outs) == 24                                           # 4! orders of the producers
    for o in outs[1:]:
        np.testing.assert_array_equal(o, outs[0])
    np.testing.assert_allclose(outs[0], A.astype(np.float64).sum(1), rtol=1e-5, atol=1e-5)
    # two row blocks: 10 tasks; walk a few thousand of its orders
    A2 = rng.standard_normal((64, 128)).astype(np.float32)
    outs2 = [sim.state["C"].copy() for sim in ts.all_orders(ts.rowsum_graph(2), ts.rowsum_state(A2), limit=2000)]
    assert len(outs2) == 2000
    for o in outs2[1:]:
        np.testing.assert_array_equal(o, outs2[0])


def test_rowsum_static_and_dynamic_schedules():
    rng = np.random.default_rng(3)
    A = rng.standard_normal((96, 128)).astype(np.float32)
    ref = ts.run_order(ts.rowsum_graph(3), ts.rowsum_state(A), lambda r: r[0]).state["C"]
    for nq in (1, 2, 4, 7):
        np.testing.assert_array_equal(ts.run_static(ts.rowsum_graph(3), ts.rowsum_state(A), nq, rng).state["C"], ref)
        np.testing.assert_array_equal(ts.run_dynamic(ts.rowsum_graph(3), ts.rowsum_state(A), nq, rng).state["C"], ref)


# ------------------------------------------------------------- failure detection on the CPU
def test_wrong_initial_count_and_bad_static_order_are_detected():
    A = np.ones((32, 128), np.float32)
    g = ts.rowsum_graph(1)
    sim = ts.Sim(g, ts.rowsum_state(A))
    sim.count["E"][0] += 1                                   # armed too high: consumer can never start
    for t in list(sim.tasks)[:4]:
        sim.execute(t)
    assert not sim.ready(sim.tasks[4])
    with pytest.raises(AssertionError):
        sim.check_final()
    # consumer placed before its producers in the only queue: the head spins for ever
    sim2 = ts.Sim(g, ts.rowsum_state(A))
    bad = [[sim2.tasks[4]] + sim2.tasks[:4]]
    with pytest.raises(ts.Deadlock):
        ts.run_static(g, ts.rowsum_state(A), 1, np.random.default_rng(0), queues=bad)
    # too low: the consumer would start early and read poison (NaN)
    sim3 = ts.Sim(g, ts.rowsum_state(A))
    sim3.count["E"][0] -= 3
    sim3.execute(sim3.tasks[0])
    sim3.execute(sim3.tasks[4])
    assert np.isnan(sim3.state["C"]).any()


# ------------------------------------------------------------- decoder layer as tiled tasks
def _mini(moe):
    base = dict(name="m", n_layers=1, H=32, nq=4, nkv=2, d=8, F=64, page=4)
    if moe:
        base.update(F=0, n_experts=6, top_k=2, moe_F=16)
    return ModelShape(**base)


def _mini_inputs(s, kv_len, seed):
    rng = np.random.default_rng(seed)
    r = lambda *sh, sc=0.2: (rng.standard_normal(sh) * sc).astype(np.float32)  # noqa: E731
    w = {"g1": 1 + r(s.H, sc=0.02), "g2": 1 + r(s.H, sc=0.02), "wq": r(s.nq * s.d, s.H), "wk": r(s.nkv * s.d, s.H),
         "wv": r(s.nkv * s.d, s.H), "wo": r(s.H, s.nq * s.d)}
    if s.is_moe:
        w.update(wr=r(s.n_experts, s.H, sc=1.0), eg=r(s.n_experts, s.moe_F, s.H), eu=r(s.n_experts, s.moe_F, s.H),
                 ed=r(s.n_experts, s.H, s.moe_F))
    else:
        w.update(wg=r(s.F, s.H), wu=r(s.F, s.H), wd=r(s.H, s.F))
    kv_len = np.asarray(kv_len, np.int32)
    npg = [pages_needed(int(l), s.page) for l in kv_len]
    indptr = np.concatenate([[0], np.cumsum(npg)]).astype(np.int32)
    n_pool = int(indptr[-1]) + 2
    step = Step(len(kv_len), kv_len, indptr, rng.permutation(n_pool)[: indptr[-1]].astype(np.int32))
    return w, step, r(n_pool, s.page, s.nkv, s.d, sc=1.0), r(n_pool, s.page, s.nkv, s.d, sc=1.0), r(len(kv_len), s.H, sc=1.0)


@pytest.mark.parametrize("moe", [False, True])
def test_layer_graph_any_order_any_scheduler_matches_operator_oracle(moe):
    s = _mini(moe)
    w, step, kpool, vpool, x = _mini_inputs(s, [9, 0, 5], seed=11 + moe)
    xo = x.copy()
    kp, vp = kpool.copy(), vpool.copy()
    ids, _ = oracle.layer(oracle.shape_of(s, tile_m=2), xo, w, kp, vp, step.kv_len, step.page_indptr, step.page_ids)

    def fresh():
        return ts.layer_state(s, step, x, w, kpool.copy(), vpool.copy(), chunk_tokens=4, n_kchunks=2)

    def graph():
        return ts.layer_graph(s, step, chunk_tokens=4, f_tile=8, n_kchunks=2, tile_m=2)

    rng = np.random.default_rng(5)
    first = ts.run_order(graph(), fresh(), lambda r: r[0])
    np.testing.assert_allclose(first.state["x_out"], xo, rtol=1e-4, atol=1e-4)
    np.testing.assert_allclose(first.state["kpool"], kp, rtol=1e-5, atol=1e-6)
    runs = [ts.run_order(graph(), fresh(), lambda r: r[-1])]
    runs += [ts.run_order(graph(), fresh(), lambda r: r[int(rng.integers(len(r)))]) for _ in range(6)]
    if not moe:
        runs += [ts.run_static(graph(), fresh(), nq, rng) for nq in (1, 3, 8)]
    runs += [ts.run_dynamic(graph(), fresh(), nw, rng) for nw in (1, 4)]
    for sim in runs:
        np.testing.assert_array_equal(sim.state["x_out"], first.state["x_out"])     # bit-identical in every order
        assert all(n == 1 for n in sim.done.values())
    if moe:
        st = first.state
        np.testing.assert_array_equal(st["topk"], ids)
        count, tok_indptr, perm, exp_indptr = oracle.group(ids, s.n_experts, 2)
        np.testing.assert_array_equal(st["count"], count)
        np.testing.assert_array_equal(st["tok_indptr"], tok_indptr)
        np.testing.assert_array_equal(st["exp_indptr"], exp_indptr)
        np.testing.assert_array_equal(st["perm"], perm)
        # data-dependent triggering: the GroupGEMM grid has exp_indptr[E] row tiles (Sec. 2.4)
        n_gg1 = sum(1 for (ci, _c) in first.tasks if first.g.calls[ci].name == "groupgemm1")
        assert n_gg1 == int(exp_indptr[-1]) * (s.moe_F // 8)


def test_shape_dynamism_same_template_two_batches():
    """One graph template, instantiated for B = 1 and B = 2 (the dynamic-shape figure of Sec. 2.3)."""
    s = _mini(False)
    sizes = {}
    for kv in ([3], [3, 6]):
        w, step, kpool, vpool, x = _mini_inputs(s, kv, seed=2)
        sim = ts.run_order(ts.layer_graph(s, step, 4, 8, 2), ts.layer_state(s, step, x, w, kpool, vpool, 4, 2),
                           lambda r: r[0])
        sizes[len(kv)] = (len(sim.tasks), sim.count["E_split"].shape)
    assert sizes[1][1] == (1, 2) and sizes[2][1] == (2, 2)
    assert sizes[2][0] > sizes[1][0]
