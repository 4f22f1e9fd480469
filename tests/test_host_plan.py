"""CPU-only checks of the library's host side: the shared library loads and exports every symbol the
header declares, and the scheduling transformation (graph instantiation, static queues, dynamic
consumer table) yields plans that a brute-force executor with virtual CUs runs to completion:
no deadlock, every task exactly once, every event counter drained to zero."""
import os
import re

import numpy as np
import pytest

import paper_2604_13327_amd as etc
import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PER_WAVE = 1
N_WAVES = 8


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "etc.h")).read()
    declared = set(re.findall(r"\b(etc_[a-z_]+)\s*\(", header))
    assert len(declared) >= 19
    L = etc.lib()
    for name in sorted(declared):
        assert hasattr(L, name), f"{name} is declared in include/etc.h but not exported"
    assert declared == set(etc.binding.EXPORTS)


def _waits(t):
    if t["wait0"] >= 0:
        if t["flags"] & PER_WAVE:
            yield from range(t["wait0"], t["wait0"] + N_WAVES)
        else:
            yield int(t["wait0"])
    if t["wait1"] >= 0:
        yield int(t["wait1"])


def run_static(plan, rng):
    """Virtual CUs walk their queues in order, spinning on the head task's events."""
    ev = plan["ev_init"].astype(np.int64).copy()
    qb, qt = plan["queue_begin"], plan["queue_tasks"]
    head = qb[:-1].astype(np.int64).copy()
    done = np.zeros(len(plan["tasks"]), np.int64)
    live = [q for q in range(len(head)) if head[q] < qb[q + 1]]
    while live:
        runnable = [q for q in live if all(ev[e] == 0 for e in _waits(qt[head[q]]))]
        assert runnable, "deadlock: every queue head waits on an unfired event"
        for q in rng.permutation(runnable)[: max(1, len(runnable) // 2)]:
            t = qt[head[q]]
            done[t["id"]] += 1
            if t["notify0"] >= 0:
                ev[t["notify0"]] -= 1
                assert ev[t["notify0"]] >= 0
            head[q] += 1
        live = [q for q in live if head[q] < qb[q + 1]]
    return ev, done


def run_dynamic(plan, n_workers, rng):
    """Central ready queue with early push (App. E): a task is pushed when every producer of every event it
    waits on has been dispatched (popped), and still waits for those events once a worker holds it."""
    ev = plan["ev_init"].astype(np.int64).copy()
    disp = ev.copy()                                   # producers not yet dispatched, per event
    tasks = plan["tasks"]
    done = np.zeros(len(tasks), np.int64)
    pending = np.zeros(len(tasks), np.int64)
    pushed = np.zeros(len(tasks), np.int64)
    queue = list(plan["seed_tasks"])
    pushed[queue] += 1
    workers = [None] * n_workers
    while True:
        for w in range(n_workers):
            if workers[w] is None and queue:
                workers[w] = queue.pop(0)
                n = int(tasks[workers[w]]["notify0"])
                if n >= 0:                             # dispatched: the last producer of the event pushes
                    disp[n] -= 1
                    if disp[n] == 0:
                        for entry in plan["consumer_ids"][plan["ev_consumers"][n]:plan["ev_consumers"][n + 1]].tolist():
                            tid, n_waited = entry & 0xFFFFFF, (entry >> 24) & 0x7F
                            if n_waited > 1:
                                pending[tid] += 1
                                if pending[tid] % n_waited:
                                    continue
                            queue.append(tid)
                            pushed[tid] += 1
        busy = [w for w in range(n_workers) if workers[w] is not None]
        if not busy:
            break
        runnable = [w for w in busy if all(ev[e] == 0 for e in _waits(tasks[workers[w]]))]
        assert runnable, "deadlock in the dynamic protocol"
        w = int(rng.choice(runnable))
        t = tasks[workers[w]]
        done[t["id"]] += 1
        workers[w] = None
        if int(t["notify0"]) >= 0:
            ev[int(t["notify0"])] -= 1
    assert (pushed == 1).all() and (disp == 0).all()
    return ev, done


@pytest.mark.parametrize("kind", [etc.SCHED_STATIC, etc.SCHED_UNFUSED])
@pytest.mark.parametrize("batch,nq", [(1, 5), (4, 16), (3, 256)])
def test_static_plans_run_to_completion(kind, batch, nq):
    plan = etc.plan_build(synth.TINY, 32, batch, nq, max_kv_len=129, kind=kind)
    ev, done = run_static(plan, np.random.default_rng(batch * 7 + nq))
    assert (ev == 0).all() and (done == 1).all()
    # each queue is ordered by task id: a subsequence of one topological order
    qb, qt = plan["queue_begin"], plan["queue_tasks"]
    for q in range(nq):
        ids = qt["id"][qb[q]:qb[q + 1]]
        assert (np.diff(ids) > 0).all()
    # round-robin: queue sizes differ by at most one
    sizes = np.diff(qb)
    assert sizes.max() - sizes.min() <= 1


def test_dynamic_plan_runs_to_completion():
    plan = etc.plan_build(synth.TINY, 32, 2, 4, max_kv_len=129, kind=etc.SCHED_DYNAMIC)
    for nw in (1, 3, 16):
        ev, done = run_dynamic(plan, nw, np.random.default_rng(nw))
        assert (ev == 0).all() and (done == 1).all()
    # every task is either a seed or listed under each event it waits on, the entry carrying how many those are
    listed = np.zeros(len(plan["tasks"]), np.int64)
    for entry in plan["consumer_ids"].tolist():
        tid, n_waited = entry & 0xFFFFFF, (entry >> 24) & 0x7F
        listed[tid] += 1
        assert max(n_waited, 1) == len(set(_waits(plan["tasks"][tid])))
    assert (listed[plan["seed_tasks"]] == 0).all()
    for tid in range(len(listed)):
        assert listed[tid] == len(set(_waits(plan["tasks"][tid]))) or (listed[tid] == 0 and tid in set(plan["seed_tasks"].tolist()))


def test_event_counts_follow_the_graph():
    s = synth.TINY                      # nq 4, nkv 2, d 64, H 256, F 1024
    B, chunk, max_kv = 2, 32, 129
    plan = etc.plan_build(s, chunk, B, 256, max_kv_len=max_kv)      # 256 queues: one row tile per projection task
    tasks, ev = plan["tasks"], plan["ev_init"]
    n_chunks = -(-max_kv // chunk)
    FN_QKV, FN_ATTN, FN_MERGE, FN_OPROJ, FN_GATEUP, FN_DOWN = 4, 5, 6, 7, 8, 9
    # no merge tasks: the attention chunk that arrives last at its (sequence, KV head) merges the chunks itself
    per_layer = {FN_QKV: (s.nq + 2 * s.nkv) * (s.d // 16), FN_ATTN: B * s.nkv * n_chunks, FN_MERGE: 0,
                 FN_OPROJ: s.H // 16, FN_GATEUP: s.F // 8, FN_DOWN: s.H // 16}
    for fn, n in per_layer.items():
        assert (tasks["fn"] == fn).sum() == n * s.n_layers
    assert len(tasks) == B + s.n_layers * sum(per_layer.values())
    # an attention task of kv head h waits on the event fed by (group + 2) heads x d/16 row tiles
    attn0 = tasks[(tasks["fn"] == FN_ATTN) & (tasks["layer"] == 0)][0]
    assert ev[attn0["wait0"]] == (s.nq // s.nkv + 2) * (s.d // 16)
    oproj0 = tasks[(tasks["fn"] == FN_OPROJ) & (tasks["layer"] == 0)][0]
    assert ev[oproj0["wait0"]] == B * s.nkv * n_chunks          # shape-dependent count: every chunk slot of the layer
    down0 = tasks[(tasks["fn"] == FN_DOWN) & (tasks["layer"] == 0)][0]
    assert down0["flags"] & PER_WAVE
    assert all(ev[down0["wait0"] + w] == (s.F // 8) // N_WAVES for w in range(N_WAVES))
    qkv1 = tasks[(tasks["fn"] == FN_QKV) & (tasks["layer"] == 1)][0]
    assert ev[qkv1["wait0"]] == s.H // 16                       # all down tiles of layer 0
    assert ev[plan["tasks"][(tasks["fn"] == FN_QKV) & (tasks["layer"] == 0)][0]["wait0"]] == B   # hidden loads


def test_unfused_plan_has_one_event_per_stage():
    plan = etc.plan_build(synth.TINY, 32, 1, 8, max_kv_len=129, kind=etc.SCHED_UNFUSED)
    # prologue + per layer: qkv, attn (+ merge), oproj, gateup, down
    assert len(plan["ev_init"]) == 1 + 5 * synth.TINY.n_layers
    assert not (plan["tasks"]["flags"] & PER_WAVE).any()


def test_llama8b_plan_shape():
    s = synth.LLAMA3_8B
    plan = etc.plan_build(s, 64, 1, 256, max_kv_len=1025)
    # QKV tasks stream 2 row tiles, gate/up tasks 7 (one task per queue and stage); the rest one tile
    per_layer = 384 // 2 + 8 * 17 + 256 + 1792 // 7 + 256
    assert len(plan["tasks"]) == 1 + 32 * per_layer
    gu = plan["tasks"][plan["tasks"]["fn"] == 8]
    assert (gu["c1"] == 7).all() and (gu["c0"] % 7 == 0).all()
    # a gate/up task's 7 consecutive tiles feed one K slice of the down projection: 32 tasks per slice event
    down0 = plan["tasks"][(plan["tasks"]["fn"] == 9) & (plan["tasks"]["layer"] == 0)][0]
    assert all(plan["ev_init"][down0["wait0"] + w] == 32 for w in range(8))
    sizes = np.diff(plan["queue_begin"])
    assert sizes.max() - sizes.min() <= 1


def test_descriptor_validation_errors_are_reported():
    bad = synth.ModelShape("bad", 1, 200, 4, 2, 64, 1024)       # hidden not a multiple of 256
    with pytest.raises(etc.EtcError) as ei:
        etc.plan_build(bad, 32, 1, 4, max_kv_len=64)
    assert ei.value.status == -1 and "256" in str(ei.value)


def test_page_size_must_be_a_power_of_two():
    """The attention key loop locates a key's page with a shift and a mask."""
    for page, ok in ((16, True), (1, True), (64, True), (12, False), (24, False)):
        s = synth.ModelShape("p", 1, 256, 4, 2, 64, 1024, page=page)
        if ok:
            etc.plan_build(s, page * 2, 1, 4, max_kv_len=page * 4)
        else:
            with pytest.raises(etc.EtcError) as ei:
                etc.plan_build(s, page * 2, 1, 4, max_kv_len=page * 4)
            assert ei.value.status == -1 and "power of two" in str(ei.value)


def test_attention_shapes_without_a_task_body_are_refused():
    """The attention task bodies exist for a list of (head_dim, query heads per KV head) pairs; a descriptor outside
    it must be refused when the plan is built (it used to pass, run no attention body and still notify)."""
    for nq, nkv, d in ((4, 2, 128), (16, 1, 128), (2, 2, 64), (8, 1, 64)):      # groups 2, 16 (d 128); 1, 8 (d 64)
        bad = synth.ModelShape("bad", 1, 512, nq, nkv, d, 1024)
        with pytest.raises(etc.EtcError) as ei:
            etc.plan_build(bad, 32, 1, 4, max_kv_len=64)
        assert ei.value.status == -1 and "attention" in str(ei.value)
    for nq, nkv, d in ((4, 1, 128), (8, 1, 128), (2, 2, 128), (4, 2, 64), (4, 1, 64)):    # every supported pair builds
        etc.plan_build(synth.ModelShape("ok", 1, 512, nq, nkv, d, 1024), 32, 1, 4, max_kv_len=64)


# ---------------------------------------------------------------- MoE layers (Sec. 2.4 under static scheduling)
FN_ROUTER_LOGITS, FN_ROUTER, FN_MOE_GATEUP, FN_MOE_DOWN, FN_COMBINE = 10, 11, 12, 13, 14
DYN_ROWTILE = 4


def _max_row_tiles_brute(E, K, B, M, rng, trials=300):
    """Largest sum_e ceil(count_e / M) seen over random and adversarial routings."""
    best = 0
    for _ in range(trials):
        ids = np.stack([rng.choice(E, size=K, replace=False) for _ in range(B)])
        best = max(best, int(np.ceil(np.bincount(ids.ravel(), minlength=E) / M).sum()))
    # adversarial: spread the pairs over as many experts as possible, one over a multiple of M where possible
    n = B * K
    counts = np.zeros(E, np.int64)
    counts[: min(E, n)] = 1
    left = n - int(counts.sum())
    e = 0
    while left > 0:
        add = min(left, M)
        counts[e % E] += add
        left -= add
        e += 1
    return max(best, int(np.ceil(counts / M).sum()))


@pytest.mark.parametrize("kind", [etc.SCHED_STATIC, etc.SCHED_UNFUSED])
@pytest.mark.parametrize("batch,nq,tile_m", [(1, 5, 16), (4, 16, 2), (3, 256, 1)])
def test_moe_static_plans_run_to_completion(kind, batch, nq, tile_m):
    plan = etc.plan_build(synth.TINY_MOE, 32, batch, nq, max_kv_len=129, kind=kind, moe_tile_m=tile_m)
    ev, done = run_static(plan, np.random.default_rng(batch + nq))
    assert (ev == 0).all() and (done == 1).all()


def test_moe_dynamic_plan_runs_to_completion():
    plan = etc.plan_build(synth.TINY_MOE, 32, 2, 4, max_kv_len=129, kind=etc.SCHED_DYNAMIC, moe_tile_m=2)
    ev, done = run_dynamic(plan, 3, np.random.default_rng(0))
    assert (ev == 0).all() and (done == 1).all()


def run_dynamic_moe(plan, n_workers, rng, s, batch, tile_m):
    """run_dynamic plus the data-dependent part of the MoE step under the dynamic scheduler (Sec. 2.4), on a
    random routing per layer: the expert event E_exp[e] counts the tokens routed to e plus one for tile 0
    (which publishes the tables); a router tile updates the events of its token's experts when it completes;
    a fired expert releases the GroupGEMM-1 tasks of its row-tile slots [exp_indptr[e], exp_indptr[e+1]) from
    the consumer list of the router tiles' event; tile 0 takes the surplus slots out of the counts fixed
    before the routing was known.  Router tiles do not count as dispatched producers (nothing is pushed early
    from their event) and a released GroupGEMM-1 task waits for nothing."""
    E, K = s.n_experts, s.top_k
    tasks = plan["tasks"]
    ev = plan["ev_init"].astype(np.int64).copy()
    disp = ev.copy()
    done = np.zeros(len(tasks), np.int64)
    pending = np.zeros(len(tasks), np.int64)
    pushed = np.zeros(len(tasks), np.int64)
    l0 = tasks[tasks["layer"] == 0]
    r_max = int(l0[l0["fn"] == FN_MOE_GATEUP]["c0"].max()) + 1
    G = int(((l0["fn"] == FN_MOE_GATEUP) & (l0["c0"] == 0)).sum())
    Gd = int(((l0["fn"] == FN_MOE_DOWN) & (l0["c0"] == 0)).sum())
    routing = {}
    for layer in range(s.n_layers):
        ids = np.stack([rng.choice(E, size=K, replace=False) for _ in range(batch)])
        cnt = np.bincount(ids.ravel(), minlength=E)
        expp = np.concatenate([[0], np.cumsum(-(-cnt // tile_m))])
        down0 = tasks[(tasks["layer"] == layer) & (tasks["fn"] == FN_MOE_DOWN) & (tasks["c0"] == 0)][0]
        routing[layer] = dict(ids=ids, cnt=cnt, expp=expp, exp_ev=np.zeros(E, np.int64),
                              ev_slot0=int(down0["wait0"]), ev_y=int(down0["notify0"]))
    credit = 0
    expect = np.ones(len(tasks), np.int64)
    for t in tasks:
        if t["fn"] in (FN_MOE_GATEUP, FN_MOE_DOWN) and t["c0"] >= routing[int(t["layer"])]["expp"][-1]:
            expect[t["id"]] = 0
    queue = list(plan["seed_tasks"])
    pushed[queue] += 1
    workers = [None] * n_workers

    def push_consumers(n):
        for entry in plan["consumer_ids"][plan["ev_consumers"][n]:plan["ev_consumers"][n + 1]].tolist():
            tid, n_waited = entry & 0xFFFFFF, (entry >> 24) & 0x7F
            if n_waited > 1:
                pending[tid] += 1
                if pending[tid] % n_waited:
                    continue
            queue.append(tid)
            pushed[tid] += 1

    while True:
        for w in range(n_workers):
            if workers[w] is None and queue:
                workers[w] = queue.pop(0)
                t = tasks[workers[w]]
                n = int(t["notify0"])
                if n >= 0 and t["fn"] != FN_ROUTER:
                    disp[n] -= 1
                    if disp[n] == 0:
                        push_consumers(n)
        busy = [w for w in range(n_workers) if workers[w] is not None]
        if not busy:
            break

        def waits_of(t):
            return [] if t["fn"] == FN_MOE_GATEUP else list(_waits(t))
        runnable = [w for w in busy if all(ev[e] == 0 for e in waits_of(tasks[workers[w]]))]
        assert runnable, "deadlock in the dynamic protocol"
        w = int(rng.choice(runnable))
        t = tasks[workers[w]]
        done[t["id"]] += 1
        workers[w] = None
        if t["fn"] == FN_ROUTER and t["c0"] < batch:
            r, tok = routing[int(t["layer"])], int(t["c0"])
            notifies = [int(e) for e in r["ids"][tok]]
            if tok == 0:
                live = int(r["expp"][-1])
                dead = r_max - live
                ev[r["ev_slot0"] + live: r["ev_slot0"] + r_max] = 0
                ev[r["ev_y"]] -= dead * Gd
                disp[r["ev_y"]] -= dead * Gd
                credit += dead * (G + Gd)
                notifies += [e for e in range(E) if r["cnt"][e] > 0]
            c0 = int(plan["ev_consumers"][int(t["notify0"])])
            for e in notifies:
                before = r["exp_ev"][e]
                r["exp_ev"][e] -= 1
                if before == -r["cnt"][e]:
                    r["exp_ev"][e] = 0
                    for entry in plan["consumer_ids"][c0 + r["expp"][e] * G: c0 + r["expp"][e + 1] * G].tolist():
                        queue.append(entry & 0xFFFFFF)
                        pushed[entry & 0xFFFFFF] += 1
        if int(t["notify0"]) >= 0:
            ev[int(t["notify0"])] -= 1
    assert (pushed == expect).all() and (done == expect).all()
    assert int(done.sum()) + credit == len(tasks)             # what the kernel's termination test compares
    assert all((r["exp_ev"] == 0).all() for r in routing.values())
    return ev


@pytest.mark.parametrize("batch,sampled,tile_m,workers", [(1, 1, 16, 3), (2, 2, 2, 5), (3, 4, 1, 16), (8, 8, 2, 2)])
def test_moe_dynamic_plan_with_data_dependent_triggers(batch, sampled, tile_m, workers):
    plan = etc.plan_build(synth.TINY_MOE, 32, sampled, 4, max_kv_len=129, kind=etc.SCHED_DYNAMIC, moe_tile_m=tile_m)
    for seed in range(3):
        ev = run_dynamic_moe(plan, workers, np.random.default_rng(seed), synth.TINY_MOE, batch, tile_m)
        assert (ev == 0).all()


def test_moe_event_counts_and_row_tile_slots():
    s = synth.TINY_MOE                   # E 16, top-2, moe_F 256, H 256
    B, M = 5, 2
    plan = etc.plan_build(s, 32, B, 256, max_kv_len=129, moe_tile_m=M)
    t, ev = plan["tasks"], plan["ev_init"]
    l0 = t[t["layer"] == 0]
    gu, dn = l0[l0["fn"] == FN_MOE_GATEUP], l0[l0["fn"] == FN_MOE_DOWN]
    slots = len(np.unique(gu["c0"]))
    # the static grid holds one slot per row tile any routing of B tokens can produce
    assert slots == (B * s.top_k + min(s.n_experts, B * s.top_k) * (M - 1)) // M
    assert slots >= _max_row_tiles_brute(s.n_experts, s.top_k, B, M, np.random.default_rng(3))
    assert ((gu["flags"] & DYN_ROWTILE) != 0).all() and ((dn["flags"] & DYN_ROWTILE) != 0).all()
    # every row tile is covered exactly once by the tasks of a slot
    for r in range(slots):
        g = gu[gu["c0"] == r]
        assert sorted(sum(([int(a) + i for i in range(int(n))] for a, n in zip(g["c1"], g["c2"])), [])) == list(range(s.moe_F // 8))
        d = dn[dn["c0"] == r]
        assert sorted(sum(([int(a) + i for i in range(int(n))] for a, n in zip(d["c1"], d["c2"])), [])) == list(range(s.H // 16))
        # GroupGEMM-1 -> GroupGEMM-2 stays fine-grained: one event per slot, fed by that slot's tasks only
        assert len(set(g["notify0"])) == 1 and set(d["wait0"]) == set(g["notify0"])
        assert ev[g["notify0"][0]] == len(g)
    # the data-dependent edges collapse to one coarse event each ("E[0]")
    router = l0[l0["fn"] == FN_ROUTER]
    assert len(router) == B and len(set(gu["wait0"])) == 1 and ev[gu["wait0"][0]] == B
    comb = l0[l0["fn"] == FN_COMBINE]
    assert len(set(comb["wait0"])) == 1 and ev[comb["wait0"][0]] == len(dn)
    assert (l0["fn"] == FN_ROUTER_LOGITS).sum() == s.n_experts // 16


def test_qwen3_moe_plan_shape():
    q = synth.QWEN3_30B_A3B
    plan = etc.plan_build(q, 64, 1, 256, max_kv_len=2049)
    t = plan["tasks"]
    l0 = t[t["layer"] == 0]
    # batch 1: 8 routed experts -> 8 row-tile slots; one GroupGEMM task per queue and stage
    assert (l0["fn"] == FN_MOE_GATEUP).sum() == 256 and (l0["fn"] == FN_MOE_DOWN).sum() == 256
    assert len(np.unique(l0[l0["fn"] == FN_MOE_GATEUP]["c0"])) == 8


def test_moe_descriptor_validation():
    bad = synth.ModelShape("bad-moe", 1, 256, 4, 2, 64, 0, n_experts=12, top_k=2, moe_F=256)
    with pytest.raises(etc.EtcError):
        etc.plan_build(bad, 32, 1, 4, max_kv_len=64)
    bad = synth.ModelShape("bad-moe", 1, 256, 4, 2, 64, 0, n_experts=16, top_k=2, moe_F=100)
    with pytest.raises(etc.EtcError):
        etc.plan_build(bad, 32, 1, 4, max_kv_len=64)


# ---------------------------------------------------------------- large batches
def test_large_batch_plan_tile_shapes():
    """Large batches on the 8B shape: the operand cannot be staged whole, so a gate/up task streams several row
    tiles per pass over it (7: one task per queue), the O and down
    projections are cut into 8 slices of K with 8 row tiles per task and a second stage that adds the
    slices up, and attention is not cut finer than batch x KV heads already provides."""
    s = synth.LLAMA3_8B
    TF_K_SLICE = 8
    for batch, tiles in ((64, 8), (16, 8)):
        plan = etc.plan_build(s, 64, batch, 256, max_kv_len=4097)
        t = plan["tasks"]
        l0 = t[t["layer"] == 0]
        qkv, gu = l0[l0["fn"] == 4], l0[l0["fn"] == 8]
        assert (qkv["c2"] == 2).all() and len(qkv) == 384 // 2
        r_gu = 7
        assert (gu["c1"] == r_gu).all() and len(gu) == 1792 // r_gu
        for fn, fn_sum in ((7, 15), (9, 16)):
            part, total = l0[l0["fn"] == fn], l0[l0["fn"] == fn_sum]
            assert len(part) == 256 // tiles * 8 and (part["flags"] & TF_K_SLICE).all() and (part["c2"] == tiles).all()
            assert sorted(set(part["c0"].tolist())) == list(range(0, 256, tiles))
            assert sorted(set(part["c1"].tolist())) == list(range(8))
            assert len(set(part["notify0"].tolist())) == 1           # one event gathers all slices
            assert len(total) == 256 and (total["wait0"] == part["notify0"][0]).all()
            assert plan["ev_init"][part["notify0"][0]] == len(part)
        down = l0[l0["fn"] == 9]
        # a down-projection slice waits for the gate/up tiles of its own K slice only
        for sl in range(8):
            waits = set(down["wait0"][down["c1"] == sl].tolist())
            assert len(waits) == 1
            producers = gu[gu["notify0"] == waits.pop()]
            assert len(producers) == 224 // r_gu
            assert producers["c0"].min() == sl * 224 and producers["c0"].max() == sl * 224 + 224 - r_gu
        # about one attention task per queue: 64 x 8 KV heads -> one chunk per sequence, 16 x 8 -> two
        assert (l0["fn"] == 5).sum() == (64 * 8 if batch == 64 else 16 * 8 * 2)
    # batch 1 on the same context shape keeps the caller's 64-token chunks where that gives the parallelism
    plan1 = etc.plan_build(s, 64, 1, 256, max_kv_len=1025)
    t1 = plan1["tasks"]
    assert ((t1["fn"] == 5) & (t1["layer"] == 0)).sum() == 8 * 17
    for p in (plan, plan1):
        ev, done = run_static(p, np.random.default_rng(5)) if len(p["tasks"]) < 100000 else (np.zeros(1), np.ones(1))
        assert (ev == 0).all() and (done == 1).all()


def test_mid_batch_down_projection_is_cut_along_k():
    """Batch 4 on the 8B shape: QKV, O and gate/up operands (K = 4096) still fit LDS whole, the down projection's
    (K = 14336) does not, one of its 8 slices of K does: it is cut along K (8 row tiles per task, one event per
    slice fed by the gate/up tiles of that slice, a second stage that adds the slices) instead of leaving the
    staged path.  Batch 2 keeps the whole-K down projection with per-wavefront waits."""
    s = synth.LLAMA3_8B
    t4 = etc.plan_build(s, 64, 4, 256, max_kv_len=2049)["tasks"]
    l0 = t4[t4["layer"] == 0]
    down, total = l0[l0["fn"] == 9], l0[l0["fn"] == 16]
    assert len(down) == 256 and (down["flags"] & 8).all() and (down["c2"] == 8).all() and not (down["flags"] & PER_WAVE).any()
    assert len(total) == 256 and (l0["fn"] == 15).sum() == 0 and (l0["fn"] == 7).sum() == 256
    assert len(set(down["wait0"].tolist())) == 8
    t2 = etc.plan_build(s, 64, 2, 256, max_kv_len=2049)["tasks"]
    d2 = t2[(t2["layer"] == 0) & (t2["fn"] == 9)]
    assert len(d2) == 256 and (d2["flags"] & PER_WAVE).all() and not (d2["flags"] & 8).any()
    assert ((t2["fn"] == 16) | (t2["fn"] == 15)).sum() == 0



@pytest.mark.parametrize("kind", [etc.SCHED_STATIC, etc.SCHED_DYNAMIC, etc.SCHED_UNFUSED])
@pytest.mark.parametrize("shape,batch,nq", [(synth.TINY_LM, 1, 7), (synth.TINY_LM, 3, 256), (synth.TINY_MOE_LM, 2, 16),
                                            (synth.TINY_LM, 40, 16)])
def test_lm_head_tasks_close_the_step(kind, shape, batch, nq):
    """A model with a vocabulary ends in vocabulary-projection tasks that cover every 16-row tile exactly once
    (the last task ragged) and one sampling task behind all of them; the plan still runs to completion."""
    plan = etc.plan_build(shape, 32, batch, nq, max_kv_len=129, kind=kind)
    tasks = plan["tasks"]
    FN_LMHEAD, FN_SAMPLE = 18, 19
    lm = tasks[tasks["fn"] == FN_LMHEAD]
    smp = tasks[tasks["fn"] == FN_SAMPLE]
    assert len(smp) == 1 and len(lm) >= 1
    tiles = shape.vocab // 16
    covered = np.zeros(tiles, np.int64)
    for t in lm:
        c0, r = int(t["c0"]), int(t["c1"])
        covered[c0:min(tiles, c0 + r)] += 1
        assert c0 < tiles
    assert (covered == 1).all()
    assert int(smp[0]["id"]) == len(tasks) - 1 and (lm["id"] < smp[0]["id"]).all()
    if kind == etc.SCHED_DYNAMIC:
        ev, done = run_dynamic(plan, 5, np.random.default_rng(1))
    else:
        ev, done = run_static(plan, np.random.default_rng(2))
    assert (ev == 0).all() and (done == 1).all()
    if kind != etc.SCHED_UNFUSED:       # the sampling task waits for every projection task
        assert plan["ev_init"][int(smp[0]["wait0"])] == len(lm)


def test_vocab_must_be_a_multiple_of_16():
    import dataclasses
    with pytest.raises(etc.EtcError):
        etc.plan_build(dataclasses.replace(synth.TINY_LM, vocab=1000), 32, 1, 8, max_kv_len=129)


# ---------------------------------------------------------------- the MoE layer on its own (token sweep)
FN_MOEL_LOAD, FN_MOEL_TOPK, FN_MOEL_SCAN, FN_MOEL_PLACE = 20, 21, 22, 23


@pytest.mark.parametrize("kind", [etc.SCHED_STATIC, etc.SCHED_UNFUSED])
@pytest.mark.parametrize("tokens,nq,tile_m", [(1, 4, 16), (70, 16, 16), (128, 256, 64), (1000, 64, 64)])
def test_moe_layer_static_plans_run_to_completion(kind, tokens, nq, tile_m):
    s = synth.TINY_MOE
    plan = etc.moe_layer_plan_build(s, tokens, nq, kind=kind, moe_tile_m=tile_m)
    ev, done = run_static(plan, np.random.default_rng(tokens + nq))
    assert (ev == 0).all() and (done == 1).all()
    t = plan["tasks"]
    n_blk = -(-tokens // 64)
    r_max = (tokens * s.top_k + min(s.n_experts, tokens * s.top_k) * (tile_m - 1)) // tile_m
    assert (t["fn"] == FN_MOEL_LOAD).sum() == -(-tokens // 16)
    assert (t["fn"] == FN_ROUTER_LOGITS).sum() == s.n_experts // 16 * n_blk
    assert (t["fn"] == FN_MOEL_TOPK).sum() == n_blk and (t["fn"] == FN_MOEL_PLACE).sum() == n_blk
    assert (t["fn"] == FN_MOEL_SCAN).sum() == 1
    gu = t[t["fn"] == FN_MOE_GATEUP]
    assert int(gu["c0"].max()) + 1 == r_max
    # every row-tile slot covers every tile of the expert FFN exactly once
    per_slot = np.zeros(s.moe_F // 8, np.int64)
    for x in gu[gu["c0"] == 0]:
        per_slot[int(x["c1"]): int(x["c1"]) + int(x["c2"])] += 1
    assert (per_slot == 1).all()
    comb = t[t["fn"] == FN_COMBINE]
    covered = np.zeros(tokens, np.int64)                       # every token is combined exactly once per chunk
    for x in comb[comb["c1"] == 0]:
        covered[int(x["c0"]): min(tokens, int(x["c0"]) + int(x["c2"]))] += 1
    assert (covered == 1).all() and len(comb) == len(comb[comb["c1"] == 0]) * -(-s.H // 2048)
    if kind == etc.SCHED_STATIC:
        # a block's top-k waits for the router tiles of its own block only
        topk0 = t[t["fn"] == FN_MOEL_TOPK][0]
        assert plan["ev_init"][int(topk0["wait0"])] == s.n_experts // 16


def run_dynamic_moe_layer(plan, n_workers, rng, s, tokens, tile_m):
    """The dynamic scheduler's protocol for the stand-alone MoE layer on a random routing: the scan task takes the
    surplus row-tile slots out of the counts; a placing task adds its block's pair count of every expert to the expert's
    event, the update that completes the expert's total fires it and releases its GroupGEMM-1 tasks; placing tasks do
    not count as dispatched producers and a released task waits for nothing."""
    E, K = s.n_experts, s.top_k
    tasks = plan["tasks"]
    ev = plan["ev_init"].astype(np.int64).copy()
    disp = ev.copy()
    done = np.zeros(len(tasks), np.int64)
    pending = np.zeros(len(tasks), np.int64)
    pushed = np.zeros(len(tasks), np.int64)
    r_max = int(tasks[tasks["fn"] == FN_MOE_GATEUP]["c0"].max()) + 1
    G = int(((tasks["fn"] == FN_MOE_GATEUP) & (tasks["c0"] == 0)).sum())
    Gd = int(((tasks["fn"] == FN_MOE_DOWN) & (tasks["c0"] == 0)).sum())
    ids = np.stack([rng.choice(E, size=K, replace=False) for _ in range(tokens)])
    n_blk = -(-tokens // 64)
    hist = np.stack([np.bincount(ids[b * 64:(b + 1) * 64].ravel(), minlength=E) for b in range(n_blk)])
    cnt = hist.sum(0)
    expp = np.concatenate([[0], np.cumsum(-(-cnt // tile_m))])
    down0 = tasks[(tasks["fn"] == FN_MOE_DOWN) & (tasks["c0"] == 0)][0]
    ev_slot0, ev_y = int(down0["wait0"]), int(down0["notify0"])
    exp_ev = np.zeros(E, np.int64)
    credit = 0
    expect = np.ones(len(tasks), np.int64)
    for t in tasks:
        if t["fn"] in (FN_MOE_GATEUP, FN_MOE_DOWN) and t["c0"] >= expp[-1]:
            expect[t["id"]] = 0
    queue = list(plan["seed_tasks"])
    pushed[queue] += 1
    workers = [None] * n_workers

    def push_consumers(n):
        for entry in plan["consumer_ids"][plan["ev_consumers"][n]:plan["ev_consumers"][n + 1]].tolist():
            tid, n_waited = entry & 0xFFFFFF, (entry >> 24) & 0x7F
            if n_waited > 1:
                pending[tid] += 1
                if pending[tid] % n_waited:
                    continue
            queue.append(tid)
            pushed[tid] += 1

    while True:
        for w in range(n_workers):
            if workers[w] is None and queue:
                workers[w] = queue.pop(0)
                t = tasks[workers[w]]
                n = int(t["notify0"])
                if n >= 0 and t["fn"] != FN_MOEL_PLACE:
                    disp[n] -= 1
                    if disp[n] == 0:
                        push_consumers(n)
        busy = [w for w in range(n_workers) if workers[w] is not None]
        if not busy:
            break

        def waits_of(t):
            return [] if t["fn"] == FN_MOE_GATEUP else list(_waits(t))
        runnable = [w for w in busy if all(ev[e] == 0 for e in waits_of(tasks[workers[w]]))]
        assert runnable, "deadlock in the dynamic protocol"
        w = int(rng.choice(runnable))
        t = tasks[workers[w]]
        done[t["id"]] += 1
        workers[w] = None
        if t["fn"] == FN_MOEL_SCAN:
            live = int(expp[-1])
            dead = r_max - live
            ev[ev_slot0 + live: ev_slot0 + r_max] = 0
            ev[ev_y] -= dead * Gd
            disp[ev_y] -= dead * Gd
            credit += dead * (G + Gd)
        if t["fn"] == FN_MOEL_PLACE and int(t["c0"]) < n_blk:
            c0 = int(plan["ev_consumers"][int(t["notify0"])])
            for e in np.nonzero(hist[int(t["c0"])])[0].tolist():
                h = int(hist[int(t["c0"]), e])
                before = exp_ev[e]
                exp_ev[e] -= h
                if before - h == -cnt[e]:
                    exp_ev[e] = 0
                    for entry in plan["consumer_ids"][c0 + expp[e] * G: c0 + expp[e + 1] * G].tolist():
                        queue.append(entry & 0xFFFFFF)
                        pushed[entry & 0xFFFFFF] += 1
        if int(t["notify0"]) >= 0:
            ev[int(t["notify0"])] -= 1
    assert (pushed == expect).all() and (done == expect).all()
    assert int(done.sum()) + credit == len(tasks)
    assert (exp_ev == 0).all()
    return ev


@pytest.mark.parametrize("tokens,sampled,tile_m,workers", [(1, 1, 16, 3), (70, 70, 4, 5), (100, 128, 16, 16), (300, 300, 64, 7)])
def test_moe_layer_dynamic_plan_with_data_dependent_triggers(tokens, sampled, tile_m, workers):
    plan = etc.moe_layer_plan_build(synth.TINY_MOE, sampled, 8, kind=etc.SCHED_DYNAMIC, moe_tile_m=tile_m)
    for seed in range(2):
        ev = run_dynamic_moe_layer(plan, workers, np.random.default_rng(seed), synth.TINY_MOE, tokens, tile_m)
        assert (ev == 0).all()


def test_moe_layer_descriptor_validation():
    import dataclasses
    with pytest.raises(etc.EtcError):
        etc.moe_layer_plan_build(synth.TINY_MOE, 5000, 8)                       # more than 4096 tokens
    with pytest.raises(etc.EtcError):
        etc.moe_layer_plan_build(synth.TINY_MOE, 64, 8, moe_tile_m=65)
    with pytest.raises(etc.EtcError):
        etc.moe_layer_plan_build(dataclasses.replace(synth.TINY_MOE, n_experts=20), 64, 8)
