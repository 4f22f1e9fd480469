"""Task-level oracle: an explicit, materialised simulation of event-tensor graphs.

TEST INFRASTRUCTURE, never the product path, and independent of the HIP code.

The paper's program form (Sec. 2.1) is a graph function made of device-function
launches; each launch has a task grid, and edges map a task coordinate to the
coordinates of the events it waits on (in-edges) or notifies (out-edges).  An
event starts at the number of tasks that notify it; notify decrements, wait
blocks until zero (Sec. 3.3).  This module materialises exactly that (the very
thing the compiled megakernel avoids doing at run time) so the scheduling
semantics can be checked by brute force:

* ``run_order``      - run tasks in an arbitrary admissible order (any topological order)
* ``all_orders``     - enumerate every topological order of a tiny static graph
* ``run_static``     - per-queue in-order execution, round-robin queue assignment (Sec. 3.1)
* ``run_dynamic``    - central ready queue with push on zero / pop when idle (Sec. 3.2, App. A)

Data-dependent graphs (Sec. 2.4): an event tensor may be armed at run time by a
task (``sim.arm``), out-edges may read run-time tensors, and a launch may take
its grid from run-time tensors once a given event has fired.

After every run the invariants of Sec. 3.3 are asserted: every counter is zero
and every task ran exactly once.
"""
from __future__ import annotations

import copy
import itertools
from dataclasses import dataclass, field
from typing import Callable

import numpy as np


@dataclass
class Call:
    """One device-function launch of the graph function."""
    name: str
    grid: Callable          # state -> list of task coordinates (tuples)
    body: Callable          # (coord, state, sim) -> None
    in_edges: Callable = lambda c, st: []    # (coord, state) -> [(event tensor, index tuple)]
    out_edges: Callable = lambda c, st: []   # (coord, state) -> [(event tensor, index tuple)]
    grid_after: tuple | None = None          # (event tensor, index): grid is read once it is zero


@dataclass
class Graph:
    events: dict                    # name -> shape tuple
    calls: list
    runtime_armed: set = field(default_factory=set)   # event tensors whose counts a task sets


class Deadlock(RuntimeError):
    pass


class Sim:
    def __init__(self, graph: Graph, state: dict):
        self.g = graph
        self.state = state
        self.count = {n: np.zeros(shape, dtype=np.int64) for n, shape in graph.events.items()}
        self.armed = {n: (n not in graph.runtime_armed) for n in graph.events}
        self.tasks: list = []            # (call index, coord)
        self.done: dict = {}             # task -> times executed
        self.materialised = [False] * len(graph.calls)
        self.trace: list = []            # (kind, ...) log for the paper's worked traces
        for ci, call in enumerate(graph.calls):
            if call.grid_after is None:
                self._materialise(ci)

    # --- graph instantiation -------------------------------------------------
    def _materialise(self, ci: int):
        call = self.g.calls[ci]
        self.materialised[ci] = True
        for c in call.grid(self.state):
            t = (ci, tuple(c))
            self.tasks.append(t)
            self.done[t] = 0
            if call.grid_after is None:
                # static producers fix the initial wait count of the events they notify
                for ev, idx in call.out_edges(tuple(c), self.state):
                    if ev not in self.g.runtime_armed:
                        self.count[ev][idx] += 1

    def arm(self, ev: str, idx, n: int):
        """A task initialises a run-time armed counter (data-dependent event update)."""
        assert ev in self.g.runtime_armed
        self.count[ev][idx] += n
        self.armed[ev] = True

    # --- task semantics --------------------------------------------------------
    def ready(self, t) -> bool:
        ci, c = t
        call = self.g.calls[ci]
        for ev, idx in call.in_edges(c, self.state):
            if not self.armed[ev] or self.count[ev][idx] != 0:
                return False
        return True

    def execute(self, t):
        ci, c = t
        call = self.g.calls[ci]
        assert self.done[t] == 0, f"task {call.name}{c} executed twice"
        assert self.ready(t), f"task {call.name}{c} started before its events fired"
        call.body(c, self.state, self)
        self.done[t] += 1
        fired = []
        for ev, idx in call.out_edges(c, self.state):
            assert self.armed[ev], f"notify on unarmed event {ev}{idx}"
            self.count[ev][idx] -= 1
            self.trace.append(("notify", call.name, c, ev, idx, int(self.count[ev][idx])))
            assert self.count[ev][idx] >= 0, f"event {ev}{idx} went negative"
            if self.count[ev][idx] == 0:
                fired.append((ev, idx))
        for cj, other in enumerate(self.g.calls):
            if not self.materialised[cj]:
                ev, idx = other.grid_after
                if self.armed[ev] and self.count[ev][idx] == 0:
                    self._materialise(cj)
        return fired

    def pending(self):
        return [t for t in self.tasks if self.done[t] == 0]

    def check_final(self):
        assert all(self.materialised), "a launch never materialised"
        for t, n in self.done.items():
            assert n == 1, f"task {t} ran {n} times"
        for ev, cnt in self.count.items():
            assert (cnt == 0).all(), f"event tensor {ev} not drained: {cnt}"


def run_order(graph: Graph, state: dict, choose: Callable) -> Sim:
    """Run in an arbitrary admissible order; ``choose(ready_list)`` picks the next task."""
    sim = Sim(graph, state)
    while True:
        pend = sim.pending()
        if not pend:
            break
        ready = [t for t in pend if sim.ready(t)]
        if not ready:
            raise Deadlock(f"no ready task among {len(pend)} pending")
        sim.execute(choose(ready))
    sim.check_final()
    return sim


def all_orders(graph: Graph, state: dict, limit: int | None = None):
    """Yield the final state of every topological order of a small static graph."""
    n_yield = 0

    def rec(sim: Sim):
        nonlocal n_yield
        pend = sim.pending()
        if not pend:
            sim.check_final()
            n_yield += 1
            yield sim
            return
        ready = [t for t in pend if sim.ready(t)]
        if not ready:
            raise Deadlock("dead end")
        for t in ready:
            if limit is not None and n_yield >= limit:
                return
            nxt = copy.deepcopy(sim)
            nxt.execute(t)
            yield from rec(nxt)

    yield from rec(Sim(graph, state))


def static_queues(sim: Sim, n_queues: int) -> list:
    """Round-robin assignment (Sec. 3.1) of tasks, enumerated launch by launch in
    row-major coordinate order, to per-CU in-order queues."""
    queues = [[] for _ in range(n_queues)]
    for i, t in enumerate(sim.tasks):
        queues[i % n_queues].append(t)
    return queues


def run_static(graph: Graph, state: dict, n_queues: int, rng: np.random.Generator,
               queues: list | None = None) -> Sim:
    """Each virtual CU walks its own queue in order, spinning on the head task's events."""
    sim = Sim(graph, state)
    assert all(sim.materialised), "static scheduling needs a fully static task grid"
    q = queues if queues is not None else static_queues(sim, n_queues)
    head = [0] * len(q)
    while any(head[i] < len(q[i]) for i in range(len(q))):
        runnable = [i for i in range(len(q)) if head[i] < len(q[i]) and sim.ready(q[i][head[i]])]
        if not runnable:
            raise Deadlock("every queue head is spinning")
        i = int(rng.choice(runnable))
        sim.execute(q[i][head[i]])
        head[i] += 1
    sim.check_final()
    return sim


def run_dynamic(graph: Graph, state: dict, n_workers: int, rng: np.random.Generator,
                trigger: Callable | None = None) -> Sim:
    """Central ready queue (Sec. 3.2): a task is pushed when its trigger event reaches
    zero (tasks with no in-edge are pushed up front); an idle worker pops the oldest
    entry, and - as with early push (App. E) - still waits for any other in-edge before
    running.  ``trigger(call, coord, state)`` names the in-edge that pushes a task
    (default: its first in-edge)."""
    sim = Sim(graph, state)
    queue: list = []
    pushed: set = set()

    def trig(t):
        ci, c = t
        call = sim.g.calls[ci]
        if trigger is not None:
            return trigger(call, c, sim.state)
        edges = call.in_edges(c, sim.state)
        return edges[0] if edges else None

    def push_ready():
        for t in sim.tasks:
            if t in pushed:
                continue
            tr = trig(t)
            if tr is None or (sim.armed[tr[0]] and sim.count[tr[0]][tr[1]] == 0):
                pushed.add(t)
                queue.append(t)
                sim.trace.append(("push", sim.g.calls[t[0]].name, t[1]))

    push_ready()
    workers: list = [None] * n_workers       # task a worker popped and is waiting on / about to run
    while True:
        for w in range(n_workers):
            if workers[w] is None and queue:
                workers[w] = queue.pop(0)
                sim.trace.append(("pop", w, sim.g.calls[workers[w][0]].name, workers[w][1]))
        busy = [w for w in range(n_workers) if workers[w] is not None]
        if not busy:
            break
        runnable = [w for w in busy if sim.ready(workers[w])]
        if not runnable:
            raise Deadlock("every worker waits on an unfired event")
        w = int(rng.choice(runnable))
        sim.execute(workers[w])
        workers[w] = None
        push_ready()
    assert not sim.pending(), "tasks were never pushed"
    sim.check_final()
    return sim


# ---------------------------------------------------------------------------
# Graph 1: the paper's split-K row sum (Sec. 2.2).  A is (n*32, 128);
# partial_sum task (i, j) writes B[32i:32i+32, j]; final_sum task (i) writes
# C[32i:32i+32]; event E[i] is notified by the 4 partial tasks of row block i.
# ---------------------------------------------------------------------------
def rowsum_graph(n: int) -> Graph:
    def partial(c, st, sim):
        i, j = c
        blk = st["A"][32 * i:32 * i + 32, 32 * j:32 * j + 32]
        acc = np.zeros(32, dtype=np.float32)
        for k in range(32):                       # fixed left-to-right order
            acc = acc + blk[:, k]
        st["B"][32 * i:32 * i + 32, j] = acc

    def final(c, st, sim):
        (i,) = c
        b = st["B"][32 * i:32 * i + 32]
        st["C"][32 * i:32 * i + 32] = ((b[:, 0] + b[:, 1]) + b[:, 2]) + b[:, 3]

    return Graph(
        events={"E": (n,)},
        calls=[Call("partial_sum", lambda st: list(itertools.product(range(n), range(4))), partial,
                    out_edges=lambda c, st: [("E", (c[0],))]),
               Call("final_sum", lambda st: [(i,) for i in range(n)], final,
                    in_edges=lambda c, st: [("E", (c[0],))])])


def rowsum_state(A: np.ndarray) -> dict:
    n32 = A.shape[0]
    return {"A": A.astype(np.float32), "B": np.full((n32, 4), np.nan, np.float32),
            "C": np.full(n32, np.nan, np.float32)}


# ---------------------------------------------------------------------------
# Graph 2: the GEMM + reduce-scatter pattern of the scheduling walk-throughs
# (Sec. 3.1, 3.2): every RS task depends on two MM tasks, so each counter starts at 2.
# ---------------------------------------------------------------------------
def mm_rs_graph(n_rs: int) -> Graph:
    def mm(c, st, sim):
        st["mm"][c[0]] = st["in"][c[0]] * 2.0

    def rs(c, st, sim):
        st["rs"][c[0]] = st["mm"][2 * c[0]] + st["mm"][2 * c[0] + 1]

    return Graph(
        events={"E": (n_rs,)},
        calls=[Call("MM", lambda st: [(i,) for i in range(2 * n_rs)], mm,
                    out_edges=lambda c, st: [("E", (c[0] // 2,))]),
               Call("RS", lambda st: [(i,) for i in range(n_rs)], rs,
                    in_edges=lambda c, st: [("E", (c[0],))])])


# ---------------------------------------------------------------------------
# Graph 3: one decoder layer as tiled tasks (dense or MoE).  Tasks write disjoint
# outputs and every reduction is an explicit task with a fixed summation order,
# so any admissible order gives bit-identical results.
# ---------------------------------------------------------------------------
def _rms(x, g, eps):
    ss = np.float32(0.0)
    for v in x:
        ss = np.float32(ss + v * v)
    r = np.float32(1.0) / np.sqrt(ss / np.float32(x.size) + np.float32(eps))
    return (x * r * g).astype(np.float32)


def _dot_rows(W, x):
    return (W.astype(np.float32) @ x.astype(np.float32)).astype(np.float32)


def _rope_head(v, pos, theta):
    d = v.size
    half = d // 2
    i = np.arange(half, dtype=np.float64)
    ang = pos * theta ** (-2.0 * i / d)
    c, s = np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
    a, b = v[:half].copy(), v[half:].copy()
    return np.concatenate([a * c - b * s, a * s + b * c]).astype(np.float32)


def _silu(z):
    return (z / (np.float32(1.0) + np.exp(-z))).astype(np.float32)


def layer_graph(s, step, chunk_tokens: int, f_tile: int, n_kchunks: int, tile_m: int = 4) -> Graph:
    """Event-tensor graph of one decoder layer for the bound step shape.

    s: model shape (H, nq, nkv, d, F | n_experts, top_k, moe_F, page, eps, theta);
    step: batch, kv_len, page_indptr, page_ids.
    State arrays: x [B,H] in, w dict, kpool/vpool, produces x_out [B,H].
    """
    B, H, d, nq, nkv = step.batch, s.H, s.d, s.nq, s.nkv
    grp = nq // nkv
    P = s.page
    n_keys = [int(l) + 1 for l in step.kv_len]
    n_chunks = [(k + chunk_tokens - 1) // chunk_tokens for k in n_keys]
    o_tile = d                      # O-projection / down row tile
    n_otiles = H // o_tile
    moe = s.n_experts > 0

    def pages(b):
        return step.page_ids[step.page_indptr[b]:step.page_indptr[b + 1]]

    def slot_row(b, j):
        pg = pages(b)
        return int(pg[j // P]), j % P

    # --- QKV head tile: norm prologue, projection rows of one head, RoPE, append ----
    def qkv(c, st, sim):
        b, hd = c
        w = st["w"]
        xn = _rms(st["x"][b], w["g1"], s.eps)
        pos = int(step.kv_len[b])
        if hd < nq:
            st["q"][b, hd] = _rope_head(_dot_rows(w["wq"][hd * d:(hd + 1) * d], xn), pos, s.theta)
        elif hd < nq + nkv:
            kh = hd - nq
            pg, sl = slot_row(b, pos)
            st["kpool"][pg, sl, kh] = _rope_head(_dot_rows(w["wk"][kh * d:(kh + 1) * d], xn), pos, s.theta)
        else:
            vh = hd - nq - nkv
            pg, sl = slot_row(b, pos)
            st["vpool"][pg, sl, vh] = _dot_rows(w["wv"][vh * d:(vh + 1) * d], xn)

    def qkv_out(c, st):
        b, hd = c
        kvh = hd // grp if hd < nq else (hd - nq) % nkv
        return [("E_qkv", (b, kvh))]

    # --- split-KV partial attention of one (sequence, kv head, chunk) ---------------
    def attn(c, st, sim):
        b, kvh, ch = c
        j0, j1 = ch * chunk_tokens, min(n_keys[b], (ch + 1) * chunk_tokens)
        where = [slot_row(b, j) for j in range(j0, j1)]
        K = np.stack([st["kpool"][pg, sl, kvh] for pg, sl in where])
        V = np.stack([st["vpool"][pg, sl, kvh] for pg, sl in where])
        for g in range(grp):
            h = kvh * grp + g
            sc = (K @ st["q"][b, h]) / np.float32(np.sqrt(d))
            m = sc.max()
            p = np.exp(sc - m).astype(np.float32)
            st["part_m"][b, h, ch] = m
            st["part_l"][b, h, ch] = p.sum(dtype=np.float32)
            st["part_o"][b, h, ch] = (p @ V).astype(np.float32)

    # --- merge of the chunk partials (fixed ascending chunk order) ------------------
    def merge(c, st, sim):
        b, kvh = c
        for g in range(grp):
            h = kvh * grp + g
            nc = n_chunks[b]
            m = st["part_m"][b, h, :nc].max()
            num = np.zeros(d, dtype=np.float32)
            den = np.float32(0.0)
            for ch in range(nc):
                sc = np.exp(st["part_m"][b, h, ch] - m).astype(np.float32)
                num = num + sc * st["part_o"][b, h, ch]
                den = den + sc * st["part_l"][b, h, ch]
            st["attn"][b, h * d:(h + 1) * d] = num / den

    def oproj(c, st, sim):
        b, t = c
        rows = slice(t * o_tile, (t + 1) * o_tile)
        st["x_mid"][b, rows] = st["x"][b, rows] + _dot_rows(st["w"]["wo"][rows], st["attn"][b])

    calls = [
        Call("qkv", lambda st: list(itertools.product(range(B), range(nq + 2 * nkv))), qkv,
             out_edges=qkv_out),
        Call("attn", lambda st: [(b, kvh, ch) for b in range(B) for kvh in range(nkv) for ch in range(n_chunks[b])],
             attn, in_edges=lambda c, st: [("E_qkv", (c[0], c[1]))],
             out_edges=lambda c, st: [("E_split", (c[0], c[1]))]),
        Call("merge", lambda st: list(itertools.product(range(B), range(nkv))), merge,
             in_edges=lambda c, st: [("E_split", (c[0], c[1]))],
             out_edges=lambda c, st: [("E_attn", (c[0],))]),
        Call("oproj", lambda st: list(itertools.product(range(B), range(n_otiles))), oproj,
             in_edges=lambda c, st: [("E_attn", (c[0],))],
             out_edges=lambda c, st: [("E_xmid", (c[0],))]),
    ]
    events = {"E_qkv": (B, nkv), "E_split": (B, nkv), "E_attn": (B,), "E_xmid": (B,), "E_x": (B,)}
    runtime_armed: set = set()

    if not moe:
        F = s.F
        n_ftiles = F // f_tile
        kchunk = F // n_kchunks
        assert kchunk % f_tile == 0

        def gateup(c, st, sim):
            b, t = c
            w = st["w"]
            xn = _rms(st["x_mid"][b], w["g2"], s.eps)
            rows = slice(t * f_tile, (t + 1) * f_tile)
            st["act"][b, rows] = _silu(_dot_rows(w["wg"][rows], xn)) * _dot_rows(w["wu"][rows], xn)

        def down(c, st, sim):
            b, t, kc = c
            rows = slice(t * o_tile, (t + 1) * o_tile)
            cols = slice(kc * kchunk, (kc + 1) * kchunk)
            st["down_part"][b, kc, rows] = _dot_rows(st["w"]["wd"][rows, cols], st["act"][b, cols])

        def reduce_(c, st, sim):
            b, t = c
            rows = slice(t * o_tile, (t + 1) * o_tile)
            acc = st["x_mid"][b, rows].copy()
            for kc in range(n_kchunks):               # fixed ascending order
                acc = acc + st["down_part"][b, kc, rows]
            st["x_out"][b, rows] = acc

        events.update({"E_act": (B, n_kchunks), "E_down": (B, n_otiles)})
        calls += [
            Call("gateup", lambda st: list(itertools.product(range(B), range(n_ftiles))), gateup,
                 in_edges=lambda c, st: [("E_xmid", (c[0],))],
                 out_edges=lambda c, st: [("E_act", (c[0], (c[1] * f_tile) // kchunk))]),
            Call("down", lambda st: list(itertools.product(range(B), range(n_otiles), range(n_kchunks))), down,
                 in_edges=lambda c, st: [("E_act", (c[0], c[2]))],
                 out_edges=lambda c, st: [("E_down", (c[0], c[1]))]),
            Call("reduce", lambda st: list(itertools.product(range(B), range(n_otiles))), reduce_,
                 in_edges=lambda c, st: [("E_down", (c[0], c[1]))],
                 out_edges=lambda c, st: [("E_x", (c[0],))]),
        ]
    else:
        E, K, F = s.n_experts, s.top_k, s.moe_F
        n_ftiles = F // f_tile
        runtime_armed = {"E_exp", "E_g1", "E_tok"}

        # TopK routing of all tokens: static dependency on the attention output;
        # arms the expert events at run time (data-dependent event update).
        def router(c, st, sim):
            w = st["w"]
            counts = np.zeros(E, dtype=np.int64)
            for b in range(B):
                xn = _rms(st["x_mid"][b], w["g2"], s.eps)
                st["xn2"][b] = xn
                lg = _dot_rows(w["wr"], xn)
                st["logits"][b] = lg
                ids = st["forced_topk"][b] if st.get("forced_topk") is not None else \
                    np.lexsort((np.arange(E), -lg))[:K]
                st["topk"][b] = ids
                sel = lg[ids].astype(np.float32)
                p = np.exp(sel - sel.max()).astype(np.float32)
                st["topk_w"][b] = p / p.sum(dtype=np.float32)
                for e in ids:
                    counts[e] += 1
            st["count"][:] = counts
            st["tok_indptr"][1:] = np.cumsum(counts)
            tiles = (counts + tile_m - 1) // tile_m
            st["exp_indptr"][1:] = np.cumsum(tiles)
            for e in range(E):
                sim.arm("E_exp", (e,), int(counts[e]))
                for mt in range(int(tiles[e])):
                    sim.arm("E_g1", (int(st["exp_indptr"][e]) + mt,), n_ftiles)
            for b in range(B):
                sim.arm("E_tok", (b,), K * n_otiles)

        # Token grouping, one tile per token: stable rank inside each expert's range.
        def grouping(c, st, sim):
            (t,) = c
            for k in range(K):
                e = int(st["topk"][t, k])
                rank = sum(1 for t2 in range(B) for k2 in range(K)
                           if st["topk"][t2, k2] == e and (t2, k2) < (t, k))
                st["perm"][st["tok_indptr"][e] + rank] = t * K + k

        def gg_grid(st):
            return [(int(ti), ft) for ti in range(int(st["exp_indptr"][E])) for ft in range(n_ftiles)]

        def tile_rows(st, ti):
            e = int(np.searchsorted(st["exp_indptr"], ti, side="right") - 1)
            mt = ti - int(st["exp_indptr"][e])
            r0 = int(st["tok_indptr"][e]) + mt * tile_m
            r1 = min(int(st["tok_indptr"][e + 1]), r0 + tile_m)
            return e, r0, r1

        def gg1(c, st, sim):
            ti, ft = c
            e, r0, r1 = tile_rows(st, ti)
            rows = slice(ft * f_tile, (ft + 1) * f_tile)
            for r in range(r0, r1):
                xn = st["xn2"][st["perm"][r] // K]
                st["eact"][r, rows] = _silu(_dot_rows(st["w"]["eg"][e][rows], xn)) * \
                    _dot_rows(st["w"]["eu"][e][rows], xn)

        def gg2_grid(st):
            return [(int(ti), ot) for ti in range(int(st["exp_indptr"][E])) for ot in range(n_otiles)]

        def gg2(c, st, sim):
            ti, ot = c
            e, r0, r1 = tile_rows(st, ti)
            rows = slice(ot * o_tile, (ot + 1) * o_tile)
            for r in range(r0, r1):
                st["ey"][r, rows] = _dot_rows(st["w"]["ed"][e][rows], st["eact"][r])

        def gg2_out(c, st):
            e, r0, r1 = tile_rows(st, c[0])
            return [("E_tok", (int(st["perm"][r]) // K,)) for r in range(r0, r1)]

        def combine(c, st, sim):
            (t,) = c
            inv = {int(p): r for r, p in enumerate(st["perm"])}
            acc = st["x_mid"][t].copy()
            for k in range(K):                                  # ascending slot order
                acc = acc + st["topk_w"][t, k] * st["ey"][inv[t * K + k]]
            st["x_out"][t] = acc

        events.update({"E_route": (1,), "E_exp": (E,), "E_g1": (B * K,), "E_tok": (B,)})
        calls += [
            Call("router", lambda st: [(0,)], router,
                 in_edges=lambda c, st: [("E_xmid", (b,)) for b in range(B)],
                 out_edges=lambda c, st: [("E_route", (0,))]),
            Call("grouping", lambda st: [(t,) for t in range(B)], grouping,
                 in_edges=lambda c, st: [("E_route", (0,))],
                 out_edges=lambda c, st: [("E_exp", (int(st["topk"][c[0], k]),)) for k in range(K)]),
            # data-dependent triggering: expert e releases tiles [exp_indptr[e], exp_indptr[e+1])
            Call("groupgemm1", gg_grid, gg1, grid_after=("E_route", (0,)),
                 in_edges=lambda c, st: [("E_exp", (tile_rows(st, c[0])[0],))],
                 out_edges=lambda c, st: [("E_g1", (c[0],))]),
            Call("groupgemm2", gg2_grid, gg2, grid_after=("E_route", (0,)),
                 in_edges=lambda c, st: [("E_g1", (c[0],))], out_edges=gg2_out),
            Call("combine", lambda st: [(t,) for t in range(B)], combine,
                 in_edges=lambda c, st: [("E_tok", (c[0],))],
                 out_edges=lambda c, st: [("E_x", (c[0],))]),
        ]

    # a sink that consumes E_x so the drained-counter invariant covers it
    calls.append(Call("epilogue", lambda st: [(b,) for b in range(B)], lambda c, st, sim: None,
                      in_edges=lambda c, st: [("E_x", (c[0],))]))
    return Graph(events=events, calls=calls, runtime_armed=runtime_armed)


def layer_state(s, step, x, w, kpool, vpool, chunk_tokens: int, n_kchunks: int, forced_topk=None) -> dict:
    B = step.batch
    max_chunks = max((int(l) + 1 + chunk_tokens - 1) // chunk_tokens for l in step.kv_len)
    nan = lambda *shape: np.full(shape, np.nan, dtype=np.float32)  # noqa: E731  poison: read-before-write shows
    st = {"x": x.astype(np.float32).copy(), "w": w, "kpool": kpool, "vpool": vpool,
          "q": nan(B, s.nq, s.d), "part_m": nan(B, s.nq, max_chunks), "part_l": nan(B, s.nq, max_chunks),
          "part_o": nan(B, s.nq, max_chunks, s.d), "attn": nan(B, s.nq * s.d), "x_mid": nan(B, s.H),
          "x_out": nan(B, s.H)}
    if s.n_experts == 0:
        st.update({"act": nan(B, s.F), "down_part": nan(B, n_kchunks, s.H)})
    else:
        E, K = s.n_experts, s.top_k
        st.update({"xn2": nan(B, s.H), "logits": nan(B, E), "topk": np.full((B, K), -1, np.int64),
                   "topk_w": nan(B, K), "count": np.zeros(E, np.int64),
                   "tok_indptr": np.zeros(E + 1, np.int64), "exp_indptr": np.zeros(E + 1, np.int64),
                   "perm": np.full(B * K, -1, np.int64), "eact": nan(B * K, s.moe_F),
                   "ey": nan(B * K, s.H), "forced_topk": forced_topk})
    return st
