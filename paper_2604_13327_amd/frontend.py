"""Front end of the event-tensor runtime: a graph description with symbolic shapes becomes a library.

The paper's compiler lowers a graph of device-function calls, gated by event tensors, to one persistent kernel:
the static transformation builds per-queue task lists and puts wait / notify around a dispatch over the device
functions (Alg. 1), the dynamic one replaces the lists by a ready queue that fired events push their consumers to
(Alg. 2); shapes stay symbolic and are bound at run time (Sec. 2.3).  This module is that flow for user-written
device functions:

  describe   Graph: symbols, event tensors, device functions (HIP source of the body of
             `void f(const Args &a, int c0, int c1, int c2)`, run by the 512 threads of a workgroup once per
             task (c0, c1, c2) of the call's grid), and calls with their in- and out-edges;
  generate   emit_dispatch_header(): the device functions and the switch that dispatches a task record to them;
  build      build_library(): hipcc over the runtime's sources around that header (generic kernel instance only);
             the result exports the C ABI of include/etc.h;
  run        CompiledGraph: declares events and calls through that ABI (device function k is ETC_FN_USER0 + k),
             binds buffers and symbol values, launches under the static, dynamic or unfused scheduler.  Task lists
             and consumer tables are instantiated by the library for every bound shape; nothing is recompiled.

Inside a device function: a.buf[slot] are the bound buffers (float *; cast for other types), a.sym[k] the bound
symbol values.  Data that another task reads must be written with the runtime's device-scope accessors (st_f32,
st_i32, ...) and read with ld_f32 / ld_i32 / ld_u64: the L2 caches of the chip's dies are not coherent with each
other, and the runtime executes no cache-wide fence.  Inputs of the whole launch may be read with plain loads.
"""
from __future__ import annotations

import dataclasses
import hashlib
import os
import subprocess
from typing import Callable, Dict, List, Sequence, Tuple

from . import binding as _b
from . import build as _build

FN_USER0 = 100                      # ETC_FN_USER0 of include/etc.h
MAX_SYMBOLS, MAX_RANK, MAX_SLOTS = 4, 3, 8


@dataclasses.dataclass(frozen=True)
class Dim:
    """mul * symbol + add (symbol < 0: the constant add)."""
    sym: int = -1
    mul: int = 0
    add: int = 0

    def eval(self, values: Sequence[int]) -> int:
        return self.add if self.sym < 0 else self.mul * values[self.sym] + self.add

    def __mul__(self, k: int) -> "Dim":
        return Dim(self.sym, self.mul * k, self.add * k)

    __rmul__ = __mul__

    def __add__(self, k: int) -> "Dim":
        return Dim(self.sym, self.mul, self.add + k)


def const(v: int) -> Dim:
    return Dim(-1, 0, int(v))


def _dim(x) -> Dim:
    return x if isinstance(x, Dim) else const(x)


@dataclasses.dataclass
class DeviceFn:
    name: str
    body: str                                           # HIP source of the function body
    buffers: Dict[int, Callable[[Dict[str, int]], int]]  # slot -> bytes the function may touch, given the symbol values


@dataclasses.dataclass
class Edge:
    """Maps a task coordinate to an element of an event tensor: per event dimension ("dim", src, div) = task
    coordinate src divided by div, or ("const", v).  Data-dependent edges (Sec. 2.4) on a rank-1 event tensor, as in
    include/etc.h: [("indirect",)] on an out-edge (task (i, ...) notifies event table[i], tables in slots 3 and 5),
    [("indptr",)] on the in-edge of a rank-1 grid (event e releases tasks indptr[e] .. indptr[e+1], slot 4)."""
    event: int
    maps: List[Tuple]


@dataclasses.dataclass
class Call:
    fn: int
    grid: List[Dim]
    waits: List[Edge]
    notifies: List[Edge]


class Graph:
    def __init__(self, name: str, symbols: Sequence[str] = ()):
        if not name.isidentifier():
            raise ValueError("graph name must be an identifier")
        if len(symbols) > MAX_SYMBOLS:
            raise ValueError(f"at most {MAX_SYMBOLS} symbols")
        self.name = name
        self.symbols = list(symbols)
        self.events: List[Tuple[str, List[Dim]]] = []
        self.fns: List[DeviceFn] = []
        self.calls: List[Call] = []

    def sym(self, name: str) -> Dim:
        return Dim(self.symbols.index(name), 1, 0)

    def event(self, name: str, shape) -> int:
        shape = [_dim(d) for d in shape]
        if not 1 <= len(shape) <= MAX_RANK:
            raise ValueError("event tensors have rank 1..3")
        self.events.append((name, shape))
        return len(self.events) - 1

    def device_fn(self, name: str, body: str, buffers: Dict[int, Callable]) -> int:
        if not name.isidentifier():
            raise ValueError("device function name must be an identifier")
        if any(f.name == name for f in self.fns):
            raise ValueError(f"device function {name} defined twice")
        if any(not 0 <= s < MAX_SLOTS for s in buffers):
            raise ValueError("buffer slots are 0..7")
        self.fns.append(DeviceFn(name, body, dict(buffers)))
        return len(self.fns) - 1

    def call(self, fn: int, grid, waits: Sequence[Edge] = (), notifies: Sequence[Edge] = ()):
        grid = [_dim(d) for d in grid]
        if not 0 <= fn < len(self.fns):
            raise ValueError("unknown device function")
        if not 1 <= len(grid) <= MAX_RANK:
            raise ValueError("task grids have rank 1..3")
        if len(waits) > 2 or len(notifies) > 1:
            raise ValueError("a call takes at most 2 in-edges and 1 out-edge")
        for e in list(waits) + list(notifies):
            if not 0 <= e.event < len(self.events) or len(e.maps) != len(self.events[e.event][1]):
                raise ValueError("an edge needs one map per dimension of its event tensor")
            for m in e.maps:
                if m[0] == "dim" and not (0 <= m[1] < len(grid) and m[2] >= 1):
                    raise ValueError("('dim', src, div): src is a grid dimension, div >= 1")
                if m[0] not in ("dim", "const", "indirect", "indptr"):
                    raise ValueError("maps are ('dim', src, div), ('const', v), ('indirect',) or ('indptr',)")
                if m[0] in ("indirect", "indptr") and len(e.maps) != 1:
                    raise ValueError("data-dependent edges take a rank-1 event tensor")
        if any(m[0] == "indirect" for e in waits for m in e.maps) or any(m[0] == "indptr" for e in notifies for m in e.maps):
            raise ValueError("('indirect',) belongs on an out-edge, ('indptr',) on an in-edge")
        if any(m[0] == "indptr" for e in waits for m in e.maps) and len(grid) != 1:
            raise ValueError("an ('indptr',) in-edge releases the tasks of a rank-1 grid")
        self.calls.append(Call(fn, grid, list(waits), list(notifies)))

    def fingerprint(self) -> str:
        return hashlib.sha256(emit_dispatch_header(self).encode()).hexdigest()[:12]


# ------------------------------------------------------------------------------------------------- generation
def emit_dispatch_header(g: Graph) -> str:
    """The generated part of the kernel: the graph's device functions and the dispatch over them.  The runtime's
    task loop (wait on the task's events, dispatch, drain, notify; or pop, dispatch, notify, push consumers) calls
    user_dispatch for every task record whose function code is FN_USER0 or above."""
    out = [f"// Generated by paper_2604_13327_amd.frontend from graph '{g.name}'.  Do not edit: change the graph description.",
           "#pragma once",
           "namespace etc_user {",
           "using namespace etc;      // the runtime's device-scope accessors: st_f32, ld_f32, st_i32, ld_i32, ld_u64, ...",
           "struct Args {",
           "    float *const *buf;    // buf[slot]: what etc_graph_bind_buffer bound",
           "    const int32_t *sym;   // sym[k]: the bound value of shape symbol k" +
           (" (" + ", ".join(f"{k} = {s}" for k, s in enumerate(g.symbols)) + ")" if g.symbols else ""),
           "};"]
    for k, f in enumerate(g.fns):
        out += ["", f"// device function {k}: {f.name}",
                f"__device__ __forceinline__ void fn{k}_{f.name}(const Args &a, int c0, int c1, int c2)",
                "{", "    (void)a; (void)c0; (void)c1; (void)c2;", f.body.strip("\n"), "}"]
    out += ["}  // namespace etc_user", "", "namespace etc {",
            f"constexpr int kUserFnCount = {len(g.fns)};",
            "__device__ __forceinline__ void user_dispatch(const Params &P, int fn, int c0, int c1, int c2)",
            "{", "    const etc_user::Args a{P.gbuf, P.gsym};", "    switch (fn) {"]
    for k, f in enumerate(g.fns):
        out.append(f"    case {k}: etc_user::fn{k}_{f.name}(a, c0, c1, c2); break;")
    out += ["    default:", "        if (threadIdx.x == 0) raise_error(P, ERR_NO_BODY, FN_USER0 + fn, fn);", "        break;",
            "    }", "}", "}  // namespace etc", ""]
    return "\n".join(out)


def generated_dir() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "_generated")


def library_path(g: Graph, out_dir: str = None) -> str:
    return os.path.join(out_dir or generated_dir(), f"libetc_{g.name}.so")


def build_library(g: Graph, out_dir: str = None, verbose: bool = False) -> str:
    """Writes the generated header and builds the graph's library with hipcc (gfx950; cross-compiles without a GPU)."""
    out_dir = out_dir or generated_dir()
    os.makedirs(out_dir, exist_ok=True)
    header = os.path.join(out_dir, f"{g.name}_dispatch.h")
    with open(header, "w") as f:
        f.write(emit_dispatch_header(g))
    lib = library_path(g, out_dir)
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-DETC_GENERIC_ONLY", f'-DETC_USER_DISPATCH_HEADER="{os.path.abspath(header)}"',
           "-o", lib] + [os.path.join(_build.CSRC, s) for s in _build.SOURCES]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd, stderr=None if verbose else subprocess.DEVNULL)
    return lib


# ------------------------------------------------------------------------------------------------- run
class CompiledGraph:
    """A graph on its generated library: declares the events and calls through the C ABI and launches them."""

    def __init__(self, g: Graph, library: str = None, kind: int = _b.SCHED_STATIC, debug_flags: int = 0,
                 spin_budget: int = 0, n_queues: int = 0):
        self.graph = g
        library = library or library_path(g)
        L = _b.load_library(library)
        import ctypes as C
        n = C.c_int32()
        L.etc_graph_user_fn_count(C.byref(n))
        if n.value != len(g.fns):
            raise RuntimeError(f"{library} carries {n.value} generated device functions, the graph has {len(g.fns)}: rebuild it")
        self.eg = _b.EventGraph(kind=kind, debug_flags=debug_flags, spin_budget=spin_budget, n_queues=n_queues,
                                library=library)
        def one_map(m):
            if m[0] == "dim":
                return (_b.MAP_DIM, m[1], m[2])
            if m[0] == "const":
                return (_b.MAP_CONST, 0, m[1])
            return (_b.MAP_INDIRECT if m[0] == "indirect" else _b.MAP_INDPTR, 0, 1)
        conv = lambda e: self.eg.edge(e.event, [one_map(m) for m in e.maps])   # noqa: E731
        for _, shape in g.events:
            self.eg.add_event([_b.DimExpr(d.sym, d.mul, d.add) for d in shape])
        for c in g.calls:
            self.eg.add_call(FN_USER0 + c.fn, [_b.DimExpr(d.sym, d.mul, d.add) for d in c.grid],
                             in_edges=[conv(e) for e in c.waits], out_edges=[conv(e) for e in c.notifies])
        self._bytes: Dict[int, int] = {}
        self._bound = False

    def bind_buffer(self, slot: int, tensor):
        self.eg.bind_buffer(slot, tensor)
        self._bytes[slot] = tensor.numel() * tensor.element_size()
        self._bound = False                     # sizes are checked against the shape again

    def bind_shape(self, **values):
        g = self.graph
        if sorted(values) != sorted(g.symbols):
            raise ValueError(f"bind_shape takes exactly the symbols {g.symbols}")
        self._values = dict(values)
        self._check_buffers()
        self.eg.bind_shape([values[s] for s in g.symbols])
        self._bound = True

    def _check_buffers(self):
        """What the library cannot know: every device function that is called must find its buffers bound and large
        enough for the bound symbol values."""
        for c in self.graph.calls:
            f = self.graph.fns[c.fn]
            for slot, need in f.buffers.items():
                nbytes = int(need(self._values))
                if slot not in self._bytes:
                    raise ValueError(f"device function {f.name} uses buffer slot {slot}, which is not bound")
                if self._bytes[slot] < nbytes:
                    raise ValueError(f"buffer slot {slot} holds {self._bytes[slot]} bytes, device function {f.name} touches "
                                     f"{nbytes} for {self._values}")

    def launch(self, stream=None):
        if not self._bound:
            if not hasattr(self, "_values"):
                raise RuntimeError("bind a shape first")
            self._check_buffers()
            self._bound = True
        self.eg.launch(stream)

    def __getattr__(self, name):                # step_info, event_counters, exec_counts, error_word, close
        if name in ("eg", "graph", "_values"):    # not set (yet): no delegation, or this would recurse
            raise AttributeError(name)
        return getattr(self.eg, name)


# ------------------------------------------------------------------------------------------------- examples
def rowsum_example() -> Graph:
    """The paper's running example (Sec. 2.2): C[r] = sum_k A[r, k] for A of (32 n, 128) fp32 as n x 4 partial-sum
    tasks over 32 x 32 tiles and n final tasks; event E[i] counts the 4 partial sums of row block i."""
    g = Graph("rowsum", ["n"])
    n = g.sym("n")
    E = g.event("E", [n])
    partial = g.device_fn("partial_sum", """
    // task (i, j): B[32 i + t, j] = sum of A[32 i + t, 32 j .. 32 j + 32), left to right
    if (threadIdx.x < 32) {
        const int row = 32 * c0 + (int)threadIdx.x;
        const float *src = a.buf[0] + (size_t)row * 128 + 32 * c1;
        float acc = 0.f;
        for (int k = 0; k < 32; ++k) acc += src[k];
        st_f32(a.buf[1] + (size_t)row * 4 + c1, acc);
    }""", {0: lambda s: s["n"] * 32 * 128 * 4, 1: lambda s: s["n"] * 32 * 4 * 4})
    final = g.device_fn("final_sum", """
    // task (i): C[32 i + t] = B[row, 0] + B[row, 1] + B[row, 2] + B[row, 3]
    if (threadIdx.x < 32) {
        const int row = 32 * c0 + (int)threadIdx.x;
        const float *b = a.buf[1] + (size_t)row * 4;
        a.buf[2][row] = ((ld_f32(b) + ld_f32(b + 1)) + ld_f32(b + 2)) + ld_f32(b + 3);
    }""", {1: lambda s: s["n"] * 32 * 4 * 4, 2: lambda s: s["n"] * 32 * 4})
    g.call(partial, [n, 4], notifies=[Edge(E, [("dim", 0, 1)])])
    g.call(final, [n], waits=[Edge(E, [("dim", 0, 1)])])
    return g


def sumsq_example() -> Graph:
    """Three stages with a tile-level event tensor in between: Y = A * A per 32 x 32 tile (event T[i, j] per tile),
    partial sums of Y per tile (each waits for ITS tile only), final sums per row block: C[r] = sum_k A[r, k]^2."""
    g = Graph("sumsq", ["n"])
    n = g.sym("n")
    T = g.event("T", [n, 4])
    E = g.event("E", [n])
    square = g.device_fn("square_tile", """
    // task (i, j): Y[32 i + r, 32 j + c] = A[.., ..]^2; thread t takes row r = t / 16 and columns c = 2 (t % 16), + 1
    {
        const int r = (int)threadIdx.x >> 4, c = ((int)threadIdx.x & 15) * 2;
        const size_t o = (size_t)(32 * c0 + r) * 128 + 32 * c1 + c;
        const float x0 = a.buf[0][o], x1 = a.buf[0][o + 1];
        st_f32(a.buf[3] + o, x0 * x0);
        st_f32(a.buf[3] + o + 1, x1 * x1);
    }""", {0: lambda s: s["n"] * 32 * 128 * 4, 3: lambda s: s["n"] * 32 * 128 * 4})
    partial = g.device_fn("partial_sum", """
    if (threadIdx.x < 32) {
        const int row = 32 * c0 + (int)threadIdx.x;
        const float *src = a.buf[3] + (size_t)row * 128 + 32 * c1;
        float acc = 0.f;
        for (int k = 0; k < 32; ++k) acc += ld_f32(src + k);
        st_f32(a.buf[1] + (size_t)row * 4 + c1, acc);
    }""", {3: lambda s: s["n"] * 32 * 128 * 4, 1: lambda s: s["n"] * 32 * 4 * 4})
    final = g.device_fn("final_sum", """
    if (threadIdx.x < 32) {
        const int row = 32 * c0 + (int)threadIdx.x;
        const float *b = a.buf[1] + (size_t)row * 4;
        a.buf[2][row] = ((ld_f32(b) + ld_f32(b + 1)) + ld_f32(b + 2)) + ld_f32(b + 3);
    }""", {1: lambda s: s["n"] * 32 * 4 * 4, 2: lambda s: s["n"] * 32 * 4})
    g.call(square, [n, 4], notifies=[Edge(T, [("dim", 0, 1), ("dim", 1, 1)])])
    g.call(partial, [n, 4], waits=[Edge(T, [("dim", 0, 1), ("dim", 1, 1)])], notifies=[Edge(E, [("dim", 0, 1)])])
    g.call(final, [n], waits=[Edge(E, [("dim", 0, 1)])])
    return g


def routed_rowsum_example(n_max: int = 24, groups: int = 5) -> Graph:
    """The two data-dependent mechanisms of Sec. 2.4 with generated device functions: n row blocks are routed to
    `groups` groups by a run-time table (slot 3); the partial sums of row block i notify the event of group table[i]
    (how often an event is notified is known at run time only: slot 5), and event g releases the final-sum tasks
    indptr[g] .. indptr[g+1] (slot 4), task t summing row block perm[t] (slot 6).  The final grid is sized for n_max
    row blocks: tasks beyond indptr[groups] have nothing to do (static rule) or are never released (ready queue)."""
    g = Graph("routed_rowsum", ["n"])
    n = g.sym("n")
    G = g.event("G", [groups])
    partial = g.device_fn("partial_sum", """
    if (threadIdx.x < 32) {
        const int row = 32 * c0 + (int)threadIdx.x;
        const float *src = a.buf[0] + (size_t)row * 128 + 32 * c1;
        float acc = 0.f;
        for (int k = 0; k < 32; ++k) acc += src[k];
        st_f32(a.buf[1] + (size_t)row * 4 + c1, acc);
    }""", {0: lambda s: s["n"] * 32 * 128 * 4, 1: lambda s: s["n"] * 32 * 4 * 4,
           3: lambda s: s["n"] * 4, 4: lambda s: (groups + 1) * 4, 5: lambda s: groups * 4})
    final = g.device_fn("final_sum_of_routed_block", f"""
    // task t of the grouped grid: row block perm[t]; tasks beyond the last group's range, and entries that name no
    // row block, do nothing
    const int32_t *indptr = reinterpret_cast<const int32_t *>(a.buf[4]), *perm = reinterpret_cast<const int32_t *>(a.buf[6]);
    if (c0 >= gld_i32(indptr + {groups})) return;
    const int r = gld_i32(perm + c0);
    if (r < 0 || r >= a.sym[0]) return;
    if (threadIdx.x < 32) {{
        const int row = 32 * r + (int)threadIdx.x;
        const float *b = a.buf[1] + (size_t)row * 4;
        a.buf[2][row] = ((ld_f32(b) + ld_f32(b + 1)) + ld_f32(b + 2)) + ld_f32(b + 3);
    }}""", {1: lambda s: s["n"] * 32 * 4 * 4, 2: lambda s: s["n"] * 32 * 4, 4: lambda s: (groups + 1) * 4,
            6: lambda s: n_max * 4})
    g.call(partial, [n, 4], notifies=[Edge(G, [("indirect",)])])
    g.call(final, [n_max], waits=[Edge(G, [("indptr",)])])
    return g


EXAMPLES = {"rowsum": rowsum_example, "sumsq": sumsq_example, "routed_rowsum": routed_rowsum_example}


def build_examples(verbose: bool = False) -> List[str]:
    return [build_library(make(), verbose=verbose) for make in EXAMPLES.values()]
