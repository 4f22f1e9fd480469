"""ctypes binding of include/etc.h.  Same names, same semantics; only marshalling happens here.

PyTorch appears only as the owner of device memory and streams: tensors are turned
into raw device pointers before they cross the C boundary.
"""
from __future__ import annotations

import ctypes as C
import functools
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))

SCHED_STATIC, SCHED_DYNAMIC, SCHED_UNFUSED = 0, 1, 2
DEBUG_EXEC_COUNT, DEBUG_LAYER_HIDDEN, DEBUG_ROUTING, DEBUG_TRACE = 1, 2, 4, 8
(DBG_ERROR_WORD, DBG_EVENT_COUNTERS, DBG_TASK_EXEC_COUNT, DBG_LAYER_HIDDEN, DBG_ROUTER_LOGITS, DBG_TOPK_IDS,
 DBG_TOPK_W, DBG_PERMUTATION, DBG_TOK_INDPTR, DBG_EXP_INDPTR, DBG_TASK_TRACE) = range(11)
FN_ROWSUM_PARTIAL, FN_ROWSUM_FINAL, FN_ROWSUM_FINAL_PERM = 1, 2, 3
MAP_DIM, MAP_CONST, MAP_INDIRECT, MAP_INDPTR = 0, 1, 2, 3

EXPORTS = ["etc_create", "etc_destroy", "etc_last_error", "etc_bind_layer_weights", "etc_bind_kv_pool",
           "etc_bind_step", "etc_force_routing", "etc_launch", "etc_launch_kernel_by_kernel", "etc_read_debug",
           "etc_bind_lm_head", "etc_launch_tokens", "etc_launch_tokens_kernel_by_kernel",
           "etc_moe_layer_create", "etc_moe_layer_bind_tokens", "etc_moe_layer_plan_build",
           "etc_get_step_info", "etc_graph_create", "etc_graph_add_event", "etc_graph_add_call",
           "etc_graph_bind_buffer", "etc_graph_bind_shape", "etc_graph_launch", "etc_plan_build", "etc_plan_free",
           "etc_rowsum_launch_noalloc", "etc_graph_user_fn_count"]
ROWSUM_NOALLOC_MAX_N = 2048


class EtcError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"etc status {status}: {msg}")
        self.status = status


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn",
                                         "n_experts", "top_k", "moe_ffn", "page_size")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float), ("qk_norm", C.c_int32), ("vocab", C.c_int32)]


class TileDesc(C.Structure):
    _fields_ = [("kv_chunk_tokens", C.c_int32), ("moe_tile_m", C.c_int32)]


class SchedDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n_sampled", C.c_int32), ("sampled_batch", C.c_int32 * 8),
                ("max_batch", C.c_int32), ("max_kv_len", C.c_int32), ("spin_budget", C.c_int64),
                ("debug_flags", C.c_uint32), ("n_queues", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd", "wr", "eg", "eu", "ed",
                                        "gq", "gk")]


class StepInfo(C.Structure):
    _fields_ = [("n_tasks", C.c_int64), ("n_events", C.c_int64), ("n_queues", C.c_int64),
                ("algorithmic_bytes", C.c_int64), ("sampled_batch", C.c_int32), ("workgroup_threads", C.c_int32),
                ("wall_clock_khz", C.c_int32), ("reserved", C.c_int32)]


class DimExpr(C.Structure):
    _fields_ = [("sym", C.c_int32), ("mul", C.c_int32), ("add", C.c_int32)]


class Edge(C.Structure):
    _fields_ = [("event", C.c_int32), ("rank", C.c_int32), ("kind", C.c_int32 * 3), ("src", C.c_int32 * 3),
                ("div", C.c_int32 * 3)]


class TaskRecord(C.Structure):
    _fields_ = [("fn", C.c_uint8), ("layer", C.c_uint8), ("flags", C.c_uint16), ("c0", C.c_int32), ("c1", C.c_int32),
                ("c2", C.c_int32), ("wait0", C.c_int32), ("wait1", C.c_int32), ("notify0", C.c_int32), ("id", C.c_int32)]


class PlanView(C.Structure):
    _fields_ = [("n_tasks", C.c_int64), ("n_events", C.c_int64), ("n_queues", C.c_int64), ("n_seed", C.c_int64),
                ("tasks", C.POINTER(TaskRecord)), ("queue_tasks", C.POINTER(TaskRecord)),
                ("queue_begin", C.POINTER(C.c_int32)), ("ev_init", C.POINTER(C.c_int32)),
                ("ev_consumers", C.POINTER(C.c_int32)), ("consumer_ids", C.POINTER(C.c_int32)),
                ("seed_tasks", C.POINTER(C.c_int32)), ("opaque", C.c_void_p)]


TASK_DTYPE = np.dtype([("fn", "u1"), ("layer", "u1"), ("flags", "<u2"), ("c0", "<i4"), ("c1", "<i4"), ("c2", "<i4"),
                       ("wait0", "<i4"), ("wait1", "<i4"), ("notify0", "<i4"), ("id", "<i4")])


def lib_path() -> str:
    return os.path.join(_HERE, "libetc.so")


def lib():
    """Loads libetc.so.  torch is imported first so that the HIP runtime torch ships is the one
    the library binds to (a second HIP runtime in the process would not know torch's allocations)."""
    return load_library(lib_path())


@functools.lru_cache(maxsize=None)
def load_library(path: str):
    """Loads a library that exports the C ABI of include/etc.h: libetc.so, or one the front end generated for a graph."""
    import torch  # noqa: F401
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first "
                          "(there is no fallback path)")
    L = C.CDLL(path)
    L.etc_last_error.restype = C.c_char_p
    L.etc_last_error.argtypes = [C.c_void_p]
    L.etc_destroy.restype = None
    L.etc_destroy.argtypes = [C.c_void_p]
    L.etc_plan_free.restype = None
    for name in EXPORTS:
        if name not in ("etc_last_error", "etc_destroy", "etc_plan_free"):
            getattr(L, name).restype = C.c_int
    L.etc_create.argtypes = [C.POINTER(ModelDesc), C.POINTER(TileDesc), C.POINTER(SchedDesc), C.POINTER(C.c_void_p)]
    L.etc_bind_layer_weights.argtypes = [C.c_void_p, C.c_int32, C.POINTER(LayerWeights)]
    L.etc_bind_kv_pool.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64]
    L.etc_bind_step.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    L.etc_force_routing.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    L.etc_launch.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.etc_launch_kernel_by_kernel.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.etc_bind_lm_head.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.etc_launch_tokens.argtypes = [C.c_void_p] * 7
    L.etc_launch_tokens_kernel_by_kernel.argtypes = [C.c_void_p] * 7
    L.etc_moe_layer_create.argtypes = [C.POINTER(ModelDesc), C.POINTER(TileDesc), C.POINTER(SchedDesc), C.POINTER(C.c_void_p)]
    L.etc_moe_layer_bind_tokens.argtypes = [C.c_void_p, C.c_int32]
    L.etc_moe_layer_plan_build.argtypes = [C.POINTER(ModelDesc), C.POINTER(TileDesc), C.POINTER(SchedDesc), C.c_int32, C.c_int32,
                                           C.POINTER(PlanView)]
    L.etc_read_debug.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t]
    L.etc_get_step_info.argtypes = [C.c_void_p, C.POINTER(StepInfo)]
    L.etc_graph_create.argtypes = [C.POINTER(SchedDesc), C.POINTER(C.c_void_p)]
    L.etc_graph_add_event.argtypes = [C.c_void_p, C.POINTER(DimExpr), C.c_int32, C.POINTER(C.c_int32)]
    L.etc_graph_add_call.argtypes = [C.c_void_p, C.c_int32, C.POINTER(DimExpr), C.c_int32, C.POINTER(Edge), C.c_int32,
                                     C.POINTER(Edge), C.c_int32]
    L.etc_graph_bind_buffer.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t]
    L.etc_graph_bind_shape.argtypes = [C.c_void_p, C.c_void_p]
    L.etc_graph_launch.argtypes = [C.c_void_p, C.c_void_p]
    L.etc_plan_build.argtypes = [C.POINTER(ModelDesc), C.POINTER(TileDesc), C.POINTER(SchedDesc), C.c_int32, C.c_int32,
                                 C.POINTER(PlanView)]
    L.etc_plan_free.argtypes = [C.POINTER(PlanView)]
    L.etc_rowsum_launch_noalloc.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
    L.etc_graph_user_fn_count.argtypes = [C.POINTER(C.c_int32)]
    return L


def _model_desc(s) -> ModelDesc:
    return ModelDesc(n_layers=s.n_layers, hidden=s.H, n_q_heads=s.nq, n_kv_heads=s.nkv, head_dim=s.d, ffn=s.F,
                     n_experts=s.n_experts, top_k=s.top_k, moe_ffn=s.moe_F, page_size=s.page, rms_eps=s.eps,
                     rope_theta=s.theta, qk_norm=1 if getattr(s, "qk_norm", False) else 0,
                     vocab=int(getattr(s, "vocab", 0) or 0))


def _sched_desc(kind, sampled_batches, max_kv_len, debug_flags=0, spin_budget=0, n_queues=0) -> SchedDesc:
    sb = sorted(int(b) for b in sampled_batches)
    sd = SchedDesc(kind=kind, n_sampled=len(sb), max_batch=sb[-1], max_kv_len=max_kv_len, spin_budget=spin_budget,
                   debug_flags=debug_flags, n_queues=n_queues)
    for i, b in enumerate(sb):
        sd.sampled_batch[i] = b
    return sd


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _plan_arrays(L, view):
    try:
        def arr(ptr, n, dtype):
            if n == 0:
                return np.zeros(0, dtype=dtype)
            buf = C.cast(ptr, C.POINTER(C.c_char * (n * np.dtype(dtype).itemsize))).contents
            return np.frombuffer(buf, dtype=dtype).copy()
        nq, ne, nt = view.n_queues, view.n_events, view.n_tasks
        ev_consumers = arr(view.ev_consumers, ne + 1, np.int32)
        return {"tasks": arr(view.tasks, nt, TASK_DTYPE), "queue_tasks": arr(view.queue_tasks, nt, TASK_DTYPE),
                "queue_begin": arr(view.queue_begin, nq + 1, np.int32), "ev_init": arr(view.ev_init, ne, np.int32),
                "ev_consumers": ev_consumers, "consumer_ids": arr(view.consumer_ids, int(ev_consumers[-1]), np.int32),
                "seed_tasks": arr(view.seed_tasks, view.n_seed, np.int32)}
    finally:
        L.etc_plan_free(C.byref(view))


def plan_build(shape, kv_chunk_tokens, sampled_batch, n_queues, max_kv_len, kind=SCHED_STATIC, moe_tile_m=16):
    """Host-only: the materialised plan of one sampled batch size as numpy arrays (copies)."""
    L = lib()
    view = PlanView()
    md, td = _model_desc(shape), TileDesc(kv_chunk_tokens, moe_tile_m)
    sd = _sched_desc(kind, [sampled_batch], max_kv_len)
    st = L.etc_plan_build(C.byref(md), C.byref(td), C.byref(sd), sampled_batch, n_queues, C.byref(view))
    if st != 0:
        raise EtcError(st, L.etc_last_error(None).decode())
    return _plan_arrays(L, view)


def moe_layer_plan_build(shape, sampled_tokens, n_queues, kind=SCHED_STATIC, moe_tile_m=16):
    """Host-only: the plan of the stand-alone MoE layer for one sampled token count."""
    L = lib()
    view = PlanView()
    md, td = _model_desc(shape), TileDesc(16, moe_tile_m)
    sd = _sched_desc(kind, [sampled_tokens], 1)
    st = L.etc_moe_layer_plan_build(C.byref(md), C.byref(td), C.byref(sd), sampled_tokens, n_queues, C.byref(view))
    if st != 0:
        raise EtcError(st, L.etc_last_error(None).decode())
    return _plan_arrays(L, view)


class _Ctx:
    def __init__(self, library: str = None):
        self._L = lib() if library is None else load_library(library)
        self._h = C.c_void_p()

    def _check(self, st: int):
        if st != 0:
            raise EtcError(st, self._L.etc_last_error(self._h).decode())

    def close(self):
        if self._h:
            self._L.etc_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def read_debug(self, kind: int, layer: int, out: np.ndarray) -> np.ndarray:
        self._check(self._L.etc_read_debug(self._h, kind, layer, out.ctypes.data, out.nbytes))
        return out

    def error_word(self):
        return self.read_debug(DBG_ERROR_WORD, 0, np.zeros(4, np.int32))


class Decoder(_Ctx):
    """describe -> bind -> launch for a decoder model (see include/etc.h)."""

    def __init__(self, shape, kv_chunk_tokens: int, sampled_batches, max_kv_len: int, kind: int = SCHED_STATIC,
                 debug_flags: int = 0, spin_budget: int = 0, n_queues: int = 0, moe_tile_m: int = 16):
        super().__init__()
        self.shape = shape
        self.kind = kind
        md, td = _model_desc(shape), TileDesc(kv_chunk_tokens, moe_tile_m)
        sd = _sched_desc(kind, sampled_batches, max_kv_len, debug_flags, spin_budget, n_queues)
        st = self._L.etc_create(C.byref(md), C.byref(td), C.byref(sd), C.byref(self._h))
        if st != 0:
            raise EtcError(st, self._L.etc_last_error(None).decode())
        self._keep = []
        self.batch = 0

    def bind_layer_weights(self, layer: int, tensors: dict):
        """tensors: name -> torch bf16 CUDA tensor (names as in etc_layer_weights)."""
        lw = LayerWeights()
        for name, t in tensors.items():
            assert t.is_cuda and t.is_contiguous() and t.element_size() == 2, name
            setattr(lw, name, t.data_ptr())
        self._keep.append(tensors)
        self._check(self._L.etc_bind_layer_weights(self._h, layer, C.byref(lw)))

    def bind_kv_pool(self, k_pages, v_pages):
        """k_pages / v_pages: torch bf16 CUDA tensors [n_layers, pages, page, nkv, d]."""
        assert k_pages.is_cuda and k_pages.is_contiguous() and v_pages.is_contiguous()
        assert k_pages.shape == v_pages.shape and k_pages.shape[0] == self.shape.n_layers
        self._keep.append((k_pages, v_pages))
        self._check(self._L.etc_bind_kv_pool(self._h, k_pages.data_ptr(), v_pages.data_ptr(), k_pages.shape[1]))

    def bind_step(self, step):
        kv, ip, ids = _i32(step.kv_len), _i32(step.page_indptr), _i32(step.page_ids)
        assert len(kv) == step.batch and len(ip) == step.batch + 1 and len(ids) >= ip[-1]
        self._check(self._L.etc_bind_step(self._h, step.batch, kv.ctypes.data, ip.ctypes.data, ids.ctypes.data))
        self.batch = step.batch

    def force_routing(self, layer: int, ids, weights=None):
        if ids is None:
            self._check(self._L.etc_force_routing(self._h, layer, None, None))
        else:
            a = _i32(ids)
            w = None if weights is None else np.ascontiguousarray(weights, dtype=np.float32)
            self._check(self._L.etc_force_routing(self._h, layer, a.ctypes.data, None if w is None else w.ctypes.data))

    def launch(self, hidden_in, hidden_out, stream=None):
        self._check(self._L.etc_launch(self._h, hidden_in.data_ptr(), hidden_out.data_ptr(), _stream_ptr(stream)))

    def launch_kernel_by_kernel(self, hidden_in, hidden_out, stream=None):
        self._check(self._L.etc_launch_kernel_by_kernel(self._h, hidden_in.data_ptr(), hidden_out.data_ptr(),
                                                        _stream_ptr(stream)))

    def bind_lm_head(self, embed, g_final, w_lm):
        """torch bf16 CUDA tensors: embed [vocab, hidden] or None, g_final [hidden], w_lm [vocab, hidden]."""
        for t in (embed, g_final, w_lm):
            assert t is None or (t.is_cuda and t.is_contiguous() and t.element_size() == 2)
        self._keep.append((embed, g_final, w_lm))
        self._check(self._L.etc_bind_lm_head(self._h, None if embed is None else embed.data_ptr(), g_final.data_ptr(),
                                             w_lm.data_ptr()))

    def launch_tokens(self, token_out, token_in=None, hidden_in=None, logits_out=None, hidden_out=None, stream=None,
                      kernel_by_kernel=False):
        """One whole decode iteration (embedding or hidden state in, greedy token and logits out)."""
        ptr = lambda t: None if t is None else t.data_ptr()      # noqa: E731
        assert token_out.dtype.itemsize == 4 and (token_in is None or token_in.dtype.itemsize == 4)
        assert logits_out is None or (logits_out.dtype.itemsize == 4 and logits_out.is_contiguous())
        fn = self._L.etc_launch_tokens_kernel_by_kernel if kernel_by_kernel else self._L.etc_launch_tokens
        self._check(fn(self._h, ptr(token_in), ptr(hidden_in), ptr(token_out), ptr(logits_out), ptr(hidden_out),
                       _stream_ptr(stream)))

    def step_info(self) -> StepInfo:
        info = StepInfo()
        self._check(self._L.etc_get_step_info(self._h, C.byref(info)))
        return info

    # evidence / debug
    def event_counters(self):
        return self.read_debug(DBG_EVENT_COUNTERS, 0, np.zeros(self.step_info().n_events, np.int32))

    def exec_counts(self):
        return self.read_debug(DBG_TASK_EXEC_COUNT, 0, np.zeros(self.step_info().n_tasks, np.int32))

    def task_trace(self):
        """uint64 [n_tasks, 8] device wall-clock marks of the last launch (needs DEBUG_TRACE)."""
        return self.read_debug(DBG_TASK_TRACE, 0, np.zeros((self.step_info().n_tasks, 8), np.uint64))

    def layer_hidden(self, layer: int):
        return self.read_debug(DBG_LAYER_HIDDEN, layer, np.zeros((self.batch, self.shape.H), np.float32))

    def routing_debug(self, kind: int, layer: int, shape, dtype):
        return self.read_debug(kind, layer, np.zeros(shape, dtype))


def rowsum_launch_noalloc(A, Cout, n: int, stream=None):
    """etc_rowsum_launch_noalloc: A fp32 [n*32, 128], Cout fp32 [n*32], CUDA tensors; allocates nothing."""
    L = lib()
    st = L.etc_rowsum_launch_noalloc(A.data_ptr(), Cout.data_ptr(), n, _stream_ptr(stream))
    if st != 0:
        raise EtcError(st, L.etc_last_error(None).decode())


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


class MoeLayer(Decoder):
    """The MoE layer on its own over a block of tokens: describe -> bind -> launch (include/etc.h).  Launches, forced
    routing and the routing dumps are the decoder's calls on layer 0."""

    def __init__(self, shape, sampled_tokens, kind: int = SCHED_STATIC, debug_flags: int = 0, spin_budget: int = 0,
                 n_queues: int = 0, moe_tile_m: int = 16):
        _Ctx.__init__(self)
        self.shape = shape
        self.kind = kind
        md, td = _model_desc(shape), TileDesc(16, moe_tile_m)
        sd = _sched_desc(kind, sampled_tokens, 1, debug_flags, spin_budget, n_queues)
        st = self._L.etc_moe_layer_create(C.byref(md), C.byref(td), C.byref(sd), C.byref(self._h))
        if st != 0:
            raise EtcError(st, self._L.etc_last_error(None).decode())
        self._keep = []
        self.batch = 0

    def bind_weights(self, tensors: dict):
        """tensors: g2, wr, eg, eu, ed as torch bf16 CUDA tensors."""
        self.bind_layer_weights(0, {k: tensors[k] for k in ("g2", "wr", "eg", "eu", "ed")})

    def bind_tokens(self, n_tokens: int):
        self._check(self._L.etc_moe_layer_bind_tokens(self._h, n_tokens))
        self.batch = n_tokens


class EventGraph(_Ctx):
    """Generic event-tensor graph (row-sum example of the paper's Sec. 2.2)."""

    def __init__(self, kind: int = SCHED_STATIC, debug_flags: int = 0, spin_budget: int = 0, n_queues: int = 0,
                 library: str = None):
        super().__init__(library)
        sd = _sched_desc(kind, [1], 1, debug_flags, spin_budget, n_queues)
        st = self._L.etc_graph_create(C.byref(sd), C.byref(self._h))
        if st != 0:
            raise EtcError(st, self._L.etc_last_error(None).decode())
        self._keep = []

    @staticmethod
    def dim(sym=-1, mul=0, add=0) -> DimExpr:
        return DimExpr(sym, mul, add)

    @staticmethod
    def edge(event: int, maps) -> Edge:
        """maps: one (kind, src, div) per event dimension."""
        e = Edge(event=event, rank=len(maps))
        for r, (k, s, d) in enumerate(maps):
            e.kind[r], e.src[r], e.div[r] = k, s, d
        return e

    def add_event(self, shape) -> int:
        arr = (DimExpr * len(shape))(*shape)
        eid = C.c_int32()
        self._check(self._L.etc_graph_add_event(self._h, arr, len(shape), C.byref(eid)))
        return eid.value

    def add_call(self, fn: int, task_shape, in_edges=(), out_edges=()):
        arr = (DimExpr * len(task_shape))(*task_shape)
        ins = (Edge * max(1, len(in_edges)))(*in_edges)
        outs = (Edge * max(1, len(out_edges)))(*out_edges)
        self._check(self._L.etc_graph_add_call(self._h, fn, arr, len(task_shape), ins, len(in_edges), outs,
                                               len(out_edges)))

    def bind_buffer(self, slot: int, tensor):
        assert tensor.is_cuda and tensor.is_contiguous()
        self._keep.append(tensor)
        self._check(self._L.etc_graph_bind_buffer(self._h, slot, tensor.data_ptr(), tensor.numel() * tensor.element_size()))

    def bind_shape(self, values):
        v = _i32(list(values) + [0] * (4 - len(values)))
        self._check(self._L.etc_graph_bind_shape(self._h, v.ctypes.data))

    def launch(self, stream=None):
        self._check(self._L.etc_graph_launch(self._h, _stream_ptr(stream)))

    def step_info(self) -> StepInfo:
        info = StepInfo()
        self._check(self._L.etc_get_step_info(self._h, C.byref(info)))
        return info

    def event_counters(self):
        return self.read_debug(DBG_EVENT_COUNTERS, 0, np.zeros(self.step_info().n_events, np.int32))

    def exec_counts(self):
        return self.read_debug(DBG_TASK_EXEC_COUNT, 0, np.zeros(self.step_info().n_tasks, np.int32))
