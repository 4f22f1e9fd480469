"""CPU oracle of the decode step  --  TEST INFRASTRUCTURE, never the product path.

ctypes front-end of ``decode_oracle.c`` (operator-level definition of one
decoder layer, fp32 storage / double accumulation) plus a driver that chains
layers.  Only tests, the smoke check and the benchmark's cpu_baseline leg may
import this package; the HIP library and its Python binding never do.
"""
from __future__ import annotations

import ctypes
import functools
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")

_f32p = ctypes.POINTER(ctypes.c_float)
_i32p = ctypes.POINTER(ctypes.c_int32)


class OrcShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("H", "nq", "nkv", "d", "F", "page", "n_experts", "top_k", "moe_F", "tile_m")] + \
               [("eps", ctypes.c_float), ("theta", ctypes.c_float), ("qk_norm", ctypes.c_int32)]


class OrcDebug(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("q_rot", "k_rot", "v_new", "attn", "x_mid", "act", "router_logits", "topk_w")]


def build(force: bool = False) -> str:
    """Compile decode_oracle.c into liboracle.so (gcc, OpenMP, no fast-math)."""
    src = os.path.join(_HERE, "decode_oracle.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC",
                               "-o", _LIB_PATH, src, "-lm"])
    return _LIB_PATH


@functools.lru_cache(maxsize=1)
def lib():
    build()
    L = ctypes.CDLL(_LIB_PATH)
    L.orc_silu.restype = ctypes.c_double
    L.orc_silu.argtypes = [ctypes.c_double]
    for name in ("orc_rmsnorm", "orc_linear", "orc_rope", "orc_attention", "orc_topk",
                 "orc_route_weights", "orc_group", "orc_layer", "orc_lm_head", "orc_moe_layer"):
        getattr(L, name).restype = None
    return L


def n_threads() -> int:
    """Threads the OpenMP loops of the oracle use."""
    env = os.environ.get("OMP_NUM_THREADS")
    return int(env) if env else (os.cpu_count() or 1)


def shape_of(s, tile_m: int = 16) -> OrcShape:
    """OrcShape from any object with the model-shape attribute names."""
    return OrcShape(H=s.H, nq=s.nq, nkv=s.nkv, d=s.d, F=s.F, page=s.page, n_experts=s.n_experts,
                    top_k=s.top_k, moe_F=s.moe_F, tile_m=tile_m, eps=s.eps, theta=s.theta,
                    qk_norm=1 if getattr(s, "qk_norm", False) else 0)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def rmsnorm(x, g, eps):
    x, g = _f(x), _f(g)
    y = np.empty_like(x)
    lib().orc_rmsnorm(_p(x), _p(g), ctypes.c_int(x.size), ctypes.c_float(eps), _p(y))
    return y


def linear(W, X):
    W, X = _f(W), _f(X)
    X2 = X.reshape(-1, X.shape[-1])
    B, K = X2.shape
    N = W.shape[0]
    assert W.shape[1] == K
    Y = np.empty((B, N), dtype=np.float32)
    lib().orc_linear(_p(W), _p(X2), ctypes.c_int(B), ctypes.c_int(N), ctypes.c_int(K), _p(Y))
    return Y.reshape(X.shape[:-1] + (N,))


def rope(v, pos, theta):
    v = _f(v).copy()
    n_heads, d = v.shape
    lib().orc_rope(_p(v), ctypes.c_int(n_heads), ctypes.c_int(d), ctypes.c_int(pos), ctypes.c_float(theta))
    return v


def silu(z: float) -> float:
    return lib().orc_silu(float(z))


def attention(shape: OrcShape, q, kpool, vpool, pages, n_keys):
    q, kpool, vpool = _f(q), _f(kpool), _f(vpool)
    pages = np.ascontiguousarray(pages, dtype=np.int32)
    out = np.empty_like(q)
    lib().orc_attention(ctypes.byref(shape), _p(q), _p(kpool), _p(vpool), _p(pages), ctypes.c_int(n_keys),
                        _p(out))
    return out


def topk(logits, K):
    logits = _f(logits)
    ids = np.empty(K, dtype=np.int32)
    lib().orc_topk(_p(logits), ctypes.c_int(logits.size), ctypes.c_int(K), _p(ids))
    return ids


def route_weights(logits, ids):
    logits = _f(logits)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    w = np.empty(ids.size, dtype=np.float32)
    lib().orc_route_weights(_p(logits), _p(ids), ctypes.c_int(ids.size), _p(w))
    return w


def group(topk_ids, E, tile_m):
    """-> count[E], tok_indptr[E+1], perm[B*K], exp_indptr[E+1] (all int32)."""
    ids = np.ascontiguousarray(topk_ids, dtype=np.int32)
    B, K = ids.shape
    count = np.empty(E, dtype=np.int32)
    tok_indptr = np.empty(E + 1, dtype=np.int32)
    perm = np.empty(B * K, dtype=np.int32)
    exp_indptr = np.empty(E + 1, dtype=np.int32)
    lib().orc_group(_p(ids), ctypes.c_int(B), ctypes.c_int(K), ctypes.c_int(E), ctypes.c_int(tile_m),
                    _p(count), _p(tok_indptr), _p(perm), _p(exp_indptr))
    return count, tok_indptr, perm, exp_indptr


_DBG_SHAPES = {"q_rot": lambda s, B: (B, s.nq * s.d), "k_rot": lambda s, B: (B, s.nkv * s.d),
               "v_new": lambda s, B: (B, s.nkv * s.d), "attn": lambda s, B: (B, s.nq * s.d),
               "x_mid": lambda s, B: (B, s.H), "act": lambda s, B: (B, max(s.F, 1)),
               "router_logits": lambda s, B: (B, max(s.n_experts, 1)),
               "topk_w": lambda s, B: (B, max(s.top_k, 1))}


def layer(shape: OrcShape, x, w: dict, kpool, vpool, kv_len, page_indptr, page_ids,
          forced_topk=None, debug: bool = False):
    """Run one decoder layer.  x [B, H] fp32 is updated in place; pools (fp32,
    [page, slot, nkv, d]) receive the appended rows.  Returns (topk_ids | None,
    debug dict | None)."""
    assert x.dtype == np.float32 and x.flags.c_contiguous
    assert kpool.dtype == np.float32 and kpool.flags.c_contiguous
    assert vpool.dtype == np.float32 and vpool.flags.c_contiguous
    B = x.shape[0]
    ww = {k: _f(v) for k, v in w.items()}
    kv_len = np.ascontiguousarray(kv_len, dtype=np.int32)
    page_indptr = np.ascontiguousarray(page_indptr, dtype=np.int32)
    page_ids = np.ascontiguousarray(page_ids, dtype=np.int32)
    ids = None
    force = 0
    if shape.n_experts:
        if forced_topk is not None:
            ids = np.ascontiguousarray(forced_topk, dtype=np.int32).copy()
            force = 1
        else:
            ids = np.empty((B, shape.top_k), dtype=np.int32)
    dbg_arrays, dbg_struct = None, None
    if debug:
        dbg_arrays = {k: np.zeros(f(shape, B), dtype=np.float32) for k, f in _DBG_SHAPES.items()}
        dbg_struct = OrcDebug(**{k: v.ctypes.data for k, v in dbg_arrays.items()})
    g = lambda name: _p(ww.get(name))  # noqa: E731
    lib().orc_layer(ctypes.byref(shape), ctypes.c_int(B), _p(x), g("g1"), g("wq"), g("wk"), g("wv"),
                    g("wo"), g("g2"), g("wg"), g("wu"), g("wd"), g("wr"), g("eg"), g("eu"), g("ed"),
                    g("gq"), g("gk"), _p(kpool), _p(vpool), _p(kv_len), _p(page_indptr), _p(page_ids), ctypes.c_int(force),
                    _p(ids), ctypes.byref(dbg_struct) if debug else None)
    return ids, dbg_arrays


def moe_layer(shape: OrcShape, x, w: dict, forced_topk=None):
    """The MoE layer on its own: x <- x + MoE(rmsnorm(x, g2)) for T tokens (paper Sec. 2.4; measured over 1 .. 4096
    tokens in Sec. 4.2 / 4.5).  x [T, H]; w holds g2, wr, eg, eu, ed.  Returns (y [T, H] fp32, top-k ids [T, K] int32,
    router logits [T, E] fp32, routing weights [T, K] fp32)."""
    y = np.array(x, dtype=np.float32, copy=True, order="C")
    T = y.shape[0]
    ww = {k: _f(v) for k, v in w.items()}
    force = 0
    if forced_topk is not None:
        ids = np.ascontiguousarray(forced_topk, dtype=np.int32).copy()
        force = 1
    else:
        ids = np.empty((T, shape.top_k), dtype=np.int32)
    logits = np.empty((T, shape.n_experts), dtype=np.float32)
    tw = np.empty((T, shape.top_k), dtype=np.float32)
    lib().orc_moe_layer(ctypes.byref(shape), ctypes.c_int(T), _p(y), _p(ww["g2"]), _p(ww["wr"]), _p(ww["eg"]), _p(ww["eu"]),
                        _p(ww["ed"]), ctypes.c_int(force), _p(ids), _p(logits), _p(tw))
    return y, ids, logits, tw


def embed(table, tokens):
    """Start of a decode iteration: the hidden state of each sequence is the embedding row of its token
    (paper Sec. 4.2 measures whole iterations, token in, token out).  table [V, H], tokens [B] -> [B, H] fp32."""
    table, tokens = _f(table), np.asarray(tokens, dtype=np.int64)
    assert tokens.min() >= 0 and tokens.max() < table.shape[0]
    return np.stack([table[int(t)] for t in tokens]).astype(np.float32)


def lm_head(shape: OrcShape, x, gf, wlm):
    """Final RMSNorm, vocabulary projection and greedy arg-max.  x [B, H], gf [H], wlm [V, H] ->
    (logits [B, V] fp32, token ids [B] int32)."""
    x, gf, wlm = _f(x), _f(gf), _f(wlm)
    B, V = x.shape[0], wlm.shape[0]
    logits = np.empty((B, V), dtype=np.float32)
    token = np.empty(B, dtype=np.int32)
    lib().orc_lm_head(ctypes.byref(shape), ctypes.c_int(B), _p(x), _p(gf), _p(wlm), ctypes.c_int(V), _p(logits), _p(token))
    return logits, token


def decode_step(s, n_layers, x0, weights_of, pools_of, step, forced_topk_of=None, tile_m: int = 16,
                keep_layers: bool = True):
    """Chain n_layers layers.  ``weights_of(layer)`` -> dict of fp32 arrays,
    ``pools_of(layer)`` -> (kpool, vpool) fp32 (modified in place), ``step`` has
    kv_len / page_indptr / page_ids.  Returns dict(final, layers[list of x after
    each layer], topk[list]).
    """
    shape = shape_of(s, tile_m)
    x = np.array(x0, dtype=np.float32, copy=True, order="C")
    per_layer, topks = [], []
    for l in range(n_layers):
        kp, vp = pools_of(l)
        forced = forced_topk_of(l) if forced_topk_of is not None else None
        ids, _ = layer(shape, x, weights_of(l), kp, vp, step.kv_len, step.page_indptr, step.page_ids,
                       forced_topk=forced)
        if keep_layers:
            per_layer.append(x.copy())
        topks.append(ids)
    return {"final": x, "layers": per_layer, "topk": topks}
