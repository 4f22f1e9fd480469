"""Pins of the operator-level CPU oracle against things other than itself:
closed forms, invariants, library routines (torch CPU / scipy in float64), a
hand-evaluated layer, brute force on tiny routings.  Each pin is chosen so that a
plausible slip (dropped term, wrong sign or index, transposed operand) fails it.
"""
import itertools
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

import oracle
from synth import ModelShape, Step, pages_needed

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(1234)


def r32(*shape, scale=1.0):
    return (rng.standard_normal(shape) * scale).astype(np.float32)


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_constant_vector_closed_form():
    H, c, eps = 64, 3.0, 1e-5
    g = r32(H)
    y = oracle.rmsnorm(np.full(H, c, np.float32), g, eps)
    np.testing.assert_allclose(y, g * c / np.sqrt(c * c + eps), rtol=1e-6)


def test_rmsnorm_unit_rms_and_scale_invariance():
    x = r32(512)
    y = oracle.rmsnorm(x, np.ones(512, np.float32), 0.0)
    assert abs(np.sqrt(np.mean(y.astype(np.float64) ** 2)) - 1.0) < 1e-6
    np.testing.assert_allclose(oracle.rmsnorm(7.5 * x, np.ones(512, np.float32), 0.0), y, rtol=2e-6)


def test_rmsnorm_matches_torch_library():
    x, g = r32(256), r32(256)
    ref = Fn.rms_norm(torch.from_numpy(x).double(), (256,), torch.from_numpy(g).double(), eps=1e-5)
    np.testing.assert_allclose(oracle.rmsnorm(x, g, 1e-5), ref.numpy(), rtol=1e-6, atol=1e-7)


# ---------------------------------------------------------------- linear
def test_linear_identity_onehot_and_orientation():
    X = r32(3, 8)
    np.testing.assert_array_equal(oracle.linear(np.eye(8, dtype=np.float32), X), X)
    W = r32(5, 8)                       # [out, in]: a one-hot input picks a COLUMN of W
    e2 = np.zeros((1, 8), np.float32)
    e2[0, 2] = 1.0
    np.testing.assert_array_equal(oracle.linear(W, e2)[0], W[:, 2])


def test_linear_matches_float64_matmul():
    W, X = r32(37, 129), r32(4, 129)
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    np.testing.assert_allclose(oracle.linear(W, X), ref, rtol=1e-6, atol=1e-6)


# ---------------------------------------------------------------- RoPE
def test_rope_position_zero_is_identity():
    v = r32(3, 16)
    np.testing.assert_array_equal(oracle.rope(v, 0, 10000.0), v)


def test_rope_onehot_closed_form_pairs_i_with_i_plus_half():
    d, theta, pos = 8, 10000.0, 5
    for i in range(d // 2):
        v = np.zeros((1, d), np.float32)
        v[0, i] = 1.0
        ang = pos * theta ** (-2.0 * i / d)
        exp = np.zeros(d)
        exp[i], exp[i + d // 2] = np.cos(ang), np.sin(ang)
        np.testing.assert_allclose(oracle.rope(v, pos, theta)[0], exp, atol=1e-6)
        v2 = np.zeros((1, d), np.float32)
        v2[0, i + d // 2] = 1.0
        exp2 = np.zeros(d)
        exp2[i], exp2[i + d // 2] = -np.sin(ang), np.cos(ang)
        np.testing.assert_allclose(oracle.rope(v2, pos, theta)[0], exp2, atol=1e-6)


def test_rope_norm_additivity_and_relative_position():
    d, theta = 32, 10000.0
    q, k = r32(1, d), r32(1, d)
    half = d // 2
    rq = oracle.rope(q, 17, theta)
    np.testing.assert_allclose(rq[0, :half] ** 2 + rq[0, half:] ** 2, q[0, :half] ** 2 + q[0, half:] ** 2,
                               rtol=1e-5)
    np.testing.assert_allclose(oracle.rope(oracle.rope(q, 5, theta), 12, theta), rq, atol=1e-5)
    # <rope(q, m), rope(k, n)> depends on m - n only
    a = float(oracle.rope(q, 40, theta)[0].astype(np.float64) @ oracle.rope(k, 33, theta)[0].astype(np.float64))
    b = float(oracle.rope(q, 7, theta)[0].astype(np.float64) @ k[0].astype(np.float64))
    assert abs(a - b) < 1e-4


# ---------------------------------------------------------------- SiLU
def test_silu_known_values():
    assert oracle.silu(0.0) == 0.0
    assert abs(oracle.silu(1.0) - 0.7310585786300049) < 1e-15
    assert abs(oracle.silu(-1.0) + 0.2689414213699951) < 1e-15
    assert abs(oracle.silu(30.0) - 30.0) < 1e-11
    z = np.linspace(-6, 6, 25)
    ref = Fn.silu(torch.from_numpy(z)).numpy()
    np.testing.assert_allclose([oracle.silu(v) for v in z], ref, rtol=1e-12, atol=1e-15)


# ---------------------------------------------------------------- attention
def _attn_setup(nq=4, nkv=2, d=16, page=4, n_keys=11, n_pool=9):
    s = ModelShape("t", 1, nq * d, nq, nkv, d, 32, page=page)
    sh = oracle.shape_of(s)
    kpool, vpool = r32(n_pool, page, nkv, d), r32(n_pool, page, nkv, d)
    pages = rng.permutation(n_pool)[: (n_keys + page - 1) // page].astype(np.int32)
    return s, sh, kpool, vpool, pages


def _contiguous(pool, pages, n_keys):
    return np.concatenate([pool[p] for p in pages])[:n_keys]      # [n_keys, nkv, d]


def test_attention_matches_torch_sdpa_with_grouped_heads():
    s, sh, kpool, vpool, pages = _attn_setup()
    n_keys = 11
    q = r32(s.nq, s.d)
    out = oracle.attention(sh, q, kpool, vpool, pages, n_keys)
    K = torch.from_numpy(_contiguous(kpool, pages, n_keys)).double().permute(1, 0, 2)   # [nkv, n, d]
    V = torch.from_numpy(_contiguous(vpool, pages, n_keys)).double().permute(1, 0, 2)
    g = s.nq // s.nkv
    K, V = K.repeat_interleave(g, dim=0), V.repeat_interleave(g, dim=0)                # head h -> kv head h // g
    ref = Fn.scaled_dot_product_attention(torch.from_numpy(q).double()[:, None, :], K, V)[:, 0, :]
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-5, atol=1e-6)


def test_attention_zero_query_gives_mean_value_and_single_key_gives_v():
    s, sh, kpool, vpool, pages = _attn_setup()
    out = oracle.attention(sh, np.zeros((s.nq, s.d), np.float32), kpool, vpool, pages, 11)
    V = _contiguous(vpool, pages, 11).astype(np.float64)
    for h in range(s.nq):
        np.testing.assert_allclose(out[h], V[:, h // (s.nq // s.nkv)].mean(0), rtol=1e-5, atol=1e-6)
    out1 = oracle.attention(sh, r32(s.nq, s.d), kpool, vpool, pages, 1)
    for h in range(s.nq):
        np.testing.assert_allclose(out1[h], vpool[pages[0], 0, h // (s.nq // s.nkv)], rtol=1e-6)


def test_attention_is_invariant_to_physical_page_placement():
    s, sh, kpool, vpool, pages = _attn_setup()
    q = r32(s.nq, s.d)
    a = oracle.attention(sh, q, kpool, vpool, pages, 11)
    perm = rng.permutation(kpool.shape[0])
    k2, v2 = np.empty_like(kpool), np.empty_like(vpool)
    k2[perm], v2[perm] = kpool, vpool                       # page p moves to perm[p]
    b = oracle.attention(sh, q, k2, v2, perm[pages].astype(np.int32), 11)
    np.testing.assert_array_equal(a, b)


def test_attention_dominant_key_selects_its_value():
    s, sh, kpool, vpool, pages = _attn_setup(nq=2, nkv=1)
    q = r32(s.nq, s.d)
    kpool[pages[1], 2, 0] = 50.0 * q[0] / np.linalg.norm(q[0])   # key index 1*4+2 = 6 aligned with q_0
    out = oracle.attention(sh, q, kpool, vpool, pages, 11)
    np.testing.assert_allclose(out[0], vpool[pages[1], 2, 0], atol=1e-3)


# ---------------------------------------------------------------- MoE integers
def test_topk_tie_break_and_lexsort_agreement():
    np.testing.assert_array_equal(oracle.topk(np.zeros(8, np.float32), 3), [0, 1, 2])
    lg = np.array([0.5, 2.0, 2.0, -1.0, 2.0, 0.5], np.float32)
    np.testing.assert_array_equal(oracle.topk(lg, 5), [1, 2, 4, 0, 5])
    for _ in range(50):
        lg = np.round(r32(16), 1)                      # rounded -> plenty of ties
        np.testing.assert_array_equal(oracle.topk(lg, 6), np.lexsort((np.arange(16), -lg))[:6])


def test_route_weights_are_softmax_over_selected():
    from scipy.special import softmax
    lg = r32(16)
    ids = oracle.topk(lg, 4)
    w = oracle.route_weights(lg, ids)
    assert abs(float(w.sum()) - 1.0) < 1e-6
    np.testing.assert_allclose(w, softmax(lg[ids].astype(np.float64)), rtol=1e-6)
    # softmax over everything, then renormalised over the selected ones: the same numbers
    p = softmax(lg.astype(np.float64))
    np.testing.assert_allclose(w, p[ids] / p[ids].sum(), rtol=1e-6)


def test_group_brute_force_on_every_tiny_routing():
    B, K, E, tile_m = 3, 2, 3, 2
    pairs = [p for p in itertools.permutations(range(E), K)]
    for combo in itertools.product(pairs, repeat=B):
        ids = np.array(combo, dtype=np.int32)
        count, tok_indptr, perm, exp_indptr = oracle.group(ids, E, tile_m)
        flat = sorted(range(B * K), key=lambda i: (ids[i // K, i % K], i // K, i % K))
        np.testing.assert_array_equal(perm, flat)
        np.testing.assert_array_equal(count, np.bincount(ids.ravel(), minlength=E))
        assert count.sum() == B * K and tok_indptr[0] == 0 and exp_indptr[0] == 0
        np.testing.assert_array_equal(np.diff(tok_indptr), count)
        np.testing.assert_array_equal(np.diff(exp_indptr), -(-count // tile_m))


# ---------------------------------------------------------------- whole layer
def _tiny(moe=False, **kw):
    base = dict(name="t", n_layers=1, H=32, nq=4, nkv=2, d=8, F=48, page=4)
    if moe:
        base.update(F=0, n_experts=6, top_k=2, moe_F=24)
    base.update(kw)
    return ModelShape(**base)


def _weights(s, scale=0.2):
    w = {"g1": 1 + r32(s.H, scale=0.02), "g2": 1 + r32(s.H, scale=0.02),
         "wq": r32(s.nq * s.d, s.H, scale=scale), "wk": r32(s.nkv * s.d, s.H, scale=scale),
         "wv": r32(s.nkv * s.d, s.H, scale=scale), "wo": r32(s.H, s.nq * s.d, scale=scale)}
    if getattr(s, "qk_norm", False):
        w.update(gq=1 + r32(s.d, scale=0.1), gk=1 + r32(s.d, scale=0.1))
    if s.is_moe:
        w.update(wr=r32(s.n_experts, s.H), eg=r32(s.n_experts, s.moe_F, s.H, scale=scale),
                 eu=r32(s.n_experts, s.moe_F, s.H, scale=scale), ed=r32(s.n_experts, s.H, s.moe_F, scale=scale))
    else:
        w.update(wg=r32(s.F, s.H, scale=scale), wu=r32(s.F, s.H, scale=scale), wd=r32(s.H, s.F, scale=scale))
    return w


def _step(s, kv_len, n_pool):
    kv_len = np.asarray(kv_len, np.int32)
    npg = [pages_needed(int(l), s.page) for l in kv_len]
    indptr = np.concatenate([[0], np.cumsum(npg)]).astype(np.int32)
    ids = rng.permutation(n_pool)[: indptr[-1]].astype(np.int32)
    return Step(len(kv_len), kv_len, indptr, ids)


def _library_layer(s, x, w, kpool, vpool, step, topk_ids=None):
    """The layer written a second, independent way: float64 torch library calls."""
    T = lambda a: torch.from_numpy(np.asarray(a)).double()  # noqa: E731
    out = []
    g = s.nq // s.nkv
    for b in range(step.batch):
        pos = int(step.kv_len[b])
        xb = T(x[b])
        xn = Fn.rms_norm(xb, (s.H,), T(w["g1"]), eps=s.eps)
        q = (T(w["wq"]) @ xn).view(s.nq, s.d)
        k = (T(w["wk"]) @ xn).view(s.nkv, s.d)
        v = (T(w["wv"]) @ xn).view(s.nkv, s.d)
        if getattr(s, "qk_norm", False):      # per-head RMSNorm over head_dim, one gain for all q heads, one for all k heads
            q = Fn.rms_norm(q, (s.d,), T(w["gq"]), eps=s.eps)
            k = Fn.rms_norm(k, (s.d,), T(w["gk"]), eps=s.eps)
        inv = s.theta ** (-torch.arange(0, s.d, 2).double() / s.d)
        cos, sin = torch.cos(pos * inv), torch.sin(pos * inv)

        def rot(t):
            a, c = t[:, : s.d // 2], t[:, s.d // 2:]
            return torch.cat([a * cos - c * sin, a * sin + c * cos], dim=1)
        q, k = rot(q), rot(k)
        pages = step.page_ids[step.page_indptr[b]:step.page_indptr[b + 1]]
        Kc = torch.cat([T(kpool[p]) for p in pages])[:pos]
        Vc = torch.cat([T(vpool[p]) for p in pages])[:pos]
        Kc = torch.cat([Kc, k[None]]).permute(1, 0, 2).repeat_interleave(g, 0)
        Vc = torch.cat([Vc, v[None]]).permute(1, 0, 2).repeat_interleave(g, 0)
        o = Fn.scaled_dot_product_attention(q[:, None, :], Kc, Vc)[:, 0, :].reshape(-1)
        xm = xb + T(w["wo"]) @ o
        xn2 = Fn.rms_norm(xm, (s.H,), T(w["g2"]), eps=s.eps)
        if not s.is_moe:
            y = T(w["wd"]) @ (Fn.silu(T(w["wg"]) @ xn2) * (T(w["wu"]) @ xn2))
        else:
            lg = T(w["wr"]) @ xn2
            ids = torch.from_numpy(np.asarray(topk_ids[b])).long()
            ww = torch.softmax(lg[ids], 0)
            y = sum(ww[i] * (T(w["ed"][e]) @ (Fn.silu(T(w["eg"][e]) @ xn2) * (T(w["eu"][e]) @ xn2)))
                    for i, e in enumerate(ids.tolist()))
        out.append((xm + y).numpy())
    return np.stack(out)


@pytest.mark.parametrize("moe", [False, True])
def test_layer_matches_independent_library_derivation(moe):
    s = _tiny(moe)
    w = _weights(s)
    step = _step(s, [9, 0, 4], n_pool=8)
    kpool, vpool = r32(8, s.page, s.nkv, s.d), r32(8, s.page, s.nkv, s.d)
    x = r32(3, s.H)
    xo = x.copy()
    kp, vp = kpool.copy(), vpool.copy()
    ids, dbg = oracle.layer(oracle.shape_of(s), xo, w, kp, vp, step.kv_len, step.page_indptr, step.page_ids,
                            debug=True)
    ref = _library_layer(s, x, w, kpool, vpool, step, ids)
    np.testing.assert_allclose(xo, ref, rtol=2e-5, atol=2e-5)
    # KV append: exactly one row per sequence changed, at (page of pos, pos % page), K stored rotated
    changed = np.argwhere((kp != kpool).any(axis=(2, 3)))
    exp = sorted((int(step.page_ids[step.page_indptr[b] + step.kv_len[b] // s.page]), int(step.kv_len[b] % s.page))
                 for b in range(3))
    assert sorted(map(tuple, changed.tolist())) == exp
    for b in range(3):
        pg, sl = exp_b = (int(step.page_ids[step.page_indptr[b] + step.kv_len[b] // s.page]),
                          int(step.kv_len[b] % s.page))
        np.testing.assert_array_equal(kp[pg, sl].ravel(), dbg["k_rot"][b])
        np.testing.assert_array_equal(vp[pg, sl].ravel(), dbg["v_new"][b])
    if moe:
        for b in range(3):
            np.testing.assert_array_equal(ids[b], np.lexsort((np.arange(s.n_experts), -dbg["router_logits"][b]))[:2])


def test_hand_evaluated_layer():
    gold = dict(l.split() for l in open(os.path.join(GOLD, "hand_layer.txt")) if not l.startswith("#"))
    s = ModelShape("hand", 1, 4, 1, 1, 4, 4, page=16)
    I = np.eye(4, dtype=np.float32)
    one = np.ones(4, np.float32)
    w = dict(g1=one, g2=one, wq=I, wk=I, wv=I, wo=I, wg=I, wu=I, wd=I)
    x = np.ones((1, 4), np.float32)
    kp, vp = np.zeros((1, 16, 1, 4), np.float32), np.zeros((1, 16, 1, 4), np.float32)
    _, dbg = oracle.layer(oracle.shape_of(s), x, w, kp, vp, [0], [0, 1], [0], debug=True)
    np.testing.assert_allclose(dbg["x_mid"][0], float(gold["x_mid"]), rtol=1e-6)
    np.testing.assert_allclose(x[0], float(gold["x_out"]), rtol=1e-6)


def test_layer_with_zero_output_projections_is_identity():
    s = _tiny()
    w = _weights(s)
    w["wo"] = np.zeros_like(w["wo"])
    w["wd"] = np.zeros_like(w["wd"])
    step = _step(s, [5], n_pool=4)
    x = r32(1, s.H)
    xo = x.copy()
    oracle.layer(oracle.shape_of(s), xo, w, r32(4, s.page, s.nkv, s.d), r32(4, s.page, s.nkv, s.d),
                 step.kv_len, step.page_indptr, step.page_ids)
    np.testing.assert_array_equal(xo, x)


def test_moe_with_identical_experts_equals_dense_ffn():
    """Routing weights sum to one, so identical experts collapse the MoE block to the dense block."""
    sm = _tiny(True)
    sd = _tiny(False, F=sm.moe_F)
    w = _weights(sm)
    for nme in ("eg", "eu", "ed"):
        w[nme] = np.repeat(w[nme][:1], sm.n_experts, axis=0)
    wd = {k: v for k, v in w.items() if k in ("g1", "g2", "wq", "wk", "wv", "wo")}
    wd.update(wg=w["eg"][0], wu=w["eu"][0], wd=w["ed"][0])
    step = _step(sm, [6, 2], n_pool=6)
    kpool, vpool = r32(6, sm.page, sm.nkv, sm.d), r32(6, sm.page, sm.nkv, sm.d)
    x = r32(2, sm.H)
    a, b = x.copy(), x.copy()
    oracle.layer(oracle.shape_of(sm), a, w, kpool.copy(), vpool.copy(), step.kv_len, step.page_indptr, step.page_ids)
    oracle.layer(oracle.shape_of(sd), b, wd, kpool.copy(), vpool.copy(), step.kv_len, step.page_indptr, step.page_ids)
    np.testing.assert_allclose(a, b, rtol=1e-5, atol=1e-6)


def test_moe_forced_routing_is_followed():
    s = _tiny(True)
    w = _weights(s)
    step = _step(s, [3], n_pool=2)
    kpool, vpool = r32(2, s.page, s.nkv, s.d), r32(2, s.page, s.nkv, s.d)
    x = r32(1, s.H)
    forced = np.array([[5, 0]], np.int32)
    xo = x.copy()
    ids, _ = oracle.layer(oracle.shape_of(s), xo, w, kpool.copy(), vpool.copy(), step.kv_len, step.page_indptr,
                          step.page_ids, forced_topk=forced)
    np.testing.assert_array_equal(ids, forced)
    ref = _library_layer(s, x, w, kpool, vpool, step, forced)
    np.testing.assert_allclose(xo, ref, rtol=2e-5, atol=2e-5)


# ---------------------------------------------------------------- the layer chain (oracle.decode_step)
@pytest.mark.parametrize("moe", [False, True])
def test_decode_step_chains_layers_like_the_library_derivation(moe):
    """Three chained layers with their own weights and their own KV pools: x after layer l is the input of
    layer l+1, layer l reads and appends to pool l only.  Checked per layer against the float64 library
    derivation of one layer applied three times by hand (a chain that fed a layer the wrong input, the wrong
    layer's weights or the wrong layer's pool fails here)."""
    s = _tiny(moe, n_layers=3)
    ws = [_weights(s) for _ in range(3)]
    n_pool = 8
    step = _step(s, [9, 0, 4], n_pool=n_pool)
    pools = [(r32(n_pool, s.page, s.nkv, s.d), r32(n_pool, s.page, s.nkv, s.d)) for _ in range(3)]
    work = [(k.copy(), v.copy()) for k, v in pools]
    x = r32(3, s.H)
    res = oracle.decode_step(s, 3, x, lambda l: ws[l], lambda l: work[l], step, tile_m=4)
    assert len(res["layers"]) == 3 and len(res["topk"]) == 3
    ref = x.astype(np.float64)
    for l in range(3):
        ref = _library_layer(s, ref.astype(np.float32), ws[l], pools[l][0], pools[l][1], step,
                             res["topk"][l] if moe else None)
        np.testing.assert_allclose(res["layers"][l], ref, rtol=5e-5, atol=5e-5, err_msg=f"layer {l}")
        # every layer appended to its own pool, and only there: one row per sequence
        assert int((work[l][0] != pools[l][0]).any(axis=(2, 3)).sum()) == 3
    np.testing.assert_array_equal(res["final"], res["layers"][-1])
    assert not np.shares_memory(res["final"], x) and np.array_equal(x, x)      # the input is not overwritten
    # forced routing is handed to the right layer
    if moe:
        forced = [np.array([[0, 1], [2, 3], [4, 5]], np.int32), np.array([[5, 4], [3, 2], [1, 0]], np.int32), None]
        work2 = [(k.copy(), v.copy()) for k, v in pools]
        res2 = oracle.decode_step(s, 3, x, lambda l: ws[l], lambda l: work2[l], step,
                                  forced_topk_of=lambda l: forced[l], tile_m=4)
        np.testing.assert_array_equal(res2["topk"][0], forced[0])
        np.testing.assert_array_equal(res2["topk"][1], forced[1])
        ref = x.astype(np.float64)
        for l in range(2):
            ref = _library_layer(s, ref.astype(np.float32), ws[l], pools[l][0], pools[l][1], step, forced[l])
        np.testing.assert_allclose(res2["layers"][1], ref, rtol=5e-5, atol=5e-5)


def test_decode_steps_in_a_row_read_back_the_rows_they_appended():
    """Three consecutive steps of one sequence on the same pools (kv_len grows by one, nothing is reset): the
    second and third step attend to the rows the earlier steps appended.  Equals one library-derivation step
    per token over a contiguous cache that is extended by hand with the oracle's own rotated K / V rows."""
    s = _tiny(False)
    w = _weights(s)
    n_pool = 4
    kpool, vpool = r32(n_pool, s.page, s.nkv, s.d), r32(n_pool, s.page, s.nkv, s.d)
    kp, vp = kpool.copy(), vpool.copy()
    pages = np.array([2, 0, 3], np.int32)                        # enough pages for kv_len up to 11
    ref_k, ref_v = kpool.copy(), vpool.copy()
    for t, L in enumerate((6, 7, 8)):                            # 7 -> 8 crosses into the third page
        step = Step(1, np.array([L], np.int32), np.array([0, pages_needed(L, s.page)], np.int32),
                    pages[: pages_needed(L, s.page)].copy())
        x = r32(1, s.H)
        xo = x.copy()
        _, dbg = oracle.layer(oracle.shape_of(s), xo, w, kp, vp, step.kv_len, step.page_indptr, step.page_ids, debug=True)
        ref = _library_layer(s, x, w, ref_k, ref_v, step)
        np.testing.assert_allclose(xo, ref, rtol=2e-5, atol=2e-5, err_msg=f"step {t}")
        # extend the reference cache by hand with the rows this step defined
        pg, sl = int(pages[L // s.page]), L % s.page
        ref_k[pg, sl] = dbg["k_rot"][0].reshape(s.nkv, s.d)
        ref_v[pg, sl] = dbg["v_new"][0].reshape(s.nkv, s.d)
        np.testing.assert_array_equal(kp, ref_k)
        np.testing.assert_array_equal(vp, ref_v)


# ---------------------------------------------------------------- per-head Q / K norm (Sec. 4.3: Q-Norm, K-Norm)
@pytest.mark.parametrize("moe", [False, True])
def test_qk_norm_layer_matches_independent_library_derivation(moe):
    s = _tiny(moe, qk_norm=True)
    w = _weights(s)
    step = _step(s, [9, 0, 4], n_pool=8)
    kpool, vpool = r32(8, s.page, s.nkv, s.d), r32(8, s.page, s.nkv, s.d)
    x = r32(3, s.H)
    xo, kp, vp = x.copy(), kpool.copy(), vpool.copy()
    ids, dbg = oracle.layer(oracle.shape_of(s), xo, w, kp, vp, step.kv_len, step.page_indptr, step.page_ids, debug=True)
    ref = _library_layer(s, x, w, kpool, vpool, step, ids)
    np.testing.assert_allclose(xo, ref, rtol=2e-5, atol=2e-5)
    # the norm is really there: without it the result differs
    s0 = _tiny(moe)
    x0 = x.copy()
    oracle.layer(oracle.shape_of(s0), x0, w, kpool.copy(), vpool.copy(), step.kv_len, step.page_indptr, step.page_ids,
                 forced_topk=ids)
    assert np.abs(x0 - xo).max() > 1e-3


def test_qk_norm_makes_the_layer_blind_to_the_scale_of_wq_and_wk():
    """A head that is normalised to unit RMS forgets how large it was: scaling Wq by 3 and Wk by 1/2 leaves the
    layer's output (nearly: eps) unchanged, and the appended key row has RMS |gk| per head at position 0."""
    s = _tiny(False, qk_norm=True, eps=1e-12)
    w = _weights(s)
    w["gk"] = np.full(s.d, 2.0, np.float32)
    step = _step(s, [0, 5], n_pool=4)
    kpool, vpool = r32(4, s.page, s.nkv, s.d), r32(4, s.page, s.nkv, s.d)
    x = r32(2, s.H)
    a, b = x.copy(), x.copy()
    kpa = kpool.copy()
    _, dbg = oracle.layer(oracle.shape_of(s), a, w, kpa, vpool.copy(), step.kv_len, step.page_indptr, step.page_ids, debug=True)
    w2 = dict(w, wq=w["wq"] * 3.0, wk=w["wk"] * 0.5)
    oracle.layer(oracle.shape_of(s), b, w2, kpool.copy(), vpool.copy(), step.kv_len, step.page_indptr, step.page_ids)
    np.testing.assert_allclose(a, b, rtol=1e-5, atol=1e-6)
    k_rows = dbg["k_rot"].reshape(2, s.nkv, s.d)          # RoPE keeps the norm of every rotated pair, hence of the head
    np.testing.assert_allclose(np.sqrt((k_rows.astype(np.float64) ** 2).mean(-1)), 2.0, rtol=1e-5)
    # constant head: every element of the normalised head equals gain * sign
    xx = np.full((1, 8), -3.0, np.float32)
    np.testing.assert_allclose(oracle.rmsnorm(xx[0], np.arange(1, 9, dtype=np.float32), 0.0), -np.arange(1, 9), rtol=1e-6)


# ---------------------------------------------------------------- final norm, vocabulary projection, greedy token
def test_lm_head_matches_float64_and_breaks_ties_to_the_lower_id():
    s = _tiny(False)
    V = 24
    x, gf, wlm = r32(3, s.H), 1 + r32(s.H, scale=0.05), r32(V, s.H, scale=0.3)
    logits, tok = oracle.lm_head(oracle.shape_of(s), x, gf, wlm)
    xd = x.astype(np.float64)
    xn = xd / np.sqrt((xd ** 2).mean(-1, keepdims=True) + s.eps) * gf.astype(np.float64)
    ref = xn @ wlm.astype(np.float64).T
    np.testing.assert_allclose(logits, ref, rtol=2e-6, atol=2e-6)
    np.testing.assert_array_equal(tok, ref.argmax(-1))
    # one-hot rows: the logit of token v is the v-th normalised input element; equal rows tie -> lower id
    eye = np.zeros((V, s.H), np.float32)
    eye[np.arange(V), np.arange(V)] = 1.0
    eye[20] = eye[5]                                        # tokens 5 and 20 have identical rows
    xo = np.zeros((1, s.H), np.float32)
    xo[0, 5], xo[0, 7] = 4.0, 4.0                            # elements 5 and 7 are the (equal) largest
    lg, tk = oracle.lm_head(oracle.shape_of(s), xo, np.ones(s.H, np.float32), eye)
    assert lg[0, 5] == lg[0, 7] == lg[0, 20] and tk[0] == 5
    np.testing.assert_allclose(lg[0, 5], 4.0 / np.sqrt(32.0 / s.H + s.eps), rtol=1e-6)


# ---------------------------------------------------------------- the MoE layer on its own
def test_moe_layer_matches_float64_library_derivation_and_the_layer_it_was_cut_from():
    """x + MoE(rmsnorm(x)) for a block of tokens, written a second way with float64 library calls (lexsort top-k,
    softmax over the selected logits, per-token expert MLPs); and the second half of the full layer, from which the
    function was extracted, gives the same bits when fed the same mid-layer residual."""
    s = _tiny(moe=True, n_experts=8, top_k=3)
    w = _weights(s)
    T_ = lambda a: torch.from_numpy(np.asarray(a)).double()  # noqa: E731
    x = r32(11, s.H)
    y, ids, logits, tw = oracle.moe_layer(oracle.shape_of(s), x, w)
    for b in range(11):
        xn = Fn.rms_norm(T_(x[b]), (s.H,), T_(w["g2"]), eps=s.eps)
        lg = T_(w["wr"]) @ xn
        np.testing.assert_allclose(logits[b], lg.numpy(), rtol=1e-5, atol=1e-6)
        order = np.lexsort((np.arange(s.n_experts), -logits[b].astype(np.float64)))[: s.top_k]
        np.testing.assert_array_equal(ids[b], order)
        ww = torch.softmax(lg[torch.from_numpy(order).long()], 0)
        np.testing.assert_allclose(tw[b], ww.numpy(), rtol=1e-5)
        ref = T_(x[b]) + sum(ww[i] * (T_(w["ed"][e]) @ (Fn.silu(T_(w["eg"][e]) @ xn) * (T_(w["eu"][e]) @ xn)))
                             for i, e in enumerate(order.tolist()))
        np.testing.assert_allclose(y[b], ref.numpy(), rtol=2e-5, atol=2e-6)
    # the same function inside the whole layer: zero attention output projection makes x_mid = x
    w0 = dict(w, wo=np.zeros_like(w["wo"]))
    n_pool = 6
    kp, vp = r32(n_pool, s.page, s.nkv, s.d), r32(n_pool, s.page, s.nkv, s.d)
    step = _step(s, [3] * 11, 11 * 2)
    kp, vp = r32(22, s.page, s.nkv, s.d), r32(22, s.page, s.nkv, s.d)
    xl = x.copy()
    oracle.layer(oracle.shape_of(s), xl, w0, kp, vp, step.kv_len, step.page_indptr, step.page_ids)
    np.testing.assert_array_equal(xl, y)
    # forced routing is followed, and the weights come from the logits at the forced ids
    forced = np.stack([rng.permutation(s.n_experts)[: s.top_k] for _ in range(11)]).astype(np.int32)
    yf, idf, _, twf = oracle.moe_layer(oracle.shape_of(s), x, w, forced_topk=forced)
    np.testing.assert_array_equal(idf, forced)
    for b in range(11):
        ww = torch.softmax(T_(logits[b])[torch.from_numpy(forced[b]).long()], 0)
        np.testing.assert_allclose(twf[b], ww.numpy(), rtol=1e-5)
    assert not np.array_equal(yf, y)
