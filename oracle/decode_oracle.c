/*
 * CPU oracle of one decoder layer of an LLM decode step  --  TEST INFRASTRUCTURE.
 *
 * This file is the definition the GPU megakernel is checked against.  It is
 * slow and plain on purpose: one operator after another, fp32 storage, every
 * reduction accumulated in double and rounded once, no tiling, no fusion, no
 * intermediate bf16 rounding.  It shares no code with the HIP path and must
 * never be called from the product path (only tests, the smoke check and the
 * benchmark's cpu_baseline leg use it).
 *
 * What is computed.  The paper names the operators of the decode pipeline its
 * megakernel covers (Sec. 4.3: Attention, RoPE, KV-cache append, Norm, MLP,
 * MoE) and describes the MoE dataflow (Sec. 2.4: TopK routing -> token
 * grouping -> GroupGEMM, with the run-time tensors topk and exp_indptr); it
 * does not restate the model equations, so they are the standard pre-norm
 * decoder of the benchmark shapes:
 *
 *   xn  = rmsnorm(x, g1)                       q,k,v = Wq xn, Wk xn, Wv xn
 *   (qk_norm models, Sec. 4.3 "Q-Norm", "K-Norm": q_h = rmsnorm(q_h, gq), k_h = rmsnorm(k_h, gk) per head, over head_dim)
 *   q,k = rope(q, pos), rope(k, pos)           append k,v at position pos
 *   o_h = softmax(q_h . K / sqrt(d)) V         over positions 0..pos, via the page table
 *   x   = x + Wo o
 *   xn2 = rmsnorm(x, g2)
 *   dense: x = x + Wd (silu(Wg xn2) * (Wu xn2))
 *   MoE  : logits = Wr xn2; S = top-k; w = softmax(logits[S]);
 *          x = x + sum_{slot} w_slot * Wd_e (silu(Wg_e xn2) * (Wu_e xn2))
 * After the last layer (models with a vocabulary: the end of a decode iteration of Sec. 4.3, whose output token
 * is the next iteration's input):
 *   logits = Wlm rmsnorm(x, gf)                token = argmax(logits), ties -> lower id
 *
 * Conventions (readings where the paper is silent):
 *   - RoPE pairs element i with i + d/2, angle = pos * theta^(-2i/d).
 *   - kv_len[b] counts cached tokens; the new token has pos = kv_len[b].
 *   - cached K is already rotated; the appended K row is stored rotated.
 *   - top-k order: larger logit first, equal logits -> lower expert id first.
 *   - routing weights: softmax over the selected logits only.
 *   - grouping order: (expert, token, slot) ascending; exp_indptr counts
 *     row tiles of tile_m tokens per expert (half-open CSR ranges).
 *   - per-head Q / K norm (Qwen3-style models only): RMSNorm over the head_dim elements of every
 *     head with one gain vector for all query heads and one for all key heads, the layer's eps,
 *     applied before RoPE; the cache holds the normalised, rotated key.
 *   - sampling: greedy (arg-max of the logits), the lower token id on equal logits.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t H, nq, nkv, d, F, page, n_experts, top_k, moe_F, tile_m;
    float eps, theta;
    int32_t qk_norm;   /* != 0: per-head RMSNorm of q and k before RoPE */
} orc_shape;

/* optional per-operator outputs for per-stage parity checks; any pointer may be NULL */
typedef struct {
    float *q_rot;   /* [B, nq*d]  after RoPE */
    float *k_rot;   /* [B, nkv*d] after RoPE (the appended row) */
    float *v_new;   /* [B, nkv*d] */
    float *attn;    /* [B, nq*d]  attention output before Wo */
    float *x_mid;   /* [B, H]     after the attention residual */
    float *act;     /* [B, F]     silu(gate)*up (dense only) */
    float *router_logits; /* [B, E] */
    float *topk_w;  /* [B, K] */
} orc_debug;

/* y = x * g / sqrt(mean(x^2) + eps) */
void orc_rmsnorm(const float *x, const float *g, int H, float eps, float *y)
{
    double ss = 0.0;
    for (int i = 0; i < H; ++i) ss += (double)x[i] * (double)x[i];
    double r = 1.0 / sqrt(ss / (double)H + (double)eps);
    for (int i = 0; i < H; ++i) y[i] = (float)((double)x[i] * r * (double)g[i]);
}

/* Y[b, n] = sum_k W[n, k] X[b, k] */
void orc_linear(const float *W, const float *X, int B, int N, int K, float *Y)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const float *w = W + (size_t)n * K;
        for (int b = 0; b < B; ++b) {
            const float *x = X + (size_t)b * K;
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int k = 0; k < K; ++k) acc += (double)w[k] * (double)x[k];
            Y[(size_t)b * N + n] = (float)acc;
        }
    }
}

/* rotate each head of v[n_heads, d] to position pos (pairs i, i + d/2) */
void orc_rope(float *v, int n_heads, int d, int pos, float theta)
{
    int half = d / 2;
    for (int h = 0; h < n_heads; ++h) {
        float *p = v + (size_t)h * d;
        for (int i = 0; i < half; ++i) {
            double ang = (double)pos * pow((double)theta, -2.0 * (double)i / (double)d);
            double c = cos(ang), s = sin(ang);
            double a = p[i], b = p[i + half];
            p[i] = (float)(a * c - b * s);
            p[i + half] = (float)(a * s + b * c);
        }
    }
}

double orc_silu(double z) { return z / (1.0 + exp(-z)); }

/*
 * Attention of one sequence's new token over n_keys positions fetched through
 * its page list.  q [nq, d]; pools [page][slot][nkv][d]; out [nq, d].
 */
void orc_attention(const orc_shape *s, const float *q, const float *kpool, const float *vpool,
                   const int32_t *pages, int n_keys, float *out)
{
    int group = s->nq / s->nkv;
    size_t row = (size_t)s->nkv * s->d;
    double *sc = (double *)malloc(sizeof(double) * (size_t)n_keys);
    for (int h = 0; h < s->nq; ++h) {
        int kvh = h / group;
        const float *qh = q + (size_t)h * s->d;
        double mx = -INFINITY;
        for (int j = 0; j < n_keys; ++j) {
            const float *kr = kpool + ((size_t)pages[j / s->page] * s->page + (size_t)(j % s->page)) * row +
                              (size_t)kvh * s->d;
            double dot = 0.0;
            for (int i = 0; i < s->d; ++i) dot += (double)qh[i] * (double)kr[i];
            sc[j] = dot / sqrt((double)s->d);
            if (sc[j] > mx) mx = sc[j];
        }
        double den = 0.0;
        for (int j = 0; j < n_keys; ++j) { sc[j] = exp(sc[j] - mx); den += sc[j]; }
        for (int i = 0; i < s->d; ++i) {
            double acc = 0.0;
            for (int j = 0; j < n_keys; ++j) {
                const float *vr = vpool + ((size_t)pages[j / s->page] * s->page + (size_t)(j % s->page)) * row +
                                  (size_t)kvh * s->d;
                acc += sc[j] * (double)vr[i];
            }
            out[(size_t)h * s->d + i] = (float)(acc / den);
        }
    }
    free(sc);
}

/* ids[0..K) = experts of the K largest logits; ties -> lower id first */
void orc_topk(const float *logits, int E, int K, int32_t *ids)
{
    char *taken = (char *)calloc((size_t)E, 1);
    for (int k = 0; k < K; ++k) {
        int best = -1;
        for (int e = 0; e < E; ++e) {
            if (taken[e]) continue;
            if (best < 0 || logits[e] > logits[best]) best = e; /* strict > keeps the lower id on ties */
        }
        ids[k] = best;
        taken[best] = 1;
    }
    free(taken);
}

/* w[k] = exp(logit[ids[k]]) / sum_k' exp(logit[ids[k']]) */
void orc_route_weights(const float *logits, const int32_t *ids, int K, float *w)
{
    double mx = -INFINITY, den = 0.0;
    for (int k = 0; k < K; ++k) if ((double)logits[ids[k]] > mx) mx = (double)logits[ids[k]];
    for (int k = 0; k < K; ++k) den += exp((double)logits[ids[k]] - mx);
    for (int k = 0; k < K; ++k) w[k] = (float)(exp((double)logits[ids[k]] - mx) / den);
}

/*
 * Token grouping (Sec. 2.4): count[e] = routed (token, slot) pairs; tok_indptr =
 * prefix sum of counts; perm lists the pairs (as token*K + slot) sorted by
 * (expert, token, slot); exp_indptr = prefix sum of ceil(count / tile_m).
 */
void orc_group(const int32_t *topk_ids, int B, int K, int E, int tile_m, int32_t *count,
               int32_t *tok_indptr, int32_t *perm, int32_t *exp_indptr)
{
    for (int e = 0; e < E; ++e) count[e] = 0;
    for (int i = 0; i < B * K; ++i) count[topk_ids[i]]++;
    tok_indptr[0] = 0;
    exp_indptr[0] = 0;
    for (int e = 0; e < E; ++e) {
        tok_indptr[e + 1] = tok_indptr[e] + count[e];
        exp_indptr[e + 1] = exp_indptr[e] + (count[e] + tile_m - 1) / tile_m;
    }
    int n = 0;
    for (int e = 0; e < E; ++e)
        for (int t = 0; t < B; ++t)
            for (int k = 0; k < K; ++k)
                if (topk_ids[t * K + k] == e) perm[n++] = t * K + k;
}

/*
 * MoE block of a layer (paper Sec. 2.4: TopK routing -> GroupGEMM-1 -> activation -> GroupGEMM-2 -> weighted combine),
 * token by token, slots in ascending order: x[b] += sum_k w[b,k] * Wd_e (silu(Wg_e xn[b]) * (Wu_e xn[b])), e = topk[b,k].
 * x [B, H] residual stream, updated in place; xn [B, H] its normalised copy.  force_routing != 0: topk_ids is an input.
 * logits_out [B, E] and topk_w_out [B, K] are optional outputs.
 */
void orc_moe_block(const orc_shape *s, int B, float *x, const float *xn, const float *wr, const float *eg, const float *eu,
                   const float *ed, int force_routing, int32_t *topk_ids, float *logits_out, float *topk_w_out)
{
    int H = s->H;
    float *y = (float *)malloc(sizeof(float) * (size_t)H);
    int E = s->n_experts, K = s->top_k, F = s->moe_F;
    float *logits = (float *)malloc(sizeof(float) * (size_t)B * E);
    float *w = (float *)malloc(sizeof(float) * (size_t)K);
    float *gt = (float *)malloc(sizeof(float) * (size_t)F);
    float *up = (float *)malloc(sizeof(float) * (size_t)F);
    double *acc = (double *)malloc(sizeof(double) * (size_t)H);
    orc_linear(wr, xn, B, E, H, logits);
    if (logits_out) memcpy(logits_out, logits, sizeof(float) * (size_t)B * E);
    for (int b = 0; b < B; ++b) {
        int32_t *ids = topk_ids + (size_t)b * K;
        const float *xb = xn + (size_t)b * H;
        if (!force_routing) orc_topk(logits + (size_t)b * E, E, K, ids);
        orc_route_weights(logits + (size_t)b * E, ids, K, w);
        if (topk_w_out) memcpy(topk_w_out + (size_t)b * K, w, sizeof(float) * (size_t)K);
        for (int i = 0; i < H; ++i) acc[i] = 0.0;
        for (int slot = 0; slot < K; ++slot) { /* ascending slot order */
            size_t e = (size_t)ids[slot];
            orc_linear(eg + e * F * H, xb, 1, F, H, gt);
            orc_linear(eu + e * F * H, xb, 1, F, H, up);
            for (int i = 0; i < F; ++i) gt[i] = (float)(orc_silu((double)gt[i]) * (double)up[i]);
            orc_linear(ed + e * H * F, gt, 1, H, F, y);
            for (int i = 0; i < H; ++i) acc[i] += (double)w[slot] * (double)y[i];
        }
        for (int i = 0; i < H; ++i) x[(size_t)b * H + i] = (float)((double)x[(size_t)b * H + i] + acc[i]);
    }
    free(logits); free(w); free(gt); free(up); free(acc); free(y);
}

/*
 * The MoE layer on its own, as the paper measures it over 1 .. 4096 tokens (Sec. 4.2, Sec. 4.5): pre-norm residual
 * block x <- x + MoE(rmsnorm(x, g)).  x [T, H] in place; the other arguments as in orc_moe_block.
 */
void orc_moe_layer(const orc_shape *s, int T, float *x, const float *g, const float *wr, const float *eg, const float *eu,
                   const float *ed, int force_routing, int32_t *topk_ids, float *logits_out, float *topk_w_out)
{
    float *xn = (float *)malloc(sizeof(float) * (size_t)T * s->H);
    for (int b = 0; b < T; ++b) orc_rmsnorm(x + (size_t)b * s->H, g, s->H, s->eps, xn + (size_t)b * s->H);
    orc_moe_block(s, T, x, xn, wr, eg, eu, ed, force_routing, topk_ids, logits_out, topk_w_out);
    free(xn);
}

/*
 * One decoder layer for a batch of B single-token sequences; x [B, H] is updated
 * in place; the K/V pools receive the appended rows (fp32) in place.
 * force_routing != 0: topk_ids is an input (weights still come from this
 * oracle's logits at those ids); otherwise it is an output.
 */
void orc_layer(const orc_shape *s, int B, float *x, const float *g1, const float *wq, const float *wk,
               const float *wv, const float *wo, const float *g2, const float *wg, const float *wu,
               const float *wd, const float *wr, const float *eg, const float *eu, const float *ed,
               const float *gq, const float *gk, float *kpool, float *vpool, const int32_t *kv_len, const int32_t *page_indptr,
               const int32_t *page_ids, int force_routing, int32_t *topk_ids, const orc_debug *dbg)
{
    int H = s->H, QD = s->nq * s->d, KD = s->nkv * s->d;
    float *xn = (float *)malloc(sizeof(float) * (size_t)B * H);
    float *q = (float *)malloc(sizeof(float) * (size_t)B * QD);
    float *k = (float *)malloc(sizeof(float) * (size_t)B * KD);
    float *v = (float *)malloc(sizeof(float) * (size_t)B * KD);
    float *o = (float *)malloc(sizeof(float) * (size_t)B * QD);
    float *y = (float *)malloc(sizeof(float) * (size_t)B * H);

    for (int b = 0; b < B; ++b) orc_rmsnorm(x + (size_t)b * H, g1, H, s->eps, xn + (size_t)b * H);
    orc_linear(wq, xn, B, QD, H, q);
    orc_linear(wk, xn, B, KD, H, k);
    orc_linear(wv, xn, B, KD, H, v);
    if (s->qk_norm) {
        for (int b = 0; b < B; ++b) {
            for (int h = 0; h < s->nq; ++h) {
                float *qh = q + (size_t)b * QD + (size_t)h * s->d;
                orc_rmsnorm(qh, gq, s->d, s->eps, qh);
            }
            for (int h = 0; h < s->nkv; ++h) {
                float *kh = k + (size_t)b * KD + (size_t)h * s->d;
                orc_rmsnorm(kh, gk, s->d, s->eps, kh);
            }
        }
    }
    for (int b = 0; b < B; ++b) {
        int pos = kv_len[b];
        orc_rope(q + (size_t)b * QD, s->nq, s->d, pos, s->theta);
        orc_rope(k + (size_t)b * KD, s->nkv, s->d, pos, s->theta);
        const int32_t *pages = page_ids + page_indptr[b];
        size_t dst = ((size_t)pages[pos / s->page] * s->page + (size_t)(pos % s->page)) * (size_t)KD;
        memcpy(kpool + dst, k + (size_t)b * KD, sizeof(float) * (size_t)KD);
        memcpy(vpool + dst, v + (size_t)b * KD, sizeof(float) * (size_t)KD);
    }
#pragma omp parallel for schedule(dynamic)
    for (int b = 0; b < B; ++b)
        orc_attention(s, q + (size_t)b * QD, kpool, vpool, page_ids + page_indptr[b], kv_len[b] + 1,
                      o + (size_t)b * QD);
    orc_linear(wo, o, B, H, QD, y);
    for (size_t i = 0; i < (size_t)B * H; ++i) x[i] = x[i] + y[i];
    if (dbg) {
        if (dbg->q_rot) memcpy(dbg->q_rot, q, sizeof(float) * (size_t)B * QD);
        if (dbg->k_rot) memcpy(dbg->k_rot, k, sizeof(float) * (size_t)B * KD);
        if (dbg->v_new) memcpy(dbg->v_new, v, sizeof(float) * (size_t)B * KD);
        if (dbg->attn) memcpy(dbg->attn, o, sizeof(float) * (size_t)B * QD);
        if (dbg->x_mid) memcpy(dbg->x_mid, x, sizeof(float) * (size_t)B * H);
    }

    for (int b = 0; b < B; ++b) orc_rmsnorm(x + (size_t)b * H, g2, H, s->eps, xn + (size_t)b * H);
    if (s->n_experts == 0) {
        int F = s->F;
        float *gt = (float *)malloc(sizeof(float) * (size_t)B * F);
        float *up = (float *)malloc(sizeof(float) * (size_t)B * F);
        orc_linear(wg, xn, B, F, H, gt);
        orc_linear(wu, xn, B, F, H, up);
        for (size_t i = 0; i < (size_t)B * F; ++i) gt[i] = (float)(orc_silu((double)gt[i]) * (double)up[i]);
        if (dbg && dbg->act) memcpy(dbg->act, gt, sizeof(float) * (size_t)B * F);
        orc_linear(wd, gt, B, H, F, y);
        for (size_t i = 0; i < (size_t)B * H; ++i) x[i] = x[i] + y[i];
        free(gt);
        free(up);
    } else {
        orc_moe_block(s, B, x, xn, wr, eg, eu, ed, force_routing, topk_ids, dbg ? dbg->router_logits : NULL,
                      dbg ? dbg->topk_w : NULL);
    }
    free(xn); free(q); free(k); free(v); free(o); free(y);
}

/*
 * End of a decode iteration: logits[b, v] = sum_i Wlm[v, i] * rmsnorm(x[b], gf)[i]; token[b] = the index of the
 * largest logit, the lower index on equal logits.  x [B, H], Wlm [V, H], logits [B, V] (output), token [B] (output).
 */
void orc_lm_head(const orc_shape *s, int B, const float *x, const float *gf, const float *wlm, int V, float *logits,
                 int32_t *token)
{
    int H = s->H;
    float *xn = (float *)malloc(sizeof(float) * (size_t)B * H);
    for (int b = 0; b < B; ++b) orc_rmsnorm(x + (size_t)b * H, gf, H, s->eps, xn + (size_t)b * H);
    orc_linear(wlm, xn, B, V, H, logits);
    for (int b = 0; b < B; ++b) {
        const float *l = logits + (size_t)b * V;
        int best = 0;
        for (int v = 1; v < V; ++v)
            if (l[v] > l[best]) best = v; /* strict >: the lower id keeps a tie */
        token[b] = best;
    }
    free(xn);
}
