// MoE routing tasks (paper Sec. 2.4): top-k routing and token grouping, the run-time resolution of a
// GroupGEMM row-tile slot, and the weighted combine of a token's expert outputs.
//
// Grouped rows.  The (token, slot) pairs of a step are sorted by (expert, token, slot); row p of the
// grouped tensors (expert activations, expert outputs) belongs to pair perm[p].  tok_indptr is the
// prefix sum of pairs per expert, exp_indptr the prefix sum of row tiles (tile_m rows each) per
// expert: expert e owns the row tiles [exp_indptr[e], exp_indptr[e+1]).  Everything is computed by
// counting and ranking, never by grabbing slots with atomics, so the permutation is the same in
// every run and under every schedule.
#pragma once
#include "device_rt.hip.h"

namespace etc {

struct RowTile {
    int expert, row0, n;     // rows [row0, row0 + n) of the grouped tensors
};

// Slot r of the static GroupGEMM grid -> its expert and rows; false for the surplus slots of this step.
__device__ __forceinline__ bool resolve_row_tile(const Params &P, int r, RowTile &rt)
{
    const int total = __builtin_amdgcn_readfirstlane(ld_i32(P.exp_indptr + P.E));
    if (r >= total) return false;
    rt.expert = __builtin_amdgcn_readfirstlane(ld_i32(P.tile_expert + r));
    rt.row0 = __builtin_amdgcn_readfirstlane(ld_i32(P.tile_row0 + r));
    rt.n = __builtin_amdgcn_readfirstlane(ld_i32(P.tile_n + r));
    return true;
}

// ---- wavefront arg-max of the router's top-k -------------------------------------------------------------
// (logit, expert) as one unsigned key: floats map to integers of the same order (sign bit flipped for
// non-negative values, all bits for negative ones), the index is complemented so that a lower index wins a tie.
__device__ __forceinline__ uint64_t topk_key(float logit, int expert)
{
    const uint32_t u = __float_as_uint(logit);
    const uint32_t ord = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ((uint64_t)ord << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)expert);
}

__device__ __forceinline__ float topk_key_logit(uint64_t key)
{
    const uint32_t ord = (uint32_t)(key >> 32);
    return __uint_as_float((ord & 0x80000000u) ? (ord & 0x7FFFFFFFu) : ~ord);
}

template <int CTRL>
__device__ __forceinline__ uint64_t dpp_max_u64(uint64_t k)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)k, CTRL, 0xF, 0xF, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(k >> 32), CTRL, 0xF, 0xF, false);
    const uint64_t o = ((uint64_t)hi << 32) | lo;
    return o > k ? o : k;
}

// Maximum over the 64 lanes, the same value in every lane: quad exchanges, half-row mirror and row mirror leave
// each row of 16 lanes with its maximum; the four row maxima are read as scalars.
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t k)
{
    k = dpp_max_u64<0xB1>(k);      // quad_perm [1,0,3,2]
    k = dpp_max_u64<0x4E>(k);      // quad_perm [2,3,0,1]
    k = dpp_max_u64<0x141>(k);     // row_half_mirror
    k = dpp_max_u64<0x140>(k);     // row_mirror
    uint64_t best = 0;
#pragma unroll
    for (int row = 0; row < 4; ++row) {
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)k, row * 16);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(k >> 32), row * 16);
        const uint64_t r = ((uint64_t)hi << 32) | lo;
        best = r > best ? r : best;
    }
    return best;
}

// Data-dependent event update and task triggering (Sec. 2.4), dynamic scheduler only.  The expert event
// tensor E_exp[e] is armed at run time with the number of tokens routed to e, plus one for tile 0, which
// publishes the per-expert tables: every tile knows that count from its own copy of the routing, so nobody
// has to write it first - a tile decrements, and the one that sees the count complete has fired the event
// (it puts the counter back to zero for the next layer).  The grouping tile of token t updates the events of
// topk[t, :]; when E_exp[e] fires, expert e releases its GroupGEMM-1 tiles, the row-tile slots
// [exp_indptr[e], exp_indptr[e+1]) of the static grid: their tasks are published to the ready queue, all
// fired experts of this tile under one reservation.  Slots beyond exp_indptr[E] are never released: tile 0
// takes them out of the counts that were fixed before the routing was known (the events between the two
// GroupGEMMs of those slots, the combine event, the number of tasks the step has to complete).
__device__ __forceinline__ void moe_update_and_trigger(const Params &P, int layer, int t, int group_ev,
                                                       const ETC_AS_LDS int32_t *ids_s, const ETC_AS_LDS int32_t *cnt,
                                                       const ETC_AS_LDS int32_t *expp)
{
    drain_vmem();            // this tile's share of the grouping (and tile 0's tables) is written
    __syncthreads();
    if (wave_id() != 0) return;
    const int lane = lane_id(), E = P.E, K = P.topk;
    const int G = P.moe_groups_gu, Gd = P.moe_groups_down;
    if (t == 0) {
        const int live = expp[E], dead = P.moe_rmax - live;
        const int ev_slot0 = gld_i32(P.moe_layer_events + 2 * layer), ev_y = gld_i32(P.moe_layer_events + 2 * layer + 1);
        for (int r = live + lane; r < P.moe_rmax; r += 64) st_i32(P.ev_cur + ev_slot0 + r, 0);
        if (lane == 0 && dead > 0) {
            __hip_atomic_fetch_sub(as_global(P.ev_cur + ev_y), dead * Gd, __ATOMIC_RELAXED, ETC_SCOPE);
            __hip_atomic_fetch_sub(as_global(P.ev_disp_cur + ev_y), dead * Gd, __ATOMIC_RELAXED, ETC_SCOPE);
            __hip_atomic_fetch_add(as_global(P.q_ctrl_cur + 3), dead * (G + Gd), __ATOMIC_RELAXED, ETC_SCOPE);
        }
        drain_vmem();        // the counts are in place before this tile's notifies can release anything
    }
    const int c0 = __builtin_amdgcn_readfirstlane(gld_i32(P.ev_consumers + group_ev));
    // Notify 0 of a lane: one pair of this token; notifies 1.. (tile 0 only): every routed expert, 64 per
    // round.  All decrements of the tile are in flight together, and what they release goes to the ready
    // queue under one reservation.
    constexpr int NV = 1 + kMaxExperts / 64;
    int ex[NV], first[NV], n_rel[NV];
    bool fired[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        ex[v] = -1;
        if (v == 0) {
            if (lane < K) ex[v] = ids_s[t * K + lane];
        } else if (t == 0) {
            const int cand = (v - 1) * 64 + lane;
            if (cand < E && cnt[cand] > 0) ex[v] = cand;
        }
    }
    int before[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v)
        before[v] = ex[v] >= 0 ? __hip_atomic_fetch_sub(as_global(P.exp_event + ex[v]), 1, __ATOMIC_RELAXED, ETC_SCOPE) : 0;
    int n_mine = 0;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        fired[v] = ex[v] >= 0 && before[v] == -cnt[ex[v]];          // this was notify number cnt[e] + 1
        if (fired[v]) st_i32(P.exp_event + ex[v], 0);
        first[v] = fired[v] ? expp[ex[v]] * G : 0;
        n_rel[v] = fired[v] ? (expp[ex[v] + 1] - expp[ex[v]]) * G : 0;
        n_mine += n_rel[v];
    }
    drain_vmem();            // the fired counters are back at zero before the tasks they release are published:
                             // nothing released here can reach the next layer's router tiles ahead of the reset
    const int total = wave_sum_i(n_mine);
    if (total == 0) return;
    const int base = q_reserve_wave(P, total);
    if (base < 0) return;
    int off = 0;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        uint64_t m = __ballot(fired[v]);
        while (m) {                                        // one fired expert after the other, 64 slots at a time
            const int src = __builtin_ctzll(m);
            m &= m - 1;
            const int s0 = __shfl(first[v], src, 64), n = __shfl(n_rel[v], src, 64);
            for (int i = lane; i < n; i += 64)
                __hip_atomic_store(as_global(P.q_slots + base + off + i),
                                   q_slot_word(P, gld_i32(P.consumer_ids + c0 + s0 + i) & 0xFFFFFF), __ATOMIC_RELAXED, ETC_SCOPE);
            off += n;
        }
    }
}

// Router tile of token t.  Every tile needs the ids of ALL tokens to rank its own pairs, so each
// recomputes the (cheap) top-k of every token from the shared logits instead of waiting one more event
// hop for them; it publishes only what belongs to token t.  Tile 0 also publishes the per-expert tables.
// Order of the selection: larger logit first, equal logits -> lower expert index first.
// Routing weights: softmax over the selected logits.
// group_ev: the event the tile notifies; under the dynamic scheduler its consumer list (the GroupGEMM-1
// tasks of the layer, row-tile slot major) is what the expert events trigger from.
__device__ __noinline__ void moe_route_and_group(const Params &P, int layer, int t, int group_ev, float *sm)
{
    layer = __builtin_amdgcn_readfirstlane(layer);
    t = __builtin_amdgcn_readfirstlane(t);
    group_ev = __builtin_amdgcn_readfirstlane(group_ev);
    const int wave = wave_id(), lane = lane_id();
    const int E = P.E, K = P.topk, B = P.B, N = B * K, M = P.tile_m;
    ETC_AS_LDS int32_t *ids_s = reinterpret_cast<ETC_AS_LDS int32_t *>(as_lds(sm));   // [B*K] expert of every pair
    ETC_AS_LDS int32_t *cnt = ids_s + kMaxBatch * kMaxTopK;                            // [E]
    ETC_AS_LDS int32_t *til = cnt + kMaxExperts;                                       // [E] row tiles per expert
    ETC_AS_LDS int32_t *tokp = til + kMaxExperts;                                      // [E+1]
    ETC_AS_LDS int32_t *expp = tokp + kMaxExperts + 1;                                 // [E+1]
    const int forced_bits = P.forced_mask != nullptr ? (int)*as_global(P.forced_mask + layer) : 0;
    const bool forced = (forced_bits & 1) != 0, forced_w = forced && (forced_bits & 2) != 0 && P.forced_w != nullptr;
    const bool dbg = (P.debug_flags & 4u) != 0 && P.dbg_logits != nullptr;
    const size_t dbg_row = (size_t)layer * P.max_batch + t;

    for (int e = threadIdx.x; e < E; e += kWgThreads) cnt[e] = 0;
    for (int b = wave; b < B; b += kWaves) {
        const float *lg = P.router_logits + (size_t)b * E;
        float v[kMaxExperts / 64];
        bool taken[kMaxExperts / 64];
#pragma unroll
        for (int j = 0; j < kMaxExperts / 64; ++j) {
            const int e = lane + 64 * j;
            taken[j] = false;
            v[j] = e < E ? ld_f32(lg + e) : -INFINITY;
            if (dbg && b == t && e < E) as_global(P.dbg_logits)[dbg_row * E + e] = v[j];
        }
        int my_id = 0;
        float my_v = -INFINITY;
        if (forced) {
            if (lane < K) {
                my_id = gld_i32(P.forced_topk + ((size_t)layer * P.max_batch + b) * K + lane);
                my_v = ld_f32(lg + my_id);
            }
        } else {
            for (int k = 0; k < K; ++k) {
                // One 64-bit key per candidate: the logit in an order-preserving integer form above, the
                // complement of the expert index below, so the largest key is the largest logit and, among equal
                // logits, the lowest index.  The wavefront maximum takes four DPP steps inside each row of 16
                // lanes and a scalar maximum over the four rows (a shuffle-based arg-max, six dependent LDS
                // round trips of two words each, made a router tile of a large batch the longest task of the layer).
                uint64_t key = 0;
#pragma unroll
                for (int j = 0; j < kMaxExperts / 64; ++j) {
                    const int e = lane + 64 * j;
                    if (e < E && !taken[j]) key = max(key, topk_key(v[j], e));
                }
                key = wave_max_u64(key);
                const int bi = (int)(0xFFFFFFFFu - (uint32_t)key);
                if (lane == k) { my_id = bi; my_v = topk_key_logit(key); }
#pragma unroll
                for (int j = 0; j < kMaxExperts / 64; ++j)
                    if (lane + 64 * j == bi) taken[j] = true;
            }
        }
        if (lane < K) ids_s[b * K + lane] = my_id;
        if (b == t) {
            float mx = lane < K ? my_v : -INFINITY;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
            const float p = lane < K ? __expf(my_v - mx) : 0.f;
            const float den = wave_sum(p);
            if (lane < K) {
                float wgt = p / den;
                if (forced_w) wgt = *as_global(P.forced_w + ((size_t)layer * P.max_batch + b) * K + lane);
                st_i32(P.topk_ids + (size_t)t * K + lane, my_id);
                st_f32(P.topk_w + (size_t)t * K + lane, wgt);
                if (dbg) {
                    as_global(P.dbg_topk_ids)[dbg_row * K + lane] = my_id;
                    as_global(P.dbg_topk_w)[dbg_row * K + lane] = wgt;
                }
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < N; i += kWgThreads)
        __hip_atomic_fetch_add(cnt + ids_s[i], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kWgThreads) til[e] = (cnt[e] + M - 1) / M;
    __syncthreads();
    for (int e = threadIdx.x; e <= E; e += kWgThreads) {
        int a = 0, c = 0;
        for (int j = 0; j < e; ++j) { a += cnt[j]; c += til[j]; }
        tokp[e] = a;
        expp[e] = c;
    }
    __syncthreads();

    // the K pairs of this token: stable rank among the pairs of the same expert
    for (int k = wave; k < K; k += kWaves) {
        const int me = t * K + k, e = ids_s[me];
        int c = 0;
        for (int i = lane; i < me; i += 64) c += ids_s[i] == e ? 1 : 0;
        c = wave_sum_i(c);
        if (lane == 0) {
            const int pos = tokp[e] + c;
            st_i32(P.perm + pos, me);
            st_i32(P.inv_perm + me, pos);
            st_i32(P.perm_tok + pos, t);
            if (dbg) as_global(P.dbg_perm)[(size_t)layer * P.max_batch * K + pos] = me;
        }
    }
    if (t == 0) {
        for (int e = threadIdx.x; e <= E; e += kWgThreads) {
            st_i32(P.tok_indptr + e, tokp[e]);
            st_i32(P.exp_indptr + e, expp[e]);
            if (dbg) {
                as_global(P.dbg_tok_indptr)[(size_t)layer * (E + 1) + e] = tokp[e];
                as_global(P.dbg_exp_indptr)[(size_t)layer * (E + 1) + e] = expp[e];
            }
        }
        for (int e = threadIdx.x; e < E; e += kWgThreads) {
            int n = cnt[e], r = expp[e], row = tokp[e];
            for (; n > 0; n -= M, ++r, row += M) {
                st_i32(P.tile_expert + r, e);
                st_i32(P.tile_row0 + r, row);
                st_i32(P.tile_n + r, n < M ? n : M);
            }
        }
    }
    if (P.moe_dd) moe_update_and_trigger(P, layer, t, group_ev, ids_s, cnt, expp);
    __syncthreads();     // the routing scratch in LDS is free again
}

// ---------------------------------------------------------------------------------------------------------
// The MoE layer on its own over a block of T tokens (Sec. 2.4; the token sweep of Sec. 4.2 / 4.5).
// One router tile per token that ranks its pairs against every other token is quadratic in the tokens, so the
// grouping runs as three counting passes over blocks of 64 tokens: (1) top-k of the block's tokens and the
// block's pair count per expert; (2) one scan over experts and blocks: totals, prefix sums, the first grouped row
// of every (block, expert) and the row-tile tables; (3) the stable rank of every pair inside its block.  The
// grouped order is the decoder's: (expert, token, slot).  Still no slot is grabbed with an atomic: the
// permutation is the same in every run and schedule.
// ---------------------------------------------------------------------------------------------------------
constexpr int kMoelBlock = 64;


// 16 tokens: x_in (bf16) -> residual stream fp32, (x * gain) split into hi + lo, per-16-element sums of squares.
// A lane takes 8 consecutive elements (one 16-byte load), two neighbouring lanes one 16-element part.
__device__ __noinline__ void moel_load(const Params &P, int blk16)
{
    blk16 = __builtin_amdgcn_readfirstlane(blk16);
    const uint16_t *g2 = (const uint16_t *)as_global(P.weights)[0].g2;
    const int n_oct = P.H / 8;
    for (int i = wave_id(); i < 16; i += kWaves) {
        const int tok = blk16 * 16 + i;
        if (tok >= P.B) break;
        for (int oct = lane_id(); oct < n_oct; oct += 64) {
            const size_t o = (size_t)tok * P.H + (size_t)oct * 8;
            const u32x4 xa = gld_16B(P.hidden_in + o), ga = gld_16B(g2 + oct * 8);
            const uint32_t xw[4] = {xa.x, xa.y, xa.z, xa.w}, gw[4] = {ga.x, ga.y, ga.z, ga.w};
            float v[8];
            uint16_t hi[8], lo[8];
            float s = 0.f;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const uint32_t xx = xw[q >> 1], gg = gw[q >> 1];
                v[q] = bf16_bits_to_f32((uint16_t)((q & 1) ? (xx >> 16) : (xx & 0xFFFFu)));
                const float gv = bf16_bits_to_f32((uint16_t)((q & 1) ? (gg >> 16) : (gg & 0xFFFFu)));
                split_bf16(v[q] * gv, hi[q], lo[q]);
                s += v[q] * v[q];
            }
#pragma unroll
            for (int q = 0; q < 8; q += 2)
                st_u64(P.x_mid + o + q, (uint64_t)__float_as_uint(v[q]) | ((uint64_t)__float_as_uint(v[q + 1]) << 32));
#pragma unroll
            for (int q = 0; q < 8; q += 4) {
                st_u64(P.xmg_hi + o + q, (uint64_t)hi[q] | ((uint64_t)hi[q + 1] << 16) | ((uint64_t)hi[q + 2] << 32) | ((uint64_t)hi[q + 3] << 48));
                st_u64(P.xmg_lo + o + q, (uint64_t)lo[q] | ((uint64_t)lo[q + 1] << 16) | ((uint64_t)lo[q + 2] << 32) | ((uint64_t)lo[q + 3] << 48));
            }
            s += dpp_f32<0xB1>(s);               // the neighbouring lane's half of the part (quad_perm [1,0,3,2])
            if ((lane_id() & 1) == 0) st_f32(P.ssq_xmid + (size_t)(oct >> 1) * (size_t)P.col_stride + tok, s);
        }
    }
}

// Block of 64 tokens: top-k ids (larger logit first, equal logits: lower expert first) and routing weights
// (softmax over the selected logits) of each token; the block's pair count per expert.
__device__ __noinline__ void moel_topk(const Params &P, int blk, float *sm)
{
    blk = __builtin_amdgcn_readfirstlane(blk);
    const int wave = wave_id(), lane = lane_id();
    const int E = P.E, K = P.topk;
    ETC_AS_LDS int32_t *cnt = reinterpret_cast<ETC_AS_LDS int32_t *>(as_lds(sm));      // [E]
    const int forced_bits = P.forced_mask != nullptr ? (int)*as_global(P.forced_mask) : 0;
    const bool forced = (forced_bits & 1) != 0, forced_w = forced && (forced_bits & 2) != 0 && P.forced_w != nullptr;
    const bool dbg = (P.debug_flags & 4u) != 0 && P.dbg_logits != nullptr;
    for (int e = threadIdx.x; e < E; e += kWgThreads) cnt[e] = 0;
    __syncthreads();
    for (int i = wave; i < kMoelBlock; i += kWaves) {
        const int b = blk * kMoelBlock + i;
        if (b >= P.B) break;
        const float *lg = P.router_logits + (size_t)b * E;
        float v[kMaxExperts / 64];
        bool taken[kMaxExperts / 64];
#pragma unroll
        for (int j = 0; j < kMaxExperts / 64; ++j) {
            const int e = lane + 64 * j;
            taken[j] = false;
            v[j] = e < E ? ld_f32(lg + e) : -INFINITY;
            if (dbg && e < E) as_global(P.dbg_logits)[(size_t)b * E + e] = v[j];
        }
        int my_id = 0;
        float my_v = -INFINITY;
        if (forced) {
            if (lane < K) {
                my_id = gld_i32(P.forced_topk + (size_t)b * K + lane);
                my_v = ld_f32(lg + my_id);
            }
        } else {
            for (int k = 0; k < K; ++k) {
                uint64_t key = 0;
#pragma unroll
                for (int j = 0; j < kMaxExperts / 64; ++j) {
                    const int e = lane + 64 * j;
                    if (e < E && !taken[j]) key = max(key, topk_key(v[j], e));
                }
                key = wave_max_u64(key);
                const int bi = (int)(0xFFFFFFFFu - (uint32_t)key);
                if (lane == k) { my_id = bi; my_v = topk_key_logit(key); }
#pragma unroll
                for (int j = 0; j < kMaxExperts / 64; ++j)
                    if (lane + 64 * j == bi) taken[j] = true;
            }
        }
        float mx = lane < K ? my_v : -INFINITY;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
        const float p = lane < K ? __expf(my_v - mx) : 0.f;
        const float den = wave_sum(p);
        if (lane < K) {
            float wgt = p / den;
            if (forced_w) wgt = *as_global(P.forced_w + (size_t)b * K + lane);
            st_i32(P.topk_ids + (size_t)b * K + lane, my_id);
            st_f32(P.topk_w + (size_t)b * K + lane, wgt);
            if (dbg) {
                as_global(P.dbg_topk_ids)[(size_t)b * K + lane] = my_id;
                as_global(P.dbg_topk_w)[(size_t)b * K + lane] = wgt;
            }
            __hip_atomic_fetch_add(cnt + my_id, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);      // integer count: order-free
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kWgThreads) st_i32(P.moel_hist + (size_t)blk * E + e, cnt[e]);
    __syncthreads();
}

// One task: pairs per expert, prefix sums over the experts (pairs and row tiles), the first grouped row of every
// (block, expert), the row-tile tables.  Under the dynamic scheduler it also takes the surplus row-tile slots of the
// static grids out of the counts that were fixed before the routing was known (as tile 0 does in a decoder).
__device__ __noinline__ void moel_scan(const Params &P, float *sm)
{
    const int E = P.E, M = P.tile_m, n_blk = (P.B + kMoelBlock - 1) / kMoelBlock;
    ETC_AS_LDS int32_t *cnt = reinterpret_cast<ETC_AS_LDS int32_t *>(as_lds(sm));      // [E]
    ETC_AS_LDS int32_t *til = cnt + kMaxExperts;                                       // [E]
    ETC_AS_LDS int32_t *tokp = til + kMaxExperts;                                      // [E+1]
    ETC_AS_LDS int32_t *expp = tokp + kMaxExperts + 1;                                 // [E+1]
    const bool dbg = (P.debug_flags & 4u) != 0 && P.dbg_logits != nullptr;
    for (int e = threadIdx.x; e < E; e += kWgThreads) {
        int n = 0;
        for (int b0 = 0; b0 < n_blk; b0 += 16) {           // 16 loads in flight: the scan is alone on the critical path
            int h[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) h[u] = b0 + u < n_blk ? ld_i32(P.moel_hist + (size_t)(b0 + u) * E + e) : 0;
#pragma unroll
            for (int u = 0; u < 16; ++u) n += h[u];
        }
        cnt[e] = n;
        til[e] = (n + M - 1) / M;
    }
    __syncthreads();
    for (int e = threadIdx.x; e <= E; e += kWgThreads) {
        int a = 0, c = 0;
        for (int j = 0; j < e; ++j) { a += cnt[j]; c += til[j]; }
        tokp[e] = a;
        expp[e] = c;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kWgThreads) {
        int row = tokp[e];
        for (int b0 = 0; b0 < n_blk; b0 += 16) {
            int h[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) h[u] = b0 + u < n_blk ? ld_i32(P.moel_hist + (size_t)(b0 + u) * E + e) : 0;
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                if (b0 + u < n_blk) st_i32(P.moel_base + (size_t)(b0 + u) * E + e, row);
                row += h[u];
            }
        }
        st_i32(P.moel_count + e, cnt[e]);
        int n = cnt[e], r = expp[e];
        row = tokp[e];
        for (; n > 0; n -= M, ++r, row += M) {
            st_i32(P.tile_expert + r, e);
            st_i32(P.tile_row0 + r, row);
            st_i32(P.tile_n + r, n < M ? n : M);
        }
    }
    for (int e = threadIdx.x; e <= E; e += kWgThreads) {
        st_i32(P.tok_indptr + e, tokp[e]);
        st_i32(P.exp_indptr + e, expp[e]);
        if (dbg) {
            as_global(P.dbg_tok_indptr)[e] = tokp[e];
            as_global(P.dbg_exp_indptr)[e] = expp[e];
        }
    }
    if (P.moe_dd && wave_id() == 0) {
        const int lane = lane_id(), G = P.moe_groups_gu, Gd = P.moe_groups_down;
        const int live = expp[E], dead = P.moe_rmax - live;
        const int ev_slot0 = gld_i32(P.moe_layer_events), ev_y = gld_i32(P.moe_layer_events + 1);
        for (int r = live + lane; r < P.moe_rmax; r += 64) st_i32(P.ev_cur + ev_slot0 + r, 0);
        if (lane == 0 && dead > 0) {
            __hip_atomic_fetch_sub(as_global(P.ev_cur + ev_y), dead * Gd, __ATOMIC_RELAXED, ETC_SCOPE);
            __hip_atomic_fetch_sub(as_global(P.ev_disp_cur + ev_y), dead * Gd, __ATOMIC_RELAXED, ETC_SCOPE);
            __hip_atomic_fetch_add(as_global(P.q_ctrl_cur + 3), dead * (G + Gd), __ATOMIC_RELAXED, ETC_SCOPE);
        }
    }
    __syncthreads();
}

// Data-dependent event update and task triggering (Sec. 2.4) of the stand-alone layer, dynamic scheduler only: the
// block adds its pair count of every expert to the expert's event at once; the total per expert is known since the
// scan, so the update that completes it has fired the event and releases the expert's GroupGEMM-1 tiles, the
// row-tile slots [exp_indptr[e], exp_indptr[e+1]), to the ready queue.
__device__ __forceinline__ void moel_update_and_trigger(const Params &P, int blk, int group_ev)
{
    drain_vmem();            // this block's share of the permutation is written
    __syncthreads();
    if (wave_id() != 0) return;
    const int lane = lane_id(), E = P.E, G = P.moe_groups_gu;
    const int c0 = __builtin_amdgcn_readfirstlane(gld_i32(P.ev_consumers + group_ev));
    for (int e0 = 0; e0 < E; e0 += 64) {
        const int e = e0 + lane;
        const int h = e < E ? ld_i32(P.moel_hist + (size_t)blk * E + e) : 0;
        const int before = h > 0 ? __hip_atomic_fetch_sub(as_global(P.exp_event + e), h, __ATOMIC_RELAXED, ETC_SCOPE) : 0;
        const bool fired = h > 0 && before - h == -ld_i32(P.moel_count + e);
        int first = 0, n_rel = 0;
        if (fired) {
            st_i32(P.exp_event + e, 0);
            const int r0 = ld_i32(P.exp_indptr + e), r1 = ld_i32(P.exp_indptr + e + 1);
            first = r0 * G;
            n_rel = (r1 - r0) * G;
        }
        drain_vmem();        // the fired counters are back at zero before the tasks they release are published
        const int total = wave_sum_i(n_rel);
        if (total == 0) continue;
        const int base = q_reserve_wave(P, total);
        if (base < 0) return;
        int off = 0;
        uint64_t m = __ballot(fired);
        while (m) {
            const int src = __builtin_ctzll(m);
            m &= m - 1;
            const int s0 = __shfl(first, src, 64), n = __shfl(n_rel, src, 64);
            for (int i = lane; i < n; i += 64)
                __hip_atomic_store(as_global(P.q_slots + base + off + i),
                                   q_slot_word(P, gld_i32(P.consumer_ids + c0 + s0 + i) & 0xFFFFFF), __ATOMIC_RELAXED, ETC_SCOPE);
            off += n;
        }
    }
}

// Block of 64 tokens: every pair's grouped row = first row of (block, expert) + its rank among the block's earlier
// pairs of the same expert (pairs in token, slot order).
__device__ __noinline__ void moel_place(const Params &P, int blk, int group_ev, float *sm)
{
    blk = __builtin_amdgcn_readfirstlane(blk);
    group_ev = __builtin_amdgcn_readfirstlane(group_ev);
    const int E = P.E, K = P.topk;
    const int n_tok = P.B - blk * kMoelBlock < kMoelBlock ? P.B - blk * kMoelBlock : kMoelBlock;
    ETC_AS_LDS int32_t *ids_s = reinterpret_cast<ETC_AS_LDS int32_t *>(as_lds(sm));    // [64 * K]
    ETC_AS_LDS int32_t *base_s = ids_s + kMoelBlock * kMaxTopK;                        // [E]
    const bool dbg = (P.debug_flags & 4u) != 0 && P.dbg_logits != nullptr;
    if (n_tok > 0) {
        const int n_pairs = n_tok * K, pair0 = blk * kMoelBlock * K;
        for (int p = threadIdx.x; p < n_pairs; p += kWgThreads) ids_s[p] = ld_i32(P.topk_ids + pair0 + p);
        for (int e = threadIdx.x; e < E; e += kWgThreads) base_s[e] = ld_i32(P.moel_base + (size_t)blk * E + e);
        __syncthreads();
        for (int p = threadIdx.x; p < n_pairs; p += kWgThreads) {
            const int e = ids_s[p];
            int rank = 0;
            for (int q = 0; q < p; ++q) rank += ids_s[q] == e ? 1 : 0;
            const int pos = base_s[e] + rank, pair = pair0 + p;
            st_i32(P.perm + pos, pair);
            st_i32(P.inv_perm + pair, pos);
            st_i32(P.perm_tok + pos, pair / K);
            if (dbg) as_global(P.dbg_perm)[pos] = pair;
        }
    }
    if (P.moe_dd) moel_update_and_trigger(P, blk, group_ev);
    __syncthreads();
}

// Combine tile (token b, 512 consecutive elements): x = x_mid + sum_k w[b,k] * y[row of pair (b,k)],
// slots in ascending order.  Like every producer of the residual stream it also prepares the next
// layer's projection operand (x * gain, split) and the partial sums of squares per 16 elements.
__device__ __forceinline__ void moe_combine(const Params &P, const Task &t)
{
    const int b = t.c0, h = t.c1 * kWgThreads + (int)threadIdx.x;
    if (h >= P.H) return;
    const int K = P.topk;
    float acc = 0.f;
    for (int k = 0; k < K; ++k) {
        const int pos = ld_i32(P.inv_perm + (size_t)b * K + k);
        acc += ld_f32(P.topk_w + (size_t)b * K + k) * ld_f32(P.ey + (size_t)pos * P.H + h);
    }
    const size_t o = (size_t)b * P.H + h;
    const float v = ld_f32(P.x_mid + o) + acc;
    st_f32(P.x + o, v);
    const bool last = (t.flags & TF_LAST_LAYER) != 0;
    if (last && P.hidden_out) gst_u16(P.hidden_out + o, f32_to_bf16_bits(v));
    if (!last || P.vocab > 0) {       // operand of the next projection: the next layer's QKV, or the vocabulary projection
        const uint16_t *g1 = last ? P.gf : (const uint16_t *)as_global(P.weights)[t.layer + 1].g1;
        uint16_t hi, lo;
        split_bf16(v * bf16_bits_to_f32(gld_u16(g1 + h)), hi, lo);
        st_u16(P.xg_hi + o, hi);
        st_u16(P.xg_lo + o, lo);
        float s = v * v;          // 16 consecutive lanes hold one 16-element part
        s = lanes_sum<16>(s);
        if ((threadIdx.x & 15) == 0) st_f32(P.ssq_x + (size_t)(h >> 4) * kMaxBatch + b, s);
    }
    if (P.debug_flags & 2u) gst_f32(P.layer_hidden + ((size_t)t.layer * kMaxBatch + b) * P.H + h, v);
}

// Combine of the stand-alone layer: task (block of `n_tok` tokens starting at tok0, 2048 consecutive elements).  One
// task per token and 512 elements would be 16 384 tasks of two dependent load rounds each at 4096 tokens (415 us for
// 320 MB); here a thread takes 4 consecutive elements (8-byte accesses) of two tokens at a time, so the row look-ups
// and expert rows of both are in flight together.  The layer's output is y; no residual copy is kept.
__device__ __forceinline__ void moel_combine(const Params &P, int tok0, int n_tok, int chunk)
{
    const int h = (chunk * kWgThreads + (int)threadIdx.x) * 4;
    if (h >= P.H) return;
    const int K = P.topk;
    constexpr int TB = 2;                        // tokens in flight per thread
    const int end = tok0 + n_tok < P.B ? tok0 + n_tok : P.B;
    for (int b0 = tok0; b0 < end; b0 += TB) {
        float acc[TB][4];
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            const int b = b0 + u < end ? b0 + u : end - 1;
            ld_f32x2(P.x_mid + (size_t)b * P.H + h, acc[u][0], acc[u][1]);
            ld_f32x2(P.x_mid + (size_t)b * P.H + h + 2, acc[u][2], acc[u][3]);
        }
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            const int b = b0 + u < end ? b0 + u : end - 1;
            float sum[4] = {0.f, 0.f, 0.f, 0.f};
            for (int k = 0; k < K; ++k) {            // slots in ascending order
                const int pos = ld_i32(P.inv_perm + (size_t)b * K + k);
                const float wk = ld_f32(P.topk_w + (size_t)b * K + k);
                float y0, y1, y2, y3;
                ld_f32x2(P.ey + (size_t)pos * P.H + h, y0, y1);
                ld_f32x2(P.ey + (size_t)pos * P.H + h + 2, y2, y3);
                sum[0] += wk * y0; sum[1] += wk * y1; sum[2] += wk * y2; sum[3] += wk * y3;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[u][q] += sum[q];
        }
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            const int b = b0 + u;
            if (b < end && P.hidden_out) {
                const uint64_t v = (uint64_t)f32_to_bf16_bits(acc[u][0]) | ((uint64_t)f32_to_bf16_bits(acc[u][1]) << 16) |
                                   ((uint64_t)f32_to_bf16_bits(acc[u][2]) << 32) | ((uint64_t)f32_to_bf16_bits(acc[u][3]) << 48);
                *as_global(reinterpret_cast<uint64_t *>(P.hidden_out + (size_t)b * P.H + h)) = v;
            }
        }
    }
}

}  // namespace etc
