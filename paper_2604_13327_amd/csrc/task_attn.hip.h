// Paged decode attention as two task kinds (split-KV):
//   attn_chunk  (sequence b, kv head, chunk): online-softmax partial (m, l, o) of the group's query
//               heads over the chunk's keys, K/V rows gathered through the page table;
//   attn_merge  (sequence b, kv head): combines the chunk partials in ascending chunk order.
// Head dim D is split 8 elements per lane (16-byte loads of a bf16 K or V row slice), so D/8 lanes
// cover one key and a wavefront covers 64/(D/8) keys per load instruction; the 8 wavefronts of the
// workgroup stride over the chunk.  Reductions are wavefront shuffles, then LDS across waves.
// Cached K/V rows are read-only during the launch (ordinary loads).  The row appended by this step is
// not read back from the cache (where it is bf16) but taken in fp32 from the projection's scratch copy,
// so the new token enters its own attention unrounded; that copy, the queries and the partials cross
// tasks and are accessed with device-scope loads / stores.
#pragma once
#include "device_rt.hip.h"

namespace etc {

// Per-wavefront partial results of a chunk in LDS: kWaves entries, and one more for the step's own token where a
// wavefront's running softmax cannot take it (the matrix-core path): [entry][g] m, l, then [entry][g][D] o.
constexpr int kAttnEnt = kWaves + 1;
template <int GRP> constexpr int kAttnOff = (2 * kAttnEnt * GRP + 3) & ~3;      // floats in front of the o rows (which are read 16 bytes at a time)

template <int D, int GRP> __device__ __forceinline__ void attn_merge_chunks(const Params &P, int b, int kvh, int nc);

// The end of a chunk task: the first n_ent LDS entries (complete, behind a barrier) are reduced to the chunk's result,
// which is the attention output itself or one of the sequence's partial results.
template <int D, int GRP>
__device__ __forceinline__ void attn_finish(const Params &P, int b, int kvh, int ch, int n_keys, int n_ent, float *sm, int task_id)
{
    ETC_AS_LDS float *s_m = as_lds(sm);
    ETC_AS_LDS float *s_l = s_m + kAttnEnt * GRP;
    ETC_AS_LDS float *s_o = s_m + kAttnOff<GRP>;
    // A sequence that is one chunk long needs no partial results, no arrival count and no merge: what a merge of one
    // chunk would compute is exactly num / den below (three memory round trips less at the end of the task).
    const int nc = (n_keys + P.kv_chunk - 1) / P.kv_chunk;
    const bool whole = nc == 1 && P.attn_arrive != nullptr;
    for (int idx = threadIdx.x; idx < GRP * D / 4; idx += kWgThreads) {      // four consecutive elements per thread: 8-byte stores
        const int g = idx / (D / 4), i = (idx % (D / 4)) * 4;
        float m = -INFINITY;
        for (int wv = 0; wv < n_ent; ++wv) m = fmaxf(m, s_m[wv * GRP + g]);
        float num[4] = {0.f, 0.f, 0.f, 0.f}, den = 0.f;
        for (int wv = 0; wv < n_ent; ++wv) {
            const float wm = s_m[wv * GRP + g];
            const float sc = (wm == -INFINITY) ? 0.f : __expf(wm - m);
            const f32x4 ov = *reinterpret_cast<ETC_AS_LDS const f32x4 *>(s_o + (size_t)(wv * GRP + g) * D + i);
#pragma unroll
            for (int q = 0; q < 4; ++q) num[q] += sc * ov[q];
            den += sc * s_l[wv * GRP + g];
        }
        const int h = kvh * GRP + g;
        if (whole) {               // the sequence's only chunk: this is the attention output (operand of the O projection)
            uint16_t hi[4], lo[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) split_bf16(num[q] / den, hi[q], lo[q]);
            const size_t o1 = (size_t)b * (size_t)(P.nq * D) + (size_t)h * D + i;
            st_u64(P.attn_hi + o1, (uint64_t)hi[0] | ((uint64_t)hi[1] << 16) | ((uint64_t)hi[2] << 32) | ((uint64_t)hi[3] << 48));
            st_u64(P.attn_lo + o1, (uint64_t)lo[0] | ((uint64_t)lo[1] << 16) | ((uint64_t)lo[2] << 32) | ((uint64_t)lo[3] << 48));
        } else {
            const size_t pidx = ((size_t)b * P.nq + h) * (size_t)P.max_chunks + ch;
            st_u64(P.part_o + pidx * D + i, (uint64_t)__float_as_uint(num[0]) | ((uint64_t)__float_as_uint(num[1]) << 32));
            st_u64(P.part_o + pidx * D + i + 2, (uint64_t)__float_as_uint(num[2]) | ((uint64_t)__float_as_uint(num[3]) << 32));
            if (i == 0) { st_f32(P.part_m + pidx, m); st_f32(P.part_l + pidx, den); }
        }
    }
    // The chunk task that arrives last at its (sequence, KV head) merges the chunks itself: the merge is no stage of
    // its own, one all-to-all hand-over less per layer.  Arrival is counted with one returning atomic per task (behind
    // the drain of the partial results); the last one puts the counter back for the next launch.  Every chunk task
    // still notifies the one event of the attention block, the merging one after its merge.
    trace_mark(P, task_id, 3);
    if (P.attn_arrive != nullptr && !whole) {
        ETC_AS_LDS int32_t *s_last = reinterpret_cast<ETC_AS_LDS int32_t *>(s_o + (size_t)kAttnEnt * GRP * D);
        drain_vmem();
        __syncthreads();
        if (threadIdx.x == 0) {
            int32_t *ctr = P.attn_arrive + (size_t)b * P.nkv + kvh;
            const int last = __hip_atomic_fetch_add(as_global(ctr), 1, __ATOMIC_RELAXED, ETC_SCOPE) + 1 == nc;
            if (last) st_i32(ctr, 0);
            *s_last = last;
        }
        __syncthreads();
        if (*s_last) attn_merge_chunks<D, GRP>(P, b, kvh, nc);
    }
}

// ev0 / ev1: the events the task waits on (the queries and this step's K / V row of the KV head).  The cached K / V
// rows do not depend on them: a chunk of one batch requests its rows BEFORE it waits, like a projection task its
// weights, so that after the wait only the queries are a round trip away (3.72 -> 3.62 ms per 8B step).
template <int D, int GRP, bool PAGES_IN_LDS>
__device__ __noinline__ void attn_chunk(const Params &P, int layer, int b, int kvh, int ch, float *sm, int ev0, int ev1, int task_id)
{
    task_id = __builtin_amdgcn_readfirstlane(task_id);
    layer = __builtin_amdgcn_readfirstlane(layer);      // uniform arguments back into scalar registers
    b = __builtin_amdgcn_readfirstlane(b);
    kvh = __builtin_amdgcn_readfirstlane(kvh);
    ch = __builtin_amdgcn_readfirstlane(ch);
    ev0 = __builtin_amdgcn_readfirstlane(ev0);
    ev1 = __builtin_amdgcn_readfirstlane(ev1);
    constexpr int LPT = D / 8;        // lanes per key
    constexpr int TPW = 64 / LPT;     // keys per wavefront step
    const int wave = wave_id(), lane = lane_id();
    const int tq = lane / LPT, dl = lane % LPT;
    const int n_keys = gld_i32(P.kv_len + b) + 1;
    const int j0 = ch * P.kv_chunk;
    const int j1 = min(n_keys, j0 + P.kv_chunk);
    const int32_t *pages = P.page_ids + gld_i32(P.page_indptr + b);
    const size_t lbase = (size_t)layer * (size_t)P.pool_layer_stride;
    const float qscale = 1.0f / sqrtf((float)D);

    // qk_norm models: 1 / rms of a head from the per-tile sums of squares its projection tasks left (D / 16 of them)
    auto head_rnorm = [&](int head) {
        const float *sp = P.qk_ssq + ((size_t)b * (P.nq + P.nkv) + head) * (size_t)(D / 16);
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < D / 16; ++i) s += ld_f32(sp + i);
        return 1.0f / sqrtf(s / (float)D + P.eps);
    };
    // What the task needs from the tasks before it, requested in ONE round trip behind the wait: the group's queries
    // (with the sums of squares of their heads on qk_norm models) and, in the sequence's last chunk, the fp32 K / V row
    // of this step's token.
    float q[GRP][8];
    auto request_queries = [&]() {
#pragma unroll
        for (int g = 0; g < GRP; ++g) {
            const float *qp = P.qbuf + (size_t)b * (size_t)(P.nq * D) + (size_t)(kvh * GRP + g) * D + dl * 8;
#pragma unroll
            for (int i = 0; i < 8; i += 2) ld_f32x2(qp + i, q[g][i], q[g][i + 1]);
        }
    };
    auto scale_queries = [&]() {
#pragma unroll
        for (int g = 0; g < GRP; ++g) {
            const float sc = P.qk_norm ? qscale * head_rnorm(kvh * GRP + g) : qscale;
#pragma unroll
            for (int i = 0; i < 8; ++i) q[g][i] *= sc;
        }
    };
    float mx[GRP], l[GRP], o[GRP][8];
#pragma unroll
    for (int g = 0; g < GRP; ++g) {
        mx[g] = -INFINITY;
        l[g] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[g][i] = 0.f;
    }

    // The chunk's slice of the page table goes to LDS first (one round trip, shared with the query loads
    // above); keys are then taken in batches of BATCH wavefront steps: all K and V rows of a batch are
    // requested, then the arithmetic runs, so a batch costs one memory round trip.
    // (The base of the dynamic LDS is a table look-up in a function that is no kernel, and the compiler repeats that
    // load where the pointer is used: inside the key loop it would drain the K / V loads in flight.  An empty asm
    // statement makes the value opaque: it is computed once.)
    uint32_t pg_base = (uint32_t)(uintptr_t)(as_lds(sm) + 10240);                   // behind the 40 KB of reduction scratch
    asm volatile("" : "+v"(pg_base));
    ETC_AS_LDS int *s_pg = reinterpret_cast<ETC_AS_LDS int *>(pg_base);
    const int psh = P.page_shift, pmask = P.page - 1;          // pages hold a power of two of tokens
    const int pg0 = j0 >> psh, n_pg = ((j1 - 1) >> psh) - pg0 + 1;
    constexpr int BATCH = GRP >= 8 ? 2 : 4;       // 8 query heads per KV head leave registers for 2 steps per batch
    constexpr int STEP = BATCH * kWaves * TPW;    // keys the workgroup covers per batch
    // requests all K and V rows of the batch that starts at key jb0 (rows beyond the chunk re-read its last key)
    auto request = [&](int jb0, u32x4 (&krs)[BATCH], u32x4 (&vrs)[BATCH]) {
        int page[BATCH], jcs[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int j = jb0 + u * kWaves * TPW + tq;
            jcs[u] = j < j1 ? j : j1 - 1;
            page[u] = PAGES_IN_LDS ? s_pg[(jcs[u] >> psh) - pg0] : gld_i32(pages + (jcs[u] >> psh));
        }
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const size_t off = lbase + ((((size_t)page[u] << psh) + (size_t)(jcs[u] & pmask)) * P.nkv + kvh) * (size_t)D + dl * 8;
            krs[u] = gld_16B(P.kpool + off);
            vrs[u] = gld_16B(P.vpool + off);
        }
    };
    // Folds the batch's keys into the running softmax of every query head of the group.  The batch is taken as a
    // whole: all scores first, one new maximum and one rescale of the running sums per head, then the weighted rows
    // (half the exponentials and multiplies of a key-by-key update).  Keys beyond the chunk, and the new token (it is
    // handled after the loop, from its fp32 row), get the score -inf, i.e. the weight 0: no branch in here.
    auto fold = [&](int jb0, const u32x4 (&krs)[BATCH], const u32x4 (&vrs)[BATCH]) {
        float p[BATCH][GRP];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int j = jb0 + u * kWaves * TPW + tq;
            const bool valid = j < j1 && j != n_keys - 1;
            const u32x4 kr = krs[u];
            float kf[8];
            kf[0] = bf16_bits_to_f32(kr.x & 0xFFFFu); kf[1] = bf16_bits_to_f32(kr.x >> 16);
            kf[2] = bf16_bits_to_f32(kr.y & 0xFFFFu); kf[3] = bf16_bits_to_f32(kr.y >> 16);
            kf[4] = bf16_bits_to_f32(kr.z & 0xFFFFu); kf[5] = bf16_bits_to_f32(kr.z >> 16);
            kf[6] = bf16_bits_to_f32(kr.w & 0xFFFFu); kf[7] = bf16_bits_to_f32(kr.w >> 16);
#pragma unroll
            for (int g = 0; g < GRP; ++g) {
                float s = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) s += q[g][i] * kf[i];
                s = lanes_sum<LPT>(s);
                p[u][g] = valid ? s : -INFINITY;
            }
        }
#pragma unroll
        for (int g = 0; g < GRP; ++g) {
            float nm = mx[g];
#pragma unroll
            for (int u = 0; u < BATCH; ++u) nm = fmaxf(nm, p[u][g]);
            const float ref = fmaxf(nm, -1e30f);           // nothing seen yet: exp(-inf - ref) = 0 instead of exp(nan)
            const float sc = __expf(mx[g] - ref);
            float ls = l[g] * sc;
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                p[u][g] = __expf(p[u][g] - ref);
                ls += p[u][g];
            }
            l[g] = ls;
            mx[g] = nm;
#pragma unroll
            for (int i = 0; i < 8; ++i) o[g][i] *= sc;
        }
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const u32x4 vr = vrs[u];
            float vf[8];
            vf[0] = bf16_bits_to_f32(vr.x & 0xFFFFu); vf[1] = bf16_bits_to_f32(vr.x >> 16);
            vf[2] = bf16_bits_to_f32(vr.y & 0xFFFFu); vf[3] = bf16_bits_to_f32(vr.y >> 16);
            vf[4] = bf16_bits_to_f32(vr.z & 0xFFFFu); vf[5] = bf16_bits_to_f32(vr.z >> 16);
            vf[6] = bf16_bits_to_f32(vr.w & 0xFFFFu); vf[7] = bf16_bits_to_f32(vr.w >> 16);
#pragma unroll
            for (int g = 0; g < GRP; ++g)
#pragma unroll
                for (int i = 0; i < 8; ++i) o[g][i] += p[u][g] * vf[i];
        }
    };
    // The token of this step (last key of the sequence's last chunk) enters the running softmax FIRST, from the fp32 row
    // the projection tasks left: key group tq == 0 of wavefront 0 takes it.  Its loads share the queries' round trip;
    // at the end of the task they would be a round trip of their own.
    const bool takes_new = j1 == n_keys && wave == 0;            // uniform per wave
    auto fold_new_token = [&](float (&kf)[8], const float (&vf)[8]) {
        if (P.qk_norm) {       // K-Norm + RoPE + CacheAppend (Sec. 4.3): the key's norm is complete here, and so is its cache row
            const float rk = head_rnorm(P.nq + kvh);
#pragma unroll
            for (int i = 0; i < 8; ++i) kf[i] *= rk;
            if (tq == 0) {
                uint16_t *dst = P.kpool + lbase + ((size_t)gld_i32(P.kv_slot + b) * P.nkv + kvh) * (size_t)D + dl * 8;
                const u32x4 row{(uint32_t)f32_to_bf16_bits(kf[0]) | ((uint32_t)f32_to_bf16_bits(kf[1]) << 16),
                                (uint32_t)f32_to_bf16_bits(kf[2]) | ((uint32_t)f32_to_bf16_bits(kf[3]) << 16),
                                (uint32_t)f32_to_bf16_bits(kf[4]) | ((uint32_t)f32_to_bf16_bits(kf[5]) << 16),
                                (uint32_t)f32_to_bf16_bits(kf[6]) | ((uint32_t)f32_to_bf16_bits(kf[7]) << 16)};
                *as_global(reinterpret_cast<u32x4 *>(dst)) = row;      // nobody reads the cache row in this launch
            }
        }
#pragma unroll
        for (int g = 0; g < GRP; ++g) {
            float sc = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) sc += q[g][i] * kf[i];
            sc = lanes_sum<LPT>(sc);
            if (tq == 0) {         // the first key of this group's running softmax: weight exp(0) = 1
                mx[g] = sc;
                l[g] = 1.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) o[g][i] = vf[i];
            }
        }
    };
    auto after_wait = [&]() {      // queries and the new token: one round trip
        trace_mark(P, task_id, 1);
        request_queries();
        float kf[8], vf[8];
        if (takes_new) {
            const float *kn = P.knew + ((size_t)b * P.nkv + kvh) * (size_t)D + dl * 8;
            const float *vn = P.vnew + ((size_t)b * P.nkv + kvh) * (size_t)D + dl * 8;
#pragma unroll
            for (int i = 0; i < 8; i += 2) {
                ld_f32x2(kn + i, kf[i], kf[i + 1]);
                ld_f32x2(vn + i, vf[i], vf[i + 1]);
            }
        }
        scale_queries();
        if (takes_new) fold_new_token(kf, vf);
    };
    const int jb_first = j0 + wave * TPW;
    // Page ids and cached K / V rows are inputs of the step, not results of its tasks: the chunk's slice of the page
    // table and the rows of the first batch are requested BEFORE the wait, like a projection task's first weights.
    if (PAGES_IN_LDS) {            // long chunks: the page ids go through LDS
        for (int i = threadIdx.x; i < n_pg; i += kWgThreads) s_pg[i] = gld_i32(pages + pg0 + i);
        __syncthreads();
        u32x4 ka[BATCH], va[BATCH];
        request(jb_first, ka, va);
        wg_wait(P, ev0, ev1, FN_ATTN);
        after_wait();
        fold(jb_first, ka, va);
        for (int jb0 = jb_first + STEP; jb0 < j1; jb0 += STEP) {     // uniform trip count per wave
            request(jb0, ka, va);      // (a second batch in flight while this one is folded measured slower with 4 query
            fold(jb0, ka, va);         //  heads per KV head; with 8 the matrix-core path below takes the long chunks)
        }
    } else {                       // chunks of (about) one batch
        u32x4 krs[BATCH], vrs[BATCH];
        request(jb_first, krs, vrs);
        wg_wait(P, ev0, ev1, FN_ATTN);
        after_wait();
        fold(jb_first, krs, vrs);
        for (int jb0 = jb_first + STEP; jb0 < j1; jb0 += STEP) {
            request(jb0, krs, vrs);
            fold(jb0, krs, vrs);
        }
    }
    trace_mark(P, task_id, 2);

    // merge the TPW key groups of the wavefront (lanes differing in tq)
#pragma unroll
    for (int off2 = LPT; off2 < 64; off2 <<= 1) {
#pragma unroll
        for (int g = 0; g < GRP; ++g) {
            const float om = __shfl_xor(mx[g], off2, 64), ol = __shfl_xor(l[g], off2, 64);
            const float nm = fmaxf(mx[g], om);
            const float sa = (mx[g] == -INFINITY) ? 0.f : __expf(mx[g] - nm);
            const float sb = (om == -INFINITY) ? 0.f : __expf(om - nm);
            l[g] = l[g] * sa + ol * sb;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float oo = __shfl_xor(o[g][i], off2, 64);
                o[g][i] = o[g][i] * sa + oo * sb;
            }
            mx[g] = nm;
        }
    }
    // across wavefronts through LDS: [wave][g] -> m, l, o[D]
    ETC_AS_LDS float *s_m = as_lds(sm);                // [kAttnEnt][GRP]
    ETC_AS_LDS float *s_l = s_m + kAttnEnt * GRP;      // [kAttnEnt][GRP]
    ETC_AS_LDS float *s_o = s_m + kAttnOff<GRP>;  // [kAttnEnt][GRP][D]
    if (tq == 0) {
#pragma unroll
        for (int g = 0; g < GRP; ++g) {
            if (dl == 0) { s_m[wave * GRP + g] = mx[g]; s_l[wave * GRP + g] = l[g]; }
#pragma unroll
            for (int i = 0; i < 8; ++i) s_o[(size_t)(wave * GRP + g) * D + dl * 8 + i] = o[g][i];
        }
    }
    __syncthreads();
    attn_finish<D, GRP>(P, b, kvh, ch, n_keys, kWaves, sm, task_id);
}

// Long chunks on the matrix cores (head dim 128, 8 query heads per KV head).  With 8 query heads per key the VALU
// form above spends about 250 vector instructions per wavefront step of 4 keys and is bound by them, not by HBM, once a
// chunk is long (with 4 heads it keeps up with the memory system, and this path measured no faster).  Here a
// wavefront takes 32 keys per step, for about 280 vector and 32 matrix instructions:
//   scores   S^T[key][head] = K[key][:] . Q[head][:]   A = K rows straight from the cache (lane (key % 16, kg) loads
//            16 bytes of its key's row: the A fragment), B = the queries as split bf16 (hi and lo: two products), heads
//            padded to 16 columns.  The result lands as lane (head, kg) <- keys blk * 16 + kg * 4 + r: eight keys of one
//            head per lane, and in exactly the order the next product wants its A fragment in;
//   softmax  per lane over its 8 keys, the maximum across the four lane groups with two shuffles, the running sum kept
//            per lane until the end;
//   output   O[head][d] += P[head][key] . V[key][d]   A = P (hi and lo) as it stands in the lanes, B = V with eight KEYS
//            per lane: the V rows go through a wavefront-private LDS tile and come back as 2-byte reads.
// K and V rows of the next step are in flight while a step computes (V from the step's start, K from the end of its
// score products); the step's own token goes into an LDS entry of its own, next to the wavefronts' partial results.
template <int GRP>
__device__ __noinline__ void attn_chunk_mfma(const Params &P, int layer, int b, int kvh, int ch, float *sm, int ev0, int ev1, int task_id)
{
    static_assert(GRP == 4 || GRP == 8, "query heads per KV head");
    constexpr int D = 128, RS = 264;                     // RS: bytes between two rows of the V tile (264 = 66 words: 2-byte reads of 4 rows x 16 columns hit 32 different banks)
    task_id = __builtin_amdgcn_readfirstlane(task_id);
    layer = __builtin_amdgcn_readfirstlane(layer);
    b = __builtin_amdgcn_readfirstlane(b);
    kvh = __builtin_amdgcn_readfirstlane(kvh);
    ch = __builtin_amdgcn_readfirstlane(ch);
    ev0 = __builtin_amdgcn_readfirstlane(ev0);
    ev1 = __builtin_amdgcn_readfirstlane(ev1);
    const int wave = wave_id(), lane = lane_id();
    const int n16 = lane & 15, kg = lane >> 4;
    const int n_keys = gld_i32(P.kv_len + b) + 1;
    const int j0 = ch * P.kv_chunk;
    const int j1 = min(n_keys, j0 + P.kv_chunk);
    const int32_t *pages = P.page_ids + gld_i32(P.page_indptr + b);
    const size_t lbase = (size_t)layer * (size_t)P.pool_layer_stride;
    const float qscale = 1.0f / sqrtf((float)D);
    const int psh = P.page_shift, pmask = P.page - 1;
    const int pg0 = j0 >> psh, n_pg = ((j1 - 1) >> psh) - pg0 + 1;
    uint32_t pg_base = (uint32_t)(uintptr_t)(as_lds(sm) + 10240);                   // behind the 40 KB of reduction scratch
    asm volatile("" : "+v"(pg_base));                                               // computed once (see attn_chunk)
    ETC_AS_LDS int *s_pg = reinterpret_cast<ETC_AS_LDS int *>(pg_base);
    ETC_AS_LDS char *vst = reinterpret_cast<ETC_AS_LDS char *>(s_pg + ((n_pg + 3) & ~3)) + wave * (32 * RS);   // this wavefront's V tile [32 keys][RS]

    auto head_rnorm = [&](int head) {
        const float *sp = P.qk_ssq + ((size_t)b * (P.nq + P.nkv) + head) * (size_t)(D / 16);
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < D / 16; ++i) s += ld_f32(sp + i);
        return 1.0f / sqrtf(s / (float)D + P.eps);
    };
    // element offsets of this lane's two key rows (keys base + blk * 16 + n16) of a step, K and V pool alike
    auto row_offsets = [&](int base, size_t (&off)[2]) {
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            const int j = base + blk * 16 + n16;
            const int jc = j < j1 ? j : j1 - 1;                  // rows beyond the chunk re-read its last key
            const int page = s_pg[(jc >> psh) - pg0];
            off[blk] = lbase + ((((size_t)page << psh) + (size_t)(jc & pmask)) * P.nkv + kvh) * (size_t)D + kg * 8;
        }
    };
    auto request = [&](const uint16_t *pool, const size_t (&off)[2], u32x4 (&r)[2][4]) {
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) r[blk][kk] = gld_16B(pool + off[blk] + kk * 32);
    };

    // page ids and the rows of the wavefront's first step: before the wait
    for (int i = threadIdx.x; i < n_pg; i += kWgThreads) s_pg[i] = gld_i32(pages + pg0 + i);
    __syncthreads();
    const int n_groups = (j1 - j0 + 31) >> 5;
    u32x4 kr[2][4], vr[2][4];
    size_t off[2];
    row_offsets(j0 + wave * 32, off);
    request(P.vpool, off, vr);
    request(P.kpool, off, kr);
    wg_wait(P, ev0, ev1, FN_ATTN);
    trace_mark(P, task_id, 1);

    // ---- queries: B fragments, lane (head n16, kg) holds elements kk * 32 + kg * 8 .. + 8 of its head, hi and lo ----
    bf16x8 qhi[4], qlo[4];
    {
        const bool real = n16 < GRP;
        const int head = kvh * GRP + (real ? n16 : 0);
        const float *qp = P.qbuf + (size_t)b * (size_t)(P.nq * D) + (size_t)head * D + kg * 8;
        float qf[4][8];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int i = 0; i < 8; i += 2) ld_f32x2(qp + kk * 32 + i, qf[kk][i], qf[kk][i + 1]);
        const float sc = real ? (P.qk_norm ? qscale * head_rnorm(head) : qscale) : 0.f;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            uint32_t wh[4], wl[4];
#pragma unroll
            for (int i = 0; i < 8; i += 2) {
                uint16_t h0, l0, h1, l1;
                split_bf16(qf[kk][i] * sc, h0, l0);
                split_bf16(qf[kk][i + 1] * sc, h1, l1);
                wh[i >> 1] = (uint32_t)h0 | ((uint32_t)h1 << 16);
                wl[i >> 1] = (uint32_t)l0 | ((uint32_t)l1 << 16);
            }
            qhi[kk] = __builtin_bit_cast(bf16x8, u32x4{wh[0], wh[1], wh[2], wh[3]});
            qlo[kk] = __builtin_bit_cast(bf16x8, u32x4{wl[0], wl[1], wl[2], wl[3]});
        }
    }
    // ---- the token of this step: an LDS entry of its own (m = its score, l = 1, o = its V row), by wavefront 0 ----
    ETC_AS_LDS float *s_m = as_lds(sm);
    ETC_AS_LDS float *s_l = s_m + kAttnEnt * GRP;
    ETC_AS_LDS float *s_o = s_m + kAttnOff<GRP>;
    const bool has_new = j1 == n_keys;
    if (has_new && wave == 0) {
        const int dl = n16, tq = kg;                    // 16 lanes x 8 elements cover a head; 4 heads at a time
        const float *kn = P.knew + ((size_t)b * P.nkv + kvh) * (size_t)D + dl * 8;
        const float *vn = P.vnew + ((size_t)b * P.nkv + kvh) * (size_t)D + dl * 8;
        float kf[8], vf[8];
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
            ld_f32x2(kn + i, kf[i], kf[i + 1]);
            ld_f32x2(vn + i, vf[i], vf[i + 1]);
        }
        if (P.qk_norm) {       // K-Norm + RoPE + CacheAppend (Sec. 4.3): the key's norm is complete here, and so is its cache row
            const float rk = head_rnorm(P.nq + kvh);
#pragma unroll
            for (int i = 0; i < 8; ++i) kf[i] *= rk;
            if (tq == 0) {
                uint16_t *dst = P.kpool + lbase + ((size_t)gld_i32(P.kv_slot + b) * P.nkv + kvh) * (size_t)D + dl * 8;
                const u32x4 row{(uint32_t)f32_to_bf16_bits(kf[0]) | ((uint32_t)f32_to_bf16_bits(kf[1]) << 16),
                                (uint32_t)f32_to_bf16_bits(kf[2]) | ((uint32_t)f32_to_bf16_bits(kf[3]) << 16),
                                (uint32_t)f32_to_bf16_bits(kf[4]) | ((uint32_t)f32_to_bf16_bits(kf[5]) << 16),
                                (uint32_t)f32_to_bf16_bits(kf[6]) | ((uint32_t)f32_to_bf16_bits(kf[7]) << 16)};
                *as_global(reinterpret_cast<u32x4 *>(dst)) = row;      // nobody reads the cache row in this launch
            }
        }
#pragma unroll
        for (int pass = 0; pass < GRP / 4; ++pass) {
            const int g = pass * 4 + tq, head = kvh * GRP + g;
            const float *qp = P.qbuf + (size_t)b * (size_t)(P.nq * D) + (size_t)head * D + dl * 8;
            float qv[8];
#pragma unroll
            for (int i = 0; i < 8; i += 2) ld_f32x2(qp + i, qv[i], qv[i + 1]);
            const float sc = P.qk_norm ? qscale * head_rnorm(head) : qscale;
            float sdot = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) sdot += qv[i] * sc * kf[i];
            sdot = lanes_sum<16>(sdot);
            if (dl == 0) { s_m[kWaves * GRP + g] = sdot; s_l[kWaves * GRP + g] = 1.f; }
#pragma unroll
            for (int i = 0; i < 8; ++i) s_o[(size_t)(kWaves * GRP + g) * D + dl * 8 + i] = vf[i];
        }
    }

    // ---- the wavefront's steps: 32 keys each -------------------------------------------------------------------
    f32x4 oacc[8];                                       // O[head kg * 4 + r][db * 16 + n16]
#pragma unroll
    for (int db = 0; db < 8; ++db) oacc[db] = f32x4{0, 0, 0, 0};
    float mrun = -INFINITY, lrun = 0.f;                  // of head n16, over the keys this lane has seen
    for (int gi = wave; gi < n_groups; gi += kWaves) {   // uniform per wavefront
        const int base = j0 + gi * 32;
        drain_vmem();                                    // K and V rows of this step are here
        // V rows -> the wavefront's LDS tile, then the next step's V rows into the same registers
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                ETC_AS_LDS uint64_t *dst = reinterpret_cast<ETC_AS_LDS uint64_t *>(vst + (blk * 16 + n16) * RS + kk * 64 + kg * 16);
                dst[0] = (uint64_t)vr[blk][kk].x | ((uint64_t)vr[blk][kk].y << 32);
                dst[1] = (uint64_t)vr[blk][kk].z | ((uint64_t)vr[blk][kk].w << 32);
            }
        row_offsets(base + kWaves * 32, off);            // beyond the chunk: its last key again, never used
        request(P.vpool, off, vr);
        // scores
        f32x4 sacc[2] = {f32x4{0, 0, 0, 0}, f32x4{0, 0, 0, 0}};
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const bf16x8 kf = __builtin_bit_cast(bf16x8, kr[blk][kk]);
                sacc[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qhi[kk], sacc[blk], 0, 0, 0);
                sacc[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qlo[kk], sacc[blk], 0, 0, 0);
            }
        __builtin_amdgcn_sched_barrier(0);               // the refill lands in the registers the products have just read
        request(P.kpool, off, kr);
        // softmax over this lane's 8 keys (blk * 16 + kg * 4 + r) of head n16
        float sv[8];
        float mloc = -INFINITY;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int key = base + (j >> 2) * 16 + kg * 4 + (j & 3);
            const bool valid = key < j1 && key != n_keys - 1;          // the step's own token: from its fp32 row, above
            sv[j] = valid ? sacc[j >> 2][j & 3] : -INFINITY;
            mloc = fmaxf(mloc, sv[j]);
        }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 16, 64));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
        const float nm = fmaxf(mrun, mloc);
        const float ref = fmaxf(nm, -1e30f);             // nothing seen yet: exp(-inf - ref) = 0 instead of exp(nan)
        const float sc = __expf(mrun - ref);
        float psum = 0.f;
        uint32_t ph[4], pl[4];
#pragma unroll
        for (int j = 0; j < 8; j += 2) {
            const float p0 = __expf(sv[j] - ref), p1 = __expf(sv[j + 1] - ref);
            psum += p0 + p1;
            uint16_t h0, l0, h1, l1;
            split_bf16(p0, h0, l0);
            split_bf16(p1, h1, l1);
            ph[j >> 1] = (uint32_t)h0 | ((uint32_t)h1 << 16);
            pl[j >> 1] = (uint32_t)l0 | ((uint32_t)l1 << 16);
        }
        lrun = lrun * sc + psum;
        mrun = nm;
        const bf16x8 phi = __builtin_bit_cast(bf16x8, u32x4{ph[0], ph[1], ph[2], ph[3]});
        const bf16x8 plo = __builtin_bit_cast(bf16x8, u32x4{pl[0], pl[1], pl[2], pl[3]});
        // running output: rows are heads kg * 4 + r, whose rescale factors sit in lanes kg * 4 + r
        if (__builtin_amdgcn_ballot_w64(sc != 1.0f) != 0) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float scr = __int_as_float(__builtin_amdgcn_ds_bpermute((kg * 4 + r) * 4, __float_as_int(sc)));
#pragma unroll
                for (int db = 0; db < 8; ++db) oacc[db][r] *= scr;
            }
        }
        // O += P . V: lane (column n16 of block db, kg) takes keys (j >> 2) * 16 + kg * 4 + (j & 3), j = 0..7, from the tile
        ETC_AS_LDS const char *vcol = vst + (kg * 4) * RS + n16 * 2;
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            uint32_t w[4];
#pragma unroll
            for (int j = 0; j < 8; j += 2) {
                const uint32_t a = *reinterpret_cast<ETC_AS_LDS const uint16_t *>(vcol + ((j >> 2) * 16 + (j & 3)) * RS + db * 32);
                const uint32_t c = *reinterpret_cast<ETC_AS_LDS const uint16_t *>(vcol + ((j >> 2) * 16 + (j & 3) + 1) * RS + db * 32);
                w[j >> 1] = a | (c << 16);
            }
            const bf16x8 vf = __builtin_bit_cast(bf16x8, u32x4{w[0], w[1], w[2], w[3]});
            oacc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(phi, vf, oacc[db], 0, 0, 0);
            oacc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(plo, vf, oacc[db], 0, 0, 0);
        }
    }
    trace_mark(P, task_id, 2);

    // ---- the wavefront's partial result: entry `wave` of the LDS table ----
    lrun += __shfl_xor(lrun, 16, 64);                    // the four lane groups saw different keys
    lrun += __shfl_xor(lrun, 32, 64);
    if (kg == 0 && n16 < GRP) { s_m[wave * GRP + n16] = mrun; s_l[wave * GRP + n16] = lrun; }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int g = kg * 4 + r;
        if (g < GRP) {
#pragma unroll
            for (int db = 0; db < 8; ++db) s_o[(size_t)(wave * GRP + g) * D + db * 16 + n16] = oacc[db][r];
        }
    }
    __syncthreads();
    attn_finish<D, GRP>(P, b, kvh, ch, n_keys, has_new ? kWaves + 1 : kWaves, sm, task_id);
}

// Merge of the chunk partials of (sequence b, KV head kvh): ascending chunk order, whoever runs it.
template <int D, int GRP>
__device__ __forceinline__ void attn_merge_chunks(const Params &P, int b, int kvh, int nc)
{
    for (int idx = threadIdx.x; idx < GRP * D; idx += kWgThreads) {
        const int g = idx / D, i = idx % D;
        const int h = kvh * GRP + g;
        const size_t p0 = ((size_t)b * P.nq + h) * (size_t)P.max_chunks;
        // one pass in ascending chunk order, 16 chunks' loads in flight at a time, running max rescaling
        float m = -INFINITY, num = 0.f, den = 0.f;
        for (int c0 = 0; c0 < nc; c0 += 16) {
            float pm[16], pl[16], po[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int c = c0 + u < nc ? c0 + u : nc - 1;
                pm[u] = ld_f32(P.part_m + p0 + c);
                pl[u] = ld_f32(P.part_l + p0 + c);
                po[u] = ld_f32(P.part_o + (p0 + c) * D + i);
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                if (c0 + u < nc) {
                    const float nm = fmaxf(m, pm[u]);
                    const float sa = __expf(m - nm), sb = __expf(pm[u] - nm);
                    num = num * sa + sb * po[u];
                    den = den * sa + sb * pl[u];
                    m = nm;
                }
            }
        }
        uint16_t hi, lo;                               // operand of the O projection: split bf16
        split_bf16(num / den, hi, lo);
        const size_t o = (size_t)b * (size_t)(P.nq * D) + (size_t)h * D + i;
        st_u16(P.attn_hi + o, hi);
        st_u16(P.attn_lo + o, lo);
    }
}

// The merge as a task of its own (graphs that keep a merge stage).
template <int D, int GRP>
__device__ __noinline__ void attn_merge(const Params &P, int b, int kvh)
{
    b = __builtin_amdgcn_readfirstlane(b);
    kvh = __builtin_amdgcn_readfirstlane(kvh);
    const int n_keys = gld_i32(P.kv_len + b) + 1;
    attn_merge_chunks<D, GRP>(P, b, kvh, (n_keys + P.kv_chunk - 1) / P.kv_chunk);
}

}  // namespace etc
