// Projection tile task: 16 weight rows x K against up to 64 activation columns, bf16 MFMA with
// fp32 accumulation (v_mfma_f32_16x16x32_bf16), weights streamed from HBM exactly once.
//
// Work split.  The 8 wavefronts of the workgroup split K; each streams its slice of all 16 rows with
// 16-byte non-temporal loads, keeping PF loads (PF KB per wave, 128 KB per CU) in flight.  The first
// PF loads are issued BEFORE the task waits on its events (weight prefetch, paper Sec. 3.4 / 4.3), so
// HBM keeps streaming while the dependency resolves.
//
// Activation operand.  Activations reach the MFMA as bf16, which alone would cost ~2^-9 relative error
// per projection and break the 2e-2 parity bar after a few dozen layers.  The PRODUCER of an activation
// therefore stores it as two bf16 numbers, hi + lo (16 mantissa bits), and the tile issues two MFMAs per
// weight fragment (hi and lo); the matrix pipe is <10 % busy in this HBM-bound regime, so this is free.
// RMSNorm is folded in the same way: the producer stores (x * gain) split, plus one partial sum of
// squares per 16-row tile; the consumer sums the partials in a fixed order and scales its accumulator
// by 1/sqrt(mean(x^2)+eps) in the epilogue (the norm factor is a per-column scalar, so it commutes
// with the contraction).  No separate norm task, no extra event hop.
//
// The 16 rows of a tile are two groups of 8 (rowsA, rowsB): a RoPE tile takes rows i..i+7 and
// i+d/2..i+d/2+7 of one head (8 rotation pairs), a SwiGLU tile takes 8 gate rows and the 8 matching
// up rows, plain tiles take 16 consecutive rows.  Partial tiles of the 8 waves are reduced through LDS
// in a fixed order (deterministic), then the epilogue runs on 8 x columns threads.
#pragma once
#include "device_rt.hip.h"

namespace etc {

struct GemmTile {
    const uint16_t *rowsA, *rowsB;   // bf16 weights, first row of each 8-row group
    int ldw;                         // weight row stride (elements)
    int K;                           // reduction length, multiple of 256
    const uint16_t *b_hi, *b_lo;     // activation operand, split bf16, [rows, ldb]
    int ldb;
    const int32_t *col_rows;         // optional gather: column n reads operand row col_rows[n]
    int n_cols;                      // valid columns (batch rows or routed tokens), <= 64
    const float *ssq_parts;          // RMSNorm: partial sums of squares [n_parts][ssq_stride], or null
    int n_parts;
    int ssq_stride;
    float eps;
    int n_tiles;                     // consecutive 16-row tiles this task streams back to back
    int tile_rows;                   // rows between consecutive tiles inside each 8-row group (8 or 16)
};

constexpr uint16_t EPF_DUMP_LAYER = 0x8000;   // epilogue also records the layer's hidden state

enum EpiKind : int { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_STORE_F32 = 3, EPI_MOE_ACT = 4, EPI_MOE_Y = 5,
                     EPI_PARTIAL = 6, EPI_LOGITS = 7 };   // PARTIAL: fp32 sums over one slice of K, [row tile][kMaxBatch][16], outf = the slice's block

struct Epilogue {
    int kind;
    int layer;
    uint16_t flags;
    int row0;                 // first output row (RESID / STORE), first f (SWIGLU), first pair index (QKV)
    int head;                 // QKV: global head index (q heads, then k heads, then v heads)
    const float *resid;       // RESID: [*, ld] fp32 added to the result
    float *outf;              // fp32 destination
    uint16_t *out_hi, *out_lo;// split-bf16 destination (operand of the consuming projection)
    const uint16_t *next_gain;// RESID: gain the consumer's RMSNorm applies (null: no operand is prepared)
    float *ssq_out;           // RESID: this tile's partial sums of squares [kMaxBatch]
    int ld;                   // destination row stride
    int col0;                 // MoE: first destination row (permuted row of column 0)
    ETC_AS_LDS unsigned long long *lds_best;   // LOGITS: the task's running maxima per column, in LDS (set by the projection path)
};

// What an epilogue thread needs from memory, fetched before the streaming loop so that the epilogue
// itself issues no load (a load issued behind the weight stream returns only after it: memory
// operations of a wavefront complete in order).
struct EpiPre {
    float a, b;       // RESID: the two residual values; QKV: cos and sin of the rotation angle
    float ga, gb;     // RESID: gains of the two rows for the consumer's operand
    int slot;         // QKV (k / v heads): KV slot of the appended row (page * page_size + position in the page)
};
__device__ __forceinline__ EpiPre epilogue_preload(const Params &P, const Epilogue &e, int col, int mp);
template <bool LM>
__device__ __forceinline__ void apply_epilogue(const Params &P, const Epilogue &e, int col, int mp, float lo, float hi,
                                               const EpiPre &pre);

constexpr int PF = 16;                            // weight loads in flight per lane (16 KB per wave)

__device__ __forceinline__ u32x4 load16_nt(const uint16_t *p) { return gld_16B_nt(p); }
__device__ __forceinline__ void ld_f32x2_pair(const float *p, float &a, float &b) { a = ld_f32(p); b = ld_f32(p + 8); }

// Waits of a projection task.  per_wave: wave w waits on ev0 + w (its own K slice) on its own.
struct TaskWaits {
    int ev0, ev1, fn;
    bool per_wave;
    int op_key;          // identifies the operand a staged copy in LDS holds (-1: never reuse a copy)
};

// State a persistent workgroup carries from task to task (uniform across the workgroup).
struct WgState {
    int zero0, zero1;    // events already seen at zero in this launch (they never re-arm inside a launch)
    int staged_key;      // operand currently staged in LDS (-1: none)
    int routed_layer;    // MoE layer whose routing tables this workgroup has already seen complete (-1: none)
};

__device__ __forceinline__ void wg_state_init(WgState &st)
{
    st.zero0 = st.zero1 = -1;
    st.staged_key = -1;
    st.routed_layer = -1;
}

__device__ __forceinline__ bool event_known_zero(const WgState &st, int ev) { return ev < 0 || ev == st.zero0 || ev == st.zero1; }

__device__ __forceinline__ const uint16_t *lane_weight_row(const GemmTile &g)
{
    const int wave = wave_id(), lane = lane_id();
    const int m = lane & 15, kg = lane >> 4;
    const int kbase = wave * (g.K / kWaves) + kg * 8;
    return (m < 8 ? g.rowsA + (size_t)m * (size_t)g.ldw : g.rowsB + (size_t)(m - 8) * (size_t)g.ldw) + kbase;
}

// Workgroup wait with a two-entry cache of events already known to have fired.
__device__ __forceinline__ void wg_wait_cached(const Params &P, WgState &st, int ev0, int ev1, int fn)
{
    const bool need0 = ev0 >= 0 && ev0 != st.zero0 && ev0 != st.zero1;
    const bool need1 = ev1 >= 0 && ev1 != st.zero0 && ev1 != st.zero1;
    if (!need0 && !need1) return;
    wg_wait(P, need0 ? ev0 : -1, need1 ? ev1 : -1, fn);
    if (need0) { st.zero1 = st.zero0; st.zero0 = ev0; }
    if (need1) { st.zero1 = st.zero0; st.zero0 = ev1; }
}

// Latency-critical path (at most 16 columns whose whole operand fits in LDS).  The operand (all columns,
// full K, hi and lo) is copied into LDS once per stage with device-scope loads and reused by every
// tile of that stage this workgroup runs.  A task streams its n_tiles row tiles back to back through a
// ring of PF weight fragments per lane that never drains between tiles; each wave parks its partial
// tile in LDS; one barrier, one reduction and one epilogue per task.
//
// Order of memory operations.  A wavefront's loads return in order, so anything issued behind the
// weight stream waits for it.  The first PF weight loads are issued BEFORE the task waits on its events
// (weight prefetch, Sec. 3.4); the epilogue's inputs are fetched before the streaming loop, so the
// epilogue issues no load.  Measured alternatives that lost: streaming the NEXT task's first fragments
// during the tail of the loop (the epilogue's loads and the drain before the notify then queue behind that
// stream: +10 % per step); keeping the polling wavefront's queue free of weight loads until the event is
// seen (+2 %); one control wavefront that polls, stages and runs the epilogue while seven wavefronts
// stream (+10 %: the compute unit's read rate follows the bytes it keeps in flight, and the gap between
// two stages is longer than what its registers can buffer either way).
//
// Shape of the streaming loop.  The task's weights are ONE linear stream of (tile, step) pairs; an issue cursor
// runs PF steps ahead of the consume cursor.  The compiler places wait counts per basic block, and what it
// cannot follow it answers with a full drain of the loads in flight, so the loop is written for it:
//   - the steady state (whole revolutions of the ring whose look-ahead steps all exist) has no branch around
//     a load, and so have the common endings (one revolution left; one and a half);
//   - a ring slot is refilled BEHIND the MFMAs that read it, so the new fragment can land in the same
//     registers: refilled in front of them it needs other registers, and the copy back at the loop's end
//     waits for every load of the revolution.
// With both, every step waits for exactly the oldest of the PF loads (4.08 -> 3.94 ms per 8B step).
template <int PRE, bool LM>
__device__ __forceinline__ void gemm_tiles_staged(const Params &P, const GemmTile &g, const Epilogue &e, const TaskWaits &w,
                                                  float *sm, WgState &st, int task_id)
{
    static_assert(PRE >= 1 && PRE <= PF, "ring slots requested before the wait");
    const int wave = wave_id(), lane = lane_id();
    const int m = lane & 15, kg = lane >> 4;
    const int Kw = g.K / kWaves, n_it = Kw >> 5;
    const int kbase = wave * Kw + kg * 8;
    const uint16_t *wcur = lane_weight_row(g);
    const size_t tile_step = (size_t)g.tile_rows * (size_t)g.ldw;

    ETC_AS_LDS float *red = as_lds(sm);               // [tile][wave][col][16 rows]
    ETC_AS_LDS float *rs = red + staged_red_floats(g.n_tiles, g.n_cols);
    ETC_AS_LDS uint16_t *op_hi = reinterpret_cast<ETC_AS_LDS uint16_t *>(rs + kRsFloats);
    const int Kp = g.K + kOpPad;                        // column stride of the operand in LDS
    ETC_AS_LDS uint16_t *op_lo = op_hi + (size_t)g.n_cols * Kp;

    const int key = w.op_key;
    const bool restage = key < 0 || key != st.staged_key;
    // The task's weights are one linear stream of (tile, step) pairs: step s of tile t sits at wcur + t * tile_step +
    // 32 s.  The issue cursor runs PF steps ahead of the consume cursor through that stream.
    const int total = g.n_tiles * n_it;
    const long long tile_jump = (long long)tile_step - (long long)n_it * 32;
    const uint16_t *ip = wcur;                        // address of the next step to request
    int is = 0;                                       // its step inside its tile
    auto advance_issue = [&]() {
        ++is;
        ip += 32;
        const bool wrap = is == n_it;
        ip += wrap ? tile_jump : 0;
        is = wrap ? 0 : is;
    };
    u32x4 wr[PF];
    // Of the PF ring slots, PRE are requested before the task waits on its events and the rest behind the
    // operand once the events have fired: the poll and the operand queue behind whatever was prefetched, which
    // costs the workgroup that arrives last (and sets the stage's end) what it gains the early ones.  Measured:
    // 8B step (staged-only instance) 8 / 10 / 12 / 14 / 16 slots = 3.95 / 3.88 / 3.88 / 3.95 / 3.92 ms; the MoE
    // step is 5 % faster with all 16 (its tasks are small and many), so the count is a parameter of the instance.
    auto prefetch_range = [&](int j0, int j1) {
#pragma unroll
        for (int j = 0; j < PF; ++j) {
            if (j >= j0 && j < j1) {
                if (j < total) {
                    wr[j] = load16_nt(ip);
                    advance_issue();
                } else {
                    wr[j] = u32x4{0, 0, 0, 0};
                }
            }
        }
    };
    auto prefetch = [&]() { prefetch_range(0, PF); };
    // A task that has nothing to wait for (its events are already known to have fired, or it runs without
    // events in the kernel-by-kernel comparator) issues its operand loads first and the weight stream right
    // behind them: loads return in order, so the operand would otherwise arrive a full round trip under load
    // later.  A task that has to wait prefetches first.  (Deciding this with one extra poll at task start was
    // measured: the round trip it adds on every workgroup costs more than it saves on the last one.)
    const bool will_wait = restage ? (!event_known_zero(st, w.ev0) || w.per_wave || !event_known_zero(st, w.ev1))
                                   : !event_known_zero(st, w.ev1);
    const bool fired = !will_wait;
    if (!fired) prefetch_range(0, PRE);

    // What the epilogue will need (single pass of the epilogue loop only) is requested right behind the operand:
    // it is back by the time the operand sits in LDS, and the streaming loop starts without another round trip.
    const int per_tile = g.n_cols * 8;
    const int n_out = g.n_tiles * per_tile;
    const bool pre_ok = n_out <= kWgThreads;
    EpiPre pre{};
    auto request_epilogue_inputs = [&]() {
        if (pre_ok && (int)threadIdx.x < n_out) {
            const int ti = (int)threadIdx.x / per_tile, r = (int)threadIdx.x - ti * per_tile;
            Epilogue et = e;
            et.row0 = e.row0 + ti * g.tile_rows;
            pre = epilogue_preload(P, et, r >> 3, r & 7);
        }
    };

    if (restage) {
        // ---- E.wait() ---------------------------------------------------------------------------
        if (fired) {
            if (!w.per_wave && !event_known_zero(st, w.ev0)) { st.zero1 = st.zero0; st.zero0 = w.ev0; }
            if (!event_known_zero(st, w.ev1)) { st.zero1 = st.zero0; st.zero0 = w.ev1; }
        } else if (w.per_wave) {    // the staged copy needs every K slice: lanes 0..7 of wave 0 poll one slice each
            if (wave == 0 && lane < kWaves) spin_until_zero(P, w.ev0 + lane, w.fn);
            if (threadIdx.x == 0 && w.ev1 >= 0) spin_until_zero(P, w.ev1, w.fn);
            __syncthreads();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        } else {
            wg_wait_cached(P, st, w.ev0, w.ev1, w.fn);
        }
        trace_mark(P, task_id, 1);
        // ---- stage the operand: all loads of a thread in flight at once ---------------------------
        constexpr int U = 8;
        const int quads = g.K >> 2;                         // 8-byte pieces per column
        const int total = g.n_cols * quads;
        float sq[8];                                        // RMSNorm: this lane's partial sums of squares of column `wave`
        const bool one_col_per_wave = g.ssq_parts != nullptr && g.n_cols <= kWaves && g.n_parts <= 512;
        if (total <= kWgThreads * U) {
            uint64_t vh[U], vl[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int idx = (int)threadIdx.x + u * kWgThreads;
                vh[u] = vl[u] = 0;
                if (idx < total) {
                    const int col = idx / quads, q = idx - col * quads;
                    int row = g.col_rows ? ld_i32(g.col_rows + col) : col;
                    if (row < 0) row = 0;
                    vh[u] = ld_u64(g.b_hi + (size_t)row * (size_t)g.ldb + q * 4);
                    vl[u] = ld_u64(g.b_lo + (size_t)row * (size_t)g.ldb + q * 4);
                }
            }
            if (one_col_per_wave && wave < g.n_cols) {
                const int row = g.col_rows ? ld_i32(g.col_rows + wave) : wave;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int pt = lane + 64 * j;
                    sq[j] = (pt < g.n_parts && row >= 0) ? ld_f32(g.ssq_parts + (size_t)pt * (size_t)g.ssq_stride + row) : 0.f;
                }
            }
            request_epilogue_inputs();
            if (fired) prefetch(); else prefetch_range(PRE, PF);   // right behind the operand loads
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int idx = (int)threadIdx.x + u * kWgThreads;
                if (idx < total) {
                    const int col = idx / quads, q = idx - col * quads;
                    *reinterpret_cast<ETC_AS_LDS uint64_t *>(op_hi + (size_t)col * Kp + q * 4) = vh[u];
                    *reinterpret_cast<ETC_AS_LDS uint64_t *>(op_lo + (size_t)col * Kp + q * 4) = vl[u];
                }
            }
        } else {
            for (int idx = threadIdx.x; idx < total; idx += kWgThreads) {
                const int col = idx / quads, q = idx - col * quads;
                int row = g.col_rows ? ld_i32(g.col_rows + col) : col;
                if (row < 0) row = 0;
                const uint64_t vh = ld_u64(g.b_hi + (size_t)row * (size_t)g.ldb + q * 4);
                const uint64_t vl = ld_u64(g.b_lo + (size_t)row * (size_t)g.ldb + q * 4);
                *reinterpret_cast<ETC_AS_LDS uint64_t *>(op_hi + (size_t)col * Kp + q * 4) = vh;
                *reinterpret_cast<ETC_AS_LDS uint64_t *>(op_lo + (size_t)col * Kp + q * 4) = vl;
            }
            if (one_col_per_wave && wave < g.n_cols) {
                const int row = g.col_rows ? ld_i32(g.col_rows + wave) : wave;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int pt = lane + 64 * j;
                    sq[j] = (pt < g.n_parts && row >= 0) ? ld_f32(g.ssq_parts + (size_t)pt * (size_t)g.ssq_stride + row) : 0.f;
                }
            }
            request_epilogue_inputs();
            if (fired) prefetch(); else prefetch_range(PRE, PF);
        }
        if (g.ssq_parts) {       // RMSNorm factor of every column: fixed-order sum of the producers' partial sums of squares
            if (one_col_per_wave) {
                if (wave < g.n_cols) {
                    float s = ((sq[0] + sq[1]) + (sq[2] + sq[3])) + ((sq[4] + sq[5]) + (sq[6] + sq[7]));
                    s = wave_sum(s);
                    if (lane == 0) rs[wave] = 1.0f / sqrtf(s / (float)g.K + g.eps);
                }
            } else {
                for (int col = wave; col < g.n_cols; col += kWaves) {
                    const int row = g.col_rows ? ld_i32(g.col_rows + col) : col;
                    float s = 0.f;
                    if (row >= 0)
                        for (int pt = lane; pt < g.n_parts; pt += 64) s += ld_f32(g.ssq_parts + (size_t)pt * (size_t)g.ssq_stride + row);
                    s = wave_sum(s);
                    if (lane == 0) rs[col] = 1.0f / sqrtf(s / (float)g.K + g.eps);
                }
            }
        }
        st.staged_key = key;
        __syncthreads();
    } else {
        if (fired) {
            if (!event_known_zero(st, w.ev1)) { st.zero1 = st.zero0; st.zero0 = w.ev1; }
            request_epilogue_inputs();
            prefetch();
        } else {
            wg_wait_cached(P, st, w.ev1, -1, w.fn);
            request_epilogue_inputs();
            prefetch_range(PRE, PF);
        }
    }
    trace_mark(P, task_id, 2);

    const bool valid = m < g.n_cols;
    ETC_AS_LDS const uint16_t *sh = op_hi + (size_t)(valid ? m : 0) * (size_t)Kp + kbase;
    ETC_AS_LDS const uint16_t *sl = op_lo + (size_t)(valid ? m : 0) * (size_t)Kp + kbase;
    // Consume cursor: step sc of tile tc.  Columns beyond n_cols read column 0's operand (never stored).
    f32x4 acc = f32x4{0, 0, 0, 0};
    int sc = 0, tc = 0;
#define ETC_STAGED_STEP(j, RELOAD)                                                                               \
    {                                                                                                             \
        const bf16x8 a = __builtin_bit_cast(bf16x8, wr[j]);                                                       \
        const u32x4 bh = *reinterpret_cast<ETC_AS_LDS const u32x4 *>(sh + sc * 32);                               \
        const u32x4 bl = *reinterpret_cast<ETC_AS_LDS const u32x4 *>(sl + sc * 32);                               \
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, bh), acc, 0, 0, 0);           \
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, bl), acc, 0, 0, 0);           \
        if (RELOAD) {           /* behind the MFMAs that read the slot: the load can land in the same registers */ \
            wr[j] = load16_nt(ip);                                                                                \
            advance_issue();                                                                                      \
        }                                                                                                         \
        if (++sc == n_it) {     /* tile done: lane holds rows 4*kg .. 4*kg+3 of column m */                       \
            if (valid)                                                                                            \
                *reinterpret_cast<ETC_AS_LDS f32x4 *>(red + ((size_t)(tc * kWaves + wave) * g.n_cols + m) * 16 + 4 * kg) = acc; \
            acc = f32x4{0, 0, 0, 0};                                                                              \
            sc = 0;                                                                                               \
            ++tc;                                                                                                 \
        }                                                                                                         \
    }
    // Steady state: whole ring revolutions whose look-ahead steps all exist.  No branch around a load here: the
    // compiler places its wait counts per basic block, and a conditional load turns the waits behind it into full
    // drains of the ring.
    int q = 0;
    for (; q + 2 * PF <= total; q += PF) {
#pragma unroll
        for (int j = 0; j < PF; ++j) ETC_STAGED_STEP(j, true)
    }
    if (total - q == PF) {                           // one whole revolution left: nothing to request, nothing to test
#pragma unroll
        for (int j = 0; j < PF; ++j) ETC_STAGED_STEP(j, false)
        q = total;
    } else if (total - q == PF + PF / 2) {           // one and a half (K = 3.5 revolutions per tile, one tile)
#pragma unroll
        for (int j = 0; j < PF / 2; ++j) ETC_STAGED_STEP(j, true)
#pragma unroll
        for (int j = PF / 2; j < PF; ++j) ETC_STAGED_STEP(j, false)
#pragma unroll
        for (int j = 0; j < PF / 2; ++j) ETC_STAGED_STEP(j, false)
        q = total;
    }
    for (; q < total; q += PF) {                     // the last revolutions of any other length
#pragma unroll
        for (int j = 0; j < PF; ++j) {
            if (q + j < total) {
                if (q + j + PF < total) ETC_STAGED_STEP(j, true)
                else ETC_STAGED_STEP(j, false)
            }
        }
    }
#undef ETC_STAGED_STEP

    // ---- one reduction (fixed wave order) and one epilogue for all tiles of the task -------------
    trace_mark(P, task_id, 3);
    ETC_AS_LDS unsigned long long *lbest = reinterpret_cast<ETC_AS_LDS unsigned long long *>(rs + kRsFloats / 2);   // [16]
    const bool to_best = LM && e.kind == EPI_LOGITS;
    if (to_best && (int)threadIdx.x < g.n_cols) lbest[threadIdx.x] = 0ull;
    __syncthreads();
    for (int idx = threadIdx.x; idx < n_out; idx += kWgThreads) {
        const int ti = idx / per_tile, r = idx - ti * per_tile;
        const int col = r >> 3, mp = r & 7;
        float lo = 0.f, hi = 0.f;
#pragma unroll
        for (int wv = 0; wv < kWaves; ++wv) {
            ETC_AS_LDS const float *base = red + ((size_t)(ti * kWaves + wv) * g.n_cols + col) * 16;
            lo += base[mp];
            hi += base[mp + 8];
        }
        if (g.ssq_parts) {
            const float rn = rs[col];
            lo *= rn;
            hi *= rn;
        }
        Epilogue et = e;
        et.row0 = e.row0 + ti * g.tile_rows;
        et.lds_best = lbest;
        if (e.ssq_out) et.ssq_out = e.ssq_out + (size_t)ti * kMaxBatch;
        if (!pre_ok) pre = epilogue_preload(P, et, col, mp);
        apply_epilogue<LM>(P, et, col, mp, lo, hi, pre);
    }
    if (to_best) {       // the task's maxima join the sequences' running maxima
        __syncthreads();
        if ((int)threadIdx.x < g.n_cols)
            __hip_atomic_fetch_max(as_global(P.best + threadIdx.x), lbest[threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Out-of-line path for batches above 16 columns, or operands too large for a whole copy in LDS.
// The operand is walked in chunks of KC elements of K: a chunk of ALL columns (hi and lo) sits in LDS,
// double buffered; while the wavefronts run the MFMAs of chunk c out of one buffer, every thread already
// has its 8-byte pieces of chunk c+1 in flight into registers and drops them into the other buffer at the
// end of the chunk: one barrier per chunk.  Within a chunk a wavefront owns 32 of every 256 elements of K
// (S = KC / 256 MFMA steps); a task streams T (4 or 8) row tiles against one pass over the operand, which
// every task has to read in full, with a ring of PFC weight fragments in flight per lane running over
// (chunk, step, tile) triples.  Register budget decides the shape: accumulators take T x NB x 4 registers,
// the ring 4 PFC, the operand pieces in flight COLS x KC / 512 - so 16 columns keep the full ring of 16, 32
// columns a ring of 8, 64 columns 4 row tiles and a ring of 4.  Nothing may spill inside the loop: a
// register reload is a memory load that queues behind the whole ring.
//
// The steady state of the loop is free of branches.  The compiler places its wait counts per basic block;
// a branch around a load (a dead tile slot, a column beyond the batch, a chunk beyond K) makes every later
// wait a full drain of the loads in flight, which halves the streaming rate.  So the steady state always
// moves T tiles (slots beyond n_tiles stream the last live tile again and are never stored), columns beyond
// n_cols read row 0, and only the last ring revolutions, whose look-ahead leaves K, run the conditional code.

// Arguments of the out-of-line path travel through LDS: passed by value they fill the argument registers and
// spill to the stack, i.e. every lane writes and reads its own copy of the same descriptors through scratch memory.
struct ChunkedArgs {
    GemmTile g;
    Epilogue e;
    TaskWaits w;
    int task_id;
};
__device__ __forceinline__ ChunkedArgs *chunked_args_slot()
{
    __shared__ ChunkedArgs slot;
    return &slot;
}

// `frame_anchor` points into the caller's stack frame and is there for the compiler alone.  A call that could be a
// tail call makes the callee save and restore every callee-saved vector register it uses, through scratch memory,
// on every call: 112 registers per lane here, at batch 64 twenty times the bytes the tasks produce.  A callee whose
// call sites all hand it a piece of the caller's frame cannot be tail-called; the compiler then tells the callers
// what the callee clobbers instead, and the callers (the task loop) have next to nothing live across the call.
template <int NB, int T>
__device__ __noinline__ void gemm_tiles_chunked(const Params &P, const ChunkedArgs *args, float *sm, int *frame_anchor)
{
    const ChunkedArgs a = lds_get_uniform(args);
    if (a.task_id == -0x7FFFFFFF) *frame_anchor = 1;      // never true (task ids are >= -1)
    const GemmTile &g = a.g;
    const Epilogue &e = a.e;
    const TaskWaits &w = a.w;
    const int task_id = a.task_id;
    static_assert(T == 1 || T == 2 || T == 4 || T == 8, "row tiles per pass");
    constexpr int PFC = NB == 1 ? (T >= 4 ? PF : 8) : (NB == 2 ? 8 : 4);   // weight loads in flight per lane, as the registers allow
    constexpr int COLS = NB * 16;
    constexpr int S = (4 / NB) < (PFC / T) ? (4 / NB) : (PFC / T);   // MFMA steps per wavefront, chunk and tile
    constexpr int KC = 256 * S;                    // K elements per chunk
    constexpr int STRIDE = KC + 8;                 // LDS column stride in elements: 16 columns cover all banks
    constexpr int PPC = KC / 4;                    // 8-byte pieces per column and half
    constexpr int U = COLS * PPC / kWgThreads;     // 8-byte pieces per thread, chunk and half
    constexpr int BUF = 2 * COLS * STRIDE;         // elements of one buffer: hi columns, then lo columns
    constexpr int CPR = PFC / (T * S);              // chunks per revolution of the ring
    static_assert(COLS * PPC == U * kWgThreads, "every thread moves U pieces of each half");
    static_assert(CPR >= 1 && CPR * T * S == PFC, "the ring holds whole chunks");
    static_assert((size_t)2 * BUF * 2 + (64 + 512) * 4 <= (size_t)kLdsBytes, "two operand buffers and the norm scratch fit");
    static_assert((size_t)kWaves * NB * 256 * 4 <= (size_t)BUF * 2, "the reduction buffer aliases one operand buffer");
    const int wave = wave_id(), lane = lane_id();
    const int m = lane & 15, kg = lane >> 4;
    const int K = __builtin_amdgcn_readfirstlane(g.K);
    const int n_chunks = (K + KC - 1) / KC;        // K is a multiple of 256; the last chunk may be partial
    const int n_full = K / KC;                     // chunks that lie inside K with all their steps
    const int n_tiles = __builtin_amdgcn_readfirstlane(g.n_tiles);
    const size_t tile_step = (size_t)g.tile_rows * (size_t)g.ldw;
    const uint16_t *wbase = (m < 8 ? g.rowsA + (size_t)m * (size_t)g.ldw : g.rowsB + (size_t)(m - 8) * (size_t)g.ldw) +
                            wave * 32 + kg * 8;
    // The steady state of the streaming loop has no branch (a branch around a load makes every later wait
    // a full drain of the loads in flight): it always moves T row tiles, slots beyond n_tiles stream the
    // last live tile again and are never stored; columns beyond n_cols read row 0.
    uint32_t toff[T];                              // uniform element offsets of the tiles: scalar registers
#pragma unroll
    for (int ti = 0; ti < T; ++ti)
        toff[ti] = __builtin_amdgcn_readfirstlane((uint32_t)((size_t)(ti < n_tiles ? ti : n_tiles - 1) * tile_step));

    ETC_AS_LDS uint16_t *buf0 = reinterpret_cast<ETC_AS_LDS uint16_t *>(as_lds(sm));
    ETC_AS_LDS float *red = as_lds(sm);                                  // after the last chunk
    ETC_AS_LDS float *rs = reinterpret_cast<ETC_AS_LDS float *>(buf0 + 2 * BUF);
    ETC_AS_LDS float *rs_part = rs + 64;                                  // [8][64]

    // ring slot j <-> (chunk j / (S*T) of the revolution, step (j / T) % S, tile j % T)
    auto step_live = [&](int c, int sidx) { return c * KC + sidx * 256 < K; };
    // ---- weight prefetch before the wait ---------------------------------------------------------------
    u32x4 wr[PFC];
#pragma unroll
    for (int j = 0; j < PFC; ++j) {
        const int c = j / (S * T), sidx = (j / T) % S, ti = j % T;
        if (step_live(c, sidx)) wr[j] = load16_nt(wbase + toff[ti] + c * KC + sidx * 256);
        else wr[j] = u32x4{0, 0, 0, 0};
    }
    // ---- E.wait(): the operand is needed in full, so every K slice event is waited for ---------------
    if (w.per_wave) {
        if (wave == 0 && lane < kWaves) spin_until_zero(P, w.ev0 + lane, w.fn);
        if (threadIdx.x == 0 && w.ev1 >= 0) spin_until_zero(P, w.ev1, w.fn);
        __syncthreads();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    } else {
        wg_wait(P, w.ev0, w.ev1, w.fn);
    }
    trace_mark(P, task_id, 1);

    // this thread's pieces of every chunk: piece tid + 512u = (column, 8-byte piece of the column's chunk)
    int rows[U], pcs[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int idx = (int)threadIdx.x + kWgThreads * u;
        const int col = idx / PPC;
        pcs[u] = idx - col * PPC;
        rows[u] = 0;
        if (col < g.n_cols) rows[u] = g.col_rows ? ld_i32(g.col_rows + col) : col;
        if (rows[u] < 0) rows[u] = 0;
    }
    uint64_t vh[U], vl[U];
    auto fetch_chunk = [&](int c) {                // any chunk: pieces beyond K are left out
#pragma unroll
        for (int u = 0; u < U; ++u) {
            vh[u] = vl[u] = 0;
            if (c * KC + pcs[u] * 4 < K) {
                const size_t off = (size_t)rows[u] * (size_t)g.ldb + (size_t)c * KC + pcs[u] * 4;
                vh[u] = ld_u64(g.b_hi + off);
                vl[u] = ld_u64(g.b_lo + off);
            }
        }
    };
    auto fetch_full_chunk = [&](int c) {           // a chunk inside K: no conditions
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t off = (size_t)rows[u] * (size_t)g.ldb + (size_t)c * KC + pcs[u] * 4;
            vh[u] = ld_u64(g.b_hi + off);
            vl[u] = ld_u64(g.b_lo + off);
        }
    };
    auto park_chunk = [&](int b) {
        ETC_AS_LDS uint16_t *hi = buf0 + b * BUF, *lo = hi + COLS * STRIDE;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int idx = (int)threadIdx.x + kWgThreads * u;
            const int col = idx / PPC;
            *reinterpret_cast<ETC_AS_LDS uint64_t *>(hi + col * STRIDE + pcs[u] * 4) = vh[u];
            *reinterpret_cast<ETC_AS_LDS uint64_t *>(lo + col * STRIDE + pcs[u] * 4) = vl[u];
        }
    };
    fetch_chunk(0);

    // ---- RMSNorm factors: thread (column, group) sums every 8th partial sum of squares, groups meet in LDS ----
    if (g.ssq_parts) {
        const int col = threadIdx.x & 63;
        int row = -1;
        if (col < g.n_cols) row = g.col_rows ? ld_i32(g.col_rows + col) : col;
        float s = 0.f;
        for (int p0 = wave; p0 < g.n_parts; p0 += 8 * 16) {
            float t[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int pt = p0 + 8 * j;
                t[j] = (pt < g.n_parts && row >= 0) ? ld_f32(g.ssq_parts + (size_t)pt * (size_t)g.ssq_stride + row) : 0.f;
            }
#pragma unroll
            for (int j = 0; j < 16; ++j) s += t[j];
        }
        rs_part[wave * 64 + col] = s;
    }
    park_chunk(0);
    __syncthreads();
    if (g.ssq_parts && threadIdx.x < 64) {
        float s = 0.f;
#pragma unroll
        for (int gq = 0; gq < 8; ++gq) s += rs_part[gq * 64 + threadIdx.x];
        rs[threadIdx.x] = 1.0f / sqrtf(s / (float)g.K + g.eps);
    }
    trace_mark(P, task_id, 2);

    f32x4 acc[T][NB];
#pragma unroll
    for (int ti = 0; ti < T; ++ti)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[ti][nb] = f32x4{0, 0, 0, 0};

    // one MFMA step of all T tiles out of ring slots j0 .. j0+T-1; RELOAD: the slots are refilled for chunk cn
#define ETC_CHUNK_STEP(hi, lo, sidx, cc, cn, RELOAD)                                                             \
    {                                                                                                             \
        u32x4 fb[NB];                                                                                             \
        _Pragma("unroll") for (int nb = 0; nb < NB; ++nb)                                                         \
            fb[nb] = *reinterpret_cast<ETC_AS_LDS const u32x4 *>(hi + nb * 16 * STRIDE + (sidx) * 256);            \
        _Pragma("unroll") for (int ti = 0; ti < T; ++ti) {                                                        \
            const bf16x8 a = __builtin_bit_cast(bf16x8, wr[((cc) * S + (sidx)) * T + ti]);                        \
            _Pragma("unroll") for (int nb = 0; nb < NB; ++nb) acc[ti][nb] =                                       \
                __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, fb[nb]), acc[ti][nb], 0, 0, 0); \
        }                                                                                                         \
        _Pragma("unroll") for (int nb = 0; nb < NB; ++nb)                                                         \
            fb[nb] = *reinterpret_cast<ETC_AS_LDS const u32x4 *>(lo + nb * 16 * STRIDE + (sidx) * 256);            \
        _Pragma("unroll") for (int ti = 0; ti < T; ++ti) {                                                        \
            const int j = ((cc) * S + (sidx)) * T + ti;                                                           \
            const bf16x8 a = __builtin_bit_cast(bf16x8, wr[j]);                                                   \
            if (RELOAD) wr[j] = load16_nt(wbase + toff[ti] + (size_t)(cn) * KC + (sidx) * 256);                   \
            _Pragma("unroll") for (int nb = 0; nb < NB; ++nb) acc[ti][nb] =                                       \
                __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, fb[nb]), acc[ti][nb], 0, 0, 0); \
        }                                                                                                         \
    }
    int c0 = 0;
    for (; c0 + 2 * CPR <= n_full; c0 += CPR) {    // steady state: this revolution, the next chunk and the chunks
#pragma unroll                                     // the ring is refilled for all lie inside K: no conditions
        for (int cc = 0; cc < CPR; ++cc) {
            const int c = c0 + cc, b = c & 1;
            fetch_full_chunk(c + 1);
            ETC_AS_LDS const uint16_t *hi = buf0 + b * BUF + m * STRIDE + wave * 32 + kg * 8;
            ETC_AS_LDS const uint16_t *lo = hi + COLS * STRIDE;
#pragma unroll
            for (int sidx = 0; sidx < S; ++sidx) ETC_CHUNK_STEP(hi, lo, sidx, cc, c + CPR, true)
            park_chunk(b ^ 1);
            __syncthreads();
        }
    }
    for (; c0 < n_chunks; c0 += CPR) {             // the last revolutions: every load and step is conditional
#pragma unroll
        for (int cc = 0; cc < CPR; ++cc) {
            const int c = c0 + cc;
            if (c < n_chunks) {                    // uniform
                const int b = c & 1;
                if (c + 1 < n_chunks) fetch_chunk(c + 1);
                ETC_AS_LDS const uint16_t *hi = buf0 + b * BUF + m * STRIDE + wave * 32 + kg * 8;
                ETC_AS_LDS const uint16_t *lo = hi + COLS * STRIDE;
#pragma unroll
                for (int sidx = 0; sidx < S; ++sidx) {
                    if (step_live(c, sidx)) {      // uniform
                        if (step_live(c + CPR, sidx)) ETC_CHUNK_STEP(hi, lo, sidx, cc, c + CPR, true)
                        else ETC_CHUNK_STEP(hi, lo, sidx, cc, c + CPR, false)
                    }
                }
                if (c + 1 < n_chunks) park_chunk(b ^ 1);
                __syncthreads();
            }
        }
    }
#undef ETC_CHUNK_STEP

    // ---- per tile: partials of the 8 wavefronts through LDS, fixed order, epilogue ----------------------
    trace_mark(P, task_id, 3);
    ETC_AS_LDS unsigned long long *lbest = reinterpret_cast<ETC_AS_LDS unsigned long long *>(rs_part);   // [64]: the norm scratch is free by now
    const bool to_best = e.kind == EPI_LOGITS;
    if (to_best && (int)threadIdx.x < g.n_cols) lbest[threadIdx.x] = 0ull;      // ordered by the barrier behind the first tile's partials
#pragma unroll
    for (int ti = 0; ti < T; ++ti) {
        if (ti < n_tiles) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                *reinterpret_cast<ETC_AS_LDS f32x4 *>(red + ((size_t)(wave * NB + nb) * 64 + lane) * 4) = acc[ti][nb];
            __syncthreads();
            Epilogue et = e;
            et.row0 = e.row0 + ti * g.tile_rows;
            et.lds_best = lbest;
            if (e.ssq_out) et.ssq_out = e.ssq_out + (size_t)ti * kMaxBatch;
            for (int idx = threadIdx.x; idx < g.n_cols * 8; idx += kWgThreads) {
                const int col = idx >> 3, mp = idx & 7;
                const int nb = col >> 4, n = col & 15;
                float lo = 0.f, hi = 0.f;
#pragma unroll
                for (int wv = 0; wv < kWaves; ++wv) {
                    ETC_AS_LDS const float *base = red + (size_t)(wv * NB + nb) * 256;
                    lo += base[(n + 16 * (mp >> 2)) * 4 + (mp & 3)];
                    hi += base[(n + 16 * ((mp + 8) >> 2)) * 4 + (mp & 3)];
                }
                if (g.ssq_parts) {
                    const float r = rs[col];
                    lo *= r;
                    hi *= r;
                }
                apply_epilogue<true>(P, et, col, mp, lo, hi, epilogue_preload(P, et, col, mp));
            }
            __syncthreads();
        }
    }
    if (to_best && (int)threadIdx.x < g.n_cols)       // behind the last tile's barrier
        __hip_atomic_fetch_max(as_global(P.best + threadIdx.x), lbest[threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Wide path: tasks of 5 or more row tiles at any column count (16 * NB columns).  The chunked path splits K over the 8
// wavefronts, so every wavefront holds accumulators for all tiles of the pass (at 64 columns a pass is 4 tiles: the
// operand, hi and lo, is read again for every 256 KB of weights) and the tiles meet in a reduction across wavefronts.
// Here the wavefronts split the OUTPUT instead: each owns TW row tiles of the pass and runs over all of K, the operand
// chunk in LDS is shared by all of them, and a pass is 8 x TW tiles.  No reduction across wavefronts; the accumulators
// go through LDS once, into the layout the epilogue threads read.  Measured against the chunked path on whole decode
// steps (8B shape): batch 16 7.30 -> 6.45 ms, batch 32 8.59 -> 7.57 ms, batch 64 14.0 -> 10.9 ms; 70B shape, batch 32,
// with 14 - 16 tiles per task (TW = 2, one task per queue instead of two): 58.1 -> 48.4 ms.
template <int TW, int NB>
__device__ __noinline__ void gemm_tiles_wide(const Params &P, const ChunkedArgs *args, float *sm, int *frame_anchor)
{
    const ChunkedArgs a = lds_get_uniform(args);
    if (a.task_id == -0x7FFFFFFF) *frame_anchor = 1;      // never true; see gemm_tiles_chunked
    const GemmTile &g = a.g;
    const Epilogue &e = a.e;
    const TaskWaits &w = a.w;
    const int task_id = a.task_id;
    constexpr int COLS = 16 * NB, KC = 256, STRIDE = KC + 8, PPC = KC / 4, U = COLS * PPC / kWgThreads;
    constexpr int BUF = 2 * COLS * STRIDE;         // elements of one operand buffer: hi columns, then lo columns
    constexpr int PASS = kWaves * TW;              // row tiles per pass
    constexpr int RING = 8 * TW;                   // weight fragments of one chunk per wavefront = loads in flight per lane
    static_assert((TW == 1 || TW == 2) && (NB == 1 || NB == 2 || NB == 4), "tiles per wavefront, column blocks");
    static_assert((size_t)2 * BUF * 2 + (64 + 512) * 4 <= (size_t)kLdsBytes, "two operand buffers and the norm scratch fit");
    static_assert((size_t)PASS * NB * 256 * 4 <= (size_t)2 * BUF * 2, "the tiles' accumulators alias the operand buffers");
    const int wave = wave_id(), lane = lane_id();
    const int m = lane & 15, kg = lane >> 4;
    const int K = __builtin_amdgcn_readfirstlane(g.K);
    const int n_chunks = K / KC;                   // K is a multiple of 256
    const int n_tiles = __builtin_amdgcn_readfirstlane(g.n_tiles);      // <= PASS
    const size_t tile_step = (size_t)g.tile_rows * (size_t)g.ldw;
    const uint16_t *wbase = (m < 8 ? g.rowsA + (size_t)m * (size_t)g.ldw : g.rowsB + (size_t)(m - 8) * (size_t)g.ldw) + kg * 8;
    // a wavefront whose tile lies beyond n_tiles streams the last live tile again and never stores it: no branch in the loop
    uint32_t toff[TW];
#pragma unroll
    for (int t = 0; t < TW; ++t) {
        const int ti = wave * TW + t;
        toff[t] = __builtin_amdgcn_readfirstlane((uint32_t)((size_t)(ti < n_tiles ? ti : n_tiles - 1) * tile_step));
    }
    ETC_AS_LDS uint16_t *buf0 = reinterpret_cast<ETC_AS_LDS uint16_t *>(as_lds(sm));
    ETC_AS_LDS float *tb = as_lds(sm);                                    // after the last chunk: [PASS][NB][64 lanes][4]
    ETC_AS_LDS float *rs = reinterpret_cast<ETC_AS_LDS float *>(buf0 + 2 * BUF);
    ETC_AS_LDS float *rs_part = rs + 64;                                  // [8][64]

    // ---- weight prefetch before the wait: the fragments of chunk 0 -----------------------------------------
    u32x4 wr[RING];
#pragma unroll
    for (int j = 0; j < RING; ++j) wr[j] = gld_16B(wbase + toff[j % TW] + (j / TW) * 32);
    if (w.per_wave) {
        if (wave == 0 && lane < kWaves) spin_until_zero(P, w.ev0 + lane, w.fn);
        if (threadIdx.x == 0 && w.ev1 >= 0) spin_until_zero(P, w.ev1, w.fn);
        __syncthreads();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    } else {
        wg_wait(P, w.ev0, w.ev1, w.fn);
    }
    trace_mark(P, task_id, 1);

    int rows[U], pcs[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int idx = (int)threadIdx.x + kWgThreads * u;
        const int col = idx / PPC;
        pcs[u] = idx - col * PPC;
        rows[u] = 0;
        if (col < g.n_cols) rows[u] = g.col_rows ? ld_i32(g.col_rows + col) : col;
        if (rows[u] < 0) rows[u] = 0;
    }
    uint64_t vh[U], vl[U];
    auto fetch_chunk = [&](int c) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t off = (size_t)rows[u] * (size_t)g.ldb + (size_t)c * KC + pcs[u] * 4;
            vh[u] = ld_u64(g.b_hi + off);
            vl[u] = ld_u64(g.b_lo + off);
        }
    };
    auto park_chunk = [&](int b) {
        ETC_AS_LDS uint16_t *hi = buf0 + b * BUF, *lo = hi + COLS * STRIDE;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int idx = (int)threadIdx.x + kWgThreads * u;
            const int col = idx / PPC;
            *reinterpret_cast<ETC_AS_LDS uint64_t *>(hi + col * STRIDE + pcs[u] * 4) = vh[u];
            *reinterpret_cast<ETC_AS_LDS uint64_t *>(lo + col * STRIDE + pcs[u] * 4) = vl[u];
        }
    };
    fetch_chunk(0);
    if (g.ssq_parts) {       // RMSNorm factors, as in the chunked path
        const int col = threadIdx.x & 63;
        int row = -1;
        if (col < g.n_cols) row = g.col_rows ? ld_i32(g.col_rows + col) : col;
        float s = 0.f;
        for (int p0 = wave; p0 < g.n_parts; p0 += 8 * 16) {
            float t[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int pt = p0 + 8 * j;
                t[j] = (pt < g.n_parts && row >= 0) ? ld_f32(g.ssq_parts + (size_t)pt * (size_t)g.ssq_stride + row) : 0.f;
            }
#pragma unroll
            for (int j = 0; j < 16; ++j) s += t[j];
        }
        rs_part[wave * 64 + col] = s;
    }
    park_chunk(0);
    __syncthreads();
    if (g.ssq_parts && threadIdx.x < 64) {
        float s = 0.f;
#pragma unroll
        for (int gq = 0; gq < 8; ++gq) s += rs_part[gq * 64 + threadIdx.x];
        rs[threadIdx.x] = 1.0f / sqrtf(s / (float)g.K + g.eps);
    }
    trace_mark(P, task_id, 2);

    f32x4 acc[TW][NB];
#pragma unroll
    for (int t = 0; t < TW; ++t)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[t][nb] = f32x4{0, 0, 0, 0};
    // one chunk: 8 steps of 32 elements of K; RELOAD: ring slots are refilled for the next chunk behind their use
#define ETC_WIDE_CHUNK(c, RELOAD)                                                                                 \
    {                                                                                                             \
        ETC_AS_LDS const uint16_t *hi = buf0 + ((c) & 1) * BUF + m * STRIDE + kg * 8;                             \
        ETC_AS_LDS const uint16_t *lo = hi + COLS * STRIDE;                                                       \
        _Pragma("unroll") for (int kk = 0; kk < 8; ++kk) {                                                        \
            u32x4 fb[NB];                                                                                         \
            _Pragma("unroll") for (int nb = 0; nb < NB; ++nb)                                                     \
                fb[nb] = *reinterpret_cast<ETC_AS_LDS const u32x4 *>(hi + nb * 16 * STRIDE + kk * 32);             \
            _Pragma("unroll") for (int t = 0; t < TW; ++t) {                                                      \
                const bf16x8 av = __builtin_bit_cast(bf16x8, wr[kk * TW + t]);                                    \
                _Pragma("unroll") for (int nb = 0; nb < NB; ++nb) acc[t][nb] =                                    \
                    __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, fb[nb]), acc[t][nb], 0, 0, 0); \
            }                                                                                                     \
            _Pragma("unroll") for (int nb = 0; nb < NB; ++nb)                                                     \
                fb[nb] = *reinterpret_cast<ETC_AS_LDS const u32x4 *>(lo + nb * 16 * STRIDE + kk * 32);             \
            _Pragma("unroll") for (int t = 0; t < TW; ++t) {                                                      \
                const bf16x8 av = __builtin_bit_cast(bf16x8, wr[kk * TW + t]);                                    \
                if (RELOAD) wr[kk * TW + t] = gld_16B(wbase + toff[t] + (size_t)((c) + 1) * KC + kk * 32);      \
                _Pragma("unroll") for (int nb = 0; nb < NB; ++nb) acc[t][nb] =                                    \
                    __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, fb[nb]), acc[t][nb], 0, 0, 0); \
            }                                                                                                     \
        }                                                                                                         \
    }
    int c = 0;
    for (; c + 1 < n_chunks; ++c) {                // every chunk but the last: the next chunk is fetched and the ring refilled
        fetch_chunk(c + 1);
        ETC_WIDE_CHUNK(c, true)
        park_chunk((c + 1) & 1);
        __syncthreads();
    }
    ETC_WIDE_CHUNK(c, false)
#undef ETC_WIDE_CHUNK
    __syncthreads();                               // every wavefront is done with the operand buffers

    // ---- accumulators through LDS into the layout of the epilogue threads, then the epilogue tile by tile ----
    trace_mark(P, task_id, 3);
#pragma unroll
    for (int t = 0; t < TW; ++t) {
        const int ti = wave * TW + t;
        if (ti < n_tiles) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                *reinterpret_cast<ETC_AS_LDS f32x4 *>(tb + ((size_t)(ti * NB + nb) * 64 + lane) * 4) = acc[t][nb];
        }
    }
    ETC_AS_LDS unsigned long long *lbest = reinterpret_cast<ETC_AS_LDS unsigned long long *>(rs_part);
    const bool to_best = e.kind == EPI_LOGITS;
    if (to_best && (int)threadIdx.x < g.n_cols) lbest[threadIdx.x] = 0ull;
    __syncthreads();
    for (int ti = 0; ti < n_tiles; ++ti) {
        Epilogue et = e;
        et.row0 = e.row0 + ti * g.tile_rows;
        et.lds_best = lbest;
        if (e.ssq_out) et.ssq_out = e.ssq_out + (size_t)ti * kMaxBatch;
        const int idx = threadIdx.x;
        if (idx < g.n_cols * 8) {
            const int col = idx >> 3, mp = idx & 7;
            const int nb = col >> 4, n = col & 15;
            ETC_AS_LDS const float *base = tb + (size_t)(ti * NB + nb) * 256;
            float lo = base[(n + 16 * (mp >> 2)) * 4 + (mp & 3)];
            float hi = base[(n + 16 * ((mp + 8) >> 2)) * 4 + (mp & 3)];
            if (g.ssq_parts) {
                const float r = rs[col];
                lo *= r;
                hi *= r;
            }
            apply_epilogue<true>(P, et, col, mp, lo, hi, epilogue_preload(P, et, col, mp));
        }
    }
    __syncthreads();                               // the next pass parks its operand over the tiles
    if (to_best && (int)threadIdx.x < g.n_cols)
        __hip_atomic_fetch_max(as_global(P.best + threadIdx.x), lbest[threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Passes of the wide path: 8 x TW row tiles each.
template <int TW, int NB>
__device__ __forceinline__ void gemm_tiles_wide_passes(const Params &PL, ChunkedArgs a, ChunkedArgs *slot, float *sm, int *frame_anchor)
{
    constexpr int PASS = kWaves * TW;
    const int total = a.g.n_tiles;
    for (int t0 = 0; t0 < total; t0 += PASS) {
        a.g.n_tiles = total - t0 < PASS ? total - t0 : PASS;
        if (t0 > 0 || a.g.n_tiles != total) {
            __syncthreads();                       // every wavefront has read the slot's current contents
            if (threadIdx.x == 0) lds_put(slot, a);
            __syncthreads();
        }
        gemm_tiles_wide<TW, NB>(PL, slot, sm, frame_anchor);
        a.g.rowsA += (size_t)PASS * a.g.tile_rows * a.g.ldw;
        a.g.rowsB += (size_t)PASS * a.g.tile_rows * a.g.ldw;
        a.e.row0 += PASS * a.g.tile_rows;
        if (a.e.ssq_out) a.e.ssq_out += (size_t)PASS * kMaxBatch;
        a.w = TaskWaits{-1, -1, a.w.fn, false, -1};
    }
}

// One call per pass over the operand: T row tiles each (the events have been seen after the first pass).
template <int NB, int T>
__device__ __forceinline__ void gemm_tiles_chunked_passes(const Params &PL, ChunkedArgs a, ChunkedArgs *slot, float *sm, int *frame_anchor)
{
    const int total = a.g.n_tiles;
    for (int t0 = 0; t0 < total; t0 += T) {
        a.g.n_tiles = total - t0 < T ? total - t0 : T;
        if (t0 > 0 || a.g.n_tiles != total) {      // the slot already holds the arguments of a single pass
            __syncthreads();                       // every wavefront has read the slot's current contents (a wavefront that
                                                   // runs ahead must not rewrite them under the others: they would disagree
                                                   // on the number of passes)
            if (threadIdx.x == 0) lds_put(slot, a);
            __syncthreads();
        }
        gemm_tiles_chunked<NB, T>(PL, slot, sm, frame_anchor);
        a.g.rowsA += (size_t)T * a.g.tile_rows * a.g.ldw;
        a.g.rowsB += (size_t)T * a.g.tile_rows * a.g.ldw;
        a.e.row0 += T * a.g.tile_rows;
        if (a.e.ssq_out) a.e.ssq_out += (size_t)T * kMaxBatch;
        a.w = TaskWaits{-1, -1, a.w.fn, false, -1};
    }
}

// Entry of the out-of-line path: one call site in the task loop.  The streaming loop always moves T row tiles, so T
// follows the task: 1, 2, 4 or 8.  Up to 32 columns a pass takes up to 8 tiles; with 64 columns the accumulators of
// 8 tiles no longer fit the register file next to the weight ring (spills inside the streaming loop queue behind the
// weight loads), so a pass takes at most 4.
__device__ __noinline__ void gemm_chunked_entry(const Params &PL, ChunkedArgs *slot, float *sm, int *frame_anchor)
{
    const ChunkedArgs a = lds_get_uniform(slot);
    if (a.task_id == -0x7FFFFFFF) *frame_anchor = 1;      // never true; see gemm_tiles_chunked
    int anchor = 0;
#define ETC_CHUNKED(NB_)                                                                         \
    {                                                                                            \
        if (a.g.n_tiles == 1) gemm_tiles_chunked_passes<NB_, 1>(PL, a, slot, sm, &anchor);      \
        else if (a.g.n_tiles == 2) gemm_tiles_chunked_passes<NB_, 2>(PL, a, slot, sm, &anchor); \
        else if (a.g.n_tiles <= 4 || NB_ == 4) gemm_tiles_chunked_passes<NB_, 4>(PL, a, slot, sm, &anchor);  \
        else gemm_tiles_chunked_passes<NB_, NB_ == 4 ? 4 : 8>(PL, a, slot, sm, &anchor);   /* several passes: crowded expert */ \
    }
    if (a.g.n_cols > 32 && a.g.n_tiles >= 16 && a.g.K % 256 == 0) gemm_tiles_wide_passes<2, 4>(PL, a, slot, sm, &anchor);
    else if (a.g.n_cols > 32 && a.g.n_tiles >= 5 && a.g.K % 256 == 0) gemm_tiles_wide_passes<1, 4>(PL, a, slot, sm, &anchor);
    else if (a.g.n_cols > 32) ETC_CHUNKED(4)
    else if (a.g.n_cols > 16 && a.g.n_tiles >= 9 && a.g.K % 256 == 0) gemm_tiles_wide_passes<2, 2>(PL, a, slot, sm, &anchor);   // 9 .. 16 tiles against ONE pass over the operand
    else if (a.g.n_cols > 16 && a.g.n_tiles >= 5 && a.g.K % 256 == 0) gemm_tiles_wide_passes<1, 2>(PL, a, slot, sm, &anchor);
    else if (a.g.n_cols > 16) ETC_CHUNKED(2)
    else if (a.g.n_tiles >= 5 && a.g.K % 256 == 0) gemm_tiles_wide_passes<1, 1>(PL, a, slot, sm, &anchor);
    else ETC_CHUNKED(1)
#undef ETC_CHUNKED
}

// The same entry with its arguments by value (some travel over the stack, which also keeps the call from being a tail
// call).  Which hand-over is cheaper is a property of the calling instance, measured: the dense large-batch steps are
// 6-7 % faster with the LDS slot (less scratch traffic per task), the MoE steps 13-18 % faster with the by-value call
// (8B batch 64: 14.4 against 15.4 ms; Qwen3 shape batch 1: 6.1 against 5.0 ms).
__device__ __noinline__ void gemm_chunked_entry_by_value(const Params &PL, GemmTile g, Epilogue e, TaskWaits w, float *sm, int task_id)
{
    const ChunkedArgs a{wave_uniform(g), wave_uniform(e), wave_uniform(w), __builtin_amdgcn_readfirstlane(task_id)};
    ChunkedArgs *slot = chunked_args_slot();
    if (threadIdx.x == 0) lds_put(slot, a);
    __syncthreads();
    int frame_anchor = 0;
    gemm_chunked_entry(PL, slot, sm, &frame_anchor);
}

// The chunked path from the task loop.  ARGS_BY_VALUE: see gemm_chunked_entry_by_value.
template <bool ARGS_BY_VALUE>
__device__ __forceinline__ void gemm_chunked_dispatch(const Params &PL, const GemmTile &g, const Epilogue &e, const TaskWaits &w,
                                                      float *sm, WgState &st, int task_id)
{
    st.staged_key = -1;
    if (ARGS_BY_VALUE) {
        gemm_chunked_entry_by_value(PL, g, e, w, sm, task_id);
        return;
    }
    ChunkedArgs *slot = chunked_args_slot();
    if (threadIdx.x == 0) lds_put(slot, ChunkedArgs{g, e, w, task_id});
    __syncthreads();
    int frame_anchor = 0;
    gemm_chunked_entry(PL, slot, sm, &frame_anchor);
}

// Second stage of a K-sliced projection: adds the partial sums of the slices in slice order (fixed, so the
// result does not depend on which slice finished first) and runs the projection's own epilogue on the 16
// rows of one row tile.  e is the epilogue of the whole projection; e.row0 = first row of the tile.
__device__ __forceinline__ void kslice_sum(const Params &P, const Epilogue &e, int n_cols, int n_slices, int n_row_tiles)
{
    const size_t slice_stride = (size_t)n_row_tiles * kMaxBatch * 16;
    const float *base = P.kpart + (size_t)(e.row0 >> 4) * kMaxBatch * 16;
    for (int idx = threadIdx.x; idx < n_cols * 8; idx += kWgThreads) {
        const int col = idx >> 3, mp = idx & 7;
        const EpiPre pre = epilogue_preload(P, e, col, mp);
        float a[8], b[8];
#pragma unroll
        for (int sl = 0; sl < 8; ++sl) {
            a[sl] = b[sl] = 0.f;
            if (sl < n_slices) ld_f32x2_pair(base + (size_t)sl * slice_stride + (size_t)col * 16 + mp, a[sl], b[sl]);
        }
        float lo = 0.f, hi = 0.f;
#pragma unroll
        for (int sl = 0; sl < 8; ++sl) {
            lo += a[sl];
            hi += b[sl];
        }
        apply_epilogue<false>(P, e, col, mp, lo, hi, pre);
    }
}

// cos / sin of the RoPE angle pos * theta^(-2i/d).  The inverse frequencies come from the host in
// double; the angle is reduced to [-pi, pi] in double (positions run into the thousands), the
// hardware sine / cosine then see a small argument.
__device__ __forceinline__ void rope_cos_sin(const Params &P, int pos, int i, float *cs, float *sn)
{
    const double ang = (double)pos * *as_global(P.rope_inv_freq + i);
    const double turns = ang * 0.15915494309189535;          // 1 / (2 pi)
    const float frac = (float)(turns - rint(turns));          // [-0.5, 0.5] turns
    const float r = frac * 6.2831853071795862f;
    *cs = __cosf(r);
    *sn = __sinf(r);
}

// Sort key of (logit, vocabulary id): larger logit first, then lower id.
__device__ __forceinline__ unsigned long long logit_key(float v, int id)
{
    const uint32_t u = __float_as_uint(v);
    const uint32_t ordered = u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
    return ((unsigned long long)ordered << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)id);
}

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

__device__ __forceinline__ void store_split(uint16_t *hi_p, uint16_t *lo_p, size_t idx, float v)
{
    uint16_t h, l;
    split_bf16(v, h, l);
    st_u16(hi_p + idx, h);
    st_u16(lo_p + idx, l);
}

__device__ __forceinline__ EpiPre epilogue_preload(const Params &P, const Epilogue &e, int col, int mp)
{
    EpiPre pre{};
    if (e.kind == EPI_QKV) {      // both resolved by the step prologue: plain independent loads, no look-up chain
        const int b = col, i = e.row0 + mp;
        if (e.head < P.nq + P.nkv) ld_f32x2(P.rope_cs + ((size_t)b * (P.d >> 1) + i) * 2, pre.a, pre.b);   // q and k heads are rotated
        if (e.head >= P.nq) pre.slot = ld_i32(P.kv_slot + b);
        if (P.qk_norm && e.head < P.nq + P.nkv) {      // gains of the two rows under the per-head norm
            const ETC_AS_GLOBAL LayerWeights *W = as_global(P.weights) + e.layer;
            const uint16_t *gn = (const uint16_t *)(e.head < P.nq ? W->gq : W->gk);
            pre.ga = bf16_bits_to_f32(gld_u16(gn + i));
            pre.gb = bf16_bits_to_f32(gld_u16(gn + i + (P.d >> 1)));
        }
    } else if (e.kind == EPI_RESID) {
        const size_t o0 = (size_t)col * e.ld + e.row0 + mp;
        pre.a = ld_f32(e.resid + o0);
        pre.b = ld_f32(e.resid + o0 + 8);
        if (e.next_gain) {
            pre.ga = bf16_bits_to_f32(gld_u16(e.next_gain + e.row0 + mp));
            pre.gb = bf16_bits_to_f32(gld_u16(e.next_gain + e.row0 + mp + 8));
        }
    }
    return pre;
}

// LM: the instance carries the vocabulary projection's epilogue.
template <bool LM>
__device__ __forceinline__ void apply_epilogue(const Params &P, const Epilogue &e, int col, int mp, float lo, float hi,
                                               const EpiPre &pre)
{
    switch (e.kind) {
    case EPI_QKV: {
        const int b = col, half = P.d >> 1, i = e.row0 + mp;
        float a = lo, c = hi;
        const bool normed = P.qk_norm && e.head < P.nq + P.nkv;
        if (normed) {
            // Per-head RMSNorm before RoPE (Sec. 4.3: Q-Norm / K-Norm).  The head's 1 / rms is a scalar, and the rotation
            // is linear, so it commutes with both: this tile leaves its share of the head's sum of squares (of the
            // raw values), applies the gains and rotates; whoever consumes the head (the attention tasks) sums the
            // tiles' shares and scales by 1 / sqrt(mean + eps).
            float sq = lo * lo + hi * hi;
            sq = lanes_sum<8>(sq);                     // the 8 threads of a column are 8 consecutive lanes
            if (mp == 0) st_f32(P.qk_ssq + ((size_t)b * (P.nq + P.nkv) + e.head) * (size_t)(P.d >> 4) + (e.row0 >> 3), sq);
            lo *= pre.ga;
            hi *= pre.gb;
            a = lo;
            c = hi;
        }
        if (e.head < P.nq + P.nkv) {
            a = lo * pre.a - hi * pre.b;
            c = lo * pre.b + hi * pre.a;
        }
        if (e.head < P.nq) {
            float *q = P.qbuf + (size_t)b * (size_t)(P.nq * P.d) + (size_t)e.head * P.d;
            st_f32(q + i, a);
            st_f32(q + i + half, c);
        } else {
            const bool is_k = e.head < P.nq + P.nkv;
            const int kvh = is_k ? e.head - P.nq : e.head - P.nq - P.nkv;
            const size_t off = (size_t)e.layer * (size_t)P.pool_layer_stride +
                               ((size_t)pre.slot * P.nkv + kvh) * (size_t)P.d;
            uint16_t *dst = (is_k ? P.kpool : P.vpool) + off;
            if (!(is_k && normed)) {       // a normalised key reaches the cache from the attention task that completes its norm
                st_u16(dst + i, f32_to_bf16_bits(a));
                st_u16(dst + i + half, f32_to_bf16_bits(c));
            }
            // this step's attention takes the new row unrounded (the cache keeps bf16)
            float *cur = (is_k ? P.knew : P.vnew) + ((size_t)b * P.nkv + kvh) * (size_t)P.d;
            st_f32(cur + i, a);
            st_f32(cur + i + half, c);
        }
        break;
    }
    case EPI_RESID: {
        const int b = col;
        const size_t o0 = (size_t)b * e.ld + e.row0 + mp, o1 = o0 + 8;
        const float v0 = pre.a + lo, v1 = pre.b + hi;
        st_f32(e.outf + o0, v0);
        st_f32(e.outf + o1, v1);
        if (e.next_gain) {   // operand of the next projection: (value * gain) split
            store_split(e.out_hi, e.out_lo, o0, v0 * pre.ga);
            store_split(e.out_hi, e.out_lo, o1, v1 * pre.gb);
        }
        float s = v0 * v0 + v1 * v1;      // this tile's sum of squares: the 8 threads of a column are 8 consecutive lanes
        s = lanes_sum<8>(s);
        if (mp == 0 && e.ssq_out) st_f32(e.ssq_out + b, s);
        if ((e.flags & TF_LAST_LAYER) && P.hidden_out) {
            gst_u16(P.hidden_out + o0, f32_to_bf16_bits(v0));
            gst_u16(P.hidden_out + o1, f32_to_bf16_bits(v1));
        }
        if (e.flags & EPF_DUMP_LAYER) {
            float *dbg = P.layer_hidden + (size_t)e.layer * (size_t)kMaxBatch * e.ld;
            gst_f32(dbg + o0, v0);
            gst_f32(dbg + o1, v1);
        }
        break;
    }
    case EPI_SWIGLU: {
        store_split(e.out_hi, e.out_lo, (size_t)col * e.ld + e.row0 + mp, silu_f(lo) * hi);
        break;
    }
    case EPI_STORE_F32: {
        st_f32(e.outf + (size_t)col * e.ld + e.row0 + mp, lo);
        st_f32(e.outf + (size_t)col * e.ld + e.row0 + mp + 8, hi);
        break;
    }
    case EPI_LOGITS: {
        if (!LM) break;
        // fp32 logits of 16 vocabulary rows, and the tile's best (logit, id) towards the sequence's running maximum.
        // The key orders like the logit (sign-folded bits) and, among equal logits, like the complement of the id,
        // so that the maximum is the greedy token with ties to the lower id; max is exact and order-free, so the
        // result does not depend on which tile arrives first.
        const int r = e.row0 + mp;
        st_f32(e.outf + (size_t)col * e.ld + r, lo);
        st_f32(e.outf + (size_t)col * e.ld + r + 8, hi);
        unsigned long long key = logit_key(lo, r), k2 = logit_key(hi, r + 8);
        key = k2 > key ? k2 : key;
#pragma unroll
        for (int off = 1; off < 8; off <<= 1) {        // the 8 threads of a column are 8 consecutive lanes
            const unsigned long long o = __shfl_xor(key, off, 64);
            key = o > key ? o : key;
        }
        // first into the task's own maxima in LDS: one device-scope atomic per task and column reaches memory
        // (thousands of them on one address are serialised there: 16 ns each, 130 us per 8B-vocabulary step)
        if (mp == 0) __hip_atomic_fetch_max(e.lds_best + col, key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        break;
    }
    case EPI_MOE_ACT: {
        store_split(e.out_hi, e.out_lo, (size_t)(e.col0 + col) * e.ld + e.row0 + mp, silu_f(lo) * hi);
        break;
    }
    case EPI_PARTIAL: {
        float *dst = e.outf + ((size_t)(e.row0 >> 4) * kMaxBatch + col) * 16 + mp;
        st_f32(dst, lo);
        st_f32(dst + 8, hi);
        break;
    }
    case EPI_MOE_Y: {
        st_f32(e.outf + (size_t)(e.col0 + col) * e.ld + e.row0 + mp, lo);
        st_f32(e.outf + (size_t)(e.col0 + col) * e.ld + e.row0 + mp + 8, hi);
        break;
    }
    }
}

}  // namespace etc
