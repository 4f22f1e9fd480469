// The persistent megakernel: dispatch loop + event runtime + task bodies in one launch.
//
// Static scheduling (paper Sec. 3.1, Alg. 1): workgroup q walks its precomputed queue; every task
// waits on its in-edge events, runs its tile, and notifies its out-edge event.
// Dynamic scheduling (Sec. 3.2, Alg. 2): workgroups pop task ids from one ready queue in HBM; the
// notify that brings an event to zero pushes that event's consumer tasks.
// A third entry point runs one stage's tasks as an ordinary kernel (kernel-by-kernel comparator).
#include <hip/hip_runtime.h>

#include "../../include/etc.h"
#include "arm_args.h"
#include "device_rt.hip.h"
#include "task_attn.hip.h"
#include "task_gemm.hip.h"
#include "task_moe.hip.h"

// Generated dispatch (paper Alg. 1 / Alg. 2 as a front end): a library built from a graph description carries the
// device functions of that graph and the switch over them in a generated header; this build includes it here.  The
// stock library has none.
#ifdef ETC_USER_DISPATCH_HEADER
#include ETC_USER_DISPATCH_HEADER
#else
namespace etc {
constexpr int kUserFnCount = 0;
__device__ __forceinline__ void user_dispatch(const Params &, int, int, int, int) {}
}  // namespace etc
#endif

namespace etc {

int user_fn_count() { return kUserFnCount; }

// ---------------------------------------------------------------------------------------------
// small task bodies
// ---------------------------------------------------------------------------------------------
// Row-sum example (Sec. 2.2): A is (n*32, 128) fp32.
__device__ __forceinline__ void rowsum_partial(const Params &P, int i, int j)
{
    // task (i, j): B[32i .. 32i+32, j] = sum_{k in [32j, 32j+32)} A[row, k], left to right
    if (threadIdx.x < 32) {
        const int row = 32 * i + threadIdx.x;
        const ETC_AS_GLOBAL float *a = as_global(P.gbuf[0]) + (size_t)row * 128 + 32 * j;
        float acc = 0.f;
        for (int k = 0; k < 32; ++k) acc += a[k];
        st_f32(P.gbuf[1] + (size_t)row * 4 + j, acc);
    }
}
__device__ __forceinline__ void rowsum_final(const Params &P, int i)
{
    if (threadIdx.x < 32) {
        const int row = 32 * i + threadIdx.x;
        const float *b = P.gbuf[1] + (size_t)row * 4;
        as_global(P.gbuf[2])[row] = ((ld_f32(b) + ld_f32(b + 1)) + ld_f32(b + 2)) + ld_f32(b + 3);
    }
}

// Task t of a grid released through indptr ranges: the final sum of row block perm[t].  Tasks beyond the last
// range (the grid is sized for the largest case) have nothing to do.
__device__ __forceinline__ void rowsum_final_perm(const Params &P, int t)
{
    const int32_t *indptr = reinterpret_cast<const int32_t *>(P.gbuf[4]), *perm = reinterpret_cast<const int32_t *>(P.gbuf[6]);
    if (t >= gld_i32(indptr + P.dd_n_events)) return;
    const int r = gld_i32(perm + t);
    if (r < 0 || r >= P.dd_table_len) {                  // an entry that names no row block: refuse, do not write
        if (threadIdx.x == 0) raise_error(P, ERR_BAD_TABLE, FN_ROWSUM_FINAL_PERM, t);
        return;
    }
    rowsum_final(P, r);
}

// Step prologue for sequence b: hidden_in (bf16) -> residual stream (fp32), the first layer's projection
// operand (x * g1, split) and the partial sums of squares per 16 elements, as every later producer does.
// Also what every layer's QKV epilogue needs of the step's shape, resolved once: the (cos, sin) of the RoPE
// angles at the sequence's position and the KV slot the new row goes to (page table look-up).
template <bool LM>
__device__ __forceinline__ void load_hidden(const Params &P, int b)
{
    const int pos = gld_i32(P.kv_len + b);
    for (int i = threadIdx.x; i < P.d / 2; i += kWgThreads) {
        float cs, sn;
        rope_cos_sin(P, pos, i, &cs, &sn);
        st_f32(P.rope_cs + ((size_t)b * (P.d / 2) + i) * 2, cs);
        st_f32(P.rope_cs + ((size_t)b * (P.d / 2) + i) * 2 + 1, sn);
    }
    if (threadIdx.x == 0) {
        const int page = gld_i32(P.page_ids + gld_i32(P.page_indptr + b) + pos / P.page);
        st_i32(P.kv_slot + b, page * P.page + pos % P.page);
    }
    // The step starts from the sequence's hidden state, or from the embedding row of its token (the token the
    // previous iteration sampled).  An id outside the table raises an error and reads row 0.
    const uint16_t *src = P.hidden_in + (size_t)b * P.H;
    if (LM && P.token_in) {
        int tok = gld_i32(P.token_in + b);
        if (tok < 0 || tok >= P.vocab) {
            if (threadIdx.x == 0) raise_error(P, ERR_BAD_TABLE, FN_LOAD_HIDDEN, tok);
            tok = 0;
        }
        src = P.embed + (size_t)tok * P.H;
    }
    if (LM && threadIdx.x == 0 && P.best)       // below the key of every logit
        __hip_atomic_store(as_global(P.best + b), 0ull, __ATOMIC_RELAXED, ETC_SCOPE);
    const uint16_t *g1 = (const uint16_t *)as_global(P.weights)[0].g1;
    for (int part = threadIdx.x; part < P.H / 16; part += kWgThreads) {
        float s = 0.f;
        for (int i = 0; i < 16; ++i) {
            const size_t o = (size_t)b * P.H + part * 16 + i;
            const float v = bf16_bits_to_f32(gld_u16(src + part * 16 + i));
            st_f32(P.x + o, v);
            uint16_t hi, lo;
            split_bf16(v * bf16_bits_to_f32(gld_u16(g1 + part * 16 + i)), hi, lo);
            st_u16(P.xg_hi + o, hi);
            st_u16(P.xg_lo + o, lo);
            s += v * v;
        }
        st_f32(P.ssq_x + (size_t)part * kMaxBatch + b, s);
    }
}

// ---------------------------------------------------------------------------------------------
// dispatch: one task, including its waits; the caller notifies
// ---------------------------------------------------------------------------------------------
// Narrows a whole-K projection task (c0 = first row tile) to K slice c1 of n_slices and c2 row tiles; the
// task then leaves fp32 partial sums instead of running the projection's epilogue.
__device__ __forceinline__ void slice_of_k(const Params &P, const Task &t, int n_slices, GemmTile &g, Epilogue &e)
{
    const int Ks = g.K / n_slices, k0 = t.c1 * Ks;
    g.rowsA += k0;
    g.rowsB += k0;
    g.b_hi += k0;
    g.b_lo += k0;
    g.K = Ks;
    g.n_tiles = t.c2;
    const int row0 = e.row0, layer = e.layer;
    e = Epilogue{};
    e.kind = EPI_PARTIAL; e.layer = layer; e.row0 = row0;
    e.outf = P.kpart + (size_t)t.c1 * (size_t)(P.H / 16) * kMaxBatch * 16;
}

// Fills the tile and epilogue descriptors of a projection task; false for every other task kind.
template <bool MOE, bool LM>
__device__ __forceinline__ bool setup_gemm(const Params &P, const Task &t, GemmTile &g, Epilogue &e)
{
    const ETC_AS_GLOBAL LayerWeights *W = as_global(P.weights) + t.layer;
    switch (t.fn) {
    case FN_QKV: {
        const int hd = t.c0, sub = t.c1;               // c2 = consecutive tiles of this head
        const int i0 = sub * 8;
        g.n_tiles = t.c2; g.tile_rows = 8;
        const uint16_t *wbase;
        if (hd < P.nq) wbase = (const uint16_t *)W->wq + (size_t)hd * P.d * P.H;
        else if (hd < P.nq + P.nkv) wbase = (const uint16_t *)W->wk + (size_t)(hd - P.nq) * P.d * P.H;
        else wbase = (const uint16_t *)W->wv + (size_t)(hd - P.nq - P.nkv) * P.d * P.H;
        g.rowsA = wbase + (size_t)i0 * P.H;
        g.rowsB = wbase + (size_t)(i0 + P.d / 2) * P.H;
        g.ldw = P.H; g.K = P.H;
        g.b_hi = P.xg_hi; g.b_lo = P.xg_lo; g.ldb = P.H;
        g.ssq_parts = P.ssq_x; g.n_parts = P.H / 16; g.eps = P.eps; g.ssq_stride = MOE ? P.col_stride : kMaxBatch;
        g.n_cols = P.B;
        e.kind = EPI_QKV; e.layer = t.layer; e.row0 = i0; e.head = hd;
        return true;
    }
    case FN_OPROJ: {
        const int r0 = t.c0 * 16, QD = P.nq * P.d;
        g.n_tiles = 1; g.tile_rows = 16;
        g.rowsA = (const uint16_t *)W->wo + (size_t)r0 * QD;
        g.rowsB = g.rowsA + (size_t)8 * QD;
        g.ldw = QD; g.K = QD;
        g.b_hi = P.attn_hi; g.b_lo = P.attn_lo; g.ldb = QD;
        g.n_cols = P.B;
        e.kind = EPI_RESID; e.layer = t.layer; e.row0 = r0; e.resid = P.x; e.outf = P.x_mid; e.ld = P.H;
        e.next_gain = (const uint16_t *)W->g2; e.out_hi = P.xmg_hi; e.out_lo = P.xmg_lo;
        e.ssq_out = P.ssq_xmid + (size_t)t.c0 * kMaxBatch;
        return true;
    }
    case FN_GATEUP: {
        const int f0 = t.c0 * 8;                       // c1 = consecutive tiles
        g.n_tiles = t.c1; g.tile_rows = 8;
        g.rowsA = (const uint16_t *)W->wg + (size_t)f0 * P.H;
        g.rowsB = (const uint16_t *)W->wu + (size_t)f0 * P.H;
        g.ldw = P.H; g.K = P.H;
        g.b_hi = P.xmg_hi; g.b_lo = P.xmg_lo; g.ldb = P.H;
        g.ssq_parts = P.ssq_xmid; g.n_parts = P.H / 16; g.eps = P.eps; g.ssq_stride = MOE ? P.col_stride : kMaxBatch;
        g.n_cols = P.B;
        e.kind = EPI_SWIGLU; e.layer = t.layer; e.row0 = f0; e.out_hi = P.act_hi; e.out_lo = P.act_lo; e.ld = P.F;
        return true;
    }
    case FN_DOWN: {
        const int r0 = t.c0 * 16;
        g.n_tiles = 1; g.tile_rows = 16;
        g.rowsA = (const uint16_t *)W->wd + (size_t)r0 * P.F;
        g.rowsB = g.rowsA + (size_t)8 * P.F;
        g.ldw = P.F; g.K = P.F;
        g.b_hi = P.act_hi; g.b_lo = P.act_lo; g.ldb = P.F;
        g.n_cols = P.B;
        e.kind = EPI_RESID; e.layer = t.layer; e.row0 = r0; e.resid = P.x_mid; e.outf = P.x; e.ld = P.H;
        e.flags = (uint16_t)((t.flags & TF_LAST_LAYER) | ((P.debug_flags & 2u) ? EPF_DUMP_LAYER : 0));
        const bool to_lm = LM && P.vocab > 0 && (t.flags & TF_LAST_LAYER);
        if (!(t.flags & TF_LAST_LAYER) || to_lm) {     // operand of the next layer's QKV projection, or of the vocabulary projection
            e.next_gain = to_lm ? P.gf : (const uint16_t *)as_global(P.weights)[t.layer + 1].g1;
            e.out_hi = P.xg_hi; e.out_lo = P.xg_lo;
            e.ssq_out = P.ssq_x + (size_t)t.c0 * kMaxBatch;
        }
        return true;
    }
    case FN_LMHEAD: {
        if (!LM) return false;
        const int tiles = P.vocab >> 4, r0 = t.c0 * 16;      // c1 = tiles per task; the last task takes what is left
        g.n_tiles = tiles - t.c0 < t.c1 ? tiles - t.c0 : t.c1; g.tile_rows = 16;
        g.rowsA = P.wlm + (size_t)r0 * P.H;
        g.rowsB = g.rowsA + (size_t)8 * P.H;
        g.ldw = P.H; g.K = P.H;
        g.b_hi = P.xg_hi; g.b_lo = P.xg_lo; g.ldb = P.H;
        g.ssq_parts = P.ssq_x; g.n_parts = P.H / 16; g.eps = P.eps; g.ssq_stride = MOE ? P.col_stride : kMaxBatch;
        g.n_cols = P.B;
        e.kind = EPI_LOGITS; e.layer = t.layer; e.row0 = r0; e.outf = P.logits; e.ld = P.vocab;
        return true;
    }
    case FN_ROUTER_LOGITS: {
        if (!MOE) return false;
        const int r0 = t.c0 * 16;
        const int cb = t.c1 * 64;      // stand-alone MoE layer: one task per block of 64 tokens (c1 = 0 in a decoder)
        g.n_tiles = 1; g.tile_rows = 16;
        g.rowsA = (const uint16_t *)W->wr + (size_t)r0 * P.H;
        g.rowsB = g.rowsA + (size_t)8 * P.H;
        g.ldw = P.H; g.K = P.H;
        g.b_hi = P.xmg_hi + (size_t)cb * P.H; g.b_lo = P.xmg_lo + (size_t)cb * P.H; g.ldb = P.H;
        g.ssq_parts = P.ssq_xmid; g.n_parts = P.H / 16; g.eps = P.eps; g.ssq_stride = MOE ? P.col_stride : kMaxBatch;
        g.ssq_parts += cb;
        g.n_cols = P.B - cb < 64 ? P.B - cb : 64;      // <= 0: a block beyond the bound tokens (the caller skips the tile)
        e.kind = EPI_STORE_F32; e.layer = t.layer; e.row0 = r0; e.outf = P.router_logits + (size_t)cb * P.E; e.ld = P.E;
        return true;
    }
    default:
        return false;
    }
}

// Second stage: the slices' partial sums of row tile c0, then the projection's own epilogue.
__device__ __noinline__ void k_slice_sum_task(const Params &PL, Task t_in, int w0, int w1)
{
    Task t = wave_uniform(t_in);
    w0 = __builtin_amdgcn_readfirstlane(w0);
    w1 = __builtin_amdgcn_readfirstlane(w1);
    GemmTile g{};
    Epilogue e{};
    const bool o_proj = t.fn == FN_OPROJ_SUM;
    t.fn = o_proj ? FN_OPROJ : FN_DOWN;
    setup_gemm<false, true>(PL, t, g, e);
    wg_wait(PL, w0, w1, t.fn);
    kslice_sum(PL, e, PL.B, o_proj ? PL.k_slices_o : PL.k_slices_d, PL.H / 16);
}

// GroupGEMM tile of a resolved row tile: the weight rows depend on the routing, so this runs after the wait.
__device__ __forceinline__ void setup_moe_gemm(const Params &P, const Task &t, const RowTile &rt, GemmTile &g, Epilogue &e)
{
    const ETC_AS_GLOBAL LayerWeights *W = as_global(P.weights) + t.layer;
    g.n_tiles = t.c2;
    g.n_cols = rt.n;
    e.layer = t.layer;
    e.col0 = rt.row0;
    if (t.fn == FN_MOE_GATEUP) {
        const int f0 = t.c1 * 8;
        const size_t off = ((size_t)rt.expert * P.moeF + f0) * (size_t)P.H;
        g.tile_rows = 8;
        g.rowsA = (const uint16_t *)W->eg + off;
        g.rowsB = (const uint16_t *)W->eu + off;
        g.ldw = P.H; g.K = P.H;
        g.b_hi = P.xmg_hi; g.b_lo = P.xmg_lo; g.ldb = P.H;
        g.col_rows = P.perm_tok + rt.row0;             // column n reads the hidden state of the row's token
        g.ssq_parts = P.ssq_xmid; g.n_parts = P.H / 16; g.eps = P.eps; g.ssq_stride = P.col_stride;
        e.kind = EPI_MOE_ACT; e.row0 = f0; e.out_hi = P.eact_hi; e.out_lo = P.eact_lo; e.ld = P.moeF;
    } else {
        const int h0 = t.c1 * 16;
        g.tile_rows = 16;
        g.rowsA = (const uint16_t *)W->ed + ((size_t)rt.expert * P.H + h0) * (size_t)P.moeF;
        g.rowsB = g.rowsA + (size_t)8 * P.moeF;
        g.ldw = P.moeF; g.K = P.moeF;
        g.b_hi = P.eact_hi + (size_t)rt.row0 * P.moeF;
        g.b_lo = P.eact_lo + (size_t)rt.row0 * P.moeF;
        g.ldb = P.moeF;
        e.kind = EPI_MOE_Y; e.row0 = h0; e.outf = P.ey; e.ld = P.H;
    }
}

// A projection task on the staged path, out of line, for every instance but the staged-only ones (whose task loop is
// built around that path).  Inlined into a task loop that also carries the MoE or the large-batch task kinds, the
// streaming loop was at the mercy of the register allocation of everything around it: builds differed by whether
// reloads of spilled registers landed inside the loop (where each queues behind the whole weight ring), 15 % of a MoE
// step.  As a function it has the register file to itself.  It takes the task record and rebuilds the tile
// descriptors itself (scalar work): 25 words of arguments travel in registers; the descriptors would spill over
// to the stack, i.e. to scratch memory, once per lane and call (3 GB per Qwen3-shape step at batch 1).
// mode 0: decoder projection, 1: GroupGEMM row tile rt, 2: K slice of a decoder projection.
template <bool MOE, bool LM>
__device__ __noinline__ WgState staged_task_out_of_line(const Params &PL, Task t_in, TaskWaits tw_in, RowTile rt_in, int mode,
                                                       float *sm, WgState st_in)
{
    const Task t = wave_uniform(t_in);
    const TaskWaits tw = wave_uniform(tw_in);
    const RowTile rt = wave_uniform(rt_in);
    WgState st = wave_uniform(st_in);
    mode = __builtin_amdgcn_readfirstlane(mode);
    GemmTile g{};
    Epilogue e{};
    if (MOE && mode == 1) {
        setup_moe_gemm(PL, t, rt, g, e);
    } else {
        setup_gemm<MOE, LM>(PL, t, g, e);
        if (mode == 2) slice_of_k(PL, t, t.fn == FN_OPROJ ? PL.k_slices_o : PL.k_slices_d, g, e);
    }
    gemm_tiles_staged<PF, LM>(PL, g, e, tw, sm, st, t.id);
    return st;
}

// Staged path (out of line, from the task record) or chunked path (out of line, from the descriptors).
template <bool MOE, bool LM>
__device__ __forceinline__ void dispatch_projection(const Params &PL, const Task &t, const TaskWaits &tw, const RowTile &rt, int mode,
                                                    const GemmTile &g, const Epilogue &e, float *sm, WgState &st)
{
    if (staged_fits(g.n_tiles, g.n_cols, g.K)) st = staged_task_out_of_line<MOE, LM>(PL, t, tw, rt, mode, sm, st);
    else gemm_chunked_dispatch<MOE>(PL, g, e, tw, sm, st, t.id);
}

// KIND: which task kinds the kernel instance carries: 0 generic graphs (the row-sum device functions), 1 dense
// decoder, 2 MoE decoder, 3 dense decoder whose projection tasks all fit the staged path (small batches), 4 the
// same with K-slice tasks (the batches at which only a slice of the down projection's operand fits).  The
// one large kernel is short of registers, and code that cannot run still costs some: the dense instance alone
// is 5 % faster than an instance that carries everything, the staged-only instance another 2 %.
constexpr int KIND_GENERIC = 0, KIND_DENSE = 1, KIND_MOE = 2, KIND_DENSE_STAGED = 3, KIND_DENSE_STAGED_K = 4;
// Added to a decoder kind: the instance also carries the end of the iteration (embedding look-up, vocabulary projection,
// sampling).  A flag of the instance for the same reason as the kinds: on the 8B step the code costs 1.5 % where it never runs.
constexpr int KIND_LM = 8;
constexpr int kind_base(int kind) { return kind & 7; }
template <bool SYNC_EVENTS, int KIND>
__device__ __forceinline__ void run_task(const Params &P, const Params &PL, const Task &t, float *sm, WgState &st)
{
    const int w0 = SYNC_EVENTS ? t.wait0 : -1, w1 = SYNC_EVENTS ? t.wait1 : -1;
    TaskWaits tw{w0, w1, (int)t.fn, (t.flags & TF_WAIT0_PER_WAVE) != 0 && SYNC_EVENTS, w0};
    GemmTile g{};
    Epilogue e{};
    constexpr int BASE = kind_base(KIND);
    constexpr bool LM = (KIND & KIND_LM) != 0;
    constexpr bool MOE = BASE == KIND_MOE;
    if (MOE && (t.flags & TF_DYN_ROWTILE)) {      // GroupGEMM tile: its weights depend on the routing
        // The routing tables of a layer are complete once the layer's router event has fired.  A GroupGEMM-2 tile
        // of a workgroup that already ran a GroupGEMM-1 tile of the same layer therefore looks its row tile
        // up at once and prefetches its weights before it waits for its own event (the activations).
        const bool routed = SYNC_EVENTS && t.fn == FN_MOE_DOWN && st.routed_layer == (int)t.layer;
        if (!routed) {
            wg_wait_cached(P, st, w0, w1, t.fn);
            if (SYNC_EVENTS) st.routed_layer = t.layer;
        }
        RowTile rt;
        if (!resolve_row_tile(P, t.c0, rt)) return;        // surplus slot of the static grid: nothing to do but notify
        setup_moe_gemm(P, t, rt, g, e);
        const int key = w0 < 0 ? -1 : w0 + ((t.c0 + 1) << 20);
        tw = routed ? TaskWaits{w0, w1, (int)t.fn, false, key} : TaskWaits{-1, -1, (int)t.fn, false, key};
        dispatch_projection<MOE, LM>(PL, t, tw, rt, 1, g, e, sm, st);
        return;
    }
    constexpr bool STAGED_ONLY = BASE == KIND_DENSE_STAGED || BASE == KIND_DENSE_STAGED_K;
    constexpr bool STAGED_SLICES = BASE == KIND_DENSE_STAGED_K;
    if (BASE != KIND_GENERIC && !STAGED_ONLY && (t.flags & TF_K_SLICE)) {      // first stage of a K-sliced projection
        setup_gemm<false, false>(P, t, g, e);
        slice_of_k(P, t, t.fn == FN_OPROJ ? P.k_slices_o : P.k_slices_d, g, e);
        if (tw.ev0 >= 0) tw.op_key = tw.ev0 + ((t.c1 + 1) << 20);      // a staged copy holds one slice
        dispatch_projection<MOE, LM>(PL, t, tw, RowTile{}, 2, g, e, sm, st);
        return;
    }
    if (BASE != KIND_GENERIC && setup_gemm<MOE, LM>(P, t, g, e)) {
        if (MOE && g.n_cols <= 0) return;         // token block beyond the bound tokens: nothing to do but notify
        if (STAGED_ONLY) {
            if (STAGED_SLICES && (t.flags & TF_K_SLICE)) {      // here a slice of K fits the staged path as well
                slice_of_k(P, t, t.fn == FN_OPROJ ? P.k_slices_o : P.k_slices_d, g, e);
                if (w0 >= 0) tw.op_key = w0 + ((t.c1 + 1) << 20);
            }
            gemm_tiles_staged<10, LM>(P, g, e, tw, sm, st, t.id);
        } else {
            dispatch_projection<MOE, LM>(PL, t, tw, RowTile{}, 0, g, e, sm, st);
        }
        return;
    }
    if (BASE == KIND_GENERIC) {
        wg_wait_cached(P, st, w0, w1, t.fn);
        if (t.fn == FN_ROWSUM_PARTIAL) rowsum_partial(P, t.c0, t.c1);
        else if (t.fn == FN_ROWSUM_FINAL) rowsum_final(P, t.c0);
        else if (t.fn == FN_ROWSUM_FINAL_PERM) rowsum_final_perm(P, t.c0);
        else if (t.fn >= FN_USER0) user_dispatch(P, t.fn - FN_USER0, t.c0, t.c1, t.c2);
        return;
    }
    switch (t.fn) {
    case FN_LOAD_HIDDEN:
        if (t.c0 < P.B) load_hidden<LM>(P, t.c0);
        break;
    case FN_SAMPLE:
        if (!LM) break;
        wg_wait_cached(P, st, w0, w1, t.fn);
        if ((int)threadIdx.x < P.B) {
            const unsigned long long key = ld_u64(P.best + threadIdx.x);
            *as_global(P.token_out + threadIdx.x) = (int32_t)(0xFFFFFFFFu - (uint32_t)(key & 0xFFFFFFFFull));
        }
        break;
    case FN_OPROJ_SUM:
    case FN_DOWN_SUM:
        if (!STAGED_ONLY || STAGED_SLICES) k_slice_sum_task(PL, t, w0, w1);
        break;
    case FN_ATTN: {
        const int b = t.c0, kvh = t.c1, ch = t.c2;
        const bool active = b < P.B && ch * P.kv_chunk < gld_i32(P.kv_len + b) + 1;
        if (active) {     // inactive slots of the sampled-shape queue neither wait nor compute; they still notify
            st.staged_key = -1;      // the attention scratch overlaps the staged operand (the task waits inside)
            const int grp = P.nq / P.nkv;
            const bool lds_pages = P.kv_chunk > 128;      // more than one batch of keys per chunk
            const bool mfma_fits = (P.kv_chunk >> P.page_shift) <= 8192;      // page ids of a chunk next to the wavefronts' V tiles in LDS
            bool ran = false;
#define ETC_ATTN(DD, GG)                                                                   \
    if (!ran && P.d == DD && grp == GG) {                                                  \
        ran = true;                                                                        \
        if constexpr (DD == 128 && GG == 8) {                                              \
            if (lds_pages && mfma_fits) attn_chunk_mfma<GG>(PL, t.layer, b, kvh, ch, sm, w0, w1, t.id);   \
            else if (lds_pages) attn_chunk<DD, GG, true>(PL, t.layer, b, kvh, ch, sm, w0, w1, t.id);       \
            else attn_chunk<DD, GG, false>(PL, t.layer, b, kvh, ch, sm, w0, w1, t.id);     \
        } else {                                                                           \
            if (lds_pages) attn_chunk<DD, GG, true>(PL, t.layer, b, kvh, ch, sm, w0, w1, t.id);  \
            else attn_chunk<DD, GG, false>(PL, t.layer, b, kvh, ch, sm, w0, w1, t.id);     \
        }                                                                                  \
    }
            ETC_ATTN_SHAPES(ETC_ATTN)
#undef ETC_ATTN
            if (!ran && threadIdx.x == 0) raise_error(P, ERR_NO_BODY, FN_ATTN, P.d * 256 + grp);   // refused at create; never silently skipped
        }
        break;
    }
    case FN_MERGE: {
        const int b = t.c0, kvh = t.c1;
        if (b < P.B) {
            wg_wait_cached(P, st, w0, w1, t.fn);
            const int grp = P.nq / P.nkv;
            bool ran = false;
#define ETC_MERGE(DD, GG)                                                                  \
    if (!ran && P.d == DD && grp == GG) {                                                  \
        ran = true;                                                                        \
        attn_merge<DD, GG>(PL, b, kvh);                                                    \
    }
            ETC_ATTN_SHAPES(ETC_MERGE)
#undef ETC_MERGE
            if (!ran && threadIdx.x == 0) raise_error(P, ERR_NO_BODY, FN_MERGE, P.d * 256 + grp);
        }
        break;
    }
    case FN_ROUTER:
        if (MOE && t.c0 < P.B) {
            wg_wait_cached(P, st, w0, w1, t.fn);
            st.staged_key = -1;      // the routing scratch overlaps the staged operand
            moe_route_and_group(PL, t.layer, t.c0, t.notify0, sm);
        }
        break;
    case FN_MOEL_LOAD:
        if (MOE) moel_load(PL, t.c0);
        break;
    case FN_MOEL_TOPK:
    case FN_MOEL_SCAN:
    case FN_MOEL_PLACE:
        if (MOE) {
            wg_wait_cached(P, st, w0, w1, t.fn);
            st.staged_key = -1;      // the routing scratch overlaps the staged operand
            if (t.fn == FN_MOEL_TOPK) moel_topk(PL, t.c0, sm);
            else if (t.fn == FN_MOEL_SCAN) moel_scan(PL, sm);
            else moel_place(PL, t.c0, t.notify0, sm);
        }
        break;
    case FN_COMBINE:
        if (MOE && t.c0 < P.B) {
            wg_wait_cached(P, st, w0, w1, t.fn);
            if (P.moel) moel_combine(P, t.c0, t.c2, t.c1);      // stand-alone layer: (first token, chunk, tokens)
            else moe_combine(P, t);
        }
        break;
    default:
        break;
    }
}

__device__ __forceinline__ Task load_task(const Task *p)
{
    // the queue is read-only for the whole launch; every lane reads the same record
    const u32x4 a = gld_16B(p), b = gld_16B(reinterpret_cast<const u32x4 *>(p) + 1);
    Task t;
    uint32_t w0 = __builtin_amdgcn_readfirstlane(a.x);
    t.fn = (uint8_t)(w0 & 0xFF);
    t.layer = (uint8_t)((w0 >> 8) & 0xFF);
    t.flags = (uint16_t)(w0 >> 16);
    t.c0 = __builtin_amdgcn_readfirstlane(a.y);
    t.c1 = __builtin_amdgcn_readfirstlane(a.z);
    t.c2 = __builtin_amdgcn_readfirstlane(a.w);
    t.wait0 = __builtin_amdgcn_readfirstlane(b.x);
    t.wait1 = __builtin_amdgcn_readfirstlane(b.y);
    t.notify0 = __builtin_amdgcn_readfirstlane(b.z);
    t.id = __builtin_amdgcn_readfirstlane(b.w);
    return t;
}

// Copies the kernel argument into LDS so that out-of-line task bodies can take it by address.
__device__ __forceinline__ void stage_params(const Params &P, Params *dst)
{
    const uint32_t *src = reinterpret_cast<const uint32_t *>(&P);
    uint32_t *d = reinterpret_cast<uint32_t *>(dst);
    for (int i = threadIdx.x; i < (int)(sizeof(Params) / 4); i += kWgThreads) d[i] = src[i];
    __syncthreads();
}

// Re-arms the event tensors of the NEXT launch from the initial counts; nothing in this launch
// touches that buffer, and the next launch starts after this kernel has ended.
__device__ __forceinline__ void rearm_next(const Params &P)
{
    for (int i = blockIdx.x * kWgThreads + threadIdx.x; i < P.n_events; i += gridDim.x * kWgThreads)
        as_global(P.ev_next)[i] = as_global(P.ev_init)[i];
}

template <int KIND>
__global__ void __launch_bounds__(kWgThreads) megakernel_static(const Params P)
{
    extern __shared__ __attribute__((aligned(16))) float sm[];
    __shared__ Params sP;
    stage_params(P, &sP);
    rearm_next(P);
    WgState st;
    wg_state_init(st);
    const int q0 = gld_i32(P.queue_begin + blockIdx.x), q1 = gld_i32(P.queue_begin + blockIdx.x + 1);
    Task t = q0 < q1 ? load_task(P.tasks + q0) : Task{};
    for (int i = q0; i < q1; ++i) {
        Task tn{};
        if (i + 1 < q1) tn = load_task(P.tasks + i + 1);      // fetched early: off the critical path of the next task
        trace_mark(P, t.id, 0);
        trace_mark(P, t.id, 7);
        run_task<true, KIND>(P, sP, t, sm, st);
        trace_mark(P, t.id, 4);
        wg_release();
        if (threadIdx.x == 0) {
            if (t.notify0 >= 0) ev_notify(P, t.notify0);
            if (P.debug_flags & 1u) atomicAdd(P.exec_count + t.id, 1);
        }
        trace_mark(P, t.id, 5);
        t = tn;
    }
}

// ---- dynamic scheduler ------------------------------------------------------------------------
// Ready queue: q_slots[ticket] = (epoch << 32) | (task id + 1).  push: reserve tickets with an atomic
// add on tail, then publish each slot; pop: take a ticket with an atomic add on head, then wait for
// that slot to carry this launch's epoch.  Control words: head, tail, -, tasks completed.  A popper
// that finds its slot empty leaves once every task of the step has counted itself completed.
// Slots and control words follow the rule of all cross-task data here: device-scope stores and loads,
// no cache-wide fence.
//
// Early push (App. E).  A task is pushed as soon as every producer of every event it waits on has been
// DISPATCHED (popped by some workgroup), not completed: each event has a second counter that a producer
// decrements when it is popped, and the workgroup that brings it to zero pushes the event's consumers
// while its own task still has to run.  The consumer keeps its waits, so it can stream its weights and
// then spin exactly like a task of a static queue; the push itself is off the critical path.  No
// deadlock: a task that spins has all its producers running on other workgroups (or spinning in turn on
// tasks dispatched before them).

// All producers of event `ev` are dispatched: publishes the consumers whose other events are that far too.
// Called by every lane of one wavefront, 64 table entries per round (one lane alone took 0.3 us per task:
// a third of a 33 000-task step).
__device__ __forceinline__ void q_push_consumers_wave(const Params &P, int ev)
{
    const int c0 = __builtin_amdgcn_readfirstlane(gld_i32(P.ev_consumers + ev));
    const int c1 = __builtin_amdgcn_readfirstlane(gld_i32(P.ev_consumers + ev + 1));
    for (int i0 = c0; i0 < c1; i0 += 64) {
        const int i = i0 + lane_id();
        bool ready = false;
        int id = 0;
        if (i < c1) {
            const int entry = gld_i32(P.consumer_ids + i);
            id = entry & 0xFFFFFF;
            const int n_waited = (entry >> 24) & 0x7F;
            ready = true;
            if (n_waited > 1) {      // the last of its events to get here pushes the task (the counter only counts up)
                const int seen = __hip_atomic_fetch_add(as_global(P.task_pending + id), 1, __ATOMIC_RELAXED, ETC_SCOPE) + 1;
                ready = seen % n_waited == 0;
            }
        }
        const uint64_t mask = __ballot(ready);
        const int cnt = __builtin_amdgcn_readfirstlane(__popcll(mask));
        if (cnt == 0) continue;
        const int base = q_reserve_wave(P, cnt);
        if (base < 0) return;
        if (ready) {
            const int pos = __popcll(mask & ((1ull << lane_id()) - 1ull));
            __hip_atomic_store(as_global(P.q_slots + base + pos), q_slot_word(P, id), __ATOMIC_RELAXED, ETC_SCOPE);
        }
    }
}

// Pop, in two halves: q_take_ticket reserves the next ticket (one lane), q_wait_slot waits for that slot to
// be published: the task id, or -1 when the step is complete (every task has counted itself done), the
// queue is exhausted or an error was raised.
__device__ __forceinline__ int q_take_ticket(const Params &P)
{
    return __hip_atomic_fetch_add(as_global(P.q_ctrl_cur + 0), 1, __ATOMIC_RELAXED, ETC_SCOPE);
}

__device__ __forceinline__ int q_wait_slot(const Params &P, int ticket)
{
    if (ticket >= P.q_capacity) return -1;
    long long spins = 0;
    for (;;) {
        const uint64_t v = ld_u64(P.q_slots + ticket);
        if ((uint32_t)(v >> 32) == P.epoch) return (int)(uint32_t)v - 1;
        if (ev_peek(P.q_ctrl_cur + 3) >= P.n_static_tasks) return -1;
        if (spins < 32) __builtin_amdgcn_s_sleep(2); else __builtin_amdgcn_s_sleep(32);
        ++spins;
        if ((spins & 63) == 0 && ev_peek(P.error_word) != 0) return -1;
        if (spins > P.spin_budget) { raise_error(P, ERR_POP_TIMEOUT, 0, ticket); return -1; }
    }
}

// Loop shape.  The lane that notifies and pops shares a wavefront with 63 lanes that do not, and
// the task id reaches the other lanes through LDS and a barrier.  The single-lane block therefore sits
// BETWEEN the task's closing barrier and the barrier that publishes the next id, inside one iteration,
// and the loop condition is a scalar: with the block split over the loop's back edge (pop at the top,
// notify at the bottom) the compiler merged the two single-lane blocks and let the other 63 lanes of
// that wavefront run ahead into the next iteration's barrier first, where every wavefront then read the
// previous id again: the same task was repeated without end and the lane that would pop never ran.
template <int KIND>
__global__ void __launch_bounds__(kWgThreads) megakernel_dynamic(const Params P)
{
    extern __shared__ __attribute__((aligned(16))) float sm[];
    __shared__ int s_task;
    __shared__ Params sP;
    stage_params(P, &sP);
    rearm_next(P);
    for (int i = blockIdx.x * kWgThreads + threadIdx.x; i < P.n_events; i += gridDim.x * kWgThreads)
        as_global(P.ev_disp_next)[i] = as_global(P.ev_init)[i];
    if (blockIdx.x == 0 && threadIdx.x == 0) {            // reset the control words of the next launch
        for (int i = 0; i < 8; ++i) P.q_ctrl_next[i] = 0;
    }
    if (kind_base(KIND) == KIND_GENERIC && P.dd_consumer_n > 0 && blockIdx.x == 0 && threadIdx.x == 0) {
        // tasks of the triggered grid beyond the last indptr range are never released: count them completed
        const int surplus = P.dd_consumer_n - gld_i32(reinterpret_cast<const int32_t *>(P.gbuf[4]) + P.dd_n_events);
        if (surplus > 0) __hip_atomic_fetch_add(as_global(P.q_ctrl_cur + 3), surplus, __ATOMIC_RELAXED, ETC_SCOPE);
    }
    // Wavefront 0 is the scheduler of its workgroup: its lane 0 notifies and pops, all its lanes push.
    const bool sched_wave = wave_id() == 0;
    if (sched_wave) {
        // seed: tasks that wait on nothing, a share per workgroup
        const int n_seed = P.n_seed > (int)blockIdx.x ? (P.n_seed - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x : 0;
        if (n_seed > 0) {
            const int base = q_reserve_wave(P, n_seed);
            if (base >= 0)
                for (int i = lane_id(); i < n_seed; i += 64)
                    __hip_atomic_store(as_global(P.q_slots + base + i),
                                       q_slot_word(P, gld_i32(P.seed_tasks + blockIdx.x + i * gridDim.x)), __ATOMIC_RELAXED,
                                       ETC_SCOPE);
        }
        if (lane_id() == 0) s_task = q_wait_slot(P, q_take_ticket(P));
    }
    __syncthreads();
    int id = __builtin_amdgcn_readfirstlane(s_task);
    // The loop has its own bound, whatever the waits inside it do: a workgroup can run each task of the step at
    // most once, so more iterations than the step has tasks mean the loop is repeating itself (a pop that
    // never ran, a stale id): the workgroup records the error and leaves, and every wait of the others then
    // gives up, so the launch drains to ETC_ETIMEOUT instead of spinning for ever.
    int iterations = 0;
    while (id >= 0) {
        if (++iterations > P.n_static_tasks + 1) {
            if (threadIdx.x == 0) raise_error(P, ERR_LOOP_BOUND, 0, id);
            break;
        }
        Task t = load_task(P.dyn_tasks + id);
        // MoE with data-dependent events (Sec. 2.4): the router tiles trigger the GroupGEMM-1 tiles of an expert
        // themselves, when the expert's event fires, so those are not pushed when the router tiles are
        // dispatched, and a triggered tile has nothing left to wait for.
        const bool dd_notify = kind_base(KIND) == KIND_GENERIC && (t.flags & TF_NOTIFY_INDIRECT);     // generic graphs (Sec. 2.4)
        const bool dd_producer = (kind_base(KIND) == KIND_MOE && P.moe_dd && (t.fn == FN_ROUTER || t.fn == FN_MOEL_PLACE)) || dd_notify;
        if (kind_base(KIND) == KIND_MOE && P.moe_dd && t.fn == FN_MOE_GATEUP) t.wait0 = -1;
        if (sched_wave) {
            // This task is dispatched: the last producer of its event to get here pushes the consumers.
            int last = 0;
            if (lane_id() == 0 && t.notify0 >= 0 && !dd_producer)
                last = __hip_atomic_fetch_sub(as_global(P.ev_disp_cur + t.notify0), 1, __ATOMIC_RELAXED, ETC_SCOPE) == 1;
            if (__builtin_amdgcn_readfirstlane(last)) q_push_consumers_wave(P, t.notify0);
        }
        WgState st;
        wg_state_init(st);
        run_task<true, KIND>(P, sP, t, sm, st);
        wg_release();                            // also: every lane has read s_task before it is written again
        if (sched_wave) {
            if (dd_notify) {
                // Data-dependent event update and trigger of a generic graph: the event is table[c0]; its count
                // (count[e], made with the table) is known at run time only, so the notifies count down from zero
                // and the one that completes the count has fired the event; it releases the tasks
                // [indptr[e], indptr[e+1]) of the triggered grid and puts the counter back.
                const int32_t *table = reinterpret_cast<const int32_t *>(P.gbuf[3]), *indptr = reinterpret_cast<const int32_t *>(P.gbuf[4]),
                              *count = reinterpret_cast<const int32_t *>(P.gbuf[5]);
                const int ev = __builtin_amdgcn_readfirstlane(gld_i32(table + t.c0));
                const bool ev_ok = ev >= 0 && ev < P.dd_n_events;
                int fired = 0;
                if (!ev_ok) {
                    if (lane_id() == 0) raise_error(P, ERR_BAD_TABLE, t.fn, t.c0);
                } else if (lane_id() == 0) {
                    const int before = __hip_atomic_fetch_sub(as_global(P.ev_cur + P.dd_event_base + ev), 1, __ATOMIC_RELAXED, ETC_SCOPE);
                    fired = before - 1 == -gld_i32(count + ev);
                    if (fired) st_i32(P.ev_cur + P.dd_event_base + ev, 0);
                }
                drain_vmem();        // the counter is back at zero before anything this event releases is published
                if (__builtin_amdgcn_readfirstlane(fired)) {
                    const int j0 = __builtin_amdgcn_readfirstlane(gld_i32(indptr + ev));
                    const int n = __builtin_amdgcn_readfirstlane(gld_i32(indptr + ev + 1)) - j0;
                    const bool range_ok = j0 >= 0 && n >= 0 && j0 + n <= P.dd_consumer_n;
                    if (!range_ok && lane_id() == 0) raise_error(P, ERR_BAD_TABLE, t.fn, ev);
                    const int base = range_ok && n > 0 ? q_reserve_wave(P, n) : -1;
                    if (base >= 0)
                        for (int i = lane_id(); i < n; i += 64)
                            __hip_atomic_store(as_global(P.q_slots + base + i), q_slot_word(P, P.dd_consumer_first + j0 + i),
                                               __ATOMIC_RELAXED, ETC_SCOPE);
                }
            }
            if (lane_id() == 0) {
                // notify and count the task done without waiting for either atomic: whoever polls an empty
                // queue compares the count with the number of tasks of the step
                if (P.debug_flags & 1u) atomicAdd(P.exec_count + t.id, 1);
                if (t.notify0 >= 0 && !dd_notify) ev_notify(P, t.notify0);
                __hip_atomic_fetch_add(as_global(P.q_ctrl_cur + 3), 1, __ATOMIC_RELAXED, ETC_SCOPE);
                // The next ticket is taken only now.  Taken a task ahead (in the round trip of the dispatch
                // decrement) it cost more than it saved: a workgroup that sits in a long wait, such as the
                // projection behind the attention chunks, then holds a task that an idle workgroup could run
                // (8B step 4.34 against 4.12 ms); taken beside the drain of the task's stores: 4.18 ms.
                s_task = q_wait_slot(P, q_take_ticket(P));
            }
        }
        __syncthreads();
        id = __builtin_amdgcn_readfirstlane(s_task);
    }
}

// One operator stage as an ordinary kernel: block i runs task first + i, no events.
template <int KIND>
__global__ void __launch_bounds__(kWgThreads) stage_kernel(const Params P, int first)
{
    extern __shared__ __attribute__((aligned(16))) float sm[];
    __shared__ Params sP;
    stage_params(P, &sP);
    const Task t = load_task(P.dyn_tasks + first + blockIdx.x);
    WgState st;
    wg_state_init(st);
    run_task<false, KIND>(P, sP, t, sm, st);
}


// ---------------------------------------------------------------------------------------------
// Allocation-free variant of the row-sum graph launch
// ---------------------------------------------------------------------------------------------
// For callers that cannot allocate (HIP graph capture, tight serving loops): everything the generic-graph
// path keeps in allocated device memory - the partial sums B, the event tensors, the materialised static
// queues and the error word - lives in one file-scope device array.  A small plan kernel instantiates the
// row-sum graph for n (tasks, round-robin queues, initial counts: what etc_graph_bind_shape computes on the
// host and uploads) and arms the counters; then the generic static megakernel runs on those tables.
// The array's name is a host-side stand-in only: its device address is looked up once per device with
// hipGetSymbolAddress and that pointer is what kernels and host code use.
constexpr int kNoAllocMaxN = ETC_ROWSUM_NOALLOC_MAX_N;      // row blocks of 32 rows
constexpr int kNoAllocMaxQueues = 1024;
constexpr size_t kNaOffB = 0;                                                     // float [n*32][4]
constexpr size_t kNaOffEvents = kNaOffB + (size_t)kNoAllocMaxN * 32 * 4 * 4;      // int32 [3][max n]: cur | init | next
constexpr size_t kNaOffTasks = kNaOffEvents + (size_t)3 * kNoAllocMaxN * 4;       // Task [5 n]
constexpr size_t kNaOffQueueBegin = kNaOffTasks + (size_t)5 * kNoAllocMaxN * sizeof(Task);
constexpr size_t kNaOffError = kNaOffQueueBegin + (size_t)(kNoAllocMaxQueues + 1) * 4 + 60;   // int32 [4]
constexpr size_t kNoAllocScratchBytes = (kNaOffError + 16 + 255) / 256 * 256;
static_assert(kNaOffEvents % 256 == 0 && kNaOffTasks % 32 == 0 && kNaOffQueueBegin % 16 == 0 && kNaOffError % 16 == 0,
              "scratch regions keep their alignment");

static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

// Instantiates the row-sum graph (Sec. 2.2) for n row blocks: tasks partial_sum(i, j) (id 4 i + j, notifies E[i])
// and final_sum(i) (id 4 n + i, waits on E[i]), dealt round-robin to the queues (task id mod queues, Sec. 3.1),
// E[i] armed with its 4 producers.  Clears the error word.  Everything the launch reads is rewritten here,
// so nothing of an earlier call survives.
__global__ void rowsum_noalloc_plan(Task *tasks, int32_t *queue_begin, int32_t *ev, int32_t *error_word, int n, int n_queues,
                                    int ev_stride)
{
    const int total = 5 * n, full = total / n_queues, rem = total % n_queues;
    const int gid = blockIdx.x * blockDim.x + threadIdx.x, stride = gridDim.x * blockDim.x;
    for (int t = gid; t < total; t += stride) {
        const int q = t % n_queues, k = t / n_queues;
        const int pos = q * full + (q < rem ? q : rem) + k;
        Task r{};
        r.wait0 = r.wait1 = r.notify0 = -1;
        r.id = t;
        if (t < 4 * n) { r.fn = FN_ROWSUM_PARTIAL; r.c0 = t >> 2; r.c1 = t & 3; r.notify0 = t >> 2; }
        else { r.fn = FN_ROWSUM_FINAL; r.c0 = t - 4 * n; r.wait0 = t - 4 * n; }
        tasks[pos] = r;
    }
    for (int q = gid; q <= n_queues; q += stride) queue_begin[q] = q * full + (q < rem ? q : rem);
    for (int i = gid; i < n; i += stride) {
        ev[i] = 4;                      // cur
        ev[ev_stride + i] = 4;          // init (the megakernel copies it into `next`)
    }
    if (gid < 4) error_word[gid] = 0;
}

hipError_t configure_kernels();
hipError_t max_resident_workgroups(int *per_cu);

namespace {
struct NoAllocDevice {
    bool ready = false;
    unsigned char *ptr = nullptr;       // this device's copy of `scratch`
    int n_queues = 0;
};
NoAllocDevice g_noalloc[64];
}  // namespace

// Per device, once: the array's address on that device, the kernels' LDS attribute, the queue count.
static hipError_t noalloc_device(NoAllocDevice **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    NoAllocDevice &d = g_noalloc[dev];
    if (!d.ready) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        e = configure_kernels();
        if (e != hipSuccess) return e;
        int cus = 0, per_cu = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        e = max_resident_workgroups(&per_cu);
        if (e != hipSuccess) return e;
        if (per_cu < 1 || cus < 1) return hipErrorLaunchOutOfResources;
        d.ptr = (unsigned char *)p;
        d.n_queues = cus < kNoAllocMaxQueues ? cus : kNoAllocMaxQueues;
        d.ready = true;
    }
    *out = &d;
    return hipSuccess;
}

hipError_t launch_rowsum_noalloc(const float *A, float *C, int n, hipStream_t s)
{
    NoAllocDevice *d = nullptr;
    hipError_t e = noalloc_device(&d);
    if (e != hipSuccess) return e;
    unsigned char *base = d->ptr;            // never the array's name: that is not a device address on the host
    Task *tasks = reinterpret_cast<Task *>(base + kNaOffTasks);
    int32_t *queue_begin = reinterpret_cast<int32_t *>(base + kNaOffQueueBegin);
    int32_t *ev = reinterpret_cast<int32_t *>(base + kNaOffEvents);
    int32_t *error_word = reinterpret_cast<int32_t *>(base + kNaOffError);
    const int plan_threads = 256, plan_blocks = (5 * n + plan_threads - 1) / plan_threads + 4;
    hipLaunchKernelGGL(rowsum_noalloc_plan, dim3(plan_blocks), dim3(plan_threads), 0, s, tasks, queue_begin, ev, error_word, n,
                       d->n_queues, kNoAllocMaxN);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    Params P{};
    P.gbuf[0] = const_cast<float *>(A);
    P.gbuf[1] = reinterpret_cast<float *>(base + kNaOffB);
    P.gbuf[2] = C;
    P.ev_cur = ev;
    P.ev_init = ev + kNoAllocMaxN;
    P.ev_next = ev + 2 * kNoAllocMaxN;
    P.n_events = n;
    P.tasks = tasks;
    P.queue_begin = queue_begin;
    P.n_queues = d->n_queues;
    P.spin_budget = 2000000;
    P.error_word = error_word;
    P.gsym[0] = n;
    hipLaunchKernelGGL(megakernel_static<KIND_GENERIC>, dim3(P.n_queues), dim3(kWgThreads), kLdsBytes, s, P);
    return hipGetLastError();
}

}  // namespace etc

// ---------------------------------------------------------------------------------------------
// host-side launch helpers (called from api.cpp)
// ---------------------------------------------------------------------------------------------
namespace etc {

hipError_t configure_kernels()
{
#ifdef ETC_GENERIC_ONLY
    const void *kernels[] = {(const void *)megakernel_static<0>, (const void *)megakernel_dynamic<0>, (const void *)stage_kernel<0>};
#else
    const void *kernels[] = {(const void *)megakernel_static<0>, (const void *)megakernel_static<1>, (const void *)megakernel_static<2>,
                             (const void *)megakernel_static<3>, (const void *)megakernel_static<4>,
                             (const void *)megakernel_dynamic<0>, (const void *)megakernel_dynamic<1>, (const void *)megakernel_dynamic<2>,
                             (const void *)megakernel_dynamic<3>, (const void *)megakernel_dynamic<4>,
                             (const void *)stage_kernel<0>, (const void *)stage_kernel<1>, (const void *)stage_kernel<2>,
                             (const void *)stage_kernel<3>, (const void *)stage_kernel<4>};
#endif
    for (const void *k : kernels) {
        hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t max_resident_workgroups(int *per_cu)
{
#ifdef ETC_GENERIC_ONLY
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(per_cu, (const void *)megakernel_static<KIND_GENERIC>, kWgThreads, kLdsBytes);
#else
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(per_cu, (const void *)megakernel_static<KIND_MOE>, kWgThreads, kLdsBytes);
#endif
}

// generic graph contexts carry no model; decoders are dense (small-batch plans: the staged-only instance) or MoE
static int kind_of(const Params &P)
{
    if (P.n_layers == 0) return KIND_GENERIC;
    const int lm = P.vocab > 0 ? KIND_LM : 0;
    if (P.E > 0) return KIND_MOE | lm;
    if (!P.all_staged) return KIND_DENSE | lm;
    return ((P.k_slices_o > 0 || P.k_slices_d > 0) ? KIND_DENSE_STAGED_K : KIND_DENSE_STAGED) | lm;
}

#ifdef ETC_GENERIC_ONLY      // a library generated for one graph: no decoder instances (they are most of the compile time)
#define ETC_LAUNCH_KIND(KERNEL, GRID, ...)                                                                          \
    if (kind_of(P) != KIND_GENERIC) return hipErrorInvalidDeviceFunction;                                          \
    hipLaunchKernelGGL(KERNEL<KIND_GENERIC>, GRID, dim3(kWgThreads), kLdsBytes, s, __VA_ARGS__);
#else
#define ETC_LAUNCH_KIND(KERNEL, GRID, ...)                                                                          \
    switch (kind_of(P)) {                                                                                          \
    case KIND_GENERIC: hipLaunchKernelGGL(KERNEL<KIND_GENERIC>, GRID, dim3(kWgThreads), kLdsBytes, s, __VA_ARGS__); break; \
    case KIND_DENSE: hipLaunchKernelGGL(KERNEL<KIND_DENSE>, GRID, dim3(kWgThreads), kLdsBytes, s, __VA_ARGS__); break;     \
    case KIND_DENSE_STAGED: hipLaunchKernelGGL(KERNEL<KIND_DENSE_STAGED>, GRID, dim3(kWgThreads), kLdsBytes, s, __VA_ARGS__); break; \
    case KIND_DENSE_STAGED_K: hipLaunchKernelGGL(KERNEL<KIND_DENSE_STAGED_K>, GRID, dim3(kWgThreads), kLdsBytes, s, __VA_ARGS__); break; \
    case KIND_MOE: hipLaunchKernelGGL(KERNEL<KIND_MOE>, GRID, dim3(kWgThreads), kLdsBytes, s, __VA_ARGS__); break;         \
    case KIND_DENSE | KIND_LM: hipLaunchKernelGGL(KERNEL<KIND_DENSE | KIND_LM>, GRID, dim3(kWgThreads), kLdsBytes, s, __VA_ARGS__); break; \
    case KIND_DENSE_STAGED | KIND_LM: hipLaunchKernelGGL(KERNEL<KIND_DENSE_STAGED | KIND_LM>, GRID, dim3(kWgThreads), kLdsBytes, s, __VA_ARGS__); break; \
    case KIND_DENSE_STAGED_K | KIND_LM: hipLaunchKernelGGL(KERNEL<KIND_DENSE_STAGED_K | KIND_LM>, GRID, dim3(kWgThreads), kLdsBytes, s, __VA_ARGS__); break; \
    default: hipLaunchKernelGGL(KERNEL<KIND_MOE | KIND_LM>, GRID, dim3(kWgThreads), kLdsBytes, s, __VA_ARGS__); break;     \
    }
#endif

hipError_t launch_static(const Params &P, hipStream_t s)
{
    ETC_LAUNCH_KIND(megakernel_static, dim3(P.n_queues), P)
    return hipGetLastError();
}

hipError_t launch_dynamic(const Params &P, hipStream_t s)
{
    ETC_LAUNCH_KIND(megakernel_dynamic, dim3(P.n_queues), P)
    return hipGetLastError();
}

// Arms the event tensors (and the dynamic scheduler's words) of the step the next launch on this stream runs.
__global__ void arm_step_kernel(const ArmArgs a)
{
    const int gid = blockIdx.x * blockDim.x + threadIdx.x, stride = gridDim.x * blockDim.x;
    if (a.ev_cur != nullptr)
        for (int i = gid; i < a.n_events; i += stride) {
            const int32_t v = a.ev_init[i];
            a.ev_cur[i] = v;
            if (a.disp_cur != nullptr) a.disp_cur[i] = v;
        }
    if (a.pending != nullptr)
        for (int i = gid; i < a.n_pending; i += stride) a.pending[i] = 0;
    if (a.exp_event != nullptr)
        for (int i = gid; i < a.n_exp; i += stride) a.exp_event[i] = 0;
    if (a.qctrl != nullptr && gid < 8) a.qctrl[gid] = 0;
    if (a.exec_count != nullptr)
        for (int i = gid; i < a.n_exec; i += stride) a.exec_count[i] = 0;
}

hipError_t launch_arm(const ArmArgs &a, hipStream_t s)
{
    hipLaunchKernelGGL(arm_step_kernel, dim3(128), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_stage(const Params &P, int first, int count, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    ETC_LAUNCH_KIND(stage_kernel, dim3(count), P, first)
    return hipGetLastError();
}

}  // namespace etc
