// Plain-data structures shared by the host scheduler and the device megakernel.
#pragma once
#include <stdint.h>

namespace etc {

constexpr int kWgThreads = 512;          // one task = one workgroup of 8 wavefronts on one CU
constexpr int kWaves = kWgThreads / 64;
constexpr int kMaxBatch = 64;
constexpr int kMaxLayers = 128;
constexpr int kMaxExperts = 256;
constexpr int kMaxTopK = 16;
constexpr int kLdsBytes = 148 * 1024;    // of the 160 KB LDS per CU: exactly one persistent workgroup per CU
constexpr int kRsFloats = 64;                     // LDS: RMSNorm factors of the columns
constexpr int kStagedMaxCols = 16;                // widest batch the staged (latency-critical) projection path takes

// LDS layout of the staged projection path: reduction buffer [tiles][waves][cols][16], norm factors, then
// the whole operand (all columns, hi and lo).  A task takes that path when this fits.
// A column of the operand is K + kOpPad elements apart from the next: with a stride of K (a multiple of the bank
// span) the 16 columns a wavefront reads in one instruction would all sit in the same banks.
constexpr int kOpPad = 8;
constexpr long long staged_red_floats(int n_tiles, int n_cols) { return (long long)n_tiles * n_cols * kWaves * 16; }
constexpr bool staged_fits(int n_tiles, int n_cols, int K)
{
    return n_cols <= kStagedMaxCols &&
           (staged_red_floats(n_tiles, n_cols) + kRsFloats) * 4 + (long long)n_cols * (K + kOpPad) * 4 <= (long long)kLdsBytes;
}

// The (head_dim, query heads per KV head) pairs the attention task bodies are instantiated for.  The device
// dispatch and the host check both read this one list: a shape outside it is refused at create.
#define ETC_ATTN_SHAPES(X) X(128, 4) X(128, 8) X(64, 2) X(128, 1) X(64, 4)
inline bool attn_shape_supported(int head_dim, int group)
{
#define ETC_ATTN_SHAPE_TEST(DD, GG) if (head_dim == DD && group == GG) return true;
    ETC_ATTN_SHAPES(ETC_ATTN_SHAPE_TEST)
#undef ETC_ATTN_SHAPE_TEST
    return false;
}

// Device functions (task bodies).  One entry of the dispatch switch each (Alg. 1 "dispatch logic").
enum Fn : uint8_t {
    FN_NOP = 0,
    FN_ROWSUM_PARTIAL = 1,
    FN_ROWSUM_FINAL = 2,
    FN_USER0 = 100,              // generic graphs: first device function of a generated dispatch switch (front end)
    FN_ROWSUM_FINAL_PERM = 17,   // generic graphs: final sum of row block perm[task], tasks beyond indptr[last] do nothing
    FN_LOAD_HIDDEN = 3,   // hidden_in bf16 -> residual stream fp32
    FN_QKV = 4,           // RMSNorm prologue, 16 rows of Wq|Wk|Wv (8 RoPE pairs), RoPE, KV append
    FN_ATTN = 5,          // split-KV partial attention of (sequence, kv head, chunk)
    FN_MERGE = 6,         // merge of the chunk partials of (sequence, kv head)
    FN_OPROJ = 7,         // 16 rows of Wo + residual
    FN_GATEUP = 8,        // RMSNorm prologue, 8 gate + 8 up rows, SiLU-mul epilogue
    FN_DOWN = 9,          // 16 rows of Wd + residual (waves split K; each waits for its own K slice)
    FN_ROUTER_LOGITS = 10,// MoE: RMSNorm prologue, 16 rows of the router matrix -> fp32 logits
    FN_ROUTER = 11,       // MoE: one tile per token: top-k ids and weights, counts, indptr, stable rank of its slots
    FN_MOE_GATEUP = 12,   // MoE: GroupGEMM-1 tile (row tile of routed tokens, 8 gate + 8 up rows), SiLU-mul
    FN_MOE_DOWN = 13,     // MoE: GroupGEMM-2 tile (row tile, 16 rows of the expert's Wd)
    FN_COMBINE = 14,      // MoE: weighted sum of a token's expert outputs in slot order + residual
    FN_OPROJ_SUM = 15,    // large batches: fixed-order sum of the K-slice partials of 16 rows of the O projection + residual
    FN_DOWN_SUM = 16,     // the same for the down projection
    FN_LMHEAD = 18,       // end of the iteration: final RMSNorm folded in, consecutive 16-row tiles of the vocabulary projection ->
                          //   fp32 logits, and each tile's best (logit, id) folded into the sequence's running maximum
    FN_SAMPLE = 19,       // greedy token of every sequence from the running maxima (ties: lower id)
    // The MoE layer on its own over a block of tokens (Sec. 2.4; token sweep of Sec. 4.2 / 4.5): grouping in three
    // counting passes instead of one tile per token, because a tile that ranks against every token is quadratic.
    FN_MOEL_LOAD = 20,    // 16 tokens: x_in bf16 -> residual fp32, (x * gain) split, per-tile sums of squares
    FN_MOEL_TOPK = 21,    // 64 tokens: top-k ids and weights of each, the block's pair count per expert
    FN_MOEL_SCAN = 22,    // one task: totals, prefix sums over experts and blocks, row-tile tables
    FN_MOEL_PLACE = 23,   // 64 tokens: stable rank of the block's pairs -> permutation; dynamic scheduler: expert events
    FN_COUNT
};

// Task flags
enum : uint16_t {
    TF_WAIT0_PER_WAVE = 1,   // wave w waits on event wait0 + w instead of the whole workgroup on wait0
    TF_LAST_LAYER = 2,       // also write hidden_out
    TF_DYN_ROWTILE = 4,      // c0 is a GroupGEMM row-tile id resolved through exp_indptr at run time
    TF_K_SLICE = 8,          // projection task over one slice of K: c1 = slice, c2 = row tiles; writes fp32 partials
    TF_NOTIFY_INDIRECT = 16, // dynamic scheduler: notifies event notify0 + table[c0] (data-dependent update, Sec. 2.4)
    TF_TRIGGERED = 32,       // dynamic scheduler: released by the event whose indptr range holds c0 (data-dependent trigger)
};

// One materialised task of a static queue (Sec. 3.1: "static execution queue"), 32 bytes.
struct Task {
    uint8_t fn;
    uint8_t layer;
    uint16_t flags;
    int32_t c0, c1, c2;      // task coordinate
    int32_t wait0, wait1;    // flat event indices to wait on (-1: none)
    int32_t notify0;         // flat event index to notify (-1: none)
    int32_t id;              // global task id (exec-count slot)
};
static_assert(sizeof(Task) == 32, "Task must stay 32 bytes");

struct LayerWeights {
    const void *g1, *wq, *wk, *wv, *wo, *g2, *wg, *wu, *wd, *wr, *eg, *eu, *ed, *gq, *gk;
};

// Error word codes
enum : int32_t { ERR_NONE = 0, ERR_WAIT_TIMEOUT = 1, ERR_QUEUE_OVERFLOW = 2, ERR_POP_TIMEOUT = 3, ERR_BAD_TABLE = 4,
                 ERR_NO_BODY = 5,        // a task kind or shape the kernel instance has no body for
                 ERR_LOOP_BOUND = 6 };   // the dynamic dispatch loop ran more iterations than the step has tasks

// Everything the megakernel needs, passed by value as the kernel argument.
struct Params {
    // model
    int32_t n_layers, H, nq, nkv, d, F, E, topk, moeF, page;
    int32_t page_shift;                // log2(page): pages hold a power of two of tokens
    float eps, theta;
    const double *rope_inv_freq;       // [d/2] theta^(-2i/d), computed on the host in double
    int32_t kv_chunk, tile_m;
    int32_t qk_norm;                   // per-head RMSNorm of q and k before RoPE (Qwen3-style)
    int32_t vocab;                     // > 0: final norm + vocabulary projection + greedy token at the end of the step
    const uint16_t *embed, *gf, *wlm;  // bf16: embedding table [vocab, H] (null: steps start from hidden states), final norm gain [H],
                                       //   vocabulary projection [vocab, H]
    const int32_t *token_in;           // [B] token ids whose embedding rows start the step (null: hidden_in does)
    int32_t *token_out;                // [B] greedy tokens
    float *logits;                     // [B, vocab] fp32
    unsigned long long *best;          // [maxB] running maximum of (ordered logit bits << 32 | ~id), cleared by the step prologue
    // resident tensors
    const LayerWeights *weights;       // [n_layers] device
    uint16_t *kpool, *vpool;           // bf16 bits
    int64_t pool_layer_stride;         // elements per layer
    // step shape
    int32_t B;                         // bound batch
    int32_t Bs;                        // sampled batch the queues were built for
    int32_t max_chunks;                // attention chunk slots per sequence in the queues
    const int32_t *kv_len, *page_indptr, *page_ids;
    const uint16_t *hidden_in;
    uint16_t *hidden_out;
    // scratch (library-owned; crosses tasks, so it is only touched with device-scope accesses)
    float *x, *x_mid;                  // residual stream before / after the attention block [maxB, H]
    uint16_t *xg_hi, *xg_lo;           // x * g1 of the consuming layer, split into bf16 hi + lo [maxB, H]
    uint16_t *xmg_hi, *xmg_lo;         // x_mid * g2, split [maxB, H]
    float *ssq_x, *ssq_xmid;           // partial sums of squares per 16-row tile [H/16][kMaxBatch]
    float *qbuf;                       // rotated queries [maxB, nq*d]
    float *knew, *vnew;                // this step's K (rotated) and V rows in fp32 [maxB, nkv*d]: the cache gets bf16
    float *qk_ssq;                     // qk_norm: sums of squares of the raw q / k heads per 16-row tile [maxB, nq + nkv, d / 16];
                                       //   qbuf / knew then hold gain-scaled, rotated but not yet normalised heads
    float *rope_cs;                    // this step's (cos, sin) of every sequence's RoPE angles [maxB, d/2, 2], from the step prologue
    int32_t *kv_slot;                  // this step's KV slot of every sequence: page * page_size + pos % page_size [maxB]
    uint16_t *attn_hi, *attn_lo;       // attention output, split [maxB, nq*d]
    uint16_t *act_hi, *act_lo;         // silu(gate)*up, split [maxB, F]
    float *part_m, *part_l, *part_o;   // split-KV partials [maxB, nq, max_chunks] (+ [d])
    int32_t *attn_arrive;              // [maxB, nkv] chunk tasks of the (sequence, KV head) that have stored their partials: the
                                       //   last one merges and puts the counter back to zero
    int32_t col_stride;                // floats between two tiles' rows of ssq_x / ssq_xmid: kMaxBatch for decoders, the
                                       //   token capacity of a stand-alone MoE layer
    float *kpart;                      // K-slice partials of a projection [slice][row tile][kMaxBatch][16], or null
    int32_t k_slices_o, k_slices_d;    // slices of K of the O / down projection tasks of the bound plan (0: whole K)
    int32_t all_staged;                // every projection task of the bound plan fits the staged path
    // MoE scratch (rows of the grouped tensors are (token, slot) pairs sorted by (expert, token, slot))
    float *router_logits;              // [maxB, E]
    int32_t *topk_ids;                 // [maxB, topk]
    float *topk_w;                     // [maxB, topk]
    int32_t *tok_indptr, *exp_indptr;  // [E+1] prefix sums of routed pairs / of row tiles per expert
    int32_t *perm, *inv_perm, *perm_tok; // [maxB*topk]: row -> pair, pair -> row, row -> token
    int32_t *tile_expert, *tile_row0, *tile_n; // [max row tiles]: expert, first row and rows of every row tile
    uint16_t *eact_hi, *eact_lo;       // expert activations, split [maxB*topk, moeF]
    float *ey;                         // expert outputs fp32 [maxB*topk, H]
    int32_t moel;                      // 1: stand-alone MoE layer over a block of B tokens
    int32_t *moel_hist;                // [token blocks of 64][E] pairs of the block routed to the expert
    int32_t *moel_base;                // [token blocks][E] first grouped row of the block's pairs of the expert
    int32_t *moel_count;               // [E] pairs routed to the expert
    const int32_t *forced_topk;        // [n_layers, maxB, topk] or null
    const uint8_t *forced_mask;        // [n_layers] or null: bit 0 = ids forced, bit 1 = weights forced as well
    const float *forced_w;             // [n_layers, maxB, topk] or null
    // per-layer copies of the routing data (debug flag 4), or null
    float *dbg_logits, *dbg_topk_w;    // [n_layers, maxB, E], [n_layers, maxB, topk]
    int32_t *dbg_topk_ids, *dbg_perm;  // [n_layers, maxB, topk], [n_layers, maxB*topk]
    int32_t *dbg_tok_indptr, *dbg_exp_indptr; // [n_layers, E+1]
    int32_t max_batch;                 // row stride of the per-layer debug copies
    // event tensors: three equal arrays [cur | init | next]; the kernel re-arms `next` from `init`
    int32_t *ev_cur;
    const int32_t *ev_init;
    int32_t *ev_next;
    int32_t n_events;
    // static queues
    const Task *tasks;                 // all queues back to back
    const int32_t *queue_begin;        // [n_queues + 1]
    int32_t n_queues;
    // dynamic scheduler
    const Task *dyn_tasks;             // task table indexed by task id
    const int32_t *ev_consumers;       // [n_events + 1] CSR: tasks that wait on the event
    const int32_t *consumer_ids;       // task id | (number of events the task waits on << 24 when that is > 1)
    int32_t *ev_disp_cur;              // per event: producers not yet dispatched (early push, App. E)
    int32_t *ev_disp_next;             //   re-armed from ev_init like the event tensors
    int32_t *task_pending;             // per task: waited events whose producers are all dispatched (counts up)
    // MoE under the dynamic scheduler: data-dependent event update and task triggering (Sec. 2.4)
    int32_t moe_dd;                    // 1: expert events armed at run time trigger the GroupGEMM-1 tiles
    int32_t *exp_event;                // [E] expert event tensor E_exp of the layer in flight
    const int32_t *moe_layer_events;   // [n_layers][2] flat ids: event of row-tile slot 0 (GroupGEMM-1 -> 2), combine event
    int32_t moe_rmax, moe_groups_gu, moe_groups_down;   // row-tile slots of the static grids, tasks per slot
    const int32_t *seed_tasks;         // tasks with no trigger edge, pushed at start
    int32_t n_seed;
    int32_t n_static_tasks;
    uint64_t *q_slots;                 // (epoch << 32 | task id + 1)
    int32_t q_capacity;
    int32_t *q_ctrl_cur;               // [head, tail, -, tasks completed, ...]
    int32_t *q_ctrl_next;
    uint32_t epoch;
    // debug / safety
    int64_t spin_budget;
    uint32_t debug_flags;
    int32_t *exec_count;
    float *layer_hidden;               // [n_layers, maxB, H]
    int32_t *error_word;               // [4]
    int32_t *error_host;               // pinned host word the first error code is mirrored to (or null)
    uint64_t *trace;                   // [n_tasks][8] wall-clock marks, or null
    // generic-graph buffers (row-sum example)
    float *gbuf[8];                    // 0..2: A, B, C of the row-sum functions; 3..6: int32 route, indptr, count, perm
    int32_t dd_event_base, dd_n_events;        // generic graphs: the data-dependently notified event tensor
    int32_t dd_consumer_first, dd_consumer_n;  // task ids of the call it triggers
    int32_t dd_table_len;                      // entries of the table = first grid extent of the notifying call
    int32_t gsym[4];
};

}  // namespace etc
