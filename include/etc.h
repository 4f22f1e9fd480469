/*
 * etc.h  --  C ABI of the event-tensor decode megakernel for AMD MI355X (gfx950).
 *
 * One persistent HIP kernel runs a whole LLM decode step as tiled tasks.  Every
 * task is gated by an event tensor (a grid of per-tile dependency counters in
 * HBM, paper Sec. 2.1): a producer tile notifies (atomic decrement, Sec. 3.3) the
 * events it feeds when it ends, a consumer tile waits (spin until zero) on the
 * events it reads when it starts.  No kernel boundary and no host launch sits
 * between operators.
 *
 * The four verbs follow the paper's statement of the problem:
 *   describe  etc_create / etc_graph_*   graph function = device-function launches with
 *                                        task shapes and event tensors (Sec. 2.1), tile
 *                                        shapes, scheduling transformation (Sec. 3.1 / 3.2)
 *   bind      etc_bind_layer_weights / etc_bind_kv_pool        resident tensors
 *   bind      etc_bind_step              symbolic shapes -> concrete (Sec. 2.3): batch,
 *                                        ragged KV lengths, page tables; no re-create
 *   launch    etc_launch                 exactly one kernel launch per decode step
 *
 * Conventions.  Plain C, no exceptions cross the boundary.  Every call returns an
 * etc_status; etc_last_error() gives the text.  A context is not thread-safe and
 * has one step in flight at a time: all launches of a context go to one stream, or the caller
 * orders them (the step's shape arrays, activations and event tensors are one set per context).
 *
 * Co-residency.  Tasks spin on events other workgroups notify (Sec. 3.3), so every persistent
 * workgroup of a launch must be resident at once: the library launches one per compute unit
 * (each takes nearly all of a unit's LDS) and needs the device to itself for the duration of a
 * launch.  A kernel of another stream or process that holds compute units while a megakernel
 * starts can keep some of its workgroups from becoming resident; their peers' waits then run
 * out of their spin budget and the launch ends with ETC_ETIMEOUT rather than hanging.
 * etc_create returns ETC_ESTATE when the device cannot hold the requested queues at all.
 *
 * Device errors.  A wait that exceeds its spin budget, a full ready queue or a bad run-time table
 * records an error word and the kernel drains (tasks still run, on stale data: the outputs of
 * that launch are garbage).  The first call that notices (etc_read_debug, or the next
 * etc_bind_step / etc_launch / etc_graph_launch after the launch has finished) returns
 * ETC_ETIMEOUT; from then on the context is dead: launches and binds return ETC_ESTATE and only
 * etc_read_debug and etc_destroy are useful (a generic-graph context is revived by
 * etc_graph_bind_shape, which rebuilds all launch state).  Pointers marked "device" are device memory
 * of the current HIP device, borrowed: the caller owns them and keeps them alive
 * until the last launch that uses them has finished.  Pointers marked "host" are
 * read during the call only.  The library owns all scratch (activations, event
 * tensors, task lists, queues).  All weights, KV pages and hidden states are bf16;
 * accumulation is fp32.
 */
#ifndef ETC_H
#define ETC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct etc_ctx etc_ctx; /* opaque, library-owned */

typedef enum {
    ETC_OK = 0,
    ETC_EINVAL = -1,   /* bad argument or descriptor */
    ETC_ENOMEM = -2,   /* host or device allocation failed */
    ETC_ESTATE = -3,   /* call order: something is not bound yet */
    ETC_EDEVICE = -4,  /* a HIP call failed */
    ETC_ETIMEOUT = -5  /* device watchdog: a wait exceeded its spin budget; the kernel drained */
} etc_status;

/* ---- describe ------------------------------------------------------------------------- */

/* Decoder shape.  Dense SwiGLU FFN when n_experts == 0, otherwise top_k-of-n_experts MoE with
 * per-expert SwiGLU width moe_ffn (Sec. 2.4, 4.2).  RoPE pairs element i with i + head_dim/2. */
typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn;
    int32_t n_experts, top_k, moe_ffn;
    int32_t page_size; /* tokens per KV page; a power of two (the paper's workloads use 16) */
    float rms_eps, rope_theta;
    int32_t qk_norm;   /* != 0: per-head RMSNorm of q and k (over head_dim, gains gq / gk, rms_eps) before RoPE: the
                          "Q-Norm + RoPE" and "K-Norm + RoPE + CacheAppend" tasks of Sec. 4.3 (Qwen3-style models) */
    int32_t vocab;     /* > 0: the model ends in a final RMSNorm and a vocabulary projection; see etc_bind_lm_head */
} etc_model_desc;

/* Tile shapes of the task grids (Sec. 2.1: tasks are CU-level tiles). */
typedef struct {
    int32_t kv_chunk_tokens; /* smallest number of keys per split-KV attention task; multiple of page_size.
                                Per sampled batch size the library enlarges it (in whole pages) until a layer
                                has about one attention task per queue. */
    int32_t moe_tile_m;      /* tokens per GroupGEMM row tile (exp_indptr unit, Sec. 2.4); 1..16 */
} etc_tile_desc;

typedef enum {
    ETC_SCHED_STATIC = 0,  /* per-CU task queues built on the host, notify / wait (Sec. 3.1, Alg. 1) */
    ETC_SCHED_DYNAMIC = 1, /* on-GPU ready queue, push / pop when idle (Sec. 3.2, Alg. 2); a task is pushed once the
                              producers of all its events are dispatched and keeps its waits (early push, App. E);
                              MoE models: expert events armed at run time release each expert's GroupGEMM row
                              tiles, surplus row-tile slots never run (Sec. 2.4) */
    ETC_SCHED_UNFUSED = 2  /* static queues, one coarse event per operator stage (Sec. 4.5 baseline) */
} etc_sched_kind;

enum {
    ETC_DEBUG_EXEC_COUNT = 1u,   /* count executions of every task */
    ETC_DEBUG_LAYER_HIDDEN = 2u, /* keep the hidden state after every layer */
    ETC_DEBUG_ROUTING = 4u,      /* keep router logits, top-k ids / weights, permutation, indptr */
    ETC_DEBUG_TRACE = 8u         /* per-task device timestamps (see ETC_DBG_TASK_TRACE) */
};

typedef struct {
    int32_t kind;             /* etc_sched_kind */
    int32_t n_sampled;        /* static: number of sampled batch sizes (Sec. 3.1), 1..8 */
    int32_t sampled_batch[8]; /* ascending; a bound batch uses the next larger sampled queue */
    int32_t max_batch;        /* <= 64 (stand-alone MoE layer: tokens, <= 4096) */
    int32_t max_kv_len;       /* largest kv_len + 1 any step will bind */
    int64_t spin_budget;      /* polls before a wait gives up (0 = default) */
    uint32_t debug_flags;
    int32_t n_queues;         /* persistent workgroups; 0 = one per compute unit */
} etc_sched_desc;

/* Builds the event-tensor graph of the decoder, the task queues for every sampled batch size
 * and all scratch.  This is the "warm-up" of Sec. 4.4: nothing is compiled or captured later. */
etc_status etc_create(const etc_model_desc *model, const etc_tile_desc *tiles, const etc_sched_desc *sched,
                      etc_ctx **out);
void etc_destroy(etc_ctx *ctx);
const char *etc_last_error(const etc_ctx *ctx); /* ctx may be NULL: error of the last failed create */

/* ---- bind ----------------------------------------------------------------------------- */

/* One layer's weights, device, bf16, row-major [out, in].  Dense layers leave the MoE
 * pointers NULL and vice versa. */
typedef struct {
    const void *g1;  /* [hidden]                 attention RMSNorm gain */
    const void *wq;  /* [n_q_heads*head_dim, hidden] */
    const void *wk;  /* [n_kv_heads*head_dim, hidden] */
    const void *wv;  /* [n_kv_heads*head_dim, hidden] */
    const void *wo;  /* [hidden, n_q_heads*head_dim] */
    const void *g2;  /* [hidden]                 FFN RMSNorm gain */
    const void *wg;  /* [ffn, hidden]            gate */
    const void *wu;  /* [ffn, hidden]            up */
    const void *wd;  /* [hidden, ffn]            down */
    const void *wr;  /* [n_experts, hidden]      router */
    const void *eg;  /* [n_experts, moe_ffn, hidden] */
    const void *eu;  /* [n_experts, moe_ffn, hidden] */
    const void *ed;  /* [n_experts, hidden, moe_ffn] */
    const void *gq;  /* [head_dim]               per-head query norm gain (qk_norm models, else NULL) */
    const void *gk;  /* [head_dim]               per-head key norm gain */
} etc_layer_weights;

/* Resident tensors of the decoder of Sec. 4.3 (attention, RoPE, norms, MLP or MoE block): recorded, not copied;
 * every weight byte is read once per step.  All pointers 16-byte aligned.  May be called again between steps. */
etc_status etc_bind_layer_weights(etc_ctx *ctx, int32_t layer, const etc_layer_weights *w);

/* Paged KV cache, device, bf16: [layer][page][page_size][n_kv_heads][head_dim] for K and for V.
 * K rows are stored already rotated.  The step appends one row per sequence (Sec. 4.3). */
etc_status etc_bind_kv_pool(etc_ctx *ctx, void *k_pages, void *v_pages, int64_t pages_per_layer);

/* Model-level tensors of a model with a vocabulary (etc_model_desc.vocab > 0), device memory, bf16, 16-byte
 * aligned, owned by the caller and kept alive while the context lives: embed [vocab, hidden] (the embedding
 * table; NULL when every step starts from hidden states), g_final [hidden] (gain of the final RMSNorm), w_lm
 * [vocab, hidden] (the vocabulary projection; may be the same memory as embed).  They close a decode
 * iteration as Sec. 4.2 measures it end to end (all transformer layers, then sampling).  ETC_ESTATE for a
 * model without a vocabulary. */
etc_status etc_bind_lm_head(etc_ctx *ctx, const void *embed, const void *g_final, const void *w_lm);

/* Dynamic shape parameters of the next step(s) (Sec. 2.3).  kv_len[b] = tokens already cached:
 * the new token has position kv_len[b], is appended there and attends to kv_len[b]+1 keys.
 * Sequence b owns page_ids[page_indptr[b] .. page_indptr[b+1]) = ceil((kv_len[b]+1)/page_size)
 * pages.  All three arrays are host memory, copied during the call (into pinned staging; they reach
 * the device by one asynchronous copy on the stream of the next launch).  Never needs a re-create
 * for batch <= max_batch and kv_len < max_kv_len (Sec. 2.3: one template, any shape), does not
 * synchronise with the device and launches nothing: it is cheap enough to run before every decode
 * step.  When the bound batch moves to another sampled batch size (Sec. 3.1), the next launch is
 * preceded by one small kernel that arms the event tensors with that plan's counts. */
etc_status etc_bind_step(etc_ctx *ctx, int32_t batch, const int32_t *kv_len, const int32_t *page_indptr,
                         const int32_t *page_ids);

/* Test hook for MoE parity (Sec. 2.4: topk is a run-time tensor): layer's routing follows ids
 * [batch, top_k] (host) instead of the device top-k; with w != NULL the routing weights are w
 * [batch, top_k] (host) instead of the softmax over the selected logits.  ids == NULL removes the
 * override (w is then ignored).  Synchronises; takes effect at the next launch. */
etc_status etc_force_routing(etc_ctx *ctx, int32_t layer, const int32_t *ids, const float *w);

/* ---- the MoE layer on its own (Sec. 2.4; measured over 1 .. 4096 tokens in Sec. 4.2 and Sec. 4.5) ------------
 * y = x + MoE(rmsnorm(x, g2)) for a block of tokens: router -> top-k -> token grouping -> GroupGEMM-1 -> SiLU-mul ->
 * GroupGEMM-2 -> weighted combine, the same event-gated tasks as the MoE block of a decoder layer, with the
 * data-dependent events of Sec. 2.4 under the dynamic scheduler; routing and grouping run as counting passes over
 * blocks of 64 tokens, so the work stays linear in the tokens.
 * Of `model` only hidden, n_experts, top_k, moe_ffn and rms_eps are read; tiles->moe_tile_m (1..64) is the row tile of
 * the GroupGEMMs; sched->max_batch is the largest token count (<= 4096), sched->sampled_batch the sampled token
 * counts (Sec. 3.1; a bound count runs the next larger one), max_kv_len is ignored.  The context takes
 * etc_bind_layer_weights(ctx, 0, w) with g2, wr, eg, eu, ed (the other pointers are ignored),
 * etc_moe_layer_bind_tokens, etc_force_routing (layer 0), etc_launch / etc_launch_kernel_by_kernel (hidden_in = x,
 * hidden_out = y, device, bf16 [n_tokens, hidden]), etc_read_debug (routing kinds, layer 0) and etc_get_step_info;
 * etc_bind_kv_pool and etc_bind_step are refused. */
etc_status etc_moe_layer_create(const etc_model_desc *model, const etc_tile_desc *tiles, const etc_sched_desc *sched,
                                etc_ctx **out);

/* Number of tokens of the next launches (a dynamic shape in the sense of Sec. 2.3: no re-create up to max_batch).
 * Host-only; after a move to another sampled token count the next launch is preceded by the arming kernel. */
etc_status etc_moe_layer_bind_tokens(etc_ctx *ctx, int32_t n_tokens);

/* ---- launch --------------------------------------------------------------------------- */

/* One decode step = one launch of the fused persistent kernel on hip_stream (a hipStream_t, may be NULL),
 * asynchronous: the scheduling transformations of Sec. 3.1 (static queues, notify / wait) or Sec. 3.2 (ready
 * queue, push / pop) applied to the whole decoder graph.  After a bind the launch is preceded on the same
 * stream by the copy of the step's shape arrays (and, after a change of plan, the arming kernel).
 * hidden_in / hidden_out: device, bf16 [batch, hidden]; may alias.  May be called repeatedly
 * for one bind: the event tensors are re-armed inside the kernel (Sec. 3.3 leaves the reset open). */
etc_status etc_launch(etc_ctx *ctx, const void *hidden_in, void *hidden_out, void *hip_stream);

/* The same task bodies, one ordinary kernel launch per operator stage (the kernel-by-kernel
 * model of Sec. 1); the launch-gap comparator.  Same arguments and results as etc_launch. */
etc_status etc_launch_kernel_by_kernel(etc_ctx *ctx, const void *hidden_in, void *hidden_out, void *hip_stream);

/* One whole decode iteration of a model with a vocabulary in one launch of the persistent kernel (Sec. 4.2: the
 * low-batch serving loop, layers then sampling): embedding look-up, all layers, final RMSNorm, vocabulary
 * projection and the greedy token of every sequence (largest logit; equal logits: the lower id), all as tasks
 * of the same event-gated graph.  Exactly one of token_in (device, int32 [batch], ids in [0, vocab), needs the
 * embedding table) and hidden_in (device, bf16 [batch, hidden]) is non-NULL.  token_out: device, int32
 * [batch].  logits_out: device, fp32 [batch, vocab], or NULL (the logits then stay in the context's own
 * buffer).  hidden_out: device, bf16 [batch, hidden] (the last layer's output before the final norm), or
 * NULL.  Asynchronous on hip_stream like etc_launch.  Iterations chain without a host round trip: bind the
 * next step's shapes (etc_bind_step does not synchronise) and launch with token_in = the previous token_out.
 * A token id outside the table raises ETC_ERR_BAD_TABLE in the error word (the context is then dead, as after
 * any device error).  ETC_ESTATE for a model without a vocabulary or before etc_bind_lm_head; on a model WITH
 * a vocabulary etc_launch / etc_launch_kernel_by_kernel are refused with ETC_ESTATE (their graph ends in
 * sampling tasks that need these buffers). */
etc_status etc_launch_tokens(etc_ctx *ctx, const int32_t *token_in, const void *hidden_in, int32_t *token_out,
                             float *logits_out, void *hidden_out, void *hip_stream);

/* The kernel-by-kernel comparator of etc_launch_tokens: same arguments and results, one launch per stage. */
etc_status etc_launch_tokens_kernel_by_kernel(etc_ctx *ctx, const int32_t *token_in, const void *hidden_in,
                                              int32_t *token_out, float *logits_out, void *hidden_out,
                                              void *hip_stream);

/* ---- evidence / debug readback (synchronises the device) -------------------------------- */
typedef enum {
    ETC_DBG_ERROR_WORD = 0,      /* int32[4]: code (0 = none), task function, event index, queue */
    ETC_DBG_EVENT_COUNTERS = 1,  /* int32[n_events] of the step that just ran: all zero when drained */
    ETC_DBG_TASK_EXEC_COUNT = 2, /* int32[n_tasks]: 1 everywhere (needs ETC_DEBUG_EXEC_COUNT) */
    ETC_DBG_LAYER_HIDDEN = 3,    /* float[batch, hidden] after `layer` (needs ETC_DEBUG_LAYER_HIDDEN) */
    ETC_DBG_ROUTER_LOGITS = 4,   /* float[batch, n_experts] of `layer`   (needs ETC_DEBUG_ROUTING) */
    ETC_DBG_TOPK_IDS = 5,        /* int32[batch, top_k] */
    ETC_DBG_TOPK_W = 6,          /* float[batch, top_k] */
    ETC_DBG_PERMUTATION = 7,     /* int32[batch*top_k]: token*top_k+slot sorted by (expert, token, slot) */
    ETC_DBG_TOK_INDPTR = 8,      /* int32[n_experts+1] prefix sum of tokens per expert */
    ETC_DBG_EXP_INDPTR = 9,      /* int32[n_experts+1] prefix sum of row tiles per expert (Sec. 2.4) */
    ETC_DBG_TASK_TRACE = 10      /* uint64[n_tasks][8] device wall-clock ticks of the last launch: 0 task fetched,
                                    1 events seen, 2 operand staged, 3 streaming done, 4 epilogue done, 5 notified,
                                    6 unused, 7 queue (workgroup) that ran the task (needs ETC_DEBUG_TRACE) */
} etc_debug_kind;

/* Evidence for the invariants of Sec. 3.3 (every counter drained, every task run once), the per-layer
 * parity checks and the run-time tensors of Sec. 2.4.  host_dst: host memory, bytes <= the item's size.
 * Synchronises the device.  Returns ETC_ETIMEOUT if the device recorded an error (the error word itself
 * can always be read). */
etc_status etc_read_debug(etc_ctx *ctx, int32_t kind, int32_t layer, void *host_dst, size_t bytes);

/* Sizes of the bound step's instantiated graph (Sec. 2.3: the template bound to concrete shapes) and the
 * bytes the roofline of the step is priced with.  No device call. */
typedef struct {
    int64_t n_tasks, n_events, n_queues;
    int64_t algorithmic_bytes; /* weights touched once + live KV once + appended rows, this step */
    int32_t sampled_batch;     /* the sampled batch size whose queues serve the bound batch */
    int32_t workgroup_threads;
    int32_t wall_clock_khz;    /* tick rate of the ETC_DBG_TASK_TRACE timestamps */
    int32_t reserved;
} etc_step_info;
etc_status etc_get_step_info(etc_ctx *ctx, etc_step_info *info);

/* ---- generic event-tensor graphs (Sec. 2.1, 2.2) ----------------------------------------
 * A graph function is a list of device-function launches over task grids plus event tensors;
 * edges map a task coordinate to an event coordinate.  Dimensions may be symbolic and are
 * bound at run time without rebuilding anything (Sec. 2.3).  Used by the row-sum example. */
typedef struct {
    int32_t sym; /* symbol id 0..3, or -1 for a constant */
    int32_t mul; /* value = mul * symbol + add */
    int32_t add;
} etc_dim_expr;

typedef enum {
    ETC_MAP_DIM = 0,      /* event coord = task coord[src] / div */
    ETC_MAP_CONST = 1,    /* event coord = div (a constant; "E[0]" style coarse event) */
    /* Data-dependent edges (Sec. 2.4) on a rank-1 event tensor, through int32 device tensors bound like buffers
     * and read at run time.  At most one such out-edge and one such in-edge per graph.
     * INDIRECT, out-edges only: task (i, ...) notifies event table[i] (slot 3, one entry per value of the first
     *   task coordinate).  How many notifies event e receives is not known before the launch: count[e] (slot 5)
     *   comes with the table, and the event fires on notify number count[e] ("initialised at run time").
     * INDPTR, in-edges of a rank-1 grid only: task j belongs to the event e with indptr[e] <= j < indptr[e+1]
     *   (slot 4, events + 1 entries, non-decreasing from 0); tasks from indptr[events] on belong to none and do
     *   nothing.  Event e releases exactly that range.
     * Dynamic scheduler: as written: a fired event pushes its range to the ready queue, tasks beyond the last
     * range never run.  Static and unfused schedulers: both edges collapse to event 0 of the tensor, fed by every
     * producer (the static rule of Sec. 3.1).  A table entry outside its range ends the launch with ETC_ETIMEOUT
     * (the error text names it); nothing is written through it. */
    ETC_MAP_INDIRECT = 2,
    ETC_MAP_INDPTR = 3
} etc_map_kind;

typedef struct {
    int32_t event;      /* id from etc_graph_add_event */
    int32_t rank;       /* rank of that event tensor, <= 3 */
    int32_t kind[3];    /* etc_map_kind per event dimension */
    int32_t src[3];
    int32_t div[3];
} etc_edge;

typedef enum {
    ETC_FN_ROWSUM_PARTIAL = 1, /* task (i, j): B[32i..32i+32, j] = sum_k A[rows, 32j..32j+32) */
    ETC_FN_ROWSUM_FINAL = 2,   /* task (i):    C[32i..32i+32]    = sum_j B[rows, j], j < 4 */
    ETC_FN_ROWSUM_FINAL_PERM = 3, /* task (t): the same for row block perm[t] (slot 6), t < indptr[events]; for grids
                                    released through ETC_MAP_INDPTR (row blocks grouped by their event) */
    ETC_FN_USER0 = 100         /* ETC_FN_USER0 + k: device function k of a GENERATED library (see below); the stock
                                    library has none and refuses these ids */
} etc_device_fn;

/* Generated dispatch (Alg. 1 and Alg. 2 read as compiler passes; Sec. 3).  The front end
 * (paper_2604_13327_amd/frontend.py) takes a graph description: shape symbols, event tensors, and calls of device
 * functions the user writes as HIP source `(const Args &a, int c0, int c1, int c2)`, one call per task of the grid.
 * It GENERATES a header with those functions and the switch that dispatches a task record to them, and builds a
 * library from this library's sources around that header (only the generic kernel instance: no decoder).  The result
 * exports this same C ABI; its etc_graph_add_call accepts ETC_FN_USER0 + k for the k-th function of the description.
 * Task lists (static queues, Alg. 1) and consumer tables (dynamic, Alg. 2) come from etc_graph_bind_shape as for the
 * built-in functions; symbols are bound at run time without rebuilding.  Device functions get the bound buffers
 * (slots 0..7 of etc_graph_bind_buffer) and symbol values; whether the buffers are large enough for a bound shape is
 * checked by the front end, which knows what the functions touch: the library cannot.
 * etc_graph_user_fn_count: how many generated device functions this library carries (0: the stock library). */
etc_status etc_graph_user_fn_count(int32_t *count);

etc_status etc_graph_create(const etc_sched_desc *sched, etc_ctx **out);
etc_status etc_graph_add_event(etc_ctx *ctx, const etc_dim_expr *shape, int32_t rank, int32_t *event_id);
etc_status etc_graph_add_call(etc_ctx *ctx, int32_t device_fn, const etc_dim_expr *task_shape, int32_t rank,
                              const etc_edge *in_edges, int32_t n_in, const etc_edge *out_edges, int32_t n_out);
/* Buffers of the device functions: slot 0 = A (fp32 [n*32, 128]), 1 = B (fp32 [n*32, 4]), 2 = C (fp32 [n*32]);
 * run-time tables (int32): 3 = table of an INDIRECT edge, 4 = indptr, 5 = count, 6 = perm.  Generated device functions
 * may use slots 0..7 as they like (3..5 keep their meaning when the graph has data-dependent edges).
 * bytes = size of the allocation, checked against the bound shape at launch. */
etc_status etc_graph_bind_buffer(etc_ctx *ctx, int32_t slot, void *device_ptr, size_t bytes);
/* Instantiates the template for concrete symbol values (values[4], host). */
etc_status etc_graph_bind_shape(etc_ctx *ctx, const int32_t *values);
etc_status etc_graph_launch(etc_ctx *ctx, void *hip_stream);

/* ---- allocation-free launch ------------------------------------------------------------------
 * For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Runs the row-sum graph (the one etc_graph_* builds from
 * ETC_FN_ROWSUM_PARTIAL over a (n, 4) grid notifying E[i] and ETC_FN_ROWSUM_FINAL over (n) waiting on E[i])
 * for n row blocks under the static scheduler, as one small plan kernel plus one launch of the same
 * megakernel etc_graph_launch uses.  The partial sums B, the event tensor, the task queues and the error
 * word sit in a device array that is part of the library image (about 1.4 MB, held by every GPU the
 * library runs on until the process ends); no context, no hipMalloc / hipFree, no memset, nothing to destroy.
 *   A  device, fp32 [n*32, 128], read only      C  device, fp32 [n*32], written      n  1..ETC_ROWSUM_NOALLOC_MAX_N
 *   hip_stream  a hipStream_t (may be NULL); the call is asynchronous on it.
 * Same results, bit for bit, as etc_graph_launch on that graph.  Returns ETC_EINVAL for a NULL pointer or n
 * outside the range (nothing is launched), ETC_EDEVICE when a HIP call fails.  All calls on one GPU share
 * the one array: every call rewrites all of it that it reads, so calls may follow each other on one stream
 * in any sizes, but calls that overlap on one GPU (different streams, different threads) race.  A wait that
 * exceeds its spin budget drains the kernel as everywhere else (C is then incomplete); the error word stays
 * in the array and is not reported by this call. */
#define ETC_ROWSUM_NOALLOC_MAX_N 2048
etc_status etc_rowsum_launch_noalloc(const float *A, float *C, int32_t n, void *hip_stream);

/* ---- host-only inspection of the scheduling transformation (no device needed) ---------------
 * Instantiates the decoder's event-tensor graph for one sampled batch size exactly as etc_create
 * does and exposes the materialised tasks, static queues (Sec. 3.1), initial event counts (Sec. 2.1)
 * and the event -> consumer table of the dynamic scheduler (Sec. 3.2).  Arrays are owned by the
 * view and released by etc_plan_free. */
typedef struct {
    uint8_t fn, layer;
    uint16_t flags;       /* bit 0: wave w of the task waits on event wait0 + w (8 waves) */
    int32_t c0, c1, c2;   /* task coordinate */
    int32_t wait0, wait1; /* flat event indices, -1 = none */
    int32_t notify0;
    int32_t id;
} etc_task_record;

typedef struct {
    int64_t n_tasks, n_events, n_queues, n_seed;
    const etc_task_record *tasks;       /* by task id */
    const etc_task_record *queue_tasks; /* static queues back to back */
    const int32_t *queue_begin;         /* [n_queues + 1] */
    const int32_t *ev_init;             /* [n_events] */
    const int32_t *ev_consumers;        /* [n_events + 1] CSR into consumer_ids: the tasks that wait on the event */
    const int32_t *consumer_ids;        /* bits 0..23 task id; bits 24..30: n when the task waits on n > 1 events
                                           (it is then listed under each of them), else 0 */
    const int32_t *seed_tasks;          /* [n_seed] tasks that wait on nothing: ready at launch */
    void *opaque;
} etc_plan_view;

etc_status etc_plan_build(const etc_model_desc *model, const etc_tile_desc *tiles, const etc_sched_desc *sched,
                          int32_t sampled_batch, int32_t n_queues, etc_plan_view *out);
/* The same for the stand-alone MoE layer graph of `sampled_tokens` tokens (etc_moe_layer_create). */
etc_status etc_moe_layer_plan_build(const etc_model_desc *model, const etc_tile_desc *tiles, const etc_sched_desc *sched,
                                    int32_t sampled_tokens, int32_t n_queues, etc_plan_view *out);
void etc_plan_free(etc_plan_view *view);

#ifdef __cplusplus
}
#endif
#endif /* ETC_H */
