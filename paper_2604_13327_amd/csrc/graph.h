// Host-side event-tensor graph IR and its instantiation into task queues.
//
// A graph function (paper Sec. 2.1) is a list of device-function launches over task
// grids plus event tensors; edges map a task coordinate to an event coordinate.  Shapes
// may contain symbols; instantiate() binds them (Sec. 2.3) and materialises
//   - the tasks with their flat wait / notify event indices,
//   - the initial wait count of every event = number of tasks that notify it (Sec. 2.1),
//   - static per-queue task lists, round-robin (Sec. 3.1, Alg. 1), or
//   - the event -> consumer-task table used by push-on-zero (Sec. 3.2, Alg. 2).
// Pure C++, no device code: it is also exercised by CPU-only tests.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "etc_types.h"

namespace etc {

struct DimExpr {
    int sym = -1, mul = 0, add = 0;   // value = mul * symbol + add
    int eval(const int *vals) const { return sym < 0 ? add : mul * vals[sym] + add; }
};
inline DimExpr dim_const(int c) { return DimExpr{-1, 0, c}; }
inline DimExpr dim_sym(int s, int mul = 1, int add = 0) { return DimExpr{s, mul, add}; }

// MAP_INDIRECT (out-edges): event coord = table[task coord 0]; MAP_INDPTR (in-edges): the event whose range
// [indptr[e], indptr[e+1]) holds task coord 0.  Both name run-time tensors (Sec. 2.4).
enum MapKind { MAP_DIM = 0, MAP_CONST = 1, MAP_INDIRECT = 2, MAP_INDPTR = 3 };

struct EdgeMap {
    int event = -1;                    // event tensor id
    int rank = 0;
    int kind[3] = {0, 0, 0};
    int src[3] = {0, 0, 0};
    int div[3] = {1, 1, 1};
};

struct EventDecl {
    DimExpr shape[3];
    int rank = 1;
};

struct CallDecl {
    int fn = FN_NOP;
    int layer = 0;
    int stage = 0;                     // operator stage (calls of one stage may run concurrently)
    DimExpr shape[3];
    int rank = 1;
    int c_mul[3] = {1, 1, 1};          // Task record coordinate = grid coordinate * c_mul + c_off ...
    int c_off[3] = {0, 0, 0};
    int c_fill[3] = {0, 0, 0};         // ... and c_fill for the coordinates beyond the grid's rank
    bool last_dim_slowest = false;     // enumeration order (balances ragged grids across queues)
    uint16_t flags = 0;
    std::vector<EdgeMap> in, out;      // at most 2 in-edges, 1 out-edge
};

struct GraphDecl {
    std::vector<EventDecl> events;
    std::vector<CallDecl> calls;
    int k_slices_o = 0, k_slices_d = 0;   // decoder graphs: slices of K of the O / down projection tasks (0: whole K)
    bool all_staged = false;              // dense decoder graphs: every projection task fits the staged path
    int add_event(std::initializer_list<DimExpr> shape);
};

struct Plan {
    std::vector<Task> tasks;           // by task id, call by call
    std::vector<int32_t> call_begin;   // [n_calls + 1] task-id ranges of the calls
    std::vector<int32_t> stage_of_call;
    std::vector<int32_t> ev_init;      // initial wait counts
    std::vector<int32_t> ev_offset;    // [n_event_tensors + 1] flat offsets
    std::vector<Task> queue_tasks;     // static queues back to back
    std::vector<int32_t> queue_begin;  // [n_queues + 1]
    std::vector<int32_t> ev_consumers; // [n_events + 1] CSR over consumer_ids
    std::vector<int32_t> consumer_ids;
    std::vector<int32_t> seed_tasks;   // tasks with no in-edge
    // data-dependent edges (dynamic scheduling only; otherwise they collapse to the tensor's event 0)
    int dd_event_base = 0, dd_n_events = 0, dd_consumer_first = 0, dd_consumer_n = 0;
    int dd_table_len = 0;              // extent of the first grid dimension of the indirectly notifying call
};

// Binds the symbols and materialises the plan.  unfused: ignore the declared edges and put one
// coarse event between consecutive stages (Sec. 4.5 baseline).  Returns "" or an error text.
// data_dependent: keep MAP_INDIRECT / MAP_INDPTR edges as run-time edges (dynamic scheduler); otherwise they are
// rewritten to the coarse event 0 of their tensor, fed by all producers (the static rule of Sec. 3.1).
std::string instantiate(const GraphDecl &g, const int *sym_values, int n_queues, bool unfused, Plan *out,
                        bool data_dependent = false);

struct ModelDims {
    int n_layers, H, nq, nkv, d, F, E, topk, moeF, page;
    int kv_chunk, tile_m;
    int vocab = 0;      // > 0: the step ends in final norm + vocabulary projection + greedy token
};

// Upper bound of sum_e ceil(count_e / tile_m) over all routings of `batch` tokens: the number of
// GroupGEMM row-tile slots a static queue holds (slots beyond exp_indptr[E] are no-ops at run time).
inline int moe_max_row_tiles(int n_experts, int top_k, int batch, int tile_m)
{
    const int n = batch * top_k, nonempty = n < n_experts ? n : n_experts;
    return (n + nonempty * (tile_m - 1)) / tile_m;
}

// Keys per split-KV attention task for one sampled batch size.  `min_chunk` is the caller's tile shape; it
// is enlarged (in whole pages) until a layer has at most one attention task per queue: every chunk costs a
// partial result the merge reads back, and a second task per queue only adds such chunks (half a task per
// queue leaves queues idle and measured slower from batch 4 on).
inline int effective_kv_chunk(int min_chunk, int page, int max_kv_len, int batch, int n_kv_heads, int n_queues)
{
    const int pairs = batch * n_kv_heads, target = n_queues;
    int chunks = target / pairs;      // at most one task per queue: a queue with a second task ends the stage a task late
                                      // (rounding up instead measured 3 - 6 % slower per step at batch 3 .. 24)
    const int most = (max_kv_len + min_chunk - 1) / min_chunk;
    if (chunks > most) chunks = most;
    if (chunks < 1) chunks = 1;
    int chunk = (max_kv_len + chunks - 1) / chunks;
    chunk = (chunk + page - 1) / page * page;
    return chunk < min_chunk ? min_chunk : chunk;
}

// Row tiles a large-batch projection task streams against one pass over its operand: 8.  (Above 32 columns the
// K-split chunked path holds accumulators for 4 tiles at most; such tasks take the wide path, one tile per wavefront.)
inline int pass_tiles_for(int batch) { (void)batch; return 8; }
// Above 16 columns the wide path takes two row tiles per wavefront: 16 tiles against one pass over the operand.  A
// projection uses that where it still leaves every queue a task: gate/up by its cost per queue (fewer rounds, each
// with one more operand pass), a projection cut along K when (row tiles / 16) x slices fill the queues.
inline int wide_pass_tiles_for(int batch) { return batch > 16 ? 16 : 8; }
inline int sliced_pass_tiles(int batch, int row_tiles, int slices, int n_queues)
{
    return (batch > 16 && slices > 0 && row_tiles % 16 == 0 && (row_tiles / 16) * slices >= n_queues) ? 16 : 8;
}

// Slices of K for a projection of a large batch: the most of 8, 4, 2 that keep a slice a multiple of the
// 256 elements one pass of the 8 wavefronts covers; 0 when K is too short to slice.
inline int k_slices_for(int K)
{
    for (int s = 8; s >= 2; s /= 2)
        if (K % (s * 256) == 0) return s;
    return 0;
}

// The decoder's graph function for one sampled batch size.  Symbol 0 = that batch size, symbol 1 =
// chunk slots per sequence.  n_queues and the batch decide how many consecutive row tiles one
// projection task streams (tile shapes are a degree of freedom of the graph, Sec. 2.1).
// moe_static_coarse: static scheduling of the data-dependent MoE stages through one coarse event
// ("E[0]" rewrite of Sec. 3.1).
std::string build_decoder_graph(const ModelDims &m, int sampled_batch, int n_queues, bool moe_static_coarse,
                                GraphDecl *out);

// The MoE layer on its own over a block of tokens (Sec. 2.4; token sweep of Sec. 4.2 / 4.5).  Only H, E, topk, moeF and
// tile_m of the dimensions are read.  The graph is built for `sampled_tokens` tokens (its grids are constants).
constexpr int kMoeLayerMaxTokens = 4096;
std::string build_moe_layer_graph(const ModelDims &m, int sampled_tokens, int n_queues, GraphDecl *out);

}  // namespace etc
