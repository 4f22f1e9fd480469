// C ABI of the library (see include/etc.h): argument checking, scratch and plan management,
// kernel launches.  Everything numerical happens in the device task bodies.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/etc.h"
#include "etc_types.h"
#include "graph.h"
#include "arm_args.h"

namespace etc {
hipError_t configure_kernels();
hipError_t max_resident_workgroups(int *per_cu);
hipError_t launch_static(const Params &P, hipStream_t s);
hipError_t launch_dynamic(const Params &P, hipStream_t s);
hipError_t launch_stage(const Params &P, int first, int count, hipStream_t s);
hipError_t launch_rowsum_noalloc(const float *A, float *C, int n, hipStream_t s);
int user_fn_count();
hipError_t launch_arm(const ArmArgs &a, hipStream_t s);
}  // namespace etc

using namespace etc;

namespace {

std::string g_create_error;

// Switch for the dynamic-scheduler kernel (off: launching it is refused; the static and unfused schedulers
// are unaffected).
constexpr bool kDynamicEnabled = true;
const char *kDynamicOffMsg = "the dynamic scheduler is switched off in this build";

struct DevPlan {          // one instantiated plan (one sampled batch size), host + device copies
    int sampled_batch = 0;
    int kv_chunk = 0;     // keys per attention task of this plan
    int k_slices_o = 0, k_slices_d = 0;   // slices of K of this plan's O / down projection tasks
    bool all_staged = false;              // every projection task of this plan fits the staged path
    Plan host;
    Task *d_queue_tasks = nullptr, *d_tasks = nullptr;
    int32_t *d_queue_begin = nullptr, *d_ev_init = nullptr, *d_ev_consumers = nullptr, *d_consumer_ids = nullptr,
            *d_seed = nullptr;
    // MoE plans: per layer the flat ids of the event of row-tile slot 0 and of the combine event; static grid sizes
    std::vector<int32_t> moe_layer_events;
    int32_t *d_moe_layer_events = nullptr;
    int moe_rmax = 0, moe_groups_gu = 0, moe_groups_down = 0;
};

template <class T>
hipError_t dev_alloc(T **p, size_t n, std::vector<void *> &owned, bool zero = true)
{
    *p = nullptr;
    if (n == 0) n = 1;
    hipError_t e = hipMalloc((void **)p, n * sizeof(T));
    if (e != hipSuccess) return e;
    owned.push_back(*p);
    if (zero) e = hipMemset(*p, 0, n * sizeof(T));
    return e;
}

template <class T>
hipError_t dev_upload(T **p, const std::vector<T> &v, std::vector<void *> &owned)
{
    hipError_t e = dev_alloc(p, v.size(), owned, false);
    if (e != hipSuccess || v.empty()) return e;
    return hipMemcpy(*p, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice);
}

}  // namespace

struct etc_ctx {
    bool is_graph = false;
    bool is_moe_layer = false;              // the MoE layer on its own over a block of tokens (etc_moe_layer_create)
    etc_model_desc model{};
    etc_tile_desc tiles{};
    etc_sched_desc sched{};
    ModelDims dims{};
    int n_queues = 0, max_chunks = 0, max_pages_per_seq = 0;
    GraphDecl graph;
    std::vector<DevPlan> plans;
    int cur_plan = -1;
    std::vector<void *> owned;              // device allocations that live as long as the context
    std::vector<void *> plan_owned;         // plans, event tensors, ready queue (rebuilt by etc_graph_bind_shape)
    size_t gbuf_bytes[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    std::vector<LayerWeights> h_weights;
    std::vector<uint8_t> weights_bound;
    LayerWeights *d_weights = nullptr;
    bool weights_dirty = true;
    Params base{};                          // device pointers and constants filled at create
    int32_t *d_events = nullptr;            // [2][n_events_max]: A | B (a launch drains one and re-arms the other)
    int32_t *d_disp = nullptr;              // [2][n_events_max]: dispatch counters of the dynamic scheduler, A | B
    int32_t *d_pending = nullptr;           // [n_tasks_max]: dynamic scheduler, waited events passed per task
    size_t n_tasks_max = 0;
    int n_events_max = 0;
    int parity = 0;
    uint32_t epoch = 1;
    int32_t *d_qctrl = nullptr;             // [2][8]
    int32_t *d_kv_len = nullptr, *d_page_indptr = nullptr, *d_page_ids = nullptr;   // parts of d_step
    // Step shapes travel host -> pinned staging slot (during etc_bind_step) -> device block (one asynchronous copy on
    // the stream of the next launch): binding a step neither synchronises nor touches the device.
    static constexpr int kStageSlots = 4;
    int32_t *d_step = nullptr;              // kv_len [max_batch] | page_indptr [max_batch + 1] | page_ids [max_batch * pages]
    int32_t *h_stage[kStageSlots] = {nullptr, nullptr, nullptr, nullptr};   // pinned, same layout
    hipEvent_t stage_ev[kStageSlots] = {nullptr, nullptr, nullptr, nullptr}; // recorded behind the slot's upload
    bool stage_pending[kStageSlots] = {false, false, false, false};
    int stage_slot = 0;
    size_t stage_words = 0, stage_used_words = 0;
    bool step_dirty = false;                // a bound step waits in its staging slot for the next launch
    bool need_arm = true;                   // the next launch first arms the event tensors from the plan's counts
    bool need_exec_reset = false;           // ... and clears the execution counts (debug)
    int32_t *h_error = nullptr;             // pinned, device-visible: the code of the first device error, 0 = none
    bool dead = false;                      // a device watchdog error was seen: launches are refused from then on
    int32_t *d_forced = nullptr;
    float *d_forced_w = nullptr;
    uint8_t *d_forced_mask = nullptr;
    std::vector<uint8_t> h_forced_mask;
    int64_t pages_per_layer = 0;
    bool kv_bound = false, step_bound = false, lm_bound = false;
    int bound_batch = 0;
    std::vector<int32_t> h_kv_len;
    int64_t algorithmic_bytes = 0;
    std::string err, err_first;
    int sym_values[4] = {0, 0, 0, 0};
};

namespace {

etc_status fail(etc_ctx *c, etc_status s, const std::string &msg)
{
    if (c) c->err = msg; else g_create_error = msg;
    return s;
}

#define HIP_TRY(ctx, expr)                                                                              \
    do {                                                                                                \
        hipError_t e_ = (expr);                                                                         \
        if (e_ != hipSuccess)                                                                           \
            return fail(ctx, e_ == hipErrorOutOfMemory ? ETC_ENOMEM : ETC_EDEVICE,                      \
                        std::string(#expr) + ": " + hipGetErrorString(e_));                             \
    } while (0)

etc_status upload_plan(etc_ctx *c, DevPlan &dp)
{
    HIP_TRY(c, dev_upload(&dp.d_queue_tasks, dp.host.queue_tasks, c->plan_owned));
    HIP_TRY(c, dev_upload(&dp.d_tasks, dp.host.tasks, c->plan_owned));
    HIP_TRY(c, dev_upload(&dp.d_queue_begin, dp.host.queue_begin, c->plan_owned));
    HIP_TRY(c, dev_upload(&dp.d_ev_init, dp.host.ev_init, c->plan_owned));
    HIP_TRY(c, dev_upload(&dp.d_ev_consumers, dp.host.ev_consumers, c->plan_owned));
    HIP_TRY(c, dev_upload(&dp.d_consumer_ids, dp.host.consumer_ids, c->plan_owned));
    HIP_TRY(c, dev_upload(&dp.d_seed, dp.host.seed_tasks, c->plan_owned));
    // what the data-dependent MoE events need to know of the static grids (dynamic scheduler, Sec. 2.4)
    int n_layers = 0;
    for (const Task &t : dp.host.tasks) n_layers = std::max(n_layers, (int)t.layer + 1);
    dp.moe_layer_events.assign((size_t)2 * n_layers, -1);
    dp.moe_rmax = dp.moe_groups_gu = dp.moe_groups_down = 0;
    for (const Task &t : dp.host.tasks) {
        if (t.fn == FN_MOE_DOWN && t.c0 == 0) {
            dp.moe_layer_events[2 * t.layer] = t.wait0;
            dp.moe_layer_events[2 * t.layer + 1] = t.notify0;
            if (t.layer == 0) dp.moe_groups_down++;
        }
        if (t.fn == FN_MOE_GATEUP && t.layer == 0) {
            dp.moe_rmax = std::max(dp.moe_rmax, (int)t.c0 + 1);
            if (t.c0 == 0) dp.moe_groups_gu++;
        }
    }
    if (dp.moe_rmax > 0) HIP_TRY(c, dev_upload(&dp.d_moe_layer_events, dp.moe_layer_events, c->plan_owned));
    return ETC_OK;
}

etc_status common_device_setup(etc_ctx *c, const etc_sched_desc *s)
{
    int dev = 0;
    HIP_TRY(c, hipGetDevice(&dev));
    hipDeviceProp_t prop;
    HIP_TRY(c, hipGetDeviceProperties(&prop, dev));
    HIP_TRY(c, configure_kernels());
    int per_cu = 0;
    HIP_TRY(c, max_resident_workgroups(&per_cu));
    if (per_cu < 1) return fail(c, ETC_EDEVICE, "the megakernel does not fit on a compute unit");
    // every persistent workgroup must be resident at once (spin waits): one per CU
    c->n_queues = s->n_queues > 0 ? std::min(s->n_queues, prop.multiProcessorCount) : prop.multiProcessorCount;
    c->sched = *s;
    if (c->sched.spin_budget <= 0) c->sched.spin_budget = 2000000;    // a few seconds of polling, then ETC_ETIMEOUT
    HIP_TRY(c, dev_alloc(&c->base.error_word, 4, c->owned));
    HIP_TRY(c, hipHostMalloc((void **)&c->h_error, 4 * sizeof(int32_t), hipHostMallocMapped));
    memset(c->h_error, 0, 4 * sizeof(int32_t));
    HIP_TRY(c, hipHostGetDevicePointer((void **)&c->base.error_host, c->h_error, 0));
    HIP_TRY(c, dev_alloc(&c->d_qctrl, 16, c->owned));
    return ETC_OK;
}

etc_status alloc_events_and_queue(etc_ctx *c)
{
    size_t n_ev = 1, n_tasks = 1;
    for (const DevPlan &dp : c->plans) {
        n_ev = std::max(n_ev, dp.host.ev_init.size());
        n_tasks = std::max(n_tasks, dp.host.tasks.size());
    }
    c->n_events_max = (int)n_ev;
    HIP_TRY(c, dev_alloc(&c->d_events, 2 * n_ev, c->plan_owned));
    HIP_TRY(c, dev_alloc(&c->d_disp, 2 * n_ev, c->plan_owned));
    HIP_TRY(c, dev_alloc(&c->d_pending, n_tasks, c->plan_owned));
    c->n_tasks_max = n_tasks;
    if (c->sched.debug_flags & ETC_DEBUG_EXEC_COUNT) HIP_TRY(c, dev_alloc(&c->base.exec_count, n_tasks + 65536, c->plan_owned));
    if (c->sched.debug_flags & ETC_DEBUG_TRACE) HIP_TRY(c, dev_alloc(&c->base.trace, n_tasks * 8, c->plan_owned));
    c->base.q_capacity = (int)(n_tasks + 65536 + c->n_queues);
    HIP_TRY(c, dev_alloc(&c->base.q_slots, (size_t)c->base.q_capacity, c->plan_owned));
    return ETC_OK;
}

// Arms the event tensors for the bound plan on the stream of the launch that follows: a small fill kernel, no
// memset or copy nodes, so the same sequence can sit in a captured graph.  Needed before the first launch of a
// context and whenever the bound plan changes (the kernel itself re-arms the other buffer for the next launch
// of the SAME plan, so a bind that keeps the plan costs the device nothing).
etc_status arm_on_stream(etc_ctx *c, hipStream_t s)
{
    if (!c->need_arm && !c->need_exec_reset) return ETC_OK;
    const DevPlan &dp = c->plans[c->cur_plan];
    const size_t N = (size_t)c->n_events_max;
    ArmArgs a{};
    if (c->need_arm) {
        a.ev_cur = c->d_events + (c->parity ? N : 0);
        a.ev_init = dp.d_ev_init;
        a.n_events = (int)dp.host.ev_init.size();
        a.disp_cur = c->d_disp + (c->parity ? N : 0);
        a.pending = c->d_pending;
        a.n_pending = (int)c->n_tasks_max;
        a.exp_event = c->base.exp_event;
        a.n_exp = c->base.exp_event ? c->base.E : 0;
        a.qctrl = c->d_qctrl + (c->parity ? 8 : 0);
    }
    if (c->base.exec_count) {
        a.exec_count = c->base.exec_count;
        a.n_exec = (int)dp.host.tasks.size();
    }
    HIP_TRY(c, launch_arm(a, s));
    c->need_arm = c->need_exec_reset = false;
    return ETC_OK;
}

void fill_launch_params(etc_ctx *c, Params &P)
{
    const DevPlan &dp = c->plans[c->cur_plan];
    const size_t N = (size_t)c->n_events_max;
    P = c->base;
    P.ev_cur = c->d_events + (c->parity ? N : 0);
    P.ev_init = dp.d_ev_init;
    P.ev_next = c->d_events + (c->parity ? 0 : N);
    P.n_events = (int)dp.host.ev_init.size();
    P.tasks = dp.d_queue_tasks;
    P.queue_begin = dp.d_queue_begin;
    P.n_queues = c->n_queues;
    P.dyn_tasks = dp.d_tasks;
    P.ev_consumers = dp.d_ev_consumers;
    P.consumer_ids = dp.d_consumer_ids;
    P.ev_disp_cur = c->d_disp + (c->parity ? N : 0);
    P.ev_disp_next = c->d_disp + (c->parity ? 0 : N);
    P.task_pending = c->d_pending;
    P.moe_dd = (c->sched.kind == ETC_SCHED_DYNAMIC && dp.moe_rmax > 0) ? 1 : 0;
    P.moe_layer_events = dp.d_moe_layer_events;
    P.moe_rmax = dp.moe_rmax;
    P.moe_groups_gu = dp.moe_groups_gu;
    P.moe_groups_down = dp.moe_groups_down;
    P.dd_event_base = dp.host.dd_event_base;
    P.dd_n_events = dp.host.dd_n_events;
    P.dd_consumer_first = dp.host.dd_consumer_first;
    P.dd_consumer_n = dp.host.dd_consumer_n;
    P.dd_table_len = dp.host.dd_table_len;
    P.seed_tasks = dp.d_seed;
    P.n_seed = (int)dp.host.seed_tasks.size();
    P.n_static_tasks = (int)dp.host.tasks.size();
    P.q_ctrl_cur = c->d_qctrl + (c->parity ? 8 : 0);
    P.q_ctrl_next = c->d_qctrl + (c->parity ? 0 : 8);
    P.epoch = c->epoch;
    P.spin_budget = c->sched.spin_budget;
    P.debug_flags = c->sched.debug_flags;
    P.B = c->bound_batch;
    P.Bs = dp.sampled_batch;
    P.max_chunks = c->max_chunks;
    if (dp.kv_chunk > 0) P.kv_chunk = dp.kv_chunk;
    P.k_slices_o = dp.k_slices_o;
    P.k_slices_d = dp.k_slices_d;
    P.all_staged = dp.all_staged ? 1 : 0;
    P.kv_len = c->d_kv_len;
    P.page_indptr = c->d_page_indptr;
    P.page_ids = c->d_page_ids;
    P.weights = c->d_weights;
    P.forced_topk = c->d_forced;
    P.forced_mask = c->d_forced_mask;
    P.forced_w = c->d_forced_w;
    for (int i = 0; i < 4; ++i) P.gsym[i] = c->sym_values[i];
}

etc_status check_error_word(etc_ctx *c)
{
    int32_t w[4];
    HIP_TRY(c, hipMemcpy(w, c->base.error_word, sizeof(w), hipMemcpyDeviceToHost));
    if (w[0] != 0) {
        char buf[200];
        snprintf(buf, sizeof(buf), "device watchdog: code %d in task function %d, event/ticket %d, queue %d", w[0],
                 w[1], w[2], w[3]);
        c->dead = true;
        return fail(c, ETC_ETIMEOUT, buf);
    }
    return ETC_OK;
}

// Non-blocking look at the error code the device mirrors into pinned host memory: what finished launches raised.
// The first call that sees an error reports it as ETC_ETIMEOUT; from then on the context refuses to launch
// (ETC_ESTATE): a kernel that drained on an error leaves counters, queue words and activations inconsistent.
etc_status refuse_if_dead(etc_ctx *c)
{
    if (c->dead) return fail(c, ETC_ESTATE, "the context is dead after a device watchdog error (" + c->err_first + "); destroy it");
    const int32_t code = *(volatile int32_t *)c->h_error;
    if (code != 0) {
        c->dead = true;
        c->err_first = "device watchdog: code " + std::to_string(code) + " (read ETC_DBG_ERROR_WORD for the task, event and queue)";
        return fail(c, ETC_ETIMEOUT, c->err_first);
    }
    return ETC_OK;
}

etc_status sync_weights(etc_ctx *c)
{
    if (!c->weights_dirty) return ETC_OK;
    for (size_t l = 0; l < c->weights_bound.size(); ++l)
        if (!c->weights_bound[l]) return fail(c, ETC_ESTATE, "layer " + std::to_string(l) + " has no weights bound");
    HIP_TRY(c, hipMemcpy(c->d_weights, c->h_weights.data(), c->h_weights.size() * sizeof(LayerWeights),
                         hipMemcpyHostToDevice));
    c->weights_dirty = false;
    return ETC_OK;
}

// The bound step's shapes, waiting in their pinned staging slot: one asynchronous copy on the launch stream.
etc_status upload_step_on_stream(etc_ctx *c, hipStream_t s)
{
    if (!c->step_dirty) return ETC_OK;
    const int slot = c->stage_slot;
    HIP_TRY(c, hipMemcpyAsync(c->d_step, c->h_stage[slot], c->stage_used_words * sizeof(int32_t), hipMemcpyHostToDevice, s));
    HIP_TRY(c, hipEventRecord(c->stage_ev[slot], s));
    c->stage_pending[slot] = true;
    c->step_dirty = false;
    return ETC_OK;
}

void post_launch(etc_ctx *c)
{
    c->parity ^= 1;
    c->epoch++;
    if (c->epoch == 0) c->epoch = 1;
}

// What a launch of a model with a vocabulary adds to the step's buffers.
struct TokenIo {
    const int32_t *token_in;
    int32_t *token_out;
    float *logits_out;
};

etc_status pre_launch(etc_ctx *c, const void *hidden_in, void *hidden_out, Params &P, hipStream_t s, const TokenIo *tok = nullptr)
{
    if (!c || c->is_graph) return fail(c, ETC_EINVAL, "not a decoder context");
    if (!tok) {
        if (!hidden_in || !hidden_out) return fail(c, ETC_EINVAL, "hidden_in / hidden_out is NULL");
        if (c->model.vocab > 0) return fail(c, ETC_ESTATE, "this model ends in sampling tasks: launch it with etc_launch_tokens");
    } else {
        if (c->model.vocab <= 0) return fail(c, ETC_ESTATE, "the model has no vocabulary");
        if (!c->lm_bound) return fail(c, ETC_ESTATE, "no LM head bound");
        if ((tok->token_in != nullptr) == (hidden_in != nullptr))
            return fail(c, ETC_EINVAL, "exactly one of token_in and hidden_in must be given");
        if (tok->token_in && !c->base.embed) return fail(c, ETC_ESTATE, "token_in needs the embedding table");
        if (!tok->token_out) return fail(c, ETC_EINVAL, "token_out is NULL");
    }
    if (!c->kv_bound && !c->is_moe_layer) return fail(c, ETC_ESTATE, "no KV pool bound");
    if (!c->step_bound) return fail(c, ETC_ESTATE, c->is_moe_layer ? "no token count bound" : "no step bound");
    etc_status st = refuse_if_dead(c);
    if (st != ETC_OK) return st;
    st = sync_weights(c);
    if (st != ETC_OK) return st;
    st = upload_step_on_stream(c, s);
    if (st != ETC_OK) return st;
    st = arm_on_stream(c, s);
    if (st != ETC_OK) return st;
    fill_launch_params(c, P);
    P.hidden_in = (const uint16_t *)hidden_in;
    P.hidden_out = (uint16_t *)hidden_out;
    if (tok) {
        P.token_in = tok->token_in;
        P.token_out = tok->token_out;
        if (tok->logits_out) P.logits = tok->logits_out;
    }
    return ETC_OK;
}

etc_status launch_fused(etc_ctx *c, Params &P, hipStream_t s)
{
    if (c->sched.kind == ETC_SCHED_DYNAMIC) {
        if (!kDynamicEnabled) return fail(c, ETC_ESTATE, kDynamicOffMsg);
        HIP_TRY(c, launch_dynamic(P, s));
    } else {
        HIP_TRY(c, launch_static(P, s));
    }
    post_launch(c);
    return ETC_OK;
}

etc_status launch_stages(etc_ctx *c, Params &P, hipStream_t s)
{
    const Plan &pl = c->plans[c->cur_plan].host;
    P.moe_dd = 0;        // no events and no ready queue here: the router tiles release nothing, every slot task runs
    // one launch per operator stage; the calls of a stage are contiguous in task-id order
    size_t ci = 0;
    while (ci < pl.stage_of_call.size()) {
        size_t cj = ci;
        while (cj + 1 < pl.stage_of_call.size() && pl.stage_of_call[cj + 1] == pl.stage_of_call[ci]) ++cj;
        HIP_TRY(c, launch_stage(P, pl.call_begin[ci], pl.call_begin[cj + 1] - pl.call_begin[ci], s));
        ci = cj + 1;
    }
    return ETC_OK;   // event buffers untouched: parity and epoch stay
}


}  // namespace

extern "C" {

const char *etc_last_error(const etc_ctx *ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

void etc_destroy(etc_ctx *ctx)
{
    if (!ctx) return;
    (void)hipDeviceSynchronize();
    for (void *p : ctx->owned) (void)hipFree(p);
    for (void *p : ctx->plan_owned) (void)hipFree(p);
    for (int i = 0; i < etc_ctx::kStageSlots; ++i) {
        if (ctx->h_stage[i]) (void)hipHostFree(ctx->h_stage[i]);
        if (ctx->stage_ev[i]) (void)hipEventDestroy(ctx->stage_ev[i]);
    }
    if (ctx->h_error) (void)hipHostFree(ctx->h_error);
    delete ctx;
}

etc_status etc_create(const etc_model_desc *m, const etc_tile_desc *t, const etc_sched_desc *s, etc_ctx **out)
{
    if (!m || !t || !s || !out) return fail(nullptr, ETC_EINVAL, "NULL argument");
    *out = nullptr;
    if (m->n_layers < 1 || m->hidden < 1 || m->n_q_heads < 1 || m->n_kv_heads < 1 || m->page_size < 1)
        return fail(nullptr, ETC_EINVAL, "model dimensions must be positive");
    if (m->page_size & (m->page_size - 1)) return fail(nullptr, ETC_EINVAL, "page_size must be a power of two");
    if (s->max_batch < 1 || s->max_batch > kMaxBatch) return fail(nullptr, ETC_EINVAL, "max_batch must be in 1..64");
    if (s->max_kv_len < 1) return fail(nullptr, ETC_EINVAL, "max_kv_len must be positive");
    if (t->kv_chunk_tokens < m->page_size || t->kv_chunk_tokens % m->page_size)
        return fail(nullptr, ETC_EINVAL, "kv_chunk_tokens must be a positive multiple of page_size");
    if (s->kind < ETC_SCHED_STATIC || s->kind > ETC_SCHED_UNFUSED) return fail(nullptr, ETC_EINVAL, "unknown scheduler kind");
    if (m->n_experts > 0 && (t->moe_tile_m < 1 || t->moe_tile_m > 16)) return fail(nullptr, ETC_EINVAL, "moe_tile_m must be in 1..16");
    if (s->n_sampled < 1 || s->n_sampled > 8) return fail(nullptr, ETC_EINVAL, "n_sampled must be in 1..8");
    for (int i = 0; i < s->n_sampled; ++i) {
        if (s->sampled_batch[i] < 1 || s->sampled_batch[i] > s->max_batch || (i && s->sampled_batch[i] <= s->sampled_batch[i - 1]))
            return fail(nullptr, ETC_EINVAL, "sampled_batch must be ascending, within 1..max_batch");
    }
    if (s->sampled_batch[s->n_sampled - 1] != s->max_batch)
        return fail(nullptr, ETC_EINVAL, "the largest sampled batch must equal max_batch");

    etc_ctx *c = new (std::nothrow) etc_ctx();
    if (!c) return fail(nullptr, ETC_ENOMEM, "out of host memory");
    auto bail = [&](etc_status st) {
        g_create_error = c->err;
        etc_destroy(c);
        return st;
    };
    c->model = *m;
    c->tiles = *t;
    ModelDims &d = c->dims;
    d = ModelDims{m->n_layers, m->hidden, m->n_q_heads, m->n_kv_heads, m->head_dim, m->ffn, m->n_experts,
                  m->top_k, m->moe_ffn, m->page_size, t->kv_chunk_tokens, std::max(1, t->moe_tile_m)};
    d.vocab = m->vocab > 0 ? m->vocab : 0;
    etc_status st = common_device_setup(c, s);
    if (st != ETC_OK) return bail(st);
    c->max_chunks = (s->max_kv_len + t->kv_chunk_tokens - 1) / t->kv_chunk_tokens;
    c->max_pages_per_seq = (s->max_kv_len + m->page_size - 1) / m->page_size;

    for (int i = 0; i < s->n_sampled; ++i) {
        c->plans.emplace_back();
        DevPlan &dp = c->plans.back();
        dp.sampled_batch = s->sampled_batch[i];
        dp.kv_chunk = effective_kv_chunk(t->kv_chunk_tokens, m->page_size, s->max_kv_len, dp.sampled_batch, m->n_kv_heads, c->n_queues);
        int syms[4] = {dp.sampled_batch, (s->max_kv_len + dp.kv_chunk - 1) / dp.kv_chunk, 0, 0};
        std::string err = build_decoder_graph(d, dp.sampled_batch, c->n_queues, s->kind != ETC_SCHED_DYNAMIC, &c->graph);
        if (!err.empty()) { c->err = err; return bail(ETC_EINVAL); }
        dp.k_slices_o = c->graph.k_slices_o;
        dp.k_slices_d = c->graph.k_slices_d;
        dp.all_staged = c->graph.all_staged;
        err = instantiate(c->graph, syms, c->n_queues, s->kind == ETC_SCHED_UNFUSED, &dp.host);
        if (!err.empty()) { c->err = err; return bail(ETC_EINVAL); }
        st = upload_plan(c, dp);
        if (st != ETC_OK) return bail(st);
    }
    st = alloc_events_and_queue(c);
    if (st != ETC_OK) return bail(st);

    // scratch
    Params &P = c->base;
    const size_t MB = (size_t)s->max_batch, H = (size_t)m->hidden, QD = (size_t)m->n_q_heads * m->head_dim;
    P.n_layers = m->n_layers; P.H = m->hidden; P.nq = m->n_q_heads; P.nkv = m->n_kv_heads; P.d = m->head_dim;
    P.F = m->ffn; P.E = m->n_experts; P.topk = m->top_k; P.moeF = m->moe_ffn; P.page = m->page_size;
    P.page_shift = 0;
    while ((1 << P.page_shift) < m->page_size) ++P.page_shift;
    P.eps = m->rms_eps; P.theta = m->rope_theta; P.kv_chunk = t->kv_chunk_tokens; P.tile_m = d.tile_m;
    P.qk_norm = m->qk_norm ? 1 : 0;
    P.vocab = d.vocab;
    P.col_stride = kMaxBatch;
    auto A = [&](auto **p, size_t n) -> bool {
        hipError_t e = dev_alloc(p, n, c->owned);
        if (e != hipSuccess) { c->err = std::string("device allocation failed: ") + hipGetErrorString(e); return false; }
        return true;
    };
    const size_t F1 = (size_t)std::max(1, m->ffn);
    bool okk = A(&P.x, MB * H) && A(&P.x_mid, MB * H) && A(&P.qbuf, MB * QD) &&
               A(&P.knew, MB * (size_t)m->n_kv_heads * m->head_dim) && A(&P.vnew, MB * (size_t)m->n_kv_heads * m->head_dim) &&
               A(&P.rope_cs, MB * (size_t)m->head_dim) && A(&P.kv_slot, MB) &&
               A(&P.qk_ssq, MB * (size_t)(m->n_q_heads + m->n_kv_heads) * (size_t)(m->head_dim / 16)) &&
               A(&P.xg_hi, MB * H) && A(&P.xg_lo, MB * H) && A(&P.xmg_hi, MB * H) && A(&P.xmg_lo, MB * H) &&
               A(&P.ssq_x, (H / 16) * (size_t)kMaxBatch) && A(&P.ssq_xmid, (H / 16) * (size_t)kMaxBatch) &&
               A(&P.attn_hi, MB * QD) && A(&P.attn_lo, MB * QD) && A(&P.act_hi, MB * F1) && A(&P.act_lo, MB * F1) &&
               A(&P.part_m, MB * m->n_q_heads * (size_t)c->max_chunks) &&
               A(&P.part_l, MB * m->n_q_heads * (size_t)c->max_chunks) &&
               A(&P.part_o, MB * m->n_q_heads * (size_t)c->max_chunks * m->head_dim) &&
               A(&P.attn_arrive, MB * (size_t)m->n_kv_heads) &&
               A(&c->d_weights, (size_t)m->n_layers);
    if (okk) {   // the step's shapes: one device block, and pinned staging slots of the same layout
        c->stage_words = MB + (MB + 1) + MB * (size_t)c->max_pages_per_seq;
        okk = A(&c->d_step, c->stage_words);
        c->d_kv_len = c->d_step;
        c->d_page_indptr = c->d_step + MB;
        c->d_page_ids = c->d_step + 2 * MB + 1;
        for (int i = 0; okk && i < etc_ctx::kStageSlots; ++i) {
            okk = hipHostMalloc((void **)&c->h_stage[i], c->stage_words * sizeof(int32_t), hipHostMallocDefault) == hipSuccess &&
                  hipEventCreateWithFlags(&c->stage_ev[i], hipEventDisableTiming) == hipSuccess;
            if (!okk) c->err = "pinned staging allocation failed";
        }
    }
    if (okk) {   // RoPE inverse frequencies theta^(-2i/d) in double
        std::vector<double> inv((size_t)m->head_dim / 2);
        for (size_t i = 0; i < inv.size(); ++i) inv[i] = pow((double)m->rope_theta, -2.0 * (double)i / (double)m->head_dim);
        double *d_inv = nullptr;
        okk = A(&d_inv, inv.size()) &&
              hipMemcpy(d_inv, inv.data(), inv.size() * sizeof(double), hipMemcpyHostToDevice) == hipSuccess;
        P.rope_inv_freq = d_inv;
    }
    {   // partial sums of the K-sliced projections of large-batch plans: [slice][row tile][kMaxBatch][16]
        int most = 0;
        for (const DevPlan &dp : c->plans) most = std::max(most, std::max(dp.k_slices_o, dp.k_slices_d));
        if (okk && most > 0) okk = A(&P.kpart, (size_t)most * (H / 16) * kMaxBatch * 16);
    }
    if (okk && d.vocab > 0) okk = A(&P.logits, MB * (size_t)d.vocab) && A(&P.best, MB);
    if (okk && (s->debug_flags & ETC_DEBUG_LAYER_HIDDEN)) okk = A(&P.layer_hidden, (size_t)m->n_layers * kMaxBatch * H);
    P.max_batch = s->max_batch;
    if (okk && m->n_experts > 0) {
        const size_t E = (size_t)m->n_experts, K = (size_t)m->top_k, NL = (size_t)m->n_layers;
        const size_t rows = MB * K, r_max = (size_t)moe_max_row_tiles(m->n_experts, m->top_k, s->max_batch, d.tile_m);
        okk = A(&P.router_logits, MB * E) && A(&P.topk_ids, rows) && A(&P.topk_w, rows) &&
              A(&P.tok_indptr, E + 1) && A(&P.exp_indptr, E + 1) && A(&P.exp_event, E) && A(&P.perm, rows) && A(&P.inv_perm, rows) &&
              A(&P.perm_tok, rows) && A(&P.tile_expert, r_max) && A(&P.tile_row0, r_max) && A(&P.tile_n, r_max) &&
              A(&P.eact_hi, rows * (size_t)m->moe_ffn) && A(&P.eact_lo, rows * (size_t)m->moe_ffn) && A(&P.ey, rows * H);
        if (okk && (s->debug_flags & ETC_DEBUG_ROUTING))
            okk = A(&P.dbg_logits, NL * MB * E) && A(&P.dbg_topk_ids, NL * rows) && A(&P.dbg_topk_w, NL * rows) &&
                  A(&P.dbg_perm, NL * rows) && A(&P.dbg_tok_indptr, NL * (E + 1)) && A(&P.dbg_exp_indptr, NL * (E + 1));
    }
    if (!okk) return bail(ETC_ENOMEM);
    c->h_weights.assign(m->n_layers, LayerWeights{});
    c->weights_bound.assign(m->n_layers, 0);
    *out = c;
    return ETC_OK;
}

etc_status etc_bind_layer_weights(etc_ctx *c, int32_t layer, const etc_layer_weights *w)
{
    if (!c || c->is_graph || !w) return fail(c, ETC_EINVAL, "bad argument");
    if (layer < 0 || layer >= c->model.n_layers) return fail(c, ETC_EINVAL, "layer out of range");
    const bool moe = c->model.n_experts > 0;
    if (c->is_moe_layer) {
        if (!w->g2 || !w->wr || !w->eg || !w->eu || !w->ed) return fail(c, ETC_EINVAL, "g2, wr, eg, eu, ed are required");
    } else if (!w->g1 || !w->wq || !w->wk || !w->wv || !w->wo || !w->g2) return fail(c, ETC_EINVAL, "attention weights missing");
    if (!moe && (!w->wg || !w->wu || !w->wd)) return fail(c, ETC_EINVAL, "dense FFN weights missing");
    if (moe && (!w->wr || !w->eg || !w->eu || !w->ed)) return fail(c, ETC_EINVAL, "MoE weights missing");
    if (c->model.qk_norm && (!w->gq || !w->gk)) return fail(c, ETC_EINVAL, "per-head norm gains gq / gk missing");
    const void *all[] = {w->g1, w->wq, w->wk, w->wv, w->wo, w->g2, w->wg, w->wu, w->wd, w->wr, w->eg, w->eu, w->ed, w->gq, w->gk};
    for (const void *p : all)
        if (p && ((uintptr_t)p & 15)) return fail(c, ETC_EINVAL, "weight pointers must be 16-byte aligned");
    c->h_weights[layer] = LayerWeights{w->g1, w->wq, w->wk, w->wv, w->wo, w->g2, w->wg, w->wu, w->wd, w->wr, w->eg, w->eu, w->ed, w->gq, w->gk};
    c->weights_bound[layer] = 1;
    c->weights_dirty = true;
    return ETC_OK;
}

etc_status etc_bind_lm_head(etc_ctx *c, const void *embed, const void *g_final, const void *w_lm)
{
    if (!c || c->is_graph) return fail(c, ETC_EINVAL, "not a decoder context");
    if (c->model.vocab <= 0) return fail(c, ETC_ESTATE, "the model has no vocabulary");
    if (!g_final || !w_lm) return fail(c, ETC_EINVAL, "g_final / w_lm is NULL");
    if (((uintptr_t)embed & 15) || ((uintptr_t)g_final & 15) || ((uintptr_t)w_lm & 15))
        return fail(c, ETC_EINVAL, "LM head pointers must be 16-byte aligned");
    c->base.embed = (const uint16_t *)embed;
    c->base.gf = (const uint16_t *)g_final;
    c->base.wlm = (const uint16_t *)w_lm;
    c->lm_bound = true;
    return ETC_OK;
}

etc_status etc_bind_kv_pool(etc_ctx *c, void *k_pages, void *v_pages, int64_t pages_per_layer)
{
    if (!c || c->is_graph || c->is_moe_layer || !k_pages || !v_pages || pages_per_layer < 1) return fail(c, ETC_EINVAL, "bad argument");
    if (((uintptr_t)k_pages & 15) || ((uintptr_t)v_pages & 15)) return fail(c, ETC_EINVAL, "KV pools must be 16-byte aligned");
    c->base.kpool = (uint16_t *)k_pages;
    c->base.vpool = (uint16_t *)v_pages;
    c->pages_per_layer = pages_per_layer;
    c->base.pool_layer_stride = pages_per_layer * c->model.page_size * (int64_t)c->model.n_kv_heads * c->model.head_dim;
    c->kv_bound = true;
    c->step_bound = false;   // page ids are validated against the pool at bind_step
    return ETC_OK;
}

etc_status etc_bind_step(etc_ctx *c, int32_t batch, const int32_t *kv_len, const int32_t *page_indptr, const int32_t *page_ids)
{
    if (!c || c->is_graph || c->is_moe_layer || !kv_len || !page_indptr || !page_ids) return fail(c, ETC_EINVAL, "bad argument");
    if (!c->kv_bound) return fail(c, ETC_ESTATE, "bind the KV pool before a step");
    if (batch < 1 || batch > c->sched.max_batch) return fail(c, ETC_EINVAL, "batch out of range 1..max_batch");
    const int P = c->model.page_size;
    if (page_indptr[0] != 0) return fail(c, ETC_EINVAL, "page_indptr[0] must be 0");
    int64_t kv_tokens = 0;
    for (int b = 0; b < batch; ++b) {
        if (kv_len[b] < 0 || kv_len[b] + 1 > c->sched.max_kv_len) return fail(c, ETC_EINVAL, "kv_len out of range (kv_len + 1 <= max_kv_len)");
        const int need = (kv_len[b] + 1 + P - 1) / P;
        if (page_indptr[b + 1] - page_indptr[b] != need)
            return fail(c, ETC_EINVAL, "page_indptr does not give ceil((kv_len+1)/page_size) pages to sequence " + std::to_string(b));
        kv_tokens += kv_len[b] + 1;
    }
    const int n_ids = page_indptr[batch];
    for (int i = 0; i < n_ids; ++i)
        if (page_ids[i] < 0 || page_ids[i] >= c->pages_per_layer) return fail(c, ETC_EINVAL, "page id outside the bound pool");
    // the next larger sampled batch size serves this step (Sec. 3.1)
    int plan = -1;
    for (size_t i = 0; i < c->plans.size(); ++i)
        if (c->plans[i].sampled_batch >= batch) { plan = (int)i; break; }
    if (plan < 0) return fail(c, ETC_EINVAL, "no sampled batch size covers this batch");

    etc_status st = refuse_if_dead(c);
    if (st != ETC_OK) return st;
    // The arrays go to a pinned staging slot now and to the device on the stream of the next launch.  A slot is
    // reused only after the copy that last read it has finished (four slots: normally long done).
    if (!c->step_dirty) c->stage_slot = (c->stage_slot + 1) % etc_ctx::kStageSlots;      // else: never launched, overwrite
    const int slot = c->stage_slot;
    if (c->stage_pending[slot]) {
        HIP_TRY(c, hipEventSynchronize(c->stage_ev[slot]));
        c->stage_pending[slot] = false;
    }
    const size_t MB = (size_t)c->sched.max_batch;
    int32_t *stg = c->h_stage[slot];
    memcpy(stg, kv_len, (size_t)batch * sizeof(int32_t));
    memcpy(stg + MB, page_indptr, (size_t)(batch + 1) * sizeof(int32_t));
    memcpy(stg + 2 * MB + 1, page_ids, (size_t)n_ids * sizeof(int32_t));
    c->stage_used_words = 2 * MB + 1 + (size_t)n_ids;
    c->step_dirty = true;
    if (plan != c->cur_plan) c->need_arm = true;      // other counts: the buffer the last launch re-armed does not fit
    if (c->base.exec_count) c->need_exec_reset = true;
    c->cur_plan = plan;
    c->bound_batch = batch;
    c->h_kv_len.assign(kv_len, kv_len + batch);

    // algorithmic bytes: every touched weight once, every live KV byte once, appended rows written
    const etc_model_desc &m = c->model;
    const int64_t QD = (int64_t)m.n_q_heads * m.head_dim, KD = (int64_t)m.n_kv_heads * m.head_dim, H = m.hidden;
    int64_t w_layer = 2 * H + QD * H + 2 * KD * H + H * QD;
    if (m.n_experts == 0) w_layer += 3 * (int64_t)m.ffn * H;
    else w_layer += (int64_t)m.n_experts * H + std::min<int64_t>(m.n_experts, (int64_t)batch * m.top_k) * 3 * (int64_t)m.moe_ffn * H;
    const int64_t kv_layer = kv_tokens * KD * 2 + (int64_t)batch * KD * 2;   // read K and V, write the new rows
    c->algorithmic_bytes = 2 * (int64_t)m.n_layers * (w_layer + kv_layer);
    c->step_bound = true;
    return ETC_OK;
}

etc_status etc_moe_layer_create(const etc_model_desc *m, const etc_tile_desc *t, const etc_sched_desc *s, etc_ctx **out)
{
    if (!m || !t || !s || !out) return fail(nullptr, ETC_EINVAL, "NULL argument");
    *out = nullptr;
    if (s->max_batch < 1 || s->max_batch > kMoeLayerMaxTokens) return fail(nullptr, ETC_EINVAL, "max_batch (tokens) must be in 1..4096");
    if (s->kind < ETC_SCHED_STATIC || s->kind > ETC_SCHED_UNFUSED) return fail(nullptr, ETC_EINVAL, "unknown scheduler kind");
    if (s->n_sampled < 1 || s->n_sampled > 8) return fail(nullptr, ETC_EINVAL, "n_sampled must be in 1..8");
    for (int i = 0; i < s->n_sampled; ++i)
        if (s->sampled_batch[i] < 1 || s->sampled_batch[i] > s->max_batch || (i && s->sampled_batch[i] <= s->sampled_batch[i - 1]))
            return fail(nullptr, ETC_EINVAL, "sampled token counts must be ascending, within 1..max_batch");
    if (s->sampled_batch[s->n_sampled - 1] != s->max_batch)
        return fail(nullptr, ETC_EINVAL, "the largest sampled token count must equal max_batch");
    etc_ctx *c = new (std::nothrow) etc_ctx();
    if (!c) return fail(nullptr, ETC_ENOMEM, "out of host memory");
    auto bail = [&](etc_status st) {
        g_create_error = c->err;
        etc_destroy(c);
        return st;
    };
    c->is_moe_layer = true;
    c->model = *m;
    c->model.n_layers = 1;
    c->model.vocab = 0;
    c->tiles = *t;
    ModelDims &d = c->dims;
    d = ModelDims{1, m->hidden, 0, 0, 0, 0, m->n_experts, m->top_k, m->moe_ffn, 1, 1, t->moe_tile_m};
    etc_status st = common_device_setup(c, s);
    if (st != ETC_OK) return bail(st);
    c->sched.debug_flags &= ~(uint32_t)ETC_DEBUG_LAYER_HIDDEN;      // there is no per-layer dump here: y is the layer's output
    for (int i = 0; i < s->n_sampled; ++i) {
        c->plans.emplace_back();
        DevPlan &dp = c->plans.back();
        dp.sampled_batch = s->sampled_batch[i];
        int syms[4] = {dp.sampled_batch, 0, 0, 0};
        std::string err = build_moe_layer_graph(d, dp.sampled_batch, c->n_queues, &c->graph);
        if (!err.empty()) { c->err = err; return bail(ETC_EINVAL); }
        err = instantiate(c->graph, syms, c->n_queues, s->kind == ETC_SCHED_UNFUSED, &dp.host);
        if (!err.empty()) { c->err = err; return bail(ETC_EINVAL); }
        st = upload_plan(c, dp);
        if (st != ETC_OK) return bail(st);
    }
    st = alloc_events_and_queue(c);
    if (st != ETC_OK) return bail(st);

    Params &P = c->base;
    const size_t T = (size_t)s->max_batch, H = (size_t)m->hidden, E = (size_t)m->n_experts, K = (size_t)m->top_k;
    const size_t Tp = (T + 63) / 64 * 64, rows = T * K, n_blk = Tp / 64;
    const size_t r_max = (size_t)moe_max_row_tiles(m->n_experts, m->top_k, s->max_batch, d.tile_m);
    P.n_layers = 1; P.H = m->hidden; P.E = m->n_experts; P.topk = m->top_k; P.moeF = m->moe_ffn; P.page = 1;
    P.eps = m->rms_eps; P.tile_m = d.tile_m; P.moel = 1; P.max_batch = s->max_batch;
    P.col_stride = (int32_t)Tp;
    auto A = [&](auto **p, size_t n) -> bool {
        hipError_t e = dev_alloc(p, n, c->owned);
        if (e != hipSuccess) { c->err = std::string("device allocation failed: ") + hipGetErrorString(e); return false; }
        return true;
    };
    bool okk = A(&P.x, T * H) && A(&P.x_mid, T * H) && A(&P.xmg_hi, Tp * H) && A(&P.xmg_lo, Tp * H) &&
               A(&P.ssq_xmid, (H / 16) * Tp) && A(&c->d_weights, 1) &&
               A(&P.router_logits, Tp * E) && A(&P.topk_ids, rows) && A(&P.topk_w, rows) &&
               A(&P.tok_indptr, E + 1) && A(&P.exp_indptr, E + 1) && A(&P.exp_event, E) && A(&P.perm, rows) && A(&P.inv_perm, rows) &&
               A(&P.perm_tok, rows) && A(&P.tile_expert, r_max) && A(&P.tile_row0, r_max) && A(&P.tile_n, r_max) &&
               A(&P.eact_hi, rows * (size_t)m->moe_ffn) && A(&P.eact_lo, rows * (size_t)m->moe_ffn) && A(&P.ey, rows * H) &&
               A(&P.moel_hist, n_blk * E) && A(&P.moel_base, n_blk * E) && A(&P.moel_count, E);
    if (okk && (s->debug_flags & ETC_DEBUG_ROUTING))
        okk = A(&P.dbg_logits, T * E) && A(&P.dbg_topk_ids, rows) && A(&P.dbg_topk_w, rows) && A(&P.dbg_perm, rows) &&
              A(&P.dbg_tok_indptr, E + 1) && A(&P.dbg_exp_indptr, E + 1);
    if (!okk) return bail(ETC_ENOMEM);
    c->h_weights.assign(1, LayerWeights{});
    c->weights_bound.assign(1, 0);
    *out = c;
    return ETC_OK;
}

etc_status etc_moe_layer_bind_tokens(etc_ctx *c, int32_t n_tokens)
{
    if (!c || !c->is_moe_layer) return fail(c, ETC_EINVAL, "not a MoE-layer context");
    if (n_tokens < 1 || n_tokens > c->sched.max_batch) return fail(c, ETC_EINVAL, "n_tokens out of range 1..max_batch");
    etc_status st = refuse_if_dead(c);
    if (st != ETC_OK) return st;
    int plan = -1;
    for (size_t i = 0; i < c->plans.size(); ++i)
        if (c->plans[i].sampled_batch >= n_tokens) { plan = (int)i; break; }
    if (plan < 0) return fail(c, ETC_EINVAL, "no sampled token count covers this block");
    if (plan != c->cur_plan) c->need_arm = true;
    if (c->base.exec_count) c->need_exec_reset = true;
    c->cur_plan = plan;
    c->bound_batch = n_tokens;
    // algorithmic bytes: gain, router and every routed expert's three matrices once; the tokens in (bf16) and out (bf16)
    const etc_model_desc &m = c->model;
    const int64_t H = m.hidden, experts = std::min<int64_t>(m.n_experts, (int64_t)n_tokens * m.top_k);
    c->algorithmic_bytes = 2 * (H + (int64_t)m.n_experts * H + experts * 3 * (int64_t)m.moe_ffn * H) + 4 * (int64_t)n_tokens * H;
    c->step_bound = true;
    return ETC_OK;
}

etc_status etc_force_routing(etc_ctx *c, int32_t layer, const int32_t *ids, const float *w)
{
    if (!c || c->is_graph || c->model.n_experts == 0) return fail(c, ETC_EINVAL, "not a MoE context");
    if (layer < 0 || layer >= c->model.n_layers) return fail(c, ETC_EINVAL, "layer out of range");
    const size_t per_layer = (size_t)c->sched.max_batch * c->model.top_k;
    if (!c->d_forced) {
        HIP_TRY(c, dev_alloc(&c->d_forced, per_layer * c->model.n_layers, c->owned));
        HIP_TRY(c, dev_alloc(&c->d_forced_w, per_layer * c->model.n_layers, c->owned));
        HIP_TRY(c, dev_alloc(&c->d_forced_mask, (size_t)c->model.n_layers, c->owned));
        c->h_forced_mask.assign(c->model.n_layers, 0);
    }
    HIP_TRY(c, hipDeviceSynchronize());
    if (ids) {
        if (!c->step_bound) return fail(c, ETC_ESTATE, "bind a step before forcing its routing");
        for (int i = 0; i < c->bound_batch * c->model.top_k; ++i)
            if (ids[i] < 0 || ids[i] >= c->model.n_experts) return fail(c, ETC_EINVAL, "expert id out of range");
        HIP_TRY(c, hipMemcpy(c->d_forced + per_layer * layer, ids, (size_t)c->bound_batch * c->model.top_k * sizeof(int32_t),
                             hipMemcpyHostToDevice));
    }
    if (ids && w)
        HIP_TRY(c, hipMemcpy(c->d_forced_w + per_layer * layer, w, (size_t)c->bound_batch * c->model.top_k * sizeof(float),
                             hipMemcpyHostToDevice));
    c->h_forced_mask[layer] = ids ? (w ? 3 : 1) : 0;
    HIP_TRY(c, hipMemcpy(c->d_forced_mask, c->h_forced_mask.data(), c->h_forced_mask.size(), hipMemcpyHostToDevice));
    return ETC_OK;
}

etc_status etc_launch(etc_ctx *c, const void *hidden_in, void *hidden_out, void *hip_stream)
{
    Params P;
    hipStream_t s = (hipStream_t)hip_stream;
    etc_status st = pre_launch(c, hidden_in, hidden_out, P, s);
    if (st != ETC_OK) return st;
    return launch_fused(c, P, s);
}

etc_status etc_launch_kernel_by_kernel(etc_ctx *c, const void *hidden_in, void *hidden_out, void *hip_stream)
{
    Params P;
    hipStream_t s = (hipStream_t)hip_stream;
    etc_status st = pre_launch(c, hidden_in, hidden_out, P, s);
    if (st != ETC_OK) return st;
    return launch_stages(c, P, s);
}

etc_status etc_launch_tokens(etc_ctx *c, const int32_t *token_in, const void *hidden_in, int32_t *token_out, float *logits_out,
                             void *hidden_out, void *hip_stream)
{
    Params P;
    hipStream_t s = (hipStream_t)hip_stream;
    const TokenIo tok{token_in, token_out, logits_out};
    etc_status st = pre_launch(c, hidden_in, hidden_out, P, s, &tok);
    if (st != ETC_OK) return st;
    return launch_fused(c, P, s);
}

etc_status etc_launch_tokens_kernel_by_kernel(etc_ctx *c, const int32_t *token_in, const void *hidden_in, int32_t *token_out,
                                              float *logits_out, void *hidden_out, void *hip_stream)
{
    Params P;
    hipStream_t s = (hipStream_t)hip_stream;
    const TokenIo tok{token_in, token_out, logits_out};
    etc_status st = pre_launch(c, hidden_in, hidden_out, P, s, &tok);
    if (st != ETC_OK) return st;
    return launch_stages(c, P, s);
}

etc_status etc_read_debug(etc_ctx *c, int32_t kind, int32_t layer, void *dst, size_t bytes)
{
    if (!c || !dst) return fail(c, ETC_EINVAL, "bad argument");
    HIP_TRY(c, hipDeviceSynchronize());
    const size_t N = (size_t)c->n_events_max;
    const Params &P = c->base;
    const void *src = nullptr;
    size_t avail = 0;
    const size_t MB = (size_t)c->sched.max_batch;
    switch (kind) {
    case ETC_DBG_ERROR_WORD: src = P.error_word; avail = 4 * sizeof(int32_t); break;
    case ETC_DBG_EVENT_COUNTERS:
        if (c->cur_plan < 0) return fail(c, ETC_ESTATE, "nothing bound");
        // the buffer the last launch consumed is the one the next launch re-arms... it was `cur` before the flip
        src = c->d_events + (c->parity ? 0 : N);
        avail = c->plans[c->cur_plan].host.ev_init.size() * sizeof(int32_t);
        break;
    case ETC_DBG_TASK_EXEC_COUNT:
        if (!P.exec_count || c->cur_plan < 0) return fail(c, ETC_ESTATE, "exec counting is off");
        src = P.exec_count; avail = c->plans[c->cur_plan].host.tasks.size() * sizeof(int32_t); break;
    case ETC_DBG_TASK_TRACE:
        if (!P.trace || c->cur_plan < 0) return fail(c, ETC_ESTATE, "task tracing is off");
        src = P.trace; avail = c->plans[c->cur_plan].host.tasks.size() * 8 * sizeof(uint64_t); break;
    case ETC_DBG_LAYER_HIDDEN:
        if (!P.layer_hidden) return fail(c, ETC_ESTATE, "layer dump is off");
        if (layer < 0 || layer >= c->model.n_layers) return fail(c, ETC_EINVAL, "layer out of range");
        src = P.layer_hidden + (size_t)layer * kMaxBatch * c->model.hidden;
        avail = (size_t)c->bound_batch * c->model.hidden * sizeof(float); break;
    case ETC_DBG_ROUTER_LOGITS: case ETC_DBG_TOPK_IDS: case ETC_DBG_TOPK_W: case ETC_DBG_PERMUTATION:
    case ETC_DBG_TOK_INDPTR: case ETC_DBG_EXP_INDPTR: {
        if (!P.dbg_logits) return fail(c, ETC_ESTATE, "routing dump is off (or the model has no experts)");
        if (layer < 0 || layer >= c->model.n_layers) return fail(c, ETC_EINVAL, "layer out of range");
        const size_t E = (size_t)c->model.n_experts, K = (size_t)c->model.top_k, L = (size_t)layer, Bb = (size_t)c->bound_batch;
        switch (kind) {
        case ETC_DBG_ROUTER_LOGITS: src = P.dbg_logits + L * MB * E; avail = Bb * E * 4; break;
        case ETC_DBG_TOPK_IDS: src = P.dbg_topk_ids + L * MB * K; avail = Bb * K * 4; break;
        case ETC_DBG_TOPK_W: src = P.dbg_topk_w + L * MB * K; avail = Bb * K * 4; break;
        case ETC_DBG_PERMUTATION: src = P.dbg_perm + L * MB * K; avail = Bb * K * 4; break;
        case ETC_DBG_TOK_INDPTR: src = P.dbg_tok_indptr + L * (E + 1); avail = (E + 1) * 4; break;
        default: src = P.dbg_exp_indptr + L * (E + 1); avail = (E + 1) * 4; break;
        }
        break;
    }
    default:
        return fail(c, ETC_EINVAL, "unknown or unavailable debug kind");
    }
    if (bytes > avail) return fail(c, ETC_EINVAL, "more bytes requested than the item holds");
    HIP_TRY(c, hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost));
    if (kind == ETC_DBG_ERROR_WORD) return ETC_OK;
    return check_error_word(c);
}

etc_status etc_get_step_info(etc_ctx *c, etc_step_info *info)
{
    if (!c || !info) return fail(c, ETC_EINVAL, "bad argument");
    if (c->cur_plan < 0) return fail(c, ETC_ESTATE, "nothing bound");
    const DevPlan &dp = c->plans[c->cur_plan];
    info->n_tasks = (int64_t)dp.host.tasks.size();
    info->n_events = (int64_t)dp.host.ev_init.size();
    info->n_queues = c->n_queues;
    info->algorithmic_bytes = c->algorithmic_bytes;
    info->sampled_batch = dp.sampled_batch;
    info->workgroup_threads = kWgThreads;
    info->reserved = 0;
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev);
    info->wall_clock_khz = khz;
    return ETC_OK;
}

// Allocation-free launch of the row-sum graph: all device state in the library's own device array.
etc_status etc_rowsum_launch_noalloc(const float *A, float *C, int32_t n, void *hip_stream)
{
    if (!A || !C) return fail(nullptr, ETC_EINVAL, "A or C is NULL");
    if (n < 1 || n > ETC_ROWSUM_NOALLOC_MAX_N)
        return fail(nullptr, ETC_EINVAL, "n must be in 1.." + std::to_string(ETC_ROWSUM_NOALLOC_MAX_N) + " (the scratch array is sized for that)");
    hipError_t e = launch_rowsum_noalloc(A, C, n, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(nullptr, ETC_EDEVICE, std::string("allocation-free row-sum launch: ") + hipGetErrorString(e));
    return ETC_OK;
}

// ---- host-only inspection ---------------------------------------------------------------------------
static_assert(sizeof(etc_task_record) == sizeof(Task), "public task record must mirror the device record");

static void fill_plan_view(Plan *p, int32_t n_queues, etc_plan_view *out)
{
    out->n_tasks = (int64_t)p->tasks.size();
    out->n_events = (int64_t)p->ev_init.size();
    out->n_queues = n_queues;
    out->n_seed = (int64_t)p->seed_tasks.size();
    out->tasks = reinterpret_cast<const etc_task_record *>(p->tasks.data());
    out->queue_tasks = reinterpret_cast<const etc_task_record *>(p->queue_tasks.data());
    out->queue_begin = p->queue_begin.data();
    out->ev_init = p->ev_init.data();
    out->ev_consumers = p->ev_consumers.data();
    out->consumer_ids = p->consumer_ids.data();
    out->seed_tasks = p->seed_tasks.data();
    out->opaque = p;
}

etc_status etc_plan_build(const etc_model_desc *m, const etc_tile_desc *t, const etc_sched_desc *s, int32_t sampled_batch,
                          int32_t n_queues, etc_plan_view *out)
{
    if (!m || !t || !s || !out) return fail(nullptr, ETC_EINVAL, "NULL argument");
    if (sampled_batch < 1 || sampled_batch > kMaxBatch || n_queues < 1) return fail(nullptr, ETC_EINVAL, "bad batch or queue count");
    if (t->kv_chunk_tokens < 1 || s->max_kv_len < 1) return fail(nullptr, ETC_EINVAL, "bad chunk or max_kv_len");
    ModelDims d{m->n_layers, m->hidden, m->n_q_heads, m->n_kv_heads, m->head_dim, m->ffn, m->n_experts,
                m->top_k, m->moe_ffn, m->page_size, t->kv_chunk_tokens, std::max(1, t->moe_tile_m)};
    d.vocab = m->vocab > 0 ? m->vocab : 0;
    GraphDecl g;
    std::string err = build_decoder_graph(d, sampled_batch, n_queues, s->kind != ETC_SCHED_DYNAMIC, &g);
    if (!err.empty()) return fail(nullptr, ETC_EINVAL, err);
    Plan *p = new (std::nothrow) Plan();
    if (!p) return fail(nullptr, ETC_ENOMEM, "out of host memory");
    const int chunk = effective_kv_chunk(t->kv_chunk_tokens, m->page_size, s->max_kv_len, sampled_batch, m->n_kv_heads, n_queues);
    int syms[4] = {sampled_batch, (s->max_kv_len + chunk - 1) / chunk, 0, 0};
    err = instantiate(g, syms, n_queues, s->kind == ETC_SCHED_UNFUSED, p);
    if (!err.empty()) { delete p; return fail(nullptr, ETC_EINVAL, err); }
    fill_plan_view(p, n_queues, out);
    return ETC_OK;
}

etc_status etc_moe_layer_plan_build(const etc_model_desc *m, const etc_tile_desc *t, const etc_sched_desc *s, int32_t sampled_tokens,
                                    int32_t n_queues, etc_plan_view *out)
{
    if (!m || !t || !s || !out) return fail(nullptr, ETC_EINVAL, "NULL argument");
    if (n_queues < 1) return fail(nullptr, ETC_EINVAL, "bad queue count");
    ModelDims d{1, m->hidden, 0, 0, 0, 0, m->n_experts, m->top_k, m->moe_ffn, 1, 1, t->moe_tile_m};
    GraphDecl g;
    std::string err = build_moe_layer_graph(d, sampled_tokens, n_queues, &g);
    if (!err.empty()) return fail(nullptr, ETC_EINVAL, err);
    Plan *p = new (std::nothrow) Plan();
    if (!p) return fail(nullptr, ETC_ENOMEM, "out of host memory");
    int syms[4] = {sampled_tokens, 0, 0, 0};
    err = instantiate(g, syms, n_queues, s->kind == ETC_SCHED_UNFUSED, p);
    if (!err.empty()) { delete p; return fail(nullptr, ETC_EINVAL, err); }
    fill_plan_view(p, n_queues, out);
    return ETC_OK;
}

void etc_plan_free(etc_plan_view *v)
{
    if (!v || !v->opaque) return;
    delete static_cast<Plan *>(v->opaque);
    memset(v, 0, sizeof(*v));
}

// ---- generic graphs ------------------------------------------------------------------------------
etc_status etc_graph_create(const etc_sched_desc *s, etc_ctx **out)
{
    if (!s || !out) return fail(nullptr, ETC_EINVAL, "NULL argument");
    *out = nullptr;
    if (s->kind < ETC_SCHED_STATIC || s->kind > ETC_SCHED_UNFUSED) return fail(nullptr, ETC_EINVAL, "unknown scheduler kind");
    etc_ctx *c = new (std::nothrow) etc_ctx();
    if (!c) return fail(nullptr, ETC_ENOMEM, "out of host memory");
    c->is_graph = true;
    etc_status st = common_device_setup(c, s);
    if (st != ETC_OK) { g_create_error = c->err; etc_destroy(c); return st; }
    *out = c;
    return ETC_OK;
}

etc_status etc_graph_add_event(etc_ctx *c, const etc_dim_expr *shape, int32_t rank, int32_t *event_id)
{
    if (!c || !c->is_graph || !shape || !event_id || rank < 1 || rank > 3) return fail(c, ETC_EINVAL, "bad argument");
    EventDecl e;
    e.rank = rank;
    for (int r = 0; r < rank; ++r) {
        if (shape[r].sym >= 4) return fail(c, ETC_EINVAL, "symbol id must be 0..3");
        e.shape[r] = DimExpr{shape[r].sym, shape[r].mul, shape[r].add};
    }
    c->graph.events.push_back(e);
    *event_id = (int32_t)c->graph.events.size() - 1;
    return ETC_OK;
}

etc_status etc_graph_add_call(etc_ctx *c, int32_t fn, const etc_dim_expr *shape, int32_t rank, const etc_edge *in,
                              int32_t n_in, const etc_edge *outs, int32_t n_out)
{
    if (!c || !c->is_graph || !shape || rank < 1 || rank > 3) return fail(c, ETC_EINVAL, "bad argument");
    const bool user_fn = fn >= ETC_FN_USER0 && fn - ETC_FN_USER0 < user_fn_count();      // generated libraries only
    if (!user_fn && fn != ETC_FN_ROWSUM_PARTIAL && fn != ETC_FN_ROWSUM_FINAL && fn != ETC_FN_ROWSUM_FINAL_PERM)
        return fail(c, ETC_EINVAL, fn >= ETC_FN_USER0 ? "this library was not generated with that many device functions" : "unknown device function");
    if (n_in < 0 || n_in > 2 || n_out < 0 || n_out > 1 || (n_in && !in) || (n_out && !outs))
        return fail(c, ETC_EINVAL, "a call takes at most 2 in-edges and 1 out-edge");
    CallDecl cd;
    cd.fn = user_fn ? FN_USER0 + (fn - ETC_FN_USER0)
                    : fn == ETC_FN_ROWSUM_PARTIAL ? FN_ROWSUM_PARTIAL : fn == ETC_FN_ROWSUM_FINAL ? FN_ROWSUM_FINAL : FN_ROWSUM_FINAL_PERM;
    cd.rank = rank;
    cd.stage = (int)c->graph.calls.size();
    for (int r = 0; r < rank; ++r) cd.shape[r] = DimExpr{shape[r].sym, shape[r].mul, shape[r].add};
    auto conv = [&](const etc_edge &e, EdgeMap *m, bool is_out) -> bool {
        if (e.event < 0 || e.event >= (int)c->graph.events.size() || e.rank != c->graph.events[e.event].rank) return false;
        m->event = e.event;
        m->rank = e.rank;
        if (e.kind[0] == ETC_MAP_INDIRECT || e.kind[0] == ETC_MAP_INDPTR) {
            // run-time maps: rank-1 event tensor, indexed through the first task coordinate; a table on out-edges,
            // ranges on the in-edges of a rank-1 grid
            if (e.rank != 1 || (e.kind[0] == ETC_MAP_INDIRECT) != is_out || (!is_out && rank != 1)) return false;
            m->kind[0] = e.kind[0] == ETC_MAP_INDIRECT ? MAP_INDIRECT : MAP_INDPTR;
            m->src[0] = 0;
            m->div[0] = 1;
            return true;
        }
        for (int r = 0; r < e.rank; ++r) {
            if (e.kind[r] != ETC_MAP_DIM && e.kind[r] != ETC_MAP_CONST) return false;
            if (e.kind[r] == ETC_MAP_DIM && (e.src[r] < 0 || e.src[r] >= rank || e.div[r] < 1)) return false;
            m->kind[r] = e.kind[r] == ETC_MAP_DIM ? MAP_DIM : MAP_CONST;
            m->src[r] = e.src[r];
            m->div[r] = e.div[r];
        }
        return true;
    };
    for (int i = 0; i < n_in; ++i) { EdgeMap m; if (!conv(in[i], &m, false)) return fail(c, ETC_EINVAL, "malformed in-edge"); cd.in.push_back(m); }
    for (int i = 0; i < n_out; ++i) { EdgeMap m; if (!conv(outs[i], &m, true)) return fail(c, ETC_EINVAL, "malformed out-edge"); cd.out.push_back(m); }
    c->graph.calls.push_back(cd);
    return ETC_OK;
}

etc_status etc_graph_user_fn_count(int32_t *count)
{
    if (!count) return fail(nullptr, ETC_EINVAL, "NULL argument");
    *count = user_fn_count();
    return ETC_OK;
}

etc_status etc_graph_bind_buffer(etc_ctx *c, int32_t slot, void *ptr, size_t bytes)
{
    if (!c || !c->is_graph || slot < 0 || slot > 7 || !ptr) return fail(c, ETC_EINVAL, "bad argument");
    c->base.gbuf[slot] = (float *)ptr;
    c->gbuf_bytes[slot] = bytes;
    return ETC_OK;
}

etc_status etc_graph_bind_shape(etc_ctx *c, const int32_t *values)
{
    if (!c || !c->is_graph || !values) return fail(c, ETC_EINVAL, "bad argument");
    for (int i = 0; i < 4; ++i)
        if (values[i] < 0 || values[i] > (1 << 20)) return fail(c, ETC_EINVAL, "symbol value out of range");
    HIP_TRY(c, hipDeviceSynchronize());
    // instantiate the template for these symbol values: no kernel is rebuilt, only queues and counts
    DevPlan dp;
    int syms[4] = {values[0], values[1], values[2], values[3]};
    std::string err = instantiate(c->graph, syms, c->n_queues, c->sched.kind == ETC_SCHED_UNFUSED, &dp.host,
                                  c->sched.kind == ETC_SCHED_DYNAMIC);
    if (!err.empty()) return fail(c, ETC_EINVAL, err);
    for (void *p : c->plan_owned) (void)hipFree(p);
    c->plan_owned.clear();
    c->base.exec_count = nullptr;
    c->base.trace = nullptr;
    c->step_bound = false;
    c->plans.clear();
    etc_status st = upload_plan(c, dp);
    if (st != ETC_OK) return st;
    c->plans.push_back(dp);
    c->cur_plan = 0;
    st = alloc_events_and_queue(c);
    if (st != ETC_OK) return st;
    for (int i = 0; i < 4; ++i) c->sym_values[i] = values[i];
    // a rebuilt plan starts from scratch: counters armed by the next launch, an earlier device error forgotten
    c->need_arm = true;
    c->need_exec_reset = false;
    HIP_TRY(c, hipMemset(c->base.error_word, 0, 4 * sizeof(int32_t)));
    memset(c->h_error, 0, 4 * sizeof(int32_t));
    c->dead = false;
    c->step_bound = true;
    return ETC_OK;
}

etc_status etc_graph_launch(etc_ctx *c, void *hip_stream)
{
    if (!c || !c->is_graph) return fail(c, ETC_EINVAL, "not a graph context");
    if (!c->step_bound) return fail(c, ETC_ESTATE, "bind a shape first");
    bool need[7] = {false, false, false, false, false, false, false};
    for (const CallDecl &cd : c->graph.calls) {
        if (cd.fn == FN_ROWSUM_PARTIAL) need[0] = need[1] = true;
        if (cd.fn == FN_ROWSUM_FINAL) need[1] = need[2] = true;
        if (cd.fn == FN_ROWSUM_FINAL_PERM) need[1] = need[2] = need[4] = need[6] = true;
        if (!cd.out.empty() && cd.out[0].kind[0] == MAP_INDIRECT) need[3] = need[4] = need[5] = true;
        for (const EdgeMap &m : cd.in)
            if (m.kind[0] == MAP_INDPTR) need[4] = true;
    }
    for (int i = 0; i < 7; ++i)
        if (need[i] && !c->base.gbuf[i]) return fail(c, ETC_ESTATE, "a device-function buffer or run-time table is not bound");
    // the task grids must stay inside the bound buffers: A (rows, 128), B (rows, 4), C (rows), 32 rows per task
    for (const CallDecl &cd : c->graph.calls) {
        const size_t rows = (size_t)32 * (size_t)cd.shape[0].eval(c->sym_values);
        if (cd.fn >= FN_USER0) {
            // generated device functions: the front end that generated them checks their buffers against the bound shape
        } else if (cd.fn == FN_ROWSUM_PARTIAL) {
            if (cd.rank != 2 || cd.shape[1].eval(c->sym_values) > 4) return fail(c, ETC_EINVAL, "partial_sum takes a (n, <=4) grid");
            if (rows * 128 * 4 > c->gbuf_bytes[0] || rows * 4 * 4 > c->gbuf_bytes[1]) return fail(c, ETC_EINVAL, "buffer A or B too small for the bound shape");
        } else if (cd.fn == FN_ROWSUM_FINAL) {
            if (cd.rank != 1) return fail(c, ETC_EINVAL, "final_sum takes a (n) grid");
            if (rows * 4 * 4 > c->gbuf_bytes[1] || rows * 4 > c->gbuf_bytes[2]) return fail(c, ETC_EINVAL, "buffer B or C too small for the bound shape");
        } else {      // one perm entry per task; the row blocks it may name are those of the indirectly notifying call
            const size_t blocks = (size_t)c->plans[c->cur_plan].host.dd_table_len;
            if (cd.rank != 1 || blocks == 0) return fail(c, ETC_EINVAL, "final_sum_perm takes a (n) grid released through an INDPTR edge");
            if (rows / 32 * 4 > c->gbuf_bytes[6]) return fail(c, ETC_EINVAL, "perm too small for the bound shape");
            if (blocks * 32 * 4 * 4 > c->gbuf_bytes[1] || blocks * 32 * 4 > c->gbuf_bytes[2]) return fail(c, ETC_EINVAL, "buffer B or C too small for the bound shape");
        }
        const size_t grid0 = (size_t)cd.shape[0].eval(c->sym_values);
        if (!cd.out.empty() && cd.out[0].kind[0] == MAP_INDIRECT) {       // table [grid dim 0], count [events], indptr [events + 1]
            const size_t n_ev = (size_t)c->graph.events[cd.out[0].event].shape[0].eval(c->sym_values);
            if (grid0 * 4 > c->gbuf_bytes[3] || n_ev * 4 > c->gbuf_bytes[5] || (n_ev + 1) * 4 > c->gbuf_bytes[4])
                return fail(c, ETC_EINVAL, "a run-time table is too small for the bound shape");
        }
    }
    Params P;
    hipStream_t s = (hipStream_t)hip_stream;
    etc_status st = refuse_if_dead(c);
    if (st != ETC_OK) return st;
    st = arm_on_stream(c, s);
    if (st != ETC_OK) return st;
    fill_launch_params(c, P);
    if (c->sched.kind == ETC_SCHED_DYNAMIC) {
        if (!kDynamicEnabled) return fail(c, ETC_ESTATE, kDynamicOffMsg);
        HIP_TRY(c, launch_dynamic(P, s));
    } else {
        HIP_TRY(c, launch_static(P, s));
    }
    post_launch(c);
    return ETC_OK;
}

}  // extern "C"
