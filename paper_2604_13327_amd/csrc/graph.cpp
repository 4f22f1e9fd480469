// Event-tensor graph IR: instantiation into tasks, event counts and queues; the decoder's graph.
#include "graph.h"

#include <algorithm>
#include <sstream>

namespace etc {

int GraphDecl::add_event(std::initializer_list<DimExpr> shape)
{
    EventDecl e;
    e.rank = (int)shape.size();
    int i = 0;
    for (const DimExpr &d : shape) e.shape[i++] = d;
    events.push_back(e);
    return (int)events.size() - 1;
}

static EdgeMap edge(int ev, std::initializer_list<int> kinds, std::initializer_list<int> srcs,
                    std::initializer_list<int> divs)
{
    EdgeMap m;
    m.event = ev;
    m.rank = (int)kinds.size();
    int i = 0;
    for (int k : kinds) m.kind[i++] = k;
    i = 0;
    for (int s : srcs) m.src[i++] = s;
    i = 0;
    for (int d : divs) m.div[i++] = d;
    return m;
}
static EdgeMap edge_const0(int ev) { return edge(ev, {MAP_CONST}, {0}, {0}); }
static EdgeMap edge_dim(int ev, int src, int div = 1) { return edge(ev, {MAP_DIM}, {src}, {div}); }

std::string instantiate(const GraphDecl &g, const int *sym, int n_queues, bool unfused, Plan *out, bool data_dependent)
{
    Plan &p = *out;
    p = Plan();
    if (n_queues <= 0) return "n_queues must be positive";

    // event tensors -> flat offsets
    std::vector<std::vector<int>> ev_dims(g.events.size());
    p.ev_offset.assign(1, 0);
    for (size_t e = 0; e < g.events.size(); ++e) {
        int n = 1;
        for (int r = 0; r < g.events[e].rank; ++r) {
            int v = g.events[e].shape[r].eval(sym);
            if (v < 0) return "negative event tensor dimension";
            ev_dims[e].push_back(v);
            n *= v;
        }
        p.ev_offset.push_back(p.ev_offset.back() + n);
    }
    int n_stages = 0;
    for (const CallDecl &c : g.calls) n_stages = std::max(n_stages, c.stage + 1);
    const int n_events = unfused ? n_stages : p.ev_offset.back();
    p.ev_init.assign(n_events, 0);

    auto flat_event = [&](const EdgeMap &m, const int *coord, int *flat) -> std::string {
        if (m.event < 0 || m.event >= (int)g.events.size()) return "edge names an unknown event tensor";
        const std::vector<int> &dims = ev_dims[m.event];
        if (m.rank != (int)dims.size()) return "edge rank differs from its event tensor's rank";
        int idx = 0;
        for (int r = 0; r < m.rank; ++r) {
            // a run-time map names the tensor's event 0 here: the coarse event of the static rule, or the base
            // the run-time index is added to
            int v = m.kind[r] == MAP_CONST ? m.div[r]
                    : (m.kind[r] == MAP_INDIRECT || m.kind[r] == MAP_INDPTR) ? 0
                                                                             : coord[m.src[r]] / std::max(1, m.div[r]);
            if (v < 0 || v >= dims[r]) {
                std::ostringstream s;
                s << "edge maps a task outside event tensor " << m.event << " (dim " << r << ": " << v
                  << " not in [0, " << dims[r] << "))";
                return s.str();
            }
            idx = idx * dims[r] + v;
        }
        *flat = p.ev_offset[m.event] + idx;
        return "";
    };

    p.call_begin.assign(1, 0);
    for (const CallDecl &c : g.calls) {
        if (c.in.size() > 2 || c.out.size() > 1) return "a call has more than 2 in-edges or 1 out-edge";
        int dims[3] = {1, 1, 1};
        for (int r = 0; r < c.rank; ++r) dims[r] = c.shape[r].eval(sym);
        const int total = dims[0] * dims[1] * dims[2];
        for (int i = 0; i < total; ++i) {
            int coord[3];
            if (c.last_dim_slowest && c.rank == 3) {      // (c2 slowest, then c0, c1)
                coord[2] = i / (dims[0] * dims[1]);
                coord[0] = (i / dims[1]) % dims[0];
                coord[1] = i % dims[1];
            } else {
                coord[0] = i / (dims[1] * dims[2]);
                coord[1] = (i / dims[2]) % dims[1];
                coord[2] = i % dims[2];
            }
            Task t{};
            t.fn = (uint8_t)c.fn;
            t.layer = (uint8_t)c.layer;
            t.flags = c.flags;
            int tc[3];
            for (int k = 0; k < 3; ++k) tc[k] = k < c.rank ? coord[k] * c.c_mul[k] + c.c_off[k] : c.c_fill[k];
            t.c0 = tc[0];
            t.c1 = tc[1];
            t.c2 = tc[2];
            t.wait0 = t.wait1 = t.notify0 = -1;
            t.id = (int32_t)p.tasks.size();
            if (unfused) {
                t.flags &= (uint16_t)~TF_WAIT0_PER_WAVE;
                if (c.stage > 0) t.wait0 = c.stage - 1;
                t.notify0 = c.stage;
                p.ev_init[c.stage]++;
            } else {
                for (size_t k = 0; k < c.in.size(); ++k) {
                    int f;
                    std::string err = flat_event(c.in[k], coord, &f);
                    if (!err.empty()) return err;
                    if (data_dependent && c.in[k].kind[0] == MAP_INDPTR) {      // released at run time, waits for nothing
                        t.flags |= TF_TRIGGERED;
                        continue;
                    }
                    (k == 0 ? t.wait0 : t.wait1) = f;
                }
                if (!c.out.empty()) {
                    int f;
                    std::string err = flat_event(c.out[0], coord, &f);
                    if (!err.empty()) return err;
                    t.notify0 = f;
                    if (data_dependent && c.out[0].kind[0] == MAP_INDIRECT) t.flags |= TF_NOTIFY_INDIRECT;   // count known at run time only
                    else p.ev_init[f]++;
                }
            }
            p.tasks.push_back(t);
        }
        p.call_begin.push_back((int32_t)p.tasks.size());
        p.stage_of_call.push_back(c.stage);
        {   // the run-time edges of the graph (the device functions bound-check their tables against these)
            if (!c.out.empty() && c.out[0].kind[0] == MAP_INDIRECT) {
                p.dd_event_base = p.ev_offset[c.out[0].event];
                p.dd_n_events = ev_dims[c.out[0].event][0];
                p.dd_table_len = dims[0];
            }
            for (const EdgeMap &m : c.in)
                if (m.kind[0] == MAP_INDPTR) {
                    p.dd_consumer_first = p.call_begin[p.call_begin.size() - 2];
                    p.dd_consumer_n = total;
                }
        }
    }

    // static queues: round-robin over the task enumeration (Sec. 3.1).  Every queue is a
    // subsequence of one topological order (calls are listed producers first), so the globally
    // oldest unfinished task always sits at some queue head with its events fired: no deadlock.
    std::vector<std::vector<Task>> q(n_queues);
    for (const Task &t : p.tasks) q[t.id % n_queues].push_back(t);
    p.queue_begin.assign(1, 0);
    for (int i = 0; i < n_queues; ++i) {
        p.queue_tasks.insert(p.queue_tasks.end(), q[i].begin(), q[i].end());
        p.queue_begin.push_back((int32_t)p.queue_tasks.size());
    }

    // dynamic scheduling with early push (App. E): a task is pushed once every producer of every event it
    // waits on has been dispatched, so it is listed under each of those events (events nobody notifies count
    // as passed, as for a wait); an entry of a task that waits on n > 1 events carries n in its top byte.
    if (p.tasks.size() >= (1u << 24)) return "more than 2^24 tasks in one plan";
    std::vector<std::vector<int32_t>> cons(n_events);
    for (const Task &t : p.tasks) {
        int trig[kWaves + 1], n = 0;
        auto add = [&](int e) {
            if (e < 0 || p.ev_init[e] <= 0) return;
            for (int k = 0; k < n; ++k)
                if (trig[k] == e) return;
            trig[n++] = e;
        };
        if (t.wait0 >= 0) {
            const int span = (t.flags & TF_WAIT0_PER_WAVE) ? kWaves : 1;
            for (int w = 0; w < span; ++w) add(t.wait0 + w);
        }
        add(t.wait1);
        if (n == 0 && !(t.flags & TF_TRIGGERED)) p.seed_tasks.push_back(t.id);
        for (int k = 0; k < n; ++k) cons[trig[k]].push_back(t.id | (n > 1 ? n << 24 : 0));
    }
    p.ev_consumers.assign(1, 0);
    for (int e = 0; e < n_events; ++e) {
        p.consumer_ids.insert(p.consumer_ids.end(), cons[e].begin(), cons[e].end());
        p.ev_consumers.push_back((int32_t)p.consumer_ids.size());
    }
    return "";
}

std::string build_decoder_graph(const ModelDims &m, int Bs, int n_queues, bool moe_static_coarse, GraphDecl *out)
{
    (void)moe_static_coarse;
    GraphDecl &g = *out;
    g = GraphDecl();
    if (m.nq % m.nkv) return "n_q_heads must be a multiple of n_kv_heads";
    if (m.d % 16 || (m.d != 64 && m.d != 128)) return "head_dim must be 64 or 128";
    if (!attn_shape_supported(m.d, m.nq / m.nkv))
        return "no attention task body for this (head_dim, n_q_heads / n_kv_heads): supported are 128 with 1, 4, 8 and 64 with 2, 4";
    if (m.H % (kWaves * 32) || (m.nq * m.d) % (kWaves * 32)) return "hidden and n_q_heads*head_dim must be multiples of 256";
    if (m.H % 16) return "hidden must be a multiple of 16";
    if (m.E == 0 && (m.F % (kWaves * 32) || (m.F / 8) % kWaves)) return "ffn must be a multiple of 256";
    if (m.n_layers > kMaxLayers) return "too many layers";
    if (m.page < 1 || (m.page & (m.page - 1))) return "page_size must be a power of two";
    if (m.E > 0) {
        if (m.E % 16 || m.E > kMaxExperts) return "n_experts must be a multiple of 16, at most 256";
        if (m.topk < 1 || m.topk > kMaxTopK || m.topk > m.E) return "top_k must be in 1..16 and at most n_experts";
        if (m.moeF < 1 || m.moeF % (kWaves * 32)) return "moe_ffn must be a multiple of 256";
        if (m.tile_m < 1 || m.tile_m > 16) return "moe_tile_m must be in 1..16";
    }
    const int grp = m.nq / m.nkv;
    const int sub = m.d / 16;                     // 16-row tiles (8 RoPE pairs) per head
    const DimExpr B = dim_sym(0), NCH = dim_sym(1), one = dim_const(1);

    // Row tiles per projection task.  When the batch is small enough for the staged path, a task
    // streams several consecutive tiles back to back (one reduction, one notify), sized so that a
    // stage is about one task per queue.
    auto staged_ok = [&](int K) {
        return staged_fits(1, Bs, K);
    };
    int r_qkv = 1, r_gu = 1;
    if (staged_ok(m.H)) {
        if ((m.nq + 2 * m.nkv) * sub > n_queues && sub % 2 == 0 && staged_fits(2, Bs, m.H)) r_qkv = 2;
        if (m.E == 0) {
            const int tiles = m.F / 8, per_slice = tiles / kWaves;
            int cand = tiles / std::max(1, n_queues);
            while (cand > 1 && (tiles % cand || per_slice % cand || !staged_fits(cand, Bs, m.H))) --cand;
            r_gu = std::max(1, cand);
            // The down projection's operand (K = ffn) leaves LDS first, at batch 3 on the 8B shape.  One slice of K
            // still fits, so it is cut along K like the large-batch projections and stays on the staged path.
            const int s_d = k_slices_for(m.F);
            if (!staged_fits(1, Bs, m.F) && s_d > 0 && staged_fits(8, Bs, m.F / s_d)) g.k_slices_d = s_d;
        }
    } else {
        // Large batches take the chunked path, where every task reads its operand from memory: traffic that
        // grows with (tasks x columns x K) and soon exceeds the weights.  A gate/up task therefore streams up to
        // 8 row tiles (4 above 32 columns) against one pass over the operand, and the O and down projections, which have only
        // hidden/16 row tiles in all, are cut along K instead: a task takes that many row tiles and one slice of K
        // and leaves fp32 partial sums, which a second, small task adds up in slice order (two-stage
        // reduction as in the row-sum example of Sec. 2.2).
        {   // row tiles per QKV task: what moves the fewest bytes through a queue, as for gate/up below (a task reads
            // the whole operand whatever it streams; two rounds of small tasks read it twice)
            const long long tile_bytes = 16LL * m.H * 2, operand_bytes = (long long)Bs * m.H * 4;
            const int tiles = (m.nq + 2 * m.nkv) * sub;
            long long best = -1;
            for (int r = 1; r <= sub; r *= 2) {
                if (sub % r) continue;
                const long long rounds = (tiles / r + n_queues - 1) / n_queues, cost = rounds * (r * tile_bytes + operand_bytes);
                if (best < 0 || cost < best || (cost == best && r == 2)) { best = cost; r_qkv = r; }
            }
        }
        g.k_slices_o = k_slices_for(m.nq * m.d);
        if (m.E == 0) {
            g.k_slices_d = k_slices_for(m.F);
            const int tiles = m.F / 8, per_slice = tiles / (g.k_slices_d ? g.k_slices_d : kWaves);
            // bytes a queue moves through the stage: rounds x (r row tiles of weights + one pass over the operand)
            const long long tile_bytes = 16LL * m.H * 2, operand_bytes = (long long)Bs * m.H * 4;
            long long best = -1;
            for (int r = 1; r <= wide_pass_tiles_for(Bs); ++r) {
                if (per_slice % r) continue;
                const long long rounds = (tiles / r + n_queues - 1) / n_queues, cost = rounds * (r * tile_bytes + operand_bytes);
                if (best < 0 || cost <= best) { best = cost; r_gu = r; }
            }
        }
    }
    const int n_ht = m.H / 16, pass_tiles = pass_tiles_for(Bs);
    const int pass_o = sliced_pass_tiles(Bs, n_ht, g.k_slices_o, n_queues), pass_d = sliced_pass_tiles(Bs, n_ht, g.k_slices_d, n_queues);
    const bool slice_o = g.k_slices_o > 0 && n_ht % pass_o == 0;
    const bool slice_d = g.k_slices_d > 0 && n_ht % pass_d == 0;
    if (!slice_o) g.k_slices_o = 0;
    if (!slice_d) g.k_slices_d = 0;
    g.all_staged = m.E == 0 && staged_fits(r_qkv, Bs, m.H) && staged_fits(r_gu, Bs, m.H) &&
                   (slice_o ? staged_fits(pass_tiles, Bs, m.nq * m.d / g.k_slices_o) : staged_fits(1, Bs, m.nq * m.d)) &&
                   (slice_d ? staged_fits(pass_tiles, Bs, m.F / g.k_slices_d) : staged_fits(1, Bs, m.F));

    int stage = 0;
    int e_x = g.add_event({one});
    {   // step prologue: hidden_in (bf16) -> residual stream
        CallDecl c;
        c.fn = FN_LOAD_HIDDEN; c.layer = 0; c.stage = stage++;
        c.rank = 1; c.shape[0] = B;
        c.out = {edge_const0(e_x)};
        g.calls.push_back(c);
    }
    for (int l = 0; l < m.n_layers; ++l) {
        const int e_qkv = g.add_event({dim_const(m.nkv)});
        const int e_attn = g.add_event({one});
        const int e_xmid = g.add_event({one});
        const int e_xnext = g.add_event({one});
        const uint16_t last = (l == m.n_layers - 1) ? TF_LAST_LAYER : 0;

        // Q, K and V row tiles: three launches of one device function, same stage (they run
        // concurrently; Sec. 4.3 names Q and K processing overlapping inside the megakernel).
        for (int part = 0; part < 3; ++part) {
            CallDecl c;
            c.fn = FN_QKV; c.layer = l; c.stage = stage;
            c.rank = 2;                                    // task record: (head, first 16-row tile of the head, tiles)
            c.shape[0] = dim_const(part == 0 ? m.nq : m.nkv);
            c.shape[1] = dim_const(sub / r_qkv);
            c.c_mul[1] = r_qkv;
            c.c_fill[2] = r_qkv;
            c.c_off[0] = part == 0 ? 0 : (part == 1 ? m.nq : m.nq + m.nkv);
            c.in = {edge_const0(e_x)};
            c.out = {edge_dim(e_qkv, 0, part == 0 ? grp : 1)};
            g.calls.push_back(c);
        }
        stage++;
        {
            CallDecl c;
            c.fn = FN_ATTN; c.layer = l; c.stage = stage++;
            c.rank = 3; c.shape[0] = B; c.shape[1] = dim_const(m.nkv); c.shape[2] = NCH;
            c.last_dim_slowest = true;
            c.in = {edge_dim(e_qkv, 1)};
            // The chunk task that arrives last at its (sequence, KV head) merges the chunks itself (counted with a
            // returning atomic outside the event tensors), so the merge is no stage and no event of its own: every
            // chunk task notifies the attention block's one event, the merging one after its merge.
            c.out = {edge_const0(e_attn)};
            g.calls.push_back(c);
        }
        if (slice_o) {
            const int e_opart = g.add_event({one});
            CallDecl c;
            c.fn = FN_OPROJ; c.layer = l; c.stage = stage++;      // task record: (first row tile, K slice, tiles)
            c.rank = 2; c.shape[0] = dim_const(n_ht / pass_o); c.shape[1] = dim_const(g.k_slices_o);
            c.c_mul[0] = pass_o; c.c_fill[2] = pass_o;
            c.flags = TF_K_SLICE;
            c.in = {edge_const0(e_attn)};
            c.out = {edge_const0(e_opart)};
            g.calls.push_back(c);
            CallDecl r;
            r.fn = FN_OPROJ_SUM; r.layer = l; r.stage = stage++;
            r.rank = 1; r.shape[0] = dim_const(n_ht);
            r.in = {edge_const0(e_opart)};
            r.out = {edge_const0(e_xmid)};
            g.calls.push_back(r);
        } else {
            CallDecl c;
            c.fn = FN_OPROJ; c.layer = l; c.stage = stage++;
            c.rank = 1; c.shape[0] = dim_const(n_ht);
            c.in = {edge_const0(e_attn)};
            c.out = {edge_const0(e_xmid)};
            g.calls.push_back(c);
        }
        if (m.E == 0) {
            const int act_slices = slice_d ? g.k_slices_d : kWaves;
            const int e_act = g.add_event({dim_const(act_slices)});
            const int tiles = m.F / 8;
            {
                CallDecl c;
                c.fn = FN_GATEUP; c.layer = l; c.stage = stage++;    // task record: (first tile, tiles)
                c.rank = 1; c.shape[0] = dim_const(tiles / r_gu);
                c.c_mul[0] = r_gu;
                c.c_fill[1] = r_gu;
                c.in = {edge_const0(e_xmid)};
                c.out = {edge_dim(e_act, 0, tiles / act_slices / r_gu)};   // K slice of the down projection it feeds
                g.calls.push_back(c);
            }
            if (slice_d) {
                const int e_dpart = g.add_event({one});
                CallDecl c;
                c.fn = FN_DOWN; c.layer = l; c.stage = stage++;      // task record: (first row tile, K slice, tiles)
                c.rank = 2; c.shape[0] = dim_const(n_ht / pass_d); c.shape[1] = dim_const(g.k_slices_d);
                c.c_mul[0] = pass_d; c.c_fill[2] = pass_d;
                c.flags = TF_K_SLICE;
                c.in = {edge_dim(e_act, 1)};                    // only the activations of its own K slice
                c.out = {edge_const0(e_dpart)};
                g.calls.push_back(c);
                CallDecl r;
                r.fn = FN_DOWN_SUM; r.layer = l; r.stage = stage++;
                r.rank = 1; r.shape[0] = dim_const(n_ht);
                r.flags = last;
                r.in = {edge_const0(e_dpart)};
                r.out = {edge_const0(e_xnext)};
                g.calls.push_back(r);
            } else {
                CallDecl c;
                c.fn = FN_DOWN; c.layer = l; c.stage = stage++;
                c.rank = 1; c.shape[0] = dim_const(n_ht);
                c.flags = (uint16_t)(TF_WAIT0_PER_WAVE | last);
                c.in = {edge_const0(e_act)};                    // wave w waits on e_act[w]
                c.out = {edge_const0(e_xnext)};
                g.calls.push_back(c);
            }
        } else {
            // MoE block (Sec. 2.4).  Static scheduling cannot follow the data-dependent edges
            // (token -> expert -> row tiles), so they collapse to one coarse event each ("E[0]",
            // Sec. 3.1): every GroupGEMM-1 tile waits for ALL router tiles, every combine tile for ALL
            // GroupGEMM-2 tiles.  The row-tile slots themselves are static, so GroupGEMM-1 ->
            // GroupGEMM-2 stays fine-grained: one event per slot.
            const int r_max = moe_max_row_tiles(m.E, m.topk, Bs, m.tile_m);
            const int n_ft = m.moeF / 8;
            // Row tiles per GroupGEMM task: what a queue takes longest over, in bytes: rounds x (fixed cost of a task +
            // tiles x bytes of a tile).  The fixed cost (slot look-up, operand gather, first chunk, epilogue, drain:
            // about 15 us) is worth 384 KB of streaming; rounds = tasks per queue, rounded up (the stage ends with
            // the queue that holds most).  Against "about three tasks per queue": Qwen3-30B-A3B shape, batch 4 9.4 -> 7.6 ms
            // per step, batch 8 12.0 -> 11.1, batch 16 .. 64 unchanged.
            auto tiles_per_task = [&](int per_slot, long long tile_bytes) {
                long long best = -1;
                int best_r = 1;
                const long long cap = 1LL << 20;      // a task streams at most 1 MB (measured on the Qwen3-30B-A3B shape, batch 4 .. 64:
                                                      // above that the rounds the model saves cost more in passes and imbalance)
                for (int r = 1; r <= per_slot; ++r) {
                    if (per_slot % r) continue;
                    if (r > 1 && r * tile_bytes > cap) continue;
                    const long long tasks = (long long)r_max * (per_slot / r), rounds = (tasks + n_queues - 1) / n_queues;
                    const long long cost = rounds * (384LL * 1024 + r * tile_bytes);
                    if (best < 0 || cost < best) { best = cost; best_r = r; }
                }
                return best_r;
            };
            const int r_g = tiles_per_task(n_ft, 16LL * m.H * 2), r_d = tiles_per_task(n_ht, 16LL * m.moeF * 2);
            const int e_logits = g.add_event({one});
            const int e_group = g.add_event({one});
            const int e_eact = g.add_event({dim_const(r_max)});
            const int e_y = g.add_event({one});
            {
                CallDecl c;
                c.fn = FN_ROUTER_LOGITS; c.layer = l; c.stage = stage++;
                c.rank = 1; c.shape[0] = dim_const(m.E / 16);
                c.in = {edge_const0(e_xmid)};
                c.out = {edge_const0(e_logits)};
                g.calls.push_back(c);
            }
            {
                CallDecl c;
                c.fn = FN_ROUTER; c.layer = l; c.stage = stage++;
                c.rank = 1; c.shape[0] = B;
                c.in = {edge_const0(e_logits)};
                c.out = {edge_const0(e_group)};
                g.calls.push_back(c);
            }
            {
                CallDecl c;
                c.fn = FN_MOE_GATEUP; c.layer = l; c.stage = stage++;     // task record: (row-tile slot, first tile, tiles)
                c.rank = 2; c.shape[0] = dim_const(r_max); c.shape[1] = dim_const(n_ft / r_g);
                c.c_mul[1] = r_g; c.c_fill[2] = r_g;
                c.flags = TF_DYN_ROWTILE;
                c.in = {edge_const0(e_group)};
                c.out = {edge_dim(e_eact, 0)};
                g.calls.push_back(c);
            }
            {
                CallDecl c;
                c.fn = FN_MOE_DOWN; c.layer = l; c.stage = stage++;
                c.rank = 2; c.shape[0] = dim_const(r_max); c.shape[1] = dim_const(n_ht / r_d);
                c.c_mul[1] = r_d; c.c_fill[2] = r_d;
                c.flags = TF_DYN_ROWTILE;
                c.in = {edge_dim(e_eact, 0)};
                c.out = {edge_const0(e_y)};
                g.calls.push_back(c);
            }
            {
                CallDecl c;
                c.fn = FN_COMBINE; c.layer = l; c.stage = stage++;        // task record: (token, chunk of 512 elements)
                c.rank = 2; c.shape[0] = B; c.shape[1] = dim_const((m.H + kWgThreads - 1) / kWgThreads);
                c.flags = last;
                c.in = {edge_const0(e_y)};
                c.out = {edge_const0(e_xnext)};
                g.calls.push_back(c);
            }
        }
        e_x = e_xnext;
    }
    if (m.vocab > 0) {
        // End of the iteration: final RMSNorm (folded into the projection like every other norm), vocabulary
        // projection and greedy token.  A projection task streams consecutive 16-row tiles of the matrix, about
        // one task per queue on the staged path; the last task is ragged.  Each tile folds its best (logit, id)
        // into the sequence's running maximum, so the sampling task that follows reads one word per sequence.
        if (m.vocab % 16) return "vocab must be a multiple of 16";
        const int tiles = m.vocab / 16;
        int r_lm = pass_tiles;
        if (staged_fits(1, Bs, m.H)) {
            r_lm = std::max(1, (tiles + n_queues - 1) / std::max(1, n_queues));
            while (r_lm > 1 && !staged_fits(r_lm, Bs, m.H)) --r_lm;
        }
        g.all_staged = g.all_staged && staged_fits(r_lm, Bs, m.H);
        const int e_logits = g.add_event({one});
        const int e_tok = g.add_event({one});
        {
            CallDecl c;
            c.fn = FN_LMHEAD; c.layer = m.n_layers - 1; c.stage = stage++;      // task record: (first tile, tiles at most)
            c.rank = 1; c.shape[0] = dim_const((tiles + r_lm - 1) / r_lm);
            c.c_mul[0] = r_lm; c.c_fill[1] = r_lm;
            c.in = {edge_const0(e_x)};
            c.out = {edge_const0(e_logits)};
            g.calls.push_back(c);
        }
        {
            CallDecl c;
            c.fn = FN_SAMPLE; c.layer = m.n_layers - 1; c.stage = stage++;
            c.rank = 1; c.shape[0] = one;
            c.in = {edge_const0(e_logits)};
            c.out = {edge_const0(e_tok)};
            g.calls.push_back(c);
        }
    }
    return "";
}

// x + MoE(rmsnorm(x)) over T tokens.  Routing and grouping run as three counting passes over blocks of 64 tokens
// (top-k and per-block expert histogram; one scan over experts and blocks; stable rank inside the block), so the work
// is linear in the tokens; the GroupGEMM grids are the row-tile slots of the decoder's MoE block (reading 19).
std::string build_moe_layer_graph(const ModelDims &m, int Ts, int n_queues, GraphDecl *out)
{
    GraphDecl &g = *out;
    g = GraphDecl();
    if (Ts < 1 || Ts > kMoeLayerMaxTokens) return "tokens must be in 1..4096";
    if (m.H % (kWaves * 32)) return "hidden must be a multiple of 256";
    if (m.E < 16 || m.E % 16 || m.E > kMaxExperts) return "n_experts must be a multiple of 16, at most 256";
    if (m.topk < 1 || m.topk > kMaxTopK || m.topk > m.E) return "top_k must be in 1..16 and at most n_experts";
    if (m.moeF < 1 || m.moeF % (kWaves * 32)) return "moe_ffn must be a multiple of 256";
    if (m.tile_m < 1 || m.tile_m > 64) return "tile_m must be in 1..64";
    const DimExpr one = dim_const(1);
    const int n_blk = (Ts + 63) / 64, n_ht = m.H / 16, n_ft = m.moeF / 8;
    const int r_max = moe_max_row_tiles(m.E, m.topk, Ts, m.tile_m);
    auto tiles_per_task = [&](int per_slot) {
        const long long total = (long long)r_max * per_slot;
        const long long want = total <= 4LL * n_queues ? n_queues : 3LL * n_queues;
        int cand = (int)std::max(1LL, total / std::max(1LL, want));
        cand = std::min(cand, per_slot);
        while (cand > 1 && per_slot % cand) --cand;
        // full row tiles of more than 32 tokens take the wide path, whose pass is 16 row tiles: whole passes, if any
        if (m.tile_m > 32 && Ts >= 512 && cand >= 16) {
            int c16 = cand / 16 * 16;
            while (c16 >= 16 && per_slot % c16) c16 -= 16;
            if (c16 >= 16) cand = c16;
        }
        return std::max(1, cand);
    };
    const int r_g = tiles_per_task(n_ft), r_d = tiles_per_task(n_ht);
    const int e_x = g.add_event({one});
    const int e_logits = g.add_event({dim_const(n_blk)});
    const int e_hist = g.add_event({one});
    const int e_scan = g.add_event({one});
    const int e_group = g.add_event({one});
    const int e_eact = g.add_event({dim_const(r_max)});
    const int e_y = g.add_event({one});
    const int e_out = g.add_event({one});
    int stage = 0;
    {
        CallDecl c;
        c.fn = FN_MOEL_LOAD; c.stage = stage++;
        c.rank = 1; c.shape[0] = dim_const((Ts + 15) / 16);
        c.out = {edge_const0(e_x)};
        g.calls.push_back(c);
    }
    {
        CallDecl c;
        c.fn = FN_ROUTER_LOGITS; c.stage = stage++;      // task record: (16 router rows, block of 64 tokens)
        c.rank = 2; c.shape[0] = dim_const(m.E / 16); c.shape[1] = dim_const(n_blk);
        c.in = {edge_const0(e_x)};
        c.out = {edge_dim(e_logits, 1)};
        g.calls.push_back(c);
    }
    {
        CallDecl c;
        c.fn = FN_MOEL_TOPK; c.stage = stage++;
        c.rank = 1; c.shape[0] = dim_const(n_blk);
        c.in = {edge_dim(e_logits, 0)};
        c.out = {edge_const0(e_hist)};
        g.calls.push_back(c);
    }
    {
        CallDecl c;
        c.fn = FN_MOEL_SCAN; c.stage = stage++;
        c.rank = 1; c.shape[0] = one;
        c.in = {edge_const0(e_hist)};
        c.out = {edge_const0(e_scan)};
        g.calls.push_back(c);
    }
    {
        CallDecl c;
        c.fn = FN_MOEL_PLACE; c.stage = stage++;
        c.rank = 1; c.shape[0] = dim_const(n_blk);
        c.in = {edge_const0(e_scan)};
        c.out = {edge_const0(e_group)};
        g.calls.push_back(c);
    }
    {
        CallDecl c;
        c.fn = FN_MOE_GATEUP; c.stage = stage++;     // task record: (row-tile slot, first tile, tiles)
        c.rank = 2; c.shape[0] = dim_const(r_max); c.shape[1] = dim_const(n_ft / r_g);
        c.c_mul[1] = r_g; c.c_fill[2] = r_g;
        c.flags = TF_DYN_ROWTILE;
        c.in = {edge_const0(e_group)};
        c.out = {edge_dim(e_eact, 0)};
        g.calls.push_back(c);
    }
    {
        CallDecl c;
        c.fn = FN_MOE_DOWN; c.stage = stage++;
        c.rank = 2; c.shape[0] = dim_const(r_max); c.shape[1] = dim_const(n_ht / r_d);
        c.c_mul[1] = r_d; c.c_fill[2] = r_d;
        c.flags = TF_DYN_ROWTILE;
        c.in = {edge_dim(e_eact, 0)};
        c.out = {edge_const0(e_y)};
        g.calls.push_back(c);
    }
    {
        CallDecl c;
        // task record: (first token, chunk of 2048 elements, tokens): blocks of tokens, about two tasks per queue
        const int n_ch = (m.H + 4 * kWgThreads - 1) / (4 * kWgThreads);
        int tb = std::max(1, Ts * n_ch / std::max(1, 2 * n_queues));
        tb = std::min(tb, 16);
        c.fn = FN_COMBINE; c.stage = stage++;
        c.rank = 2; c.shape[0] = dim_const((Ts + tb - 1) / tb); c.shape[1] = dim_const(n_ch);
        c.c_mul[0] = tb; c.c_fill[2] = tb;
        c.flags = TF_LAST_LAYER;
        c.in = {edge_const0(e_y)};
        c.out = {edge_const0(e_out)};
        g.calls.push_back(c);
    }
    return "";
}

}  // namespace etc
