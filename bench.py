#!/usr/bin/env python3
"""Decode-step benchmark of the event-tensor megakernel on one MI355X.

Workload (the configuration the headline metric is quoted on): Llama-3-8B-shaped decoder, 32 layers,
random-init bf16 weights, batch 1, 1024 cached tokens in 16-token pages behind a random permuted page
table, LM head excluded.  One step = one launch of the persistent megakernel = the whole hot path.
Prints ONE JSON line (see the keys below); inputs are resident in HBM before the timed region.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0       # dense bf16 matrix-core peak of MI355X
T_PROCESS_START = time.time()


FN_NAMES = {3: "load_hidden", 4: "qkv", 5: "attn_chunk", 6: "attn_merge", 7: "o_proj", 8: "gate_up", 9: "down",
            10: "router_logits", 11: "router", 12: "moe_gate_up", 13: "moe_down", 14: "combine", 15: "o_proj_sum",
            16: "down_sum"}


def print_timeline(dec, etc, shape, args, B, L, f):
    """Per stage of one layer, from the per-task device trace of the last launch: number of tasks and queues
    (= compute units) that ran them, first task start, last weight-loop start, last loop end, last notify (us
    from the layer's first task start), the weight bytes the stage streams and the rate over its span."""
    import numpy as np
    info = dec.step_info()
    tr = dec.task_trace().astype(np.int64)
    plan = etc.plan_build(shape, args.kv_chunk, info.sampled_batch, int(info.n_queues), L + 1, kind=dec.kind)
    tasks = plan["tasks"]
    khz = float(info.wall_clock_khz)
    us = lambda t: t / khz * 1e3                                     # noqa: E731
    layer = args.timeline
    sel_l = (tasks["layer"] == layer) & (tasks["fn"] != 3) & (tr[tasks["id"], 0] > 0)
    t0 = tr[tasks["id"][sel_l], 0].min()
    H, QD, KD, F = shape.H, shape.nq * shape.d, shape.nkv * shape.d, shape.F
    wbytes = {4: 2 * H * (QD + 2 * KD), 7: 2 * H * QD, 8: 4 * F * H, 9: 2 * F * H, 5: 4 * KD * (L + 1) * B}
    print(f"# per-stage timeline, layer {layer}, {shape.name} batch {B} kv_len {L}, scheduler {args.sched}; times in us "
          f"from the layer's first task start", file=f)
    print("| stage | tasks | CUs | first start | events seen p50 / max | loop start p50 / max | loop end p50 / max | notify p50 / max | MB | GB/s over span |", file=f)
    print("|---|---|---|---|---|---|---|---|---|---|", file=f)
    end_prev = 0.0
    for fn in sorted(set(tasks["fn"][sel_l].tolist())):
        sel = sel_l & (tasks["fn"] == fn)
        T = tr[tasks["id"][sel]]
        first, notified = us(T[:, 0].min() - t0), us(T[:, 5].max() - t0)
        def p50max(col):
            v = T[:, col][T[:, col] > 0]
            return f"{us(np.median(v) - t0):.1f} / {us(v.max() - t0):.1f}" if len(v) else "-"
        mb = wbytes.get(fn, 0) / 1e6
        rate = f"{wbytes[fn] / ((notified - first) * 1e-6) / 1e9:.0f}" if fn in wbytes and notified > first else "-"
        print(f"| {FN_NAMES.get(fn, fn)} | {int(sel.sum())} | {len(set(T[:, 7].tolist()))} | {first:.1f} | {p50max(1)} | {p50max(2)} | "
              f"{p50max(3)} | {p50max(5)} | {mb:.1f} | {rate} |", file=f)
        end_prev = max(end_prev, notified)
    nxt = (tasks["layer"] == layer + 1) & (tr[tasks["id"], 0] > 0)
    if nxt.any():
        print(f"layer span (first task start of this layer to first task start of the next): "
              f"{us(tr[tasks['id'][nxt], 0].min() - t0):.1f} us; last notify of the layer at {end_prev:.1f} us", file=f)
    print(f"whole step: {us(tr[:, 5].max() - tr[:, 0][tr[:, 0] > 0].min()):.1f} us (with tracing on)", file=f)


def bench_moe_layer(args) -> int:
    """The MoE layer on its own (paper Sec. 4.2 / 4.5, the token sweep of the ablation): Qwen3-30B-A3B layer shape,
    --batch tokens, one launch per step.  Reports the step time, the HBM fraction on the algorithmic bytes (weights of
    the routed experts once, tokens in and out) and the matrix-core fraction on the algorithmic flops."""
    import numpy as np
    import torch

    import paper_2604_13327_amd as etc
    import synth
    from synth.workloads import weight_specs

    s, T = synth.QWEN3_30B_A3B, args.batch
    torch.manual_seed(2024)
    w = {name: torch.empty(shp, dtype=torch.bfloat16, device="cuda").normal_(mean, sigma)
         for name, shp, mean, sigma in weight_specs(s) if name in ("g2", "wr", "eg", "eu", "ed")}
    x = torch.empty(T, s.H, dtype=torch.bfloat16, device="cuda").normal_()
    y = torch.empty_like(x)
    kind = {"static": etc.SCHED_STATIC, "dynamic": etc.SCHED_DYNAMIC, "unfused": etc.SCHED_UNFUSED}[args.sched]
    layer = etc.MoeLayer(s, [T], kind=kind, moe_tile_m=args.moe_tile_m, debug_flags=etc.DEBUG_ROUTING)
    layer.bind_weights(w)
    layer.bind_tokens(T)
    launch = layer.launch_kernel_by_kernel if args.kernel_by_kernel else layer.launch
    for _ in range(args.warmup + 1):
        launch(x, y)
    torch.cuda.synchronize()
    assert (layer.error_word() == 0).all()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a, b in ev:
        a.record()
        launch(x, y)
        b.record()
    torch.cuda.synchronize()
    per = np.array([a.elapsed_time(b) * 1e3 for a, b in ev])
    us = float(ev[0][0].elapsed_time(ev[-1][1]) * 1e3 / args.steps)
    from paper_2604_13327_amd import binding as b_
    ids = layer.routing_debug(b_.DBG_TOPK_IDS, 0, (T, s.top_k), np.int32)
    n_exp = int(len(np.unique(ids)))
    tiles = int(layer.routing_debug(b_.DBG_EXP_INDPTR, 0, (s.n_experts + 1,), np.int32)[-1])
    alg_bytes = 2 * (s.H + s.n_experts * s.H + n_exp * 3 * s.moe_F * s.H) + 4 * T * s.H
    flops = T * (2 * s.H * s.n_experts + s.top_k * 3 * 2 * s.H * s.moe_F)
    info = layer.step_info()
    kern_us = float(per.mean())
    hbm = alg_bytes / (kern_us * 1e-6) / 1e9
    tfl = flops / (kern_us * 1e-6) / 1e12
    bound = "mfma" if tfl / MFMA_BF16_PEAK_TFLOPS > hbm / HBM_PEAK_GBS else "hbm"
    result = {
        "metric": "moe_layer_latency_us", "value": round(us, 2), "unit": "us", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(us / 1e3, 5), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic (torch generator)",
        "config": {"workload": f"qwen3-30b-a3b MoE layer, {T} tokens, row tiles of {args.moe_tile_m}",
                   "scheduler": args.sched + (" (kernel by kernel)" if args.kernel_by_kernel else ""),
                   "tasks_per_step": int(info.n_tasks), "events_per_step": int(info.n_events),
                   "experts_routed": n_exp, "row_tiles": tiles},
        "tokens_per_s": round(T / (us * 1e-6), 1),
        "roofline": {"bound": bound, "kernel": "megakernel_dynamic" if args.sched == "dynamic" else "megakernel_static",
                     "achieved": round(tfl, 2) if bound == "mfma" else round(hbm, 1),
                     "peak": MFMA_BF16_PEAK_TFLOPS if bound == "mfma" else HBM_PEAK_GBS,
                     "unit": "TFLOP/s" if bound == "mfma" else "GB/s",
                     "frac": round(tfl / MFMA_BF16_PEAK_TFLOPS if bound == "mfma" else hbm / HBM_PEAK_GBS, 4),
                     "hbm_gbs": round(hbm, 1), "hbm_frac": round(hbm / HBM_PEAK_GBS, 4), "tflops": round(tfl, 2),
                     "mfma_frac": round(tfl / MFMA_BF16_PEAK_TFLOPS, 4), "algorithmic_bytes_per_launch": int(alg_bytes),
                     "algorithmic_flops_per_launch": int(flops), "avg_launch_us": round(kern_us, 2), "traffic": None},
    }
    layer.close()
    print(json.dumps(result))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="llama3-8b",
                    help="llama3-8b (headline) | any shape of synth.SHAPES | moe-layer (the MoE layer alone, --batch tokens)")
    ap.add_argument("--sched", default="static", choices=["static", "dynamic", "unfused"])
    ap.add_argument("--kv-len", type=int, default=1024)
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--kv-chunk", type=int, default=128, help="smallest number of keys per split-KV attention task")
    ap.add_argument("--moe-tile-m", type=int, default=64, help="moe-layer workload: tokens per GroupGEMM row tile")
    ap.add_argument("--kernel-by-kernel", action="store_true", help="moe-layer workload: one launch per stage")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-comparators", action="store_true")
    ap.add_argument("--cpu-layers", type=int, default=0, help="layers the CPU oracle runs (0 = all)")
    ap.add_argument("--timeline", type=int, default=-1, metavar="LAYER",
                    help="also print a per-stage timeline of that layer from the per-task device trace (to stderr)")
    ap.add_argument("--bind-every-step", action="store_true",
                    help="also time a chain of steps whose kv_len grows by one, each bound before its launch")
    ap.add_argument("--fast-fill", action="store_true",
                    help="fill weights and KV pool with torch's own normal generator (same distributions, not the seeded "
                         "generator the oracle shares: timing / counter runs only, no parity leg)")
    ap.add_argument("--launch-at", type=float, default=0.0, metavar="SECONDS",
                    help="sleep until that many seconds after process start before the first launch (lets a profiler's "
                         "collection period skip the synthetic weight fill)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures the one-GPU path only (this build has no multi-GPU sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2604_13327_amd as etc
    import synth
    from harness import GpuModel, bf16_to_f32_np, fixed_step, rel_err

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.workload == "moe-layer":
        return bench_moe_layer(args)
    shape = synth.SHAPES[args.workload]
    seed, B, L = 2024, args.batch, args.kv_len
    n_pool = B * synth.pages_needed(L, shape.page) + 16

    t0 = time.time()
    if args.fast_fill:
        args.no_cpu_baseline = True

        class FastModel(GpuModel):               # same tensors, values from torch's generator
            def __init__(self, shape, seed, n_pool_pages):
                torch.manual_seed(seed)
                self.shape, self.seed, self.n_pool_pages, self.device = shape, seed, n_pool_pages, "cuda"
                self.weights = [{name: torch.empty(shp, dtype=torch.bfloat16, device="cuda").normal_(mean, sigma)
                                 for name, shp, mean, sigma in synth.weight_specs(shape)} for _ in range(shape.n_layers)]
                pshape = (shape.n_layers,) + synth.kv_pool_shape(shape, n_pool_pages)
                self.kpool = torch.empty(pshape, dtype=torch.bfloat16, device="cuda").normal_()
                self.vpool = torch.empty(pshape, dtype=torch.bfloat16, device="cuda").normal_()

            def reset_pools(self):
                pass

            def hidden(self, step_index, batch):
                return torch.empty(batch, self.shape.H, dtype=torch.bfloat16, device="cuda").normal_()
        model = FastModel(shape, seed, n_pool)
    else:
        model = GpuModel(shape, seed, n_pool)
    torch.cuda.synchronize()
    t_fill = time.time() - t0

    if args.launch_at > 0:
        time.sleep(max(0.0, args.launch_at - (time.time() - T_PROCESS_START)))

    # ---- warm-up in the paper's sense (Sec. 4.4): engine start to first step served, minus model load
    t0 = time.time()
    kind = {"static": etc.SCHED_STATIC, "dynamic": etc.SCHED_DYNAMIC, "unfused": etc.SCHED_UNFUSED}[args.sched]
    dec = etc.Decoder(shape, kv_chunk_tokens=args.kv_chunk, sampled_batches=[B], max_kv_len=L + 1, kind=kind)
    model.bind(dec)
    step = fixed_step(shape, B, [L] * B, n_pool, seed=7)
    dec.bind_step(step)
    x = model.hidden(0, B)
    out = torch.empty_like(x)
    dec.launch(x, out)
    torch.cuda.synchronize()
    t_warmup = time.time() - t0
    first_out = bf16_to_f32_np(out)
    info = dec.step_info()

    def timed(launch, steps, warmup):
        for _ in range(warmup):
            launch(x, out)
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t_a = time.perf_counter()
        for a, b in ev:
            a.record()
            launch(x, out)
            b.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t_a) / steps * 1e6
        per = np.array([a.elapsed_time(b) * 1e3 for a, b in ev])          # us, device time per launch
        span = ev[0][0].elapsed_time(ev[-1][1]) * 1e3 / steps              # us per step over the whole region
        return per, span, wall

    per, span, wall = timed(dec.launch, args.steps, args.warmup)
    us = float(span)                       # whole timed region / K: what a serving loop would see
    kern_us = float(per.mean())            # average device duration of the megakernel launch
    alg = int(info.algorithmic_bytes)
    achieved = alg / (kern_us * 1e-6) / 1e9

    result = {
        "metric": "decode_step_latency_us", "value": round(us, 2), "unit": "us", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(us / 1e3, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic (torch generator)" if args.fast_fill else "synthetic",
        "config": {"workload": f"{shape.name} decode, batch {B}, kv_len {L}, page 16, random page table, "
                               f"{shape.n_layers} layers, LM head excluded",
                   "scheduler": args.sched, "kv_chunk_tokens": args.kv_chunk,
                   "tasks_per_step": int(info.n_tasks), "events_per_step": int(info.n_events),
                   "persistent_workgroups": int(info.n_queues)},
        "tokens_per_s": round(B / (us * 1e-6), 1),
        "latency_us": {"median": round(float(np.median(per)), 2), "p10": round(float(np.percentile(per, 10)), 2),
                       "p90": round(float(np.percentile(per, 90)), 2), "host_wall_per_step": round(wall, 2)},
        "roofline": {"bound": "hbm", "kernel": "megakernel_dynamic" if args.sched == "dynamic" else "megakernel_static", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "algorithmic_bytes_per_launch": alg, "avg_launch_us": round(kern_us, 2), "traffic": None},
        "warmup_s": {"create_bind_first_step": round(t_warmup, 3), "synthetic_weight_fill": round(t_fill, 3)},
    }

    # HBM traffic of this workload as last measured with rocprofv3 --pmc (see profiles/); null if never measured
    try:
        tr = json.load(open(os.path.join(ROOT, "paper_2604_13327_amd", "measured_traffic.json")))
        key = f"{shape.name}/{args.sched}/b{B}/kv{L}"
        if key in tr:
            result["roofline"]["traffic"] = tr[key]["fetch_bytes"] + tr[key]["write_bytes"]
            result["roofline"]["traffic_source"] = tr[key]["source"]
            result["roofline"]["traffic_measured_at_commit"] = tr[key].get("measured_at_commit")
    except OSError:
        pass

    if args.calib_copy:      # a plain copy kernel of known size: 2^30 bytes read, 2^30 bytes written
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        result["calib_copy_bytes"] = 1 << 30
        del src, dst

    # ---- per-stage timeline of one layer from the per-task device trace -------------------------------------
    if args.timeline >= 0:
        tdec = etc.Decoder(shape, kv_chunk_tokens=args.kv_chunk, sampled_batches=[B], max_kv_len=L + 1, kind=kind,
                           debug_flags=etc.DEBUG_TRACE)
        model.bind(tdec)
        tdec.bind_step(step)
        for _ in range(3):
            tdec.launch(x, out)
        torch.cuda.synchronize()
        print_timeline(tdec, etc, shape, args, B, L, sys.stderr)
        tdec.close()

    # ---- comparators on identical task bodies -------------------------------------------------------
    if not args.no_comparators:
        k = max(5, min(20, args.steps))
        per_kbk, span_kbk, _ = timed(dec.launch_kernel_by_kernel, k, 2)
        result["kernel_by_kernel_us"] = round(float(span_kbk), 2)
        result["launch_gap_removed_us"] = round(float(span_kbk) - us, 2)
        if args.sched == "static":
            un = etc.Decoder(shape, kv_chunk_tokens=args.kv_chunk, sampled_batches=[B], max_kv_len=L + 1,
                             kind=etc.SCHED_UNFUSED)
            model.bind(un)
            un.bind_step(step)
            _, span_un, _ = timed(un.launch, k, 2)
            result["unfused_megakernel_us"] = round(float(span_un), 2)
            result["speedup_vs_unfused"] = round(float(span_un) / us, 4)
            un.close()
            # the dynamic scheduler (Alg. 2) on the same task bodies: its time, and that its output is the same bits
            try:
                dy = etc.Decoder(shape, kv_chunk_tokens=args.kv_chunk, sampled_batches=[B], max_kv_len=L + 1,
                                 kind=etc.SCHED_DYNAMIC)
                model.bind(dy)
                dy.bind_step(step)
                out_dy = torch.empty_like(x)
                dy.launch(x, out_dy)
                torch.cuda.synchronize()
                result["dynamic_matches_static_bitwise"] = bool((bf16_to_f32_np(out_dy) == first_out).all())
                _, span_dy, _ = timed(dy.launch, k, 2)
                result["dynamic_megakernel_us"] = round(float(span_dy), 2)
                dy.close()
            except etc.EtcError as err:          # a comparator must not cost the headline line
                result["dynamic_megakernel_error"] = str(err)

    # ---- the whole decode iteration (Sec. 4.2 measures iterations: token in, layers, sampling, token out) ------
    # The same step with embedding look-up, final norm, vocabulary projection and greedy token inside the
    # megakernel, each launch reading the token the previous one wrote (no host round trip).
    vocab = {"llama3-8b": 128256, "llama3-70b": 128256, "qwen3-32b": 151936, "qwen3-30b-a3b": 151936, "tiny": 1024}.get(args.workload, 0)
    if not args.no_comparators and vocab:
        import dataclasses
        from synth import gpu as sgpu
        shape_lm = dataclasses.replace(shape, vocab=vocab)
        if args.fast_fill:
            lm = {n: torch.empty(shp, dtype=torch.bfloat16, device="cuda").normal_(mean, sigma)
                  for n, shp, mean, sigma in synth.lm_specs(shape_lm)}
        else:
            lm = sgpu.lm_weights_gpu(shape_lm, seed)
        it = etc.Decoder(shape_lm, kv_chunk_tokens=args.kv_chunk, sampled_batches=[B], max_kv_len=L + 1, kind=kind)
        model.bind(it)
        it.bind_lm_head(lm["embed"], lm["gf"], lm["wlm"])
        it.bind_step(step)
        toks = torch.randint(0, vocab, (2, B), dtype=torch.int32, device="cuda")
        flip = [0]

        def iteration(_x, _out):
            it.launch_tokens(toks[flip[0] ^ 1], token_in=toks[flip[0]])
            flip[0] ^= 1
        k = max(5, min(20, args.steps))
        _, span_it, _ = timed(iteration, k, 2)
        lm_bytes = vocab * shape.H * 2
        result["iteration_with_sampling_us"] = round(float(span_it), 2)
        result["lm_head_and_sampling_us"] = round(float(span_it) - us, 2)
        result["lm_head_gbs"] = round(lm_bytes / max(1e-9, (float(span_it) - us) * 1e-6) / 1e9, 1)
        result["iteration_hbm_frac"] = round((alg + lm_bytes) / (float(span_it) * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
        assert (it.error_word() == 0).all()
        it.close()
        del lm

    # ---- the cost of binding a step on the real per-step path: kv_len grows by one every step -------------
    # (last of the GPU measurements: these steps append rows at other positions of the KV pool)
    if args.bind_every_step or not args.no_comparators:
        K = args.steps
        chain = [fixed_step(shape, B, [max(0, L - K + 1 + i)] * B, n_pool, seed=7) for i in range(K)]
        for st_ in chain[:3]:
            dec.bind_step(st_)
            dec.launch(x, out)
        torch.cuda.synchronize()
        # host cost of one bind (validation, copy into pinned staging; no device call), device idle
        t_bind = 0.0
        for st_ in chain[: min(K, 20)]:
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            dec.bind_step(st_)
            t_bind += time.perf_counter() - t1
            dec.launch(x, out)
        torch.cuda.synchronize()
        result["bind_step_us"] = round(t_bind / min(K, 20) * 1e6, 2)
        # the serving loop: bind, launch, bind, launch ... with no synchronisation in between
        ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ea.record()
        for st_ in chain:
            dec.bind_step(st_)
            dec.launch(x, out)
        eb.record()
        torch.cuda.synchronize()
        result["step_incl_bind_us"] = round(float(ea.elapsed_time(eb) * 1e3 / K), 2)
        dec.bind_step(step)

    # ---- CPU oracle on the host cores: reported baseline + end-to-end parity of this very workload ----
    if not args.no_cpu_baseline:
        import oracle
        n_l = args.cpu_layers if args.cpu_layers > 0 else shape.n_layers
        xo = synth.hidden_f32(shape, seed, 0, B)
        oshape = oracle.shape_of(shape)
        t_orc = 0.0
        for l in range(n_l):
            w = synth.layer_weights_f32(shape, seed, l)
            kp, vp = synth.kv_pool_f32(shape, seed, l, n_pool)
            t1 = time.perf_counter()
            oracle.layer(oshape, xo, w, kp, vp, step.kv_len, step.page_indptr, step.page_ids)
            t_orc += time.perf_counter() - t1
        scale = shape.n_layers / n_l
        result["cpu_baseline"] = {"value": round(t_orc * scale * 1e6, 1), "unit": "us", "cores": oracle.n_threads(),
                                  "kind": "oracle",
                                  "sample": f"{n_l} of {shape.n_layers} layers of the same step, oracle compute only "
                                            f"(input generation excluded), scaled x{scale:g}"}
        if n_l == shape.n_layers:
            result["parity_vs_oracle_final"] = round(rel_err(first_out, xo), 5)

    dec.close()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
