#!/usr/bin/env python3
"""Benchmark of the MoE draft+verify layer on one MI355X.

One *step* is one speculative cycle of one MoE layer (every row of the hot path once):
K draft calls (moe_draft_layer_int4, one token each, int4 experts, expert ids written into the
window buffer), one moe_expert_union over the window's ids against the slot table, and one
moe_verify_layer_bf16 over the K+1 tokens (bf16 experts through the slot table).  Successive
steps rotate over a stack of distinct layers so that weights come from HBM, not from a cache.

For a workload whose experts are not all resident (dsv2lite: 16 of 64 per layer) a step is the
same cycle of one layer inside a whole-stack cycle: all layers draft first, the experts the
union reports missing are copied from pinned host memory on a side stream
(moe_expert_copy_async) while earlier layers verify, and experts that only the verify call
itself discovers are fetched on demand and added with an ACCUMULATE|ONLY_LISTED call.

Prints ONE JSON line: value = token passes per second = (K + K+1) / step time, with the
`roofline` of the kernel that takes the most time and the `cpu_baseline` (the fp64 oracle on
the host cores).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
METRIC = "MoE-layer draft+verify tokens/s and achieved HBM GB/s vs peak, 1 GPU"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(cfg, T, mean_u, symmetric=False):
    """Bytes the method has to move per call (selected experts' weights once + small operands)."""
    H, E, I, k, S, g = cfg.hidden, cfg.n_experts, cfg.inter, cfg.top_k, cfg.n_shared, cfg.group_size
    P = 3 * H * I
    int4_expert = P // 2 + (P // g) * (2 if symmetric else 4)      # codes + fp16 scale (+ fp16 zero)
    return {
        "draft_call": k * int4_expert + S * 2 * P + E * H * 2 + H * 2 + H * 4,              # one token
        "verify_call": mean_u * 2 * P + S * 2 * P + E * H * 2 + T * H * 4,
        "draft_fused_kernel": k * int4_expert + E * H * 2 + H * 2 + H * 4,
        "bf16_gateup_kernel": (mean_u + S) * (2 * H * I * 2) + T * H * 2,
        "bf16_down_kernel": (mean_u + S) * (H * I * 2) + T * k * I * 2,
    }


def roofline_table(cfg, kern, nbytes, root):
    """Per-kernel achieved GB/s from the event-pair times; returns (dominant entry, table)."""
    traffic = {}
    tpath = os.path.join(root, "profiles", "pmc_traffic.json")   # HBM bytes per launch from committed PMC runs
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(cfg.name, {})
        except Exception:
            traffic = {}
    table = {}
    for name in ("draft_fused_kernel", "bf16_gateup_kernel", "bf16_down_kernel"):
        kk = kern.get(name)
        if not kk or (cfg.n_shared > 0 and name != "draft_fused_kernel"):
            continue        # with shared experts the bf16 kernels also run inside draft calls
        ach = nbytes[name] / (kk["us_avg"] * 1e-6) / 1e9
        table[name] = {"kernel": name, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                       "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                       "traffic": traffic.get(name),
                       "traffic_source": "profiles/pmc_traffic.json: fabric-side FETCH_SIZE + WRITE_SIZE per launch from "
                                         "committed rocprofv3 --pmc runs of this command, not measured in this run"
                                         if traffic.get(name) else None,
                       "bytes_per_launch": int(nbytes[name]),
                       "us_per_launch": round(kk["us_avg"], 2), "launches": kk["launches"],
                       "ms_total": round(kk["ms_total"], 3)}
    dominant = max(table.values(), key=lambda r: r["ms_total"]) if table else None   # most time in the timed region
    return dominant, table


def read_profile(ctx):
    prof = ctx.profile_read()
    return {n: {"ms_total": ms, "launches": cnt, "us_avg": 1e3 * ms / cnt} for n, (ms, cnt) in prof.items() if cnt}


def cpu_baseline(cfg, L0, K, T):
    """The oracle as it stands on layer 0's step: about 10 s of host work on all threads the process
    has, then a few steps on one thread."""
    import synth
    from oracle import oracle as orc
    from oracle.layer_check import oracle_arrays, oracle_draft, oracle_verify
    A = oracle_arrays(L0)

    def run(budget_s, max_reps):
        tc = time.time()
        reps = 0
        while (time.time() - tc < budget_s and reps < max_reps) or reps == 0:
            x0 = synth.make_tokens(cfg, T, layer=0, step=reps)
            oracle_draft(A, x0[:K])
            oracle_verify(A, x0)
            reps += 1
        return reps, time.time() - tc
    threads = orc.num_threads()
    reps, dt = run(10.0, 64)
    orc.set_num_threads(1)
    reps1, dt1 = run(4.0, 8)
    orc.set_num_threads(threads)
    return {"value": round(reps * (2 * K + 1) / dt, 3), "unit": "tokens/s", "cores": threads,
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": "%d steps of layer 0 (fresh tokens each): %d draft tokens (int4) + one verify of %d "
                      "tokens (bf16) per step" % (reps, K, T),
            "single_thread": {"value": round(reps1 * (2 * K + 1) / dt1, 3), "unit": "tokens/s", "cores": 1,
                              "seconds": round(dt1, 2), "steps": reps1}}


def stream_ceiling(ctx, torch, blobs, nbytes, grid, reps=64):
    """moe_stream_read_probe over `nbytes` of each blob in turn (cold data every launch)."""
    sink = torch.zeros(1, dtype=torch.int32, device=blobs[0].device)
    nbytes = nbytes // 1024 * 1024
    for b in blobs:
        ctx.stream_read_probe(b, nbytes, grid, sink)
    torch.cuda.synchronize()
    ctx.profile_enable(True)
    for i in range(reps):
        ctx.stream_read_probe(blobs[i % len(blobs)], nbytes, grid, sink)
    torch.cuda.synchronize()
    kk = read_profile(ctx).get("stream_read_kernel")
    ctx.profile_enable(False)
    us = kk["us_avg"]
    return {"bytes": nbytes, "workgroups": grid, "us": round(us, 2), "GBs": round(nbytes / us / 1e3, 1)}


def emit(cfg, args, K, T, n_layers, ms_step, ms_eager, launch, mean_u, nbytes, roofline, cpu, extra):
    H, E, I, k, S, g = cfg.hidden, cfg.n_experts, cfg.inter, cfg.top_k, cfg.n_shared, cfg.group_size
    tokens = 2 * K + 1
    out = {
        "metric": METRIC, "value": round(tokens / (ms_step * 1e-3), 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int4+bf16 (fp32 accumulate)", "data": "synthetic",
        "config": {"workload": "%s-shaped MoE layer: H%d E%d I%d top%d g%d S%d, K=%d draft tokens + verify of %d, "
                               "%d distinct layers" % (cfg.name, H, E, I, k, g, S, K, T, n_layers),
                   "launch": launch, "tokens_per_step": tokens,
                   "mean_distinct_experts_per_verify": round(mean_u, 2)},
        "ms_per_step_eager": None if ms_eager is None else round(ms_eager, 4),
        "ms_per_step_hipgraph": extra.pop("ms_graph", None),
        "algorithmic_GBs_step": round((K * nbytes["draft_call"] + nbytes["verify_call"]) / (ms_step * 1e-3) / 1e9, 1),
        "roofline": roofline, "cpu_baseline": cpu,
    }
    out.update(extra)
    print(json.dumps(out), flush=True)


# ------------------------------------------------------------------------------------------------
def resident_leg(args, cfg, ctx, dev):
    """Every expert has a slot: K draft calls + union + verify per step, rotating over the layers."""
    import numpy as np
    import torch
    import synth
    from paper_2511_14102_amd.harness import DeviceLayer

    T = max(cfg.verify_tokens)
    K = T - 1
    n_layers = args.layers or cfg.bench_layers
    H, E, k = cfg.hidden, cfg.n_experts, cfg.top_k

    # ---- layers: layer 0 from the CPU streams (the oracle can see it), the rest drawn on the GPU
    t0 = time.time()
    layers, xs = [], []
    sym = args.int4 == "symmetric"
    L0 = synth.make_layer(cfg, 0, quant_device=dev, symmetric=sym)
    for li in range(n_layers):
        L = L0 if li == 0 else synth.make_layer(cfg, li, device=dev, symmetric=sym)
        layers.append(DeviceLayer(ctx, cfg, L, max_tokens=T, symmetric=sym))
        xs.append(synth.make_tokens(cfg, T, layer=li).to(dev))
        if li:
            del L
        if li % 4 == 0:
            log("  layer %d/%d on device (%.0f s)" % (li + 1, n_layers, time.time() - t0))
    torch.cuda.synchronize()
    log("setup %.1f s, %.1f GB allocated" % (time.time() - t0, torch.cuda.memory_allocated() / 1e9))

    # ---- static per-layer buffers
    bufs = []
    for li in range(n_layers):
        bufs.append(dict(
            yd=torch.empty((K, H), dtype=torch.float32, device=dev),
            win=torch.empty((K, k), dtype=torch.int32, device=dev),
            conf=torch.empty((K, k), dtype=torch.float32, device=dev),
            yv=torch.empty((T, H), dtype=torch.bfloat16, device=dev),
            idv=torch.empty((T, k), dtype=torch.int32, device=dev),
            mask=torch.empty((E + 63) // 64, dtype=torch.int64, device=dev),
            lst=torch.empty(E, dtype=torch.int32, device=dev),
            miss=torch.empty(E, dtype=torch.int32, device=dev),
            nl=torch.empty(1, dtype=torch.int32, device=dev),
            nm=torch.empty(1, dtype=torch.int32, device=dev)))

    def step(li):
        D, x, b = layers[li], xs[li], bufs[li]
        for i in range(K):
            D.draft(x[i:i + 1], y=b["yd"][i:i + 1], ids=b["win"][i:i + 1], conf=b["conf"][i:i + 1])
        ctx.expert_union(b["win"], K * k, E, D.slot_of_expert, b["mask"], b["lst"], b["nl"], b["miss"], b["nm"])
        D.verify(x, y=b["yv"], ids=b["idv"])

    def timed(fn, n_warm, n_steps, passes=5):
        """Median over `passes` timed passes of exactly n_steps steps each, after n_warm warm-up steps."""
        for i in range(n_warm):
            fn(i % n_layers)
        torch.cuda.synchronize()
        per_step = []
        for p in range(passes):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for i in range(n_steps):
                fn((n_warm + i) % n_layers)
            e1.record()
            torch.cuda.synchronize()
            per_step.append(e0.elapsed_time(e1) / n_steps)
        return float(np.median(per_step)), per_step

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ms_eager, passes_eager = timed(step, args.warmup, args.steps)
    log("eager: %.3f ms/step (passes: %s)" % (ms_eager, " ".join("%.3f" % v for v in passes_eager)))
    ms_step, launch = ms_eager, "eager"
    if args.mode == "graph":
        graphs = []
        side = torch.cuda.Stream()
        for li in range(n_layers):
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph, stream=side):
                step(li)
            graphs.append(gph)
        torch.cuda.synchronize()
        ms_graph, passes_graph = timed(lambda li: graphs[li].replay(), args.warmup, args.steps)
        log("graph: %.3f ms/step (passes: %s)" % (ms_graph, " ".join("%.3f" % v for v in passes_graph)))
        if ms_graph < ms_eager:
            ms_step, launch = ms_graph, "hipgraph"

    # ---- what the steps computed: distinct experts per verify call, from the ids of the layers the
    # timed steps ran on (weighted by how often each ran)
    torch.cuda.synchronize()
    ran = [(args.warmup + i) % n_layers for i in range(args.steps)]
    uniq = {li: len(set(bufs[li]["idv"].cpu().numpy().reshape(-1).tolist())) for li in sorted(set(ran))}
    mean_u = float(np.mean([uniq[li] for li in ran]))
    nbytes = algorithmic_bytes(cfg, T, mean_u, sym)

    # ---- per-kernel time (eager, event pairs around every kernel launch)
    roofline, extra = None, {}
    if sym:
        extra["int4_format"] = "symmetric (z = 8, scale blobs)"
    extra["timing"] = {"passes": 5, "ms_per_step_each_pass": [round(v, 4) for v in (passes_graph if launch == "hipgraph" else passes_eager)],
                       "reported": "median"}
    if args.mode == "graph":
        extra["ms_graph"] = round(ms_graph, 4)
    if not args.no_profile:
        ctx.profile_enable(True)
        for i in range(args.steps):
            step((args.warmup + i) % n_layers)
        torch.cuda.synchronize()
        kern = read_profile(ctx)
        ctx.profile_enable(False)
        roofline, table = roofline_table(cfg, kern, nbytes, ROOT)
        extra["kernels"] = table
        extra["kernel_us"] = {n: round(v["us_avg"], 2) for n, v in kern.items()}
        # the same bytes as one draft call, read by a kernel that only reads (practical ceiling)
        grid = k * cfg.inter // 32
        extra["stream_read_ceiling"] = stream_ceiling(ctx, torch, [D.q_blob for D in layers],
                                                      nbytes["draft_fused_kernel"], grid)
        # the same draft call with the layer changing from call to call: no expert is read twice within
        # the reach of the memory-side cache (in a step the K draft calls hit one layer, whose popular
        # expert may be served from that cache)
        ctx.profile_enable(True)
        for i in range(4 * n_layers):
            li = i % n_layers
            layers[li].draft(xs[li][i % K:i % K + 1], y=bufs[li]["yd"][0:1], ids=bufs[li]["win"][0:1], conf=bufs[li]["conf"][0:1])
        torch.cuda.synchronize()
        rot = read_profile(ctx).get("draft_fused_kernel")
        ctx.profile_enable(False)
        if rot:
            extra["draft_kernel_us_layer_rotating"] = round(rot["us_avg"], 2)
        extra["per_call"] = {
            "draft_us": round(kern["draft_fused_kernel"]["us_avg"], 2),
            "draft_tokens_per_s": round(1e6 / kern["draft_fused_kernel"]["us_avg"], 1),
            "verify_us": round(sum(kern[n]["us_avg"] for n in ("route_kernel", "plan_kernel", "bf16_gateup_kernel",
                                                                 "bf16_down_kernel", "combine_kernel") if n in kern), 2),
        }
        extra["per_call"]["verify_tokens_per_s"] = round(T * 1e6 / extra["per_call"]["verify_us"], 1)

    # ---- one isolated call, host clock from launch to completion (the per-call figures above are
    # kernel times of back-to-back launches)
    def latency(fn, reps=20):
        out = []
        for i in range(reps + 3):
            li = i % n_layers
            torch.cuda.synchronize()
            t = time.perf_counter()
            fn(li)
            torch.cuda.synchronize()
            if i >= 3:
                out.append((time.perf_counter() - t) * 1e6)
        return round(float(np.median(out)), 1)
    extra["single_call_latency_us"] = {
        "draft": latency(lambda li: layers[li].draft(xs[li][0:1], y=bufs[li]["yd"][0:1], ids=bufs[li]["win"][0:1], conf=bufs[li]["conf"][0:1])),
        "verify": latency(lambda li: layers[li].verify(xs[li], y=bufs[li]["yv"], ids=bufs[li]["idv"])),
        "note": "host wall clock of one call with a synchronise before and after, median of 20, layers rotating"}

    # ---- layer 0's step as the timed launches left it, against the oracle (same buffers, same path)
    if not args.no_cpu_baseline:
        from oracle.layer_check import oracle_arrays, oracle_draft, oracle_verify, rel_err
        step(0)
        torch.cuda.synchronize()
        A0 = oracle_arrays(L0)
        x0 = xs[0].cpu()
        rd, rv = oracle_draft(A0, x0[:K]), oracle_verify(A0, x0)
        b0 = bufs[0]
        e_d = rel_err(b0["yd"].cpu().numpy().astype(np.float64), rd["y"])
        e_v = rel_err(b0["yv"].float().cpu().numpy().astype(np.float64), rv["y"])
        assert np.array_equal(b0["win"].cpu().numpy(), rd["ids"]) and np.array_equal(b0["idv"].cpu().numpy(), rv["ids"]), \
            "layer 0 routing disagrees with the oracle"
        assert e_d <= 1e-3 and e_v <= 2e-2, "layer 0 outputs disagree with the oracle: %g %g" % (e_d, e_v)
        extra["layer0_rel_err_vs_oracle"] = {"draft": float("%.3e" % e_d), "verify": float("%.3e" % e_v)}
    cpu = None if args.no_cpu_baseline else cpu_baseline(cfg, L0, K, T)
    emit(cfg, args, K, T, n_layers, ms_step, ms_eager, launch, mean_u, nbytes, roofline, cpu, extra)


# ------------------------------------------------------------------------------------------------
def prefill_leg(args, cfg, ctx, dev):
    """--prefill T: the draft layer over T tokens in one call (moe_draft_prefill_int4), rotating over
    distinct layers.  A side measurement, not the headline metric: a step is one call."""
    import numpy as np
    import torch
    import synth
    from paper_2511_14102_amd.harness import DeviceLayer

    T = args.prefill
    n_layers = args.layers or 4
    sym = args.int4 == "symmetric"
    L0 = synth.make_layer(cfg, 0, quant_device=dev, symmetric=sym)
    layers = []
    for li in range(n_layers):
        L = L0 if li == 0 else synth.make_layer(cfg, li, device=dev, symmetric=sym)
        layers.append(DeviceLayer(ctx, cfg, L, max_tokens=8, verify=False, symmetric=sym))
    x = synth.make_tokens(cfg, T, kind="iid").to(dev)
    H, k = cfg.hidden, cfg.top_k
    y = torch.empty((T, H), dtype=torch.float32, device=dev)
    ids = torch.empty((T, k), dtype=torch.int32, device=dev)
    conf = torch.empty((T, k), dtype=torch.float32, device=dev)
    for i in range(args.warmup):
        layers[i % n_layers].prefill(x, y=y, ids=ids, conf=conf)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(args.steps):
        layers[(args.warmup + i) % n_layers].prefill(x, y=y, ids=ids, conf=conf)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    ctx.profile_enable(True)
    for i in range(min(args.steps, 8)):
        layers[i % n_layers].prefill(x, y=y, ids=ids, conf=conf)
    torch.cuda.synchronize()
    kern = read_profile(ctx)
    ctx.profile_enable(False)
    cnt = np.bincount(ids.cpu().numpy().reshape(-1), minlength=cfg.n_experts)
    items = int(np.sum((cnt + 63) // 64))
    distinct = int((cnt > 0).sum())
    I, g = cfg.inter, cfg.group_size
    entry = 2 if sym else 4
    n = T * k
    # weights-once bytes of the two contractions (every distinct expert's part read once) plus the
    # operand tiles they read and write; flops of the assignments that exist
    gu_bytes = distinct * (H * I + 2 * H * I // g * entry) + n * H * 2 + n * I * 4
    dn_bytes = distinct * (H * I // 2 + H * I // g * entry) + n * I * 4 + n * H * 4
    gu_us, dn_us = kern["prefill_gateup_kernel"]["us_avg"], kern["prefill_down_kernel"]["us_avg"]

    def roof(name, nbytes, flops, us):
        return {"kernel": name, "bound": "hbm", "achieved": round(nbytes / us / 1e3, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4), "traffic": None,
                "bytes_per_launch": nbytes, "us_per_launch": round(us, 2),
                "mfma": {"TFLOPs": round(flops / us / 1e6, 1), "peak": 2500.0, "frac": round(flops / us / 1e6 / 2500.0, 4)}}
    roofs = {"prefill_gateup_kernel": roof("prefill_gateup_kernel", gu_bytes, 4.0 * n * H * I, gu_us),
             "prefill_down_kernel": roof("prefill_down_kernel", dn_bytes, 2.0 * n * H * I, dn_us)}
    out = {"metric": "draft prefill tokens/s per MoE layer, 1 GPU", "value": round(T / (ms * 1e-3), 1), "unit": "tokens/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
           "higher_is_better": True, "dtype": "int4 (fp32 accumulate)", "data": "synthetic",
           "config": {"workload": "%s-shaped MoE layer, one moe_draft_prefill_int4 call over %d tokens, %d distinct layers"
                                  % (cfg.name, T, n_layers)},
           "us_per_token": round(ms * 1e3 / T, 3),
           "work_items": items, "distinct_experts": distinct,
           "kernel_us": {n_: round(v["us_avg"], 2) for n_, v in kern.items()},
           "roofline": roofs["prefill_gateup_kernel"], "kernels": roofs,
           "note": "algorithmic bytes = each distinct expert's weights once + operand tiles; an expert with more "
                   "than 64 assignments is streamed once per item of 64 (the repeats hit the caches)"}
    print(json.dumps(out), flush=True)


# ------------------------------------------------------------------------------------------------
def offload_leg(args, cfg, ctx, dev):
    """n_resident of the E experts of every layer start in the expert cache; all experts also sit in
    pinned host memory.  The Expert Scheduler (moe_elb_*, moe_cache_*, moe_sched_*) decides what
    to fetch and what to evict; the copies run on a side stream.

    One stack cycle: the K draft tokens go through all layers token by token; after each token its
    expert ids (one D2H per token) enter the lookahead buffer and a prefetch phase is planned
    (first token: priming, middle tokens: budgeted prefetch, last token: saturation) whose copies
    overlap the next token's drafting; then every layer verifies its K+1 rows as soon as its
    copies are in; experts only the verify call discovers are fetched on demand and added with an
    ACCUMULATE|ONLY_LISTED call.  Every cycle sees new tokens."""
    import numpy as np
    import torch
    import synth
    from paper_2511_14102_amd import binding as B
    from paper_2511_14102_amd import sched as S
    from paper_2511_14102_amd.harness import DeviceLayer

    T = max(cfg.verify_tokens)
    K = T - 1
    n_layers = args.layers or cfg.bench_layers
    H, E, k = cfg.hidden, cfg.n_experts, cfg.top_k
    n_res = cfg.n_resident
    n_slots = args.slots or (n_res + min(E, T * k))          # default: residents + room for one window's union
    cycles = max(1, args.steps // n_layers)
    warm_cycles = max(1, args.warmup // n_layers)
    n_tok_sets = warm_cycles + cycles

    t0 = time.time()
    layers, host = [], []
    L0 = synth.make_layer(cfg, 0, quant_device=dev)
    for li in range(n_layers):
        L = L0 if li == 0 else synth.make_layer(cfg, li, device=dev)
        D = DeviceLayer(ctx, cfg, L, max_tokens=T, resident=list(range(n_res)), n_slots=n_slots)
        hb = torch.empty((E, D.bf16_bytes), dtype=torch.uint8, pin_memory=True)
        for e in range(E):
            hb[e].copy_(D._pack_bf16(L, e))
        layers.append(D)
        host.append(hb)
        if li:
            del L
        if li % 4 == 0:
            log("  layer %d/%d on device, its %d experts in pinned host memory (%.0f s)" % (li + 1, n_layers, E, time.time() - t0))
    xs = [torch.stack([synth.make_tokens(cfg, T, layer=li, step=c) for li in range(n_layers)]).to(dev) for c in range(n_tok_sets)]
    xin = torch.empty((n_layers, T, H), dtype=xs[0].dtype, device=dev)       # what the launches read (fixed addresses)
    torch.cuda.synchronize()
    blob = layers[0].bf16_bytes
    log("setup %.1f s, %.1f GB in HBM, %.1f GB pinned, %d slots per layer" %
        (time.time() - t0, torch.cuda.memory_allocated() / 1e9, n_layers * E * blob / 1e9, n_slots))

    yd = torch.empty((K, n_layers, H), dtype=torch.float32, device=dev)
    win = torch.empty((K, n_layers, k), dtype=torch.int32, device=dev)          # [step, layer, k]: one D2H per token
    wconf = torch.empty((K, n_layers, k), dtype=torch.float32, device=dev)
    h_win, h_wconf = win.cpu().pin_memory(), wconf.cpu().pin_memory()
    yv = torch.empty((n_layers, T, H), dtype=torch.bfloat16, device=dev)
    idv = torch.empty((n_layers, T, k), dtype=torch.int32, device=dev)
    miss = torch.zeros((n_layers, E), dtype=torch.int32, device=dev)
    nm = torch.zeros(n_layers, dtype=torch.int32, device=dev)
    h_idv, h_miss, h_nm = idv.cpu().pin_memory(), miss.cpu().pin_memory(), nm.cpu().pin_memory()
    h_table = [torch.empty(E, dtype=torch.int32).pin_memory() for _ in range(n_layers)]
    for li, D in enumerate(layers):
        D.missing, D.n_missing = miss[li], nm[li:li + 1]
    copy_stream = torch.cuda.Stream()
    ready = [torch.cuda.Event() for _ in range(n_layers)]        # the layer's copies and slot table are in
    verified = [torch.cuda.Event() for _ in range(n_layers)]     # the layer's verify results are in host memory
    drafted = [torch.cuda.Event() for _ in range(K)]
    main = torch.cuda.current_stream()
    state = {"cache": None, "guided_budget": 8}

    def draft_token(i):
        for li, D in enumerate(layers):
            D.draft(xin[li, i:i + 1], y=yd[i, li:li + 1], ids=win[i, li:li + 1], conf=wconf[i, li:li + 1])

    # one HIP graph per drafted token: its n_layers draft calls (the leg was bound by the host's launch
    # rate before: n_layers x K separate calls per cycle)
    draft_graphs = None
    if args.mode == "graph":
        xin.copy_(xs[0])
        draft_token(0)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        draft_graphs = []
        for i in range(K):
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph, stream=side):
                draft_token(i)
            draft_graphs.append(gph)
        torch.cuda.synchronize()

    def run_draft(i):
        if draft_graphs is not None:
            draft_graphs[i].replay()
        else:
            draft_token(i)

    def new_cache():
        c = S.Cache(n_layers, E, n_slots)
        for li in range(n_layers):
            for e in range(n_res):
                c.place(li, e, e)
        return c

    def reset_residency():
        """Back to the initial residents (the slot pools still hold their blobs in slots 0..n_res-1
        only if nothing overwrote them, so they are copied again)."""
        state["cache"] = new_cache()
        for li, D in enumerate(layers):
            for e in range(n_res):
                ctx.expert_copy_async(D.slot_view(e), host[li][e], blob, copy_stream, None)
            h_table[li].copy_(torch.tensor(state["cache"].slot_table(li), dtype=torch.int32))
            with torch.cuda.stream(copy_stream):
                D.slot_of_expert.copy_(h_table[li], non_blocking=True)
        torch.cuda.synchronize()

    def wall(fn):
        torch.cuda.synchronize()
        t = time.perf_counter()
        r = fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3, r

    # ---- constants of this machine and this stack, measured before the cycles: the link rate (copies of
    # resident blobs onto themselves) and the time to draft one token through all layers.  The
    # phase II budget follows from them: twice what the link moves while one token drafts, so that the
    # copy queue does not run dry between two planning steps.
    reset_residency()
    xin.copy_(xs[0])

    def link_probe():
        for j in range(32):
            li, e = j % n_layers, j % n_res
            ctx.expert_copy_async(layers[li].slot_view(e), host[li][e], blob, copy_stream, None)
    wall(link_probe)
    link_rate = 32 * blob / (min(wall(link_probe)[0] for _ in range(3)) * 1e-3)

    def draft_only():
        for i in range(K):
            run_draft(i)
    draft_only()
    t_draft_phase = min(wall(draft_only)[0] for _ in range(3)) * 1e-3
    state["guided_budget"] = max(1, int(np.ceil(2.0 * (t_draft_phase / K) * link_rate / blob)))
    log("link %.1f GB/s, draft %.3f ms per token (%s), phase II budget %d experts per token" %
        (link_rate / 1e9, t_draft_phase / K * 1e3, "one graph per token" if draft_graphs else "eager", state["guided_budget"]))

    def issue(fetches, log_list=None, marks=None):
        """Copies for a list of (layer, expert, slot, evicted), layer by layer in ascending order; after a
        layer's copies its slot table is uploaded and its event recorded, so that the layer's verify
        call waits for its own experts only."""
        by_layer = {}
        for f in fetches:
            by_layer.setdefault(f[0], []).append(f)
        for li in sorted(by_layer):
            for (_li, e, slot, _ev) in by_layer[li]:
                if marks is not None and marks.get("first") is None:
                    marks["first"] = torch.cuda.Event(enable_timing=True)
                    marks["first"].record(copy_stream)
                ctx.expert_copy_async(layers[li].slot_view(slot), host[li][e], blob, copy_stream, None)
            h_table[li].copy_(torch.tensor(state["cache"].slot_table(li), dtype=torch.int32))
            with torch.cuda.stream(copy_stream):
                layers[li].slot_of_expert.copy_(h_table[li], non_blocking=True)
            ready[li].record(copy_stream)
        if log_list is not None:
            log_list.extend(fetches)
        return sorted(by_layer)

    def plan_step(i, elb, waiting, fetch_log, marks):
        elb.put_step(i, h_win[i].tolist(), h_wconf[i].tolist())
        phase = S.PHASE_SATURATE if i == K - 1 else (S.PHASE_PRIME if i == 0 else S.PHASE_GUIDED)
        fetches = state["cache"].plan(elb, phase, state["guided_budget"], 0.0)
        for li in issue(fetches, fetch_log, marks):
            waiting.add(li)
        return len(fetches)

    def cycle(x, prefetch=True, fetch_log=None, timeline=None):
        cache = state["cache"]
        elb = S.Elb(n_layers, K, k)
        waiting = set()
        counts = {"predicted": 0, "on_demand": 0}
        marks = {"first": None}
        ev = {n: torch.cuda.Event(enable_timing=True) for n in ("start", "drafted", "prefetched", "verified", "end")}
        tables0 = [cache.slot_table(li) for li in range(n_layers)]
        ev["start"].record(main)
        h0 = time.perf_counter()
        host = {}
        xin.copy_(x)
        for i in range(K):                                   # draft, token-major
            run_draft(i)
            h_win[i].copy_(win[i], non_blocking=True)
            h_wconf[i].copy_(wconf[i], non_blocking=True)
            drafted[i].record(main)
            if i < 2:
                host["launched_token_%d" % i] = (time.perf_counter() - h0) * 1e3
            if prefetch and i:                               # plan token i-1 while token i drafts
                drafted[i - 1].synchronize()
                if i == 1:
                    host["token_0_ids_on_host"] = (time.perf_counter() - h0) * 1e3
                counts["predicted"] += plan_step(i - 1, elb, waiting, fetch_log, marks)
                if i == 1:
                    host["token_0_planned_and_issued"] = (time.perf_counter() - h0) * 1e3
        ev["drafted"].record(main)
        drafted[K - 1].synchronize()
        if prefetch:
            counts["predicted"] += plan_step(K - 1, elb, waiting, fetch_log, marks)
        ev["prefetched"].record(copy_stream)
        # |E_new(k)| of the governor's model: experts of the first k drafted tokens that the cache
        # lacked when the cycle began
        ids_np = h_win.numpy()
        counts["n_new_by_k"] = [0] + [sum(len({int(e) for e in ids_np[:kk, li].reshape(-1) if tables0[li][int(e)] < 0})
                                          for li in range(n_layers)) for kk in range(1, K + 1)]
        for li, D in enumerate(layers):                      # verify, each layer as soon as its own experts are in
            if li in waiting:
                main.wait_event(ready[li])
            D.verify(xin[li], y=yv[li], ids=idv[li])
            h_idv[li].copy_(idv[li], non_blocking=True)
            h_miss[li].copy_(miss[li], non_blocking=True)
            h_nm[li:li + 1].copy_(nm[li:li + 1], non_blocking=True)
            verified[li].record(main)
        ev["verified"].record(main)
        for li in range(n_layers):                           # coverage accounting; on-demand fetches as results arrive
            verified[li].synchronize()
            cache.use(li, h_idv[li].reshape(-1).tolist())
            n = int(h_nm[li])
            if n:
                fetches = cache.on_demand(li, h_miss[li, :n].tolist())
                issue(fetches, fetch_log, marks)
                counts["on_demand"] += n
                main.wait_event(ready[li])
                layers[li].verify(xin[li], flags=B.MOE_VERIFY_ACCUMULATE | B.MOE_VERIFY_ONLY_LISTED, y=yv[li], ids=idv[li])
        ev["end"].record(main)
        cache.end_window()
        elb.close()
        torch.cuda.synchronize()
        if timeline is not None:
            t = {n: ev["start"].elapsed_time(ev[n]) for n in ("drafted", "prefetched", "verified", "end")}
            t["first_copy"] = ev["start"].elapsed_time(marks["first"]) if marks["first"] is not None else None
            t["host"] = {n: round(v, 3) for n, v in host.items()}
            timeline.append(t)
        return counts

    # ---- copies and compute together, new tokens every cycle, cache carried from cycle to cycle
    reset_residency()
    t_both, per_cycle, fetch_log, timeline = [], [], [], []
    for c in range(n_tok_sets):
        log_c, tl = [], []
        ms, counts = wall(lambda: cycle(xs[c], True, log_c, tl))
        if c >= warm_cycles:
            t_both.append(ms)
            per_cycle.append(counts)
            timeline.append(tl[0])
            fetch_log = log_c
        log("cycle %d: %.2f ms, %d predicted + %d on demand experts fetched" % (c, ms, counts["predicted"], counts["on_demand"]))
    hits, misses = state["cache"].stats()
    last = n_tok_sets - 1

    # ---- compute alone: the last cycle's tokens again, everything it needs is resident now
    t_compute = []
    for c in range(warm_cycles + cycles):
        ms, counts = wall(lambda: cycle(xs[last], True))
        assert counts["predicted"] == 0 and counts["on_demand"] == 0, "compute-only cycle still fetches"
        if c >= warm_cycles:
            t_compute.append(ms)

    # ---- copies alone: the last timed cycle's fetch list, nothing else running
    def copies_only():
        for (li, e, slot, _ev) in fetch_log:
            ctx.expert_copy_async(layers[li].slot_view(slot), host[li][e], blob, copy_stream, None)
    t_copy = []
    for c in range(3):
        ms, _ = wall(copies_only)
        if c:
            t_copy.append(ms)
    tb, tc, tp = float(np.median(t_both)), float(np.median(t_compute)), float(np.median(t_copy))
    copy_bytes = len(fetch_log) * blob
    uniq = [len(set(h_idv[li].reshape(-1).tolist())) for li in range(n_layers)]
    mean_u = float(np.mean(uniq))
    nbytes = algorithmic_bytes(cfg, T, mean_u)
    # The last timed cycle on the GPU's clock (events; ms from the cycle's start): the first copy can
    # only start once the first token's experts are known; from there to `drafted` the remaining
    # tokens draft while the link is busy.
    tl = timeline[-1]
    draft_hidden = None if tl["first_copy"] is None else max(0.0, 1.0 - tl["first_copy"] / tl["drafted"])
    n_pred_last, n_od_last = per_cycle[-1]["predicted"], per_cycle[-1]["on_demand"]
    offload = {
        "layers": n_layers, "resident_per_layer": n_res, "slots_per_layer": n_slots, "cycles": cycles,
        "draft_launch": "one HIP graph per drafted token" if draft_graphs else "eager calls",
        "t_both_ms": round(tb, 3), "t_compute_ms": round(tc, 3), "t_copy_ms": round(tp, 3),
        "overlap": round((tp + tc - tb) / min(tp, tc), 3),       # (t_copy + t_compute - t_both) / min(t_copy, t_compute)
        "compute_hidden_under_copies": round((tp + tc - tb) / min(tp, tc), 3),
        "timeline_last_cycle_ms": {n: (v if isinstance(v, dict) or v is None else round(v, 3)) for n, v in tl.items()},
        "draft_phase_hidden_under_copies": None if draft_hidden is None else round(draft_hidden, 3),
        "link_busy_share_of_cycle": round(tp / tb, 3),
        "copy_GB_last_cycle": round(copy_bytes / 1e9, 3), "h2d_GBs": round(copy_bytes / (tp * 1e-3) / 1e9, 1),
        "phase2_budget_experts_per_token": state["guided_budget"],
        "fetched_predicted_per_layer": round(float(np.mean([c["predicted"] for c in per_cycle])) / n_layers, 2),
        "fetched_on_demand_per_layer": round(float(np.mean([c["on_demand"] for c in per_cycle])) / n_layers, 2),
        "cache_coverage_pct": round(100.0 * hits / max(hits + misses, 1), 2),
        "compute_ms_per_layer": round(tc / n_layers, 4),
    }
    log("offload:", json.dumps(offload))

    # ---- per-kernel time on the compute-only cycle (eager calls: the event pairs cannot be captured)
    roofline, extra = None, {"offload": offload}
    if not args.no_profile:
        saved, draft_graphs = draft_graphs, None
        ctx.profile_enable(True)
        cycle(xs[last], True)
        torch.cuda.synchronize()
        kern = read_profile(ctx)
        ctx.profile_enable(False)
        draft_graphs = saved
        roofline, table = roofline_table(cfg, kern, nbytes, ROOT)
        extra["kernels"] = table
        extra["kernel_us"] = {n: round(v["us_avg"], 2) for n, v in kern.items()}

    # ---- the Speculative Governor on what was just measured (Eq. 3): T_draft(k) linear in k (the draft
    # phase is token-major), T_verify profiled at three token counts with everything resident, the link
    # rate from the copies-alone pass; |E_new(k)| from the last timed cycle (against the cache as it was
    # when that cycle began).  Its cycle time for the drafted length beside the measured one.
    n_new = per_cycle[-1]["n_new_by_k"]
    xin.copy_(xs[last])
    v_tokens = sorted({max(1, T // 3), max(2, (2 * T) // 3), T})
    v_seconds = []
    for tv in v_tokens:
        def verify_only():
            for li, D in enumerate(layers):
                D.verify(xin[li, :tv], y=yv[li, :tv], ids=idv[li, :tv])
        verify_only()
        v_seconds.append(min(wall(verify_only)[0] for _ in range(3)) * 1e-3)
    rate = copy_bytes / (tp * 1e-3) if copy_bytes else link_rate
    gov_cfg = dict(t_draft_base=0.0, t_draft_token=t_draft_phase / K, t_pcie_init=blob / rate,
                   t_pcie_overhead=0.0, b_pcie=rate, s_expert=float(blob),
                   verify_tokens=v_tokens, verify_seconds=v_seconds, ema_alpha=0.1, p_init=0.8, k_min=1, k_max=K)
    gov = S.Governor(gov_cfg)
    k_star, theta_star = gov.choose_k(n_new)
    model_new = gov.cycle_time(K, n_new[K]) * 1e3
    model_fetched = gov.cycle_time(K, n_pred_last + n_od_last) * 1e3
    measured_last = t_both[-1]
    extra["governor"] = {
        "inputs": {kk: ([round(x, 6) for x in v] if isinstance(v, list) and v and isinstance(v[0], float)
                        else (round(v, 6) if isinstance(v, float) else v)) for kk, v in gov_cfg.items()},
        "n_new_by_k": n_new, "theta_by_k": [round(gov.evaluate(kk, n_new[kk])[0], 2) for kk in range(1, K + 1)],
        "k_star": k_star, "theta_star_tokens_per_s": round(theta_star, 2),
        "cycle_time_model_ms": {"k": K, "n_new": n_new[K], "with_n_new": round(model_new, 3),
                                "fetched_last_cycle": n_pred_last + n_od_last, "with_fetched": round(model_fetched, 3)},
        "t_both_last_cycle_ms": round(measured_last, 3),
        "measured_over_model": {"with_n_new": round(measured_last / model_new, 3),
                                "with_fetched": round(measured_last / model_fetched, 3)},
        "note": "acceptance probability 0.8 per token assumed (no model to measure it on).  The model charges every "
                "new expert's copy after the draft phase; the measured cycle also fetches what the draft pass "
                "mispredicted (fetched > n_new) and hides part of the draft and verify phases under the copies."}
    gov.close()

    # ---- the last cycle's result on layer 0 against the oracle (same launch path as timed)
    if not args.no_cpu_baseline:
        from oracle.layer_check import oracle_arrays, oracle_verify, rel_err
        ref = oracle_verify(oracle_arrays(L0), xs[last][0].cpu())
        err = rel_err(yv[0].float().cpu().numpy().astype(np.float64), ref["y"])
        assert np.array_equal(idv[0].cpu().numpy(), ref["ids"]) and err <= 2e-2, "layer 0 of the cycle disagrees with the oracle"
        extra["layer0_verify_rel_err_vs_oracle"] = float("%.3e" % err)
    cpu = None if args.no_cpu_baseline else cpu_baseline(cfg, L0, K, T)
    # the step time of this workload includes the expert copies it cannot avoid
    emit(cfg, args, K, T, n_layers, tb / n_layers, None, "eager, copies on a side stream", mean_u, nbytes, roofline, cpu, extra)


def draft_table_leg(args, cfg, ctx, dev):
    """--draft-table: the draft kernel's duration (kernel-stamped events) for calls of 1, 2, 4 and 8 tokens,
    rotating over distinct layers, with the bytes each call has to move (the distinct experts its tokens
    select, once each).  A side measurement: one JSON line, no headline metric."""
    import numpy as np
    import torch
    import synth
    from paper_2511_14102_amd.harness import DeviceLayer

    sym = args.int4 == "symmetric"
    H, E, I, k, g = cfg.hidden, cfg.n_experts, cfg.inter, cfg.top_k, cfg.group_size
    P = 3 * H * I
    expert_bytes = P // 2 + (P // g) * (2 if sym else 4)
    n_layers = args.layers or (12 if expert_bytes * E < 2e9 else 6)
    layers = [DeviceLayer(ctx, cfg, synth.make_layer(cfg, li, device=dev, symmetric=sym), max_tokens=8, verify=False,
                          symmetric=sym) for li in range(n_layers)]
    xs = [synth.make_tokens(cfg, 8, layer=li).to(dev) for li in range(n_layers)]
    ids = torch.empty((8, k), dtype=torch.int32, device=dev)
    rows = {}
    for T in (1, 2, 4, 8):
        for i in range(n_layers):
            layers[i].draft(xs[i][:T])
        torch.cuda.synchronize()
        distinct = []
        ctx.profile_enable(True)
        for i in range(8 * n_layers):
            r = layers[i % n_layers].draft(xs[i % n_layers][(i // n_layers) % (9 - T):][:T], ids=ids[:T])
            if i < n_layers:
                distinct.append(len(set(r["ids"].cpu().numpy().reshape(-1).tolist())))
        torch.cuda.synchronize()
        prof = read_profile(ctx)
        ctx.profile_enable(False)
        us = prof["draft_fused_kernel"]["us_avg"]
        n_calls = prof["draft_fused_kernel"]["launches"]
        call_us = sum(v["us_avg"] for v in prof.values() if v["launches"] == n_calls)   # + shared-expert kernels, if any
        nbytes = float(np.mean(distinct)) * expert_bytes + E * H * 2 + T * H * 2 + T * H * 4
        rows[str(T)] = {"us": round(us, 2), "all_kernels_of_the_call_us": round(call_us, 2),
                        "mean_distinct_experts": round(float(np.mean(distinct)), 2),
                        "bytes": int(nbytes), "GBs": round(nbytes / us / 1e3, 1), "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4),
                        "launches": n_calls}
    print(json.dumps({"metric": "draft kernel duration by tokens per call, 1 GPU", "unit": "us", "data": "synthetic",
                      "config": {"workload": "%s-shaped MoE layer, %d distinct layers rotating, int4 %s" %
                                 (cfg.name, n_layers, "symmetric" if sym else "asymmetric")},
                      "tokens_per_call": rows}), flush=True)


def read_probe_leg(args, cfg, ctx, dev):
    """--read-probe: moe_stream_read_probe (a kernel that only reads) over the bytes of one one-token draft call,
    cold data (the int4 blobs of distinct layers in rotation), for several grids: the draft kernel's own launch
    shape (k I / 32 workgroups) and grids that fill the compute units evenly.  A side measurement."""
    import torch
    import synth
    from paper_2511_14102_amd.harness import DeviceLayer

    n_layers = args.layers or 12
    layers = [DeviceLayer(ctx, cfg, synth.make_layer(cfg, li, device=dev), max_tokens=8, verify=False) for li in range(n_layers)]
    blobs = [D.q_blob for D in layers]
    nbytes = algorithmic_bytes(cfg, 1, 1.0)["draft_fused_kernel"]
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    own = cfg.top_k * cfg.inter // 32
    rows = {}
    for rep in range(3):                                     # three rounds: the scatter between them is part of the result
        for grid in sorted({n_cu, own, 2 * n_cu, 2 * own, 4 * n_cu}):
            r = stream_ceiling(ctx, torch, blobs, nbytes, grid, reps=96)
            rows.setdefault(str(grid), []).append(r["us"])
    print(json.dumps({"metric": "read-only kernel over the bytes of one draft call, 1 GPU", "unit": "us", "data": "synthetic",
                      "config": {"workload": "%s-shaped MoE layer, %d distinct layers rotating" % (cfg.name, n_layers)},
                      "bytes": nbytes // 1024 * 1024, "compute_units": n_cu, "draft_kernel_workgroups": own,
                      "us_by_workgroups": rows}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--config", default="phi")
    ap.add_argument("--layers", type=int, default=0, help="distinct layers to rotate over (0 = config default)")
    ap.add_argument("--mode", default="graph", choices=["graph", "eager"],
                    help="how the timed steps are launched (per-kernel timing always runs eagerly)")
    ap.add_argument("--int4", default="asymmetric", choices=["asymmetric", "symmetric"],
                    help="draft weight format: scale + zero per group (default) or scales only with z = 8")
    ap.add_argument("--prefill", type=int, default=0,
                    help="side measurement: one moe_draft_prefill_int4 call over this many tokens per step")
    ap.add_argument("--draft-table", action="store_true",
                    help="side measurement: the draft kernel's duration for calls of 1, 2, 4 and 8 tokens")
    ap.add_argument("--read-probe", action="store_true",
                    help="side measurement: a kernel that only reads one draft call's bytes, for several grids")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--slots", type=int, default=0,
                    help="expert-cache slots per layer for workloads with non-resident experts (0: residents + one window's union)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (known HBM traffic, for PMC scaling)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    from paper_2511_14102_amd import binding as B

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = synth.config_by_name(args.config)
    ctx = B.Context(0)
    if args.read_probe:
        read_probe_leg(args, cfg, ctx, "cuda:0")
    elif args.draft_table:
        draft_table_leg(args, cfg, ctx, "cuda:0")
    elif args.prefill:
        prefill_leg(args, cfg, ctx, "cuda:0")
    elif cfg.n_resident and cfg.n_resident < cfg.n_experts:
        offload_leg(args, cfg, ctx, "cuda:0")
    else:
        resident_leg(args, cfg, ctx, "cuda:0")


if __name__ == "__main__":
    main()
