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


def algorithmic_bytes(cfg, T, mean_u):
    """Bytes the method has to move per call (selected experts' weights once + small operands)."""
    H, E, I, k, S, g = cfg.hidden, cfg.n_experts, cfg.inter, cfg.top_k, cfg.n_shared, cfg.group_size
    P = 3 * H * I
    int4_expert = P // 2 + (P // g) * 4
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
                       "traffic": traffic.get(name), "bytes_per_launch": int(nbytes[name]),
                       "us_per_launch": round(kk["us_avg"], 2), "launches": kk["launches"],
                       "ms_total": round(kk["ms_total"], 3)}
    dominant = max(table.values(), key=lambda r: r["ms_total"]) if table else None   # most time in the timed region
    return dominant, table


def read_profile(ctx):
    prof = ctx.profile_read()
    return {n: {"ms_total": ms, "launches": cnt, "us_avg": 1e3 * ms / cnt} for n, (ms, cnt) in prof.items() if cnt}


def cpu_baseline(cfg, L0, K, T):
    """The oracle as it stands on layer 0's step, for at least 10 s of host work."""
    import synth
    from oracle import oracle as orc
    from tests.common import oracle_arrays, oracle_draft, oracle_verify
    A = oracle_arrays(L0)
    tc = time.time()
    reps = 0
    while time.time() - tc < 10.0 and reps < 64:
        x0 = synth.make_tokens(cfg, T, layer=0, step=reps)
        oracle_draft(A, x0[:K])
        oracle_verify(A, x0)
        reps += 1
    dt = time.time() - tc
    return {"value": round(reps * (2 * K + 1) / dt, 3), "unit": "tokens/s", "cores": orc.num_threads(),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": "%d steps of layer 0 (fresh tokens each): %d draft tokens (int4) + one verify of %d "
                      "tokens (bf16) per step" % (reps, K, T)}


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
    L0 = synth.make_layer(cfg, 0, quant_device=dev)
    for li in range(n_layers):
        L = L0 if li == 0 else synth.make_layer(cfg, li, device=dev)
        layers.append(DeviceLayer(ctx, cfg, L, max_tokens=T))
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

    def timed(fn, n_warm, n_steps):
        for i in range(n_warm):
            fn(i % n_layers)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n_steps):
            fn((n_warm + i) % n_layers)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n_steps

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ms_eager = timed(step, args.warmup, args.steps)
    log("eager: %.3f ms/step" % ms_eager)
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
        ms_graph = timed(lambda li: graphs[li].replay(), args.warmup, args.steps)
        log("graph: %.3f ms/step" % ms_graph)
        if ms_graph < ms_eager:
            ms_step, launch = ms_graph, "hipgraph"

    # ---- what the steps computed: distinct experts per verify call, from the ids
    torch.cuda.synchronize()
    uniq = [len(set(bufs[li]["idv"].cpu().numpy().reshape(-1).tolist())) for li in range(n_layers)]
    mean_u = float(np.mean(uniq))
    mean_u_run = float(np.mean([uniq[(args.warmup + i) % n_layers] for i in range(args.steps)]))
    nbytes = algorithmic_bytes(cfg, T, mean_u_run)

    # ---- per-kernel time (eager, event pairs around every kernel launch)
    roofline, extra = None, {}
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
        extra["per_call"] = {
            "draft_us": round(kern["draft_fused_kernel"]["us_avg"], 2),
            "draft_tokens_per_s": round(1e6 / kern["draft_fused_kernel"]["us_avg"], 1),
            "verify_us": round(sum(kern[n]["us_avg"] for n in ("route_kernel", "plan_kernel", "bf16_gateup_kernel",
                                                                 "bf16_down_kernel", "combine_kernel") if n in kern), 2),
        }
        extra["per_call"]["verify_tokens_per_s"] = round(T * 1e6 / extra["per_call"]["verify_us"], 1)

    cpu = None if args.no_cpu_baseline else cpu_baseline(cfg, L0, K, T)
    emit(cfg, args, K, T, n_layers, ms_step, ms_eager, launch, mean_u, nbytes, roofline, cpu, extra)


# ------------------------------------------------------------------------------------------------
def offload_leg(args, cfg, ctx, dev):
    """n_resident of the E experts of every layer start in slots; the rest sit in pinned host memory."""
    import numpy as np
    import torch
    import synth
    from paper_2511_14102_amd import binding as B
    from paper_2511_14102_amd.harness import DeviceLayer

    T = max(cfg.verify_tokens)
    K = T - 1
    n_layers = args.layers or cfg.bench_layers
    H, E, k = cfg.hidden, cfg.n_experts, cfg.top_k
    n_res = cfg.n_resident
    n_stage = min(E, T * k)                      # staging slots behind the resident ones
    cycles = max(1, args.steps // n_layers)
    warm_cycles = max(1, args.warmup // n_layers)

    t0 = time.time()
    layers, xs, host = [], [], []
    L0 = synth.make_layer(cfg, 0, quant_device=dev)
    for li in range(n_layers):
        L = L0 if li == 0 else synth.make_layer(cfg, li, device=dev)
        D = DeviceLayer(ctx, cfg, L, max_tokens=T, resident=list(range(n_res)), n_slots=n_res + n_stage)
        hb = torch.empty((E - n_res, D.bf16_bytes), dtype=torch.uint8, pin_memory=True)
        for e in range(n_res, E):
            hb[e - n_res].copy_(D._pack_bf16(L, e))
        layers.append(D)
        host.append(hb)
        xs.append(synth.make_tokens(cfg, T, layer=li).to(dev))
        if li:
            del L
        if li % 4 == 0:
            log("  layer %d/%d on device, %d experts in pinned host memory (%.0f s)" % (li + 1, n_layers, E - n_res, time.time() - t0))
    torch.cuda.synchronize()
    blob = layers[0].bf16_bytes
    log("setup %.1f s, %.1f GB in HBM, %.1f GB pinned" % (time.time() - t0, torch.cuda.memory_allocated() / 1e9,
                                                          n_layers * (E - n_res) * blob / 1e9))

    yd = torch.empty((n_layers, K, H), dtype=torch.float32, device=dev)
    win = torch.empty((n_layers, K, k), dtype=torch.int32, device=dev)
    conf = torch.empty((n_layers, K, k), dtype=torch.float32, device=dev)
    yv = torch.empty((n_layers, T, H), dtype=torch.bfloat16, device=dev)
    idv = torch.empty((n_layers, T, k), dtype=torch.int32, device=dev)
    mask = torch.empty((E + 63) // 64, dtype=torch.int64, device=dev)
    lst = torch.empty(E, dtype=torch.int32, device=dev)
    nl = torch.empty(1, dtype=torch.int32, device=dev)
    miss1 = torch.zeros((n_layers, E), dtype=torch.int32, device=dev)      # predicted misses (union)
    nm1 = torch.zeros(n_layers, dtype=torch.int32, device=dev)
    miss2 = torch.zeros((n_layers, E), dtype=torch.int32, device=dev)      # found by the verify call
    nm2 = torch.zeros(n_layers, dtype=torch.int32, device=dev)
    h_miss1, h_nm1 = miss1.cpu().pin_memory(), nm1.cpu().pin_memory()
    h_miss2, h_nm2 = miss2.cpu().pin_memory(), nm2.cpu().pin_memory()
    table0 = [D.slot_of_expert.clone() for D in layers]
    h_table = [D.slot_host.clone().pin_memory() for D in layers]
    for li, D in enumerate(layers):
        D.missing, D.n_missing = miss2[li], nm2[li:li + 1]
    copy_stream = torch.cuda.Stream()
    events = [torch.cuda.Event() for _ in range(n_layers)]
    main = torch.cuda.current_stream()

    def reset_tables():
        for li, D in enumerate(layers):
            D.slot_of_expert.copy_(table0[li])
            h_table[li].copy_(D.slot_host)
        torch.cuda.synchronize()

    drafted = [torch.cuda.Event() for _ in range(n_layers)]

    def draft_phase(base=None):
        """K draft calls + union per layer; the layer's missing list goes to the host right behind
        it, and (base given) its copies are issued while the next layer's drafts already run."""
        for li, D in enumerate(layers):
            x = xs[li]
            for i in range(K):
                D.draft(x[i:i + 1], y=yd[li, i:i + 1], ids=win[li, i:i + 1], conf=conf[li, i:i + 1])
            ctx.expert_union(win[li], K * k, E, D.slot_of_expert, mask, lst, nl, miss1[li], nm1[li:li + 1])
            h_miss1[li].copy_(miss1[li], non_blocking=True)
            h_nm1[li:li + 1].copy_(nm1[li:li + 1], non_blocking=True)
            drafted[li].record(main)
            if base is not None and li:
                drafted[li - 1].synchronize()
                issue_copies(h_miss1, h_nm1, base, wait_main=False, only=li - 1)
        drafted[n_layers - 1].synchronize()
        if base is not None:
            return issue_copies(h_miss1, h_nm1, base, wait_main=False, only=n_layers - 1)

    def issue_copies(h_miss, h_nm, base, wait_main, only=None):
        """Copies the listed experts of every layer (or of layer `only`) into staging slots
        base[li]+j; returns bytes."""
        total = 0
        if wait_main:
            copy_stream.wait_stream(main)
        for li, D in enumerate(layers):
            if only is not None and li != only:
                continue
            n = int(h_nm[li])
            if n == 0:
                continue
            for j in range(n):
                e = int(h_miss[li, j])
                slot = n_res + base[li] + j
                ctx.expert_copy_async(D.slot_view(slot), host[li][e - n_res], blob, copy_stream, None)
                h_table[li][e] = slot
            with torch.cuda.stream(copy_stream):
                D.slot_of_expert.copy_(h_table[li], non_blocking=True)
            events[li].record(copy_stream)
            base[li] += n
            total += n * blob
        return total

    def verify_phase(wait):
        for li, D in enumerate(layers):
            if wait and int(h_nm1[li]):
                main.wait_event(events[li])
            D.verify(xs[li], y=yv[li], ids=idv[li])
        h_miss2.copy_(miss2, non_blocking=True)
        h_nm2.copy_(nm2, non_blocking=True)
        main.synchronize()

    def demand_phase(base):
        """Experts the draft window did not predict: fetch, then add their share."""
        todo = [li for li in range(n_layers) if int(h_nm2[li])]
        nbytes = issue_copies(h_miss2, h_nm2, base, wait_main=True)
        for li in todo:
            main.wait_event(events[li])
            layers[li].verify(xs[li], flags=B.MOE_VERIFY_ACCUMULATE | B.MOE_VERIFY_ONLY_LISTED, y=yv[li], ids=idv[li])
        return nbytes, len(todo)

    def cycle():
        base = [0] * n_layers
        draft_phase(base)
        b1 = int(h_nm1.sum()) * blob
        verify_phase(wait=True)
        b2, n_demand_layers = demand_phase(base)
        torch.cuda.synchronize()
        return b1, b2, n_demand_layers

    def wall(fn):
        torch.cuda.synchronize()
        t = time.perf_counter()
        r = fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3, r

    # ---- copies and compute together
    t_both, copied = [], None
    for c in range(warm_cycles + cycles):
        reset_tables()
        ms, copied = wall(cycle)
        if c >= warm_cycles:
            t_both.append(ms)
        log("cycle %d: %.2f ms, %.2f GB predicted + %.2f GB on demand (%d layers)" % (c, ms, copied[0] / 1e9, copied[1] / 1e9, copied[2]))
    n_pred = h_nm1.numpy().astype(np.int64).copy()
    n_dem = h_nm2.numpy().astype(np.int64).copy()
    pred_list, dem_list = h_miss1.clone(), h_miss2.clone()
    pred_n, dem_n = h_nm1.clone(), h_nm2.clone()

    # ---- compute alone: everything the cycle needs is resident now (tables left as they are)
    def compute_only():
        draft_phase()
        verify_phase(wait=False)
    t_compute = []
    for c in range(warm_cycles + cycles):
        ms, _ = wall(compute_only)
        if c >= warm_cycles:
            t_compute.append(ms)
    assert int(h_nm1.sum()) == 0 and int(h_nm2.sum()) == 0, "compute-only cycle still reports missing experts"

    # ---- copies alone: the same list of experts, nothing else running
    def copies_only():
        base = [0] * n_layers
        issue_copies(pred_list, pred_n, base, wait_main=False)
        issue_copies(dem_list, dem_n, base, wait_main=False)
    t_copy = []
    for c in range(cycles + 1):
        reset_tables()
        ms, _ = wall(copies_only)
        if c >= 1:
            t_copy.append(ms)
    # leave the tables pointing at the fetched experts for the profile pass below
    tb, tc, tp = float(np.median(t_both)), float(np.median(t_compute)), float(np.median(t_copy))
    copy_bytes = copied[0] + copied[1]
    uniq = [len(set(idv[li].cpu().numpy().reshape(-1).tolist())) for li in range(n_layers)]
    mean_u = float(np.mean(uniq))
    nbytes = algorithmic_bytes(cfg, T, mean_u)
    offload = {
        "layers": n_layers, "resident_per_layer": n_res, "staging_slots": n_stage, "cycles": cycles,
        "t_both_ms": round(tb, 3), "t_compute_ms": round(tc, 3), "t_copy_ms": round(tp, 3),
        "overlap": round((tp + tc - tb) / min(tp, tc), 3),
        "copy_GB_per_cycle": round(copy_bytes / 1e9, 3), "h2d_GBs": round(copy_bytes / (tp * 1e-3) / 1e9, 1),
        "missing_predicted_per_layer": round(float(n_pred.mean()), 2),
        "missing_on_demand_per_layer": round(float(n_dem.mean()), 2),
        "compute_ms_per_layer": round(tc / n_layers, 4),
    }
    log("offload:", json.dumps(offload))

    # ---- per-kernel time on the compute-only cycle
    roofline, extra = None, {"offload": offload}
    if not args.no_profile:
        ctx.profile_enable(True)
        compute_only()
        torch.cuda.synchronize()
        kern = read_profile(ctx)
        ctx.profile_enable(False)
        roofline, table = roofline_table(cfg, kern, nbytes, ROOT)
        extra["kernels"] = table
        extra["kernel_us"] = {n: round(v["us_avg"], 2) for n, v in kern.items()}

    # ---- the cycle's result on layer 0 against the oracle (same launch path as timed)
    if not args.no_cpu_baseline:
        from tests.common import oracle_arrays, oracle_verify, rel_err
        ref = oracle_verify(oracle_arrays(L0), xs[0].cpu())
        err = rel_err(yv[0].float().cpu().numpy().astype(np.float64), ref["y"])
        assert np.array_equal(idv[0].cpu().numpy(), ref["ids"]) and err <= 2e-2, "layer 0 of the cycle disagrees with the oracle"
        extra["layer0_verify_rel_err_vs_oracle"] = float("%.3e" % err)
    cpu = None if args.no_cpu_baseline else cpu_baseline(cfg, L0, K, T)
    # the step time of this workload includes the expert copies it cannot avoid
    emit(cfg, args, K, T, n_layers, tb / n_layers, None, "eager, copies on a side stream", mean_u, nbytes, roofline, cpu, extra)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--config", default="phi")
    ap.add_argument("--layers", type=int, default=0, help="distinct layers to rotate over (0 = config default)")
    ap.add_argument("--mode", default="graph", choices=["graph", "eager"],
                    help="how the timed steps are launched (per-kernel timing always runs eagerly)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
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
    if cfg.n_resident and cfg.n_resident < cfg.n_experts:
        offload_leg(args, cfg, ctx, "cuda:0")
    else:
        resident_leg(args, cfg, ctx, "cuda:0")


if __name__ == "__main__":
    main()
