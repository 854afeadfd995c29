#!/usr/bin/env python3
"""Benchmark of the MoE draft+verify layer on one MI355X.

One *step* is one speculative cycle of one MoE layer (every row of the hot path once):
K draft calls (moe_draft_layer_int4, one token each, int4 experts, expert ids written into the
window buffer), one moe_expert_union over the window's ids against the slot table, and one
moe_verify_layer_bf16 over the K+1 tokens (bf16 experts through the slot table).  Successive
steps rotate over a stack of distinct layers so that weights come from HBM, not from a cache.
For workloads with non-resident experts (dsv2lite) the step also copies the missing experts
from pinned host memory on a side stream (moe_expert_copy_async) before the verify call.

Prints ONE JSON line: value = token passes per second = (K + K+1) / step time, with the
`roofline` of the dominant kernel and the `cpu_baseline` (the fp64 oracle on the host cores).
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


def log(*a):
    print(*a, file=sys.stderr, flush=True)


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

    import numpy as np
    import torch
    import synth
    from paper_2511_14102_amd import binding as B
    from paper_2511_14102_amd.harness import DeviceLayer

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.config_by_name(args.config)
    T = max(cfg.verify_tokens)
    K = T - 1
    n_layers = args.layers or cfg.bench_layers
    ctx = B.Context(0)
    H, E, I, k, S, g = cfg.hidden, cfg.n_experts, cfg.inter, cfg.top_k, cfg.n_shared, cfg.group_size

    # ---- layers: layer 0 from the CPU streams (the oracle can see it), the rest drawn on the GPU
    t0 = time.time()
    layers, xs = [], []
    L0 = synth.make_layer(cfg, 0, quant_device=dev)
    n_res = cfg.n_resident or E
    for li in range(n_layers):
        L = L0 if li == 0 else synth.make_layer(cfg, li, device=dev)
        D = DeviceLayer(ctx, cfg, L, max_tokens=T, resident=list(range(n_res)),
                        n_slots=n_res + (min(E, T * k) if n_res < E else 0))
        layers.append(D)
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

    # ---- eager timing
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
        ms_step, launch = ms_graph, "hipgraph"

    # ---- what the steps computed: distinct experts per verify call, from the ids
    torch.cuda.synchronize()
    uniq = [len(set(bufs[li]["idv"].cpu().numpy().reshape(-1).tolist())) for li in range(n_layers)]
    mean_u = float(np.mean(uniq))

    # ---- per-kernel time (eager, event pairs around every kernel launch)
    kern = {}
    if not args.no_profile:
        ctx.profile_enable(True)
        for i in range(args.steps):
            step((args.warmup + i) % n_layers)
        torch.cuda.synchronize()
        prof = ctx.profile_read()
        ctx.profile_enable(False)
        kern = {n: {"ms_total": ms, "launches": cnt, "us_avg": 1e3 * ms / cnt} for n, (ms, cnt) in prof.items() if cnt}

    # ---- algorithmic bytes
    P = 3 * H * I
    int4_expert = P // 2 + (P // g) * 4
    draft_bytes = k * int4_expert + S * 2 * P + E * H * 2 + H * 2 + H * 4          # one token
    mean_u_run = float(np.mean([uniq[(args.warmup + i) % n_layers] for i in range(args.steps)]))
    verify_bytes = mean_u_run * 2 * P + S * 2 * P + E * H * 2 + T * H * 4
    # per-launch algorithmic bytes of the three weight-streaming kernels (what the method must
    # move: the selected experts' weights once, plus the small operands)
    kbytes = {
        "draft_fused_kernel": k * int4_expert + E * H * 2 + H * 2 + H * 4,
        "bf16_gateup_kernel": (mean_u_run + S) * (2 * H * I * 2) + T * H * 2,
        "bf16_down_kernel": (mean_u_run + S) * (H * I * 2) + T * k * I * 2,
    }
    traffic = {}
    tpath = os.path.join(ROOT, "profiles", "pmc_traffic.json")   # HBM bytes per launch from committed PMC runs
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(cfg.name, {})
        except Exception:
            traffic = {}
    roofline, extra = None, {}
    if kern:
        table = {}
        for name, nbytes in kbytes.items():
            kk = kern.get(name)
            if not kk or (S > 0 and name != "draft_fused_kernel"):
                continue        # with shared experts the bf16 kernels also run inside draft calls
            ach = nbytes / (kk["us_avg"] * 1e-6) / 1e9
            table[name] = {"kernel": name, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                           "traffic": traffic.get(name), "bytes_per_launch": int(nbytes),
                           "us_per_launch": round(kk["us_avg"], 2), "launches": kk["launches"],
                           "ms_total": round(kk["ms_total"], 3)}
        if table:
            roofline = max(table.values(), key=lambda r: r["ms_total"])      # most time in the timed region
            extra["kernels"] = table
        extra["kernel_us"] = {n: round(v["us_avg"], 2) for n, v in kern.items()}

    # ---- CPU baseline: the oracle on layer 0's step
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        from tests.common import oracle_arrays, oracle_draft, oracle_verify
        A = oracle_arrays(L0)
        tc = time.time()
        reps = 0
        while time.time() - tc < 10.0 and reps < 64:         # bounded sample: >= 10 s of oracle work
            x0 = synth.make_tokens(cfg, T, layer=0, step=reps)
            oracle_draft(A, x0[:K])
            oracle_verify(A, x0)
            reps += 1
        dt = time.time() - tc
        cpu = {"value": round(reps * (2 * K + 1) / dt, 3), "unit": "tokens/s", "cores": orc.num_threads(),
               "kind": "oracle", "seconds": round(dt, 2),
               "sample": "%d steps of layer 0 (fresh tokens each): %d draft tokens (int4) + one verify of %d "
                         "tokens (bf16) per step" % (reps, K, T)}

    tokens = 2 * K + 1
    out = {
        "metric": "MoE-layer draft+verify tokens/s and achieved HBM GB/s vs peak, 1 GPU", "value": round(tokens / (ms_step * 1e-3), 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int4+bf16 (fp32 accumulate)", "data": "synthetic",
        "config": {"workload": "%s-shaped MoE layer: H%d E%d I%d top%d g%d S%d, K=%d draft tokens + verify of %d, "
                               "%d distinct layers" % (cfg.name, H, E, I, k, g, S, K, T, n_layers),
                   "launch": launch, "tokens_per_step": tokens,
                   "mean_distinct_experts_per_verify": round(mean_u, 2)},
        "ms_per_step_eager": round(ms_eager, 4),
        "algorithmic_GBs_step": round((K * draft_bytes + verify_bytes) / (ms_step * 1e-3) / 1e9, 1),
        "roofline": roofline, "cpu_baseline": cpu,
    }
    out.update(extra)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
