"""Cache-coverage experiment of the paper's "Impact of Prefetch Strategy" study (its hit-rate
table), on synthetic routing: expert ids come from moe_route_topk on the GPU over a stack of
layers and a stream of tokens (AR(1) activations, so that neighbouring tokens share experts), the
caching strategies are played on the host with the Expert Scheduler (moe_elb_*, moe_cache_*,
moe_sched_*).

A decoding cycle verifies K drafted tokens and one more (K + 1 rows); the draft pass has routed
the first K of them, so those K rows are what the lookahead buffer can hold.  After the cycle
a + 1 tokens are kept (a = accepted drafts, drawn with a fixed per-token acceptance probability)
and the stream moves on by that much.  Coverage = of the distinct experts a layer's verify step
needs, the share resident when it starts (summed over layers and cycles), the metric of that table.

Strategies: lru (no prefetch, misses loaded on demand), lru with more slots, single prefetch (the
buffer holds one drafted token: the first = "sooner", the last = "later"), speculative (the whole
window).  Run:  python -m paper_2511_14102_amd.cache_sim [--config dsv2lite] [--tokens 600]
"""
import argparse
import json
import sys

import numpy as np


def route_stream(cfg, n_tokens, n_layers, kind="ar1"):
    """ids [n_layers, n_tokens, k] (int), conf the same shape, from the GPU router."""
    import torch
    import synth
    from . import binding as B
    ctx = B.Context(0)
    desc = B.LayerDesc.from_config(cfg)
    k = cfg.top_k
    ids_all = np.empty((n_layers, n_tokens, k), dtype=np.int32)
    conf_all = np.empty((n_layers, n_tokens, k), dtype=np.float32)
    for li in range(n_layers):
        router = synth.make_router(cfg, li).cuda()
        x = synth.make_tokens(cfg, n_tokens, layer=li, kind=kind).cuda()
        ids = torch.empty((n_tokens, k), dtype=torch.int32, device="cuda")
        w = torch.empty((n_tokens, k), dtype=torch.float32, device="cuda")
        conf = torch.empty((n_tokens, k), dtype=torch.float32, device="cuda")
        for t0 in range(0, n_tokens, 16):
            t1 = min(n_tokens, t0 + 16)
            ctx.route_topk(desc, x[t0:t1], router, None, t1 - t0, ids[t0:t1], w[t0:t1], conf[t0:t1])
        torch.cuda.synchronize()
        ids_all[li] = ids.cpu().numpy()
        conf_all[li] = conf.cpu().numpy()
    return ids_all, conf_all


def play(ids, conf, n_experts, n_slots, K, strategy, accept_p, seed=0, metric="window"):
    """Returns (hits, misses, experts fetched) of one strategy over the stream.

    metric "window": a layer's step is the verify call over all K + 1 rows at once (what
    moe_verify_layer_bf16 does), so the cache has to hold the union of the window.
    metric "token": a step is one token of the window (K + 1 steps per layer and cycle, each needing
    its top-k experts), the paper's per-decoding-step view; a drafted token's experts are fetched
    right before its step, the last token of the window is never predicted."""
    from . import sched as S
    L, N, k = ids.shape
    cache = S.Cache(L, n_experts, n_slots)
    elb = S.Elb(L, K, k)
    rng = np.random.default_rng(seed)
    pos, fetched = 0, 0
    predicted = {"lru": [], "single_sooner": [0], "single_later": [K - 1], "speculative": list(range(K))}[strategy]

    def demand(li, need):
        table = cache.slot_table(li)
        missing = sorted({e for e in need if table[e] < 0})
        # a step may need more experts than the layer has slots: load what fits (the rest would
        # take a further pass; they are counted as misses already)
        return len(cache.on_demand(li, missing[:n_slots]))

    while pos + K + 1 <= N:
        if metric == "window":
            if predicted:
                elb.reset()
                for step, row in enumerate(predicted):
                    elb.put_step(step, ids[:, pos + row, :].tolist(), conf[:, pos + row, :].tolist())
                fetched += len(cache.plan(elb, S.PHASE_SATURATE))
            for li in range(L):
                need = ids[li, pos:pos + K + 1, :].reshape(-1).tolist()
                cache.use(li, need)
                fetched += demand(li, need)
            cache.end_window()
        else:
            for row in range(K + 1):
                if row in predicted:
                    elb.reset()
                    elb.put_step(0, ids[:, pos + row, :].tolist(), conf[:, pos + row, :].tolist())
                    fetched += len(cache.plan(elb, S.PHASE_SATURATE))
                for li in range(L):
                    need = ids[li, pos + row, :].tolist()
                    cache.use(li, need)
                    fetched += demand(li, need)
                cache.end_window()
        a = 0
        while a < K and rng.random() < accept_p:
            a += 1
        pos += a + 1
    h, m = cache.stats()
    cache.close()
    elb.close()
    return h, m, fetched


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="dsv2lite")
    ap.add_argument("--tokens", type=int, default=600)
    ap.add_argument("--layers", type=int, default=0)
    ap.add_argument("--K", type=int, default=0, help="drafted tokens per cycle (0: the config's verify length - 1)")
    ap.add_argument("--accept", type=float, default=0.8)
    ap.add_argument("--slots", default="6,16,32")
    ap.add_argument("--scaled", default="22,32,48", help="slot counts of the 'lru (scaled)' rows, one per --slots entry")
    ap.add_argument("--metric", default="both", choices=["window", "token", "both"])
    args = ap.parse_args(argv)
    import synth
    cfg = synth.config_by_name(args.config)
    L = args.layers or cfg.n_layers or cfg.bench_layers
    K = args.K or (max(cfg.verify_tokens) - 1)
    ids, conf = route_stream(cfg, args.tokens, L)
    E = cfg.n_experts
    rows = []
    for metric in (["window", "token"] if args.metric == "both" else [args.metric]):
        for C, Cs in zip([int(v) for v in args.slots.split(",")], [int(v) for v in args.scaled.split(",")]):
            for name, slots, strat in (("lru", C, "lru"), ("lru (scaled)", min(Cs, E), "lru"),
                                       ("single prefetch (sooner)", C, "single_sooner"),
                                       ("single prefetch (later)", C, "single_later"),
                                       ("speculative", C, "speculative")):
                h, m, f = play(ids, conf, E, slots, K, strat, args.accept, metric=metric)
                rows.append({"metric": metric, "capacity": C, "method": name, "slots": slots,
                             "coverage_pct": round(100.0 * h / (h + m), 2), "fetched_experts": f})
                print("%-6s %-3d %-26s slots %-3d coverage %6.2f %%  fetched %d" %
                      (metric, C, name, slots, rows[-1]["coverage_pct"], f), file=sys.stderr, flush=True)
    print(json.dumps({"config": cfg.name, "layers": L, "tokens": args.tokens, "K": K, "accept_p": args.accept,
                      "distinct_needed_per_layer_step": round(float(np.mean(
                          [len(set(ids[li, p:p + K + 1].reshape(-1).tolist())) for li in range(L)
                           for p in range(0, args.tokens - K - 1, K + 1)])), 2),
                      "rows": rows}))


if __name__ == "__main__":
    main()
