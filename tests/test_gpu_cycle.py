"""A draft -> prefetch -> verify cycle over a stack with the Expert Scheduler in charge of the
expert cache: draft calls emit ids, the lookahead buffer and the three-phase plan decide the
copies (pinned host -> slot, side stream, ordered by events), the verify calls read through the
scheduler's slot tables, misses are fetched on demand and accumulated.  Every layer's draft and
verify output is compared with the fp64 oracle, over several cycles with a cache too small for
everything.

Two stacks: the tiny shape (3 layers, 5 slots), and the DeepSeek-V2-Lite-shaped workload in its
own form (paper sections 3.3.2 and 4.1.2, Table 1): 64 routed + 2 shared experts, top-6, 16 of the
64 resident at the start in slot numbers that are neither the expert numbers nor ascending, 52
slots per layer, all 64 experts of every layer in pinned host memory."""
import numpy as np
import pytest
import torch

import synth
from paper_2511_14102_amd import binding as B
from paper_2511_14102_amd import pack
from paper_2511_14102_amd import sched as S
from paper_2511_14102_amd.harness import DeviceLayer
from tests.common import oracle_arrays, oracle_draft, oracle_verify, rel_err
from tests.gpu_common import TOL_DRAFT, TOL_VERIFY, build_layer, say, to_np, tokens_with_clear_routing

pytestmark = pytest.mark.gpu


def run_stack_cycles(cfg, n_layers, n_slots, residents, T, cycles, guided_budget):
    """residents: per layer a list of (expert, slot) pairs that are in the cache at the start."""
    ctx = B.Context(0)
    E, k = cfg.n_experts, cfg.top_k
    K = T - 1
    layers, host, As = [], [], []
    cache = S.Cache(n_layers, E, n_slots)
    for li in range(n_layers):
        L = build_layer(cfg, li)
        As.append(oracle_arrays(L))
        D = DeviceLayer(ctx, cfg, L, max_tokens=T, resident=[], n_slots=n_slots)
        hb = torch.empty((E, D.bf16_bytes), dtype=torch.uint8).pin_memory()
        for e in range(E):
            hb[e].copy_(pack.pack_bf16_expert(L["gate"][e].cuda(), L["up"][e].cuda(), L["down"][e].cuda()))
        # slots start out holding bf16 NaN patterns: whatever a verify call reads before its copy
        # has landed shows in the result
        D.slot_pool.fill_(0xFF)
        for (e, slot) in residents[li]:
            D.slot_view(slot).copy_(hb[e])
            D.set_slot(e, slot)
            cache.place(li, e, slot)
        layers.append(D)
        host.append(hb)
        del L
        say("  layer %d on the device, %d resident experts" % (li, len(residents[li])))
    blob = layers[0].bf16_bytes
    copy_stream = torch.cuda.Stream()
    main = torch.cuda.current_stream()
    done = [torch.cuda.Event() for _ in range(n_layers)]

    def apply(fetches):
        """Poison each destination slot, copy the expert in on the side stream, upload the touched
        layers' slot tables behind the copies and record the layer's event; the compute stream
        waits for the events."""
        touched = []
        for (li, e, slot, _ev) in fetches:
            with torch.cuda.stream(copy_stream):
                layers[li].slot_view(slot).fill_(0xFF)
            ctx.expert_copy_async(layers[li].slot_view(slot), host[li][e], blob, copy_stream, None)
            if li not in touched:
                touched.append(li)
        for li in touched:
            table = torch.tensor(cache.slot_table(li), dtype=torch.int32).pin_memory()
            with torch.cuda.stream(copy_stream):
                layers[li].slot_of_expert.copy_(table, non_blocking=True)
            done[li].record(copy_stream)
            main.wait_event(done[li])

    total_fetch, on_demand = 0, 0
    for cyc in range(cycles):
        say("cycle", cyc)
        xs = [tokens_with_clear_routing(cfg, As[li], T, layer=li, step=50 + cyc) for li in range(n_layers)]
        xd = [x.cuda() for x in xs]
        yd = torch.empty((n_layers, K, cfg.hidden), dtype=torch.float32, device="cuda")
        win = torch.empty((K, n_layers, k), dtype=torch.int32, device="cuda")       # [step, layer, k]
        wconf = torch.empty((K, n_layers, k), dtype=torch.float32, device="cuda")
        elb = S.Elb(n_layers, K, k)
        for i in range(K):                                   # draft token by token through the stack
            for li, D in enumerate(layers):
                D.draft(xd[li][i:i + 1], y=yd[li, i:i + 1], ids=win[i, li:li + 1], conf=wconf[i, li:li + 1])
            torch.cuda.synchronize()
            elb.put_step(i, win[i].cpu().tolist(), wconf[i].cpu().tolist())
            phase = S.PHASE_SATURATE if i == K - 1 else (S.PHASE_PRIME if i == 0 else S.PHASE_GUIDED)
            copy_stream.wait_stream(main)
            fetches = cache.plan(elb, phase, guided_budget, 0.0)
            total_fetch += len(fetches)
            apply(fetches)
        for li, D in enumerate(layers):
            ref_d = oracle_draft(As[li], xs[li][:K])
            assert np.array_equal(to_np(win[:, li]), ref_d["ids"])
            ed = rel_err(to_np(yd[li]), ref_d["y"])
            assert ed <= TOL_DRAFT, "layer %d draft rel err %.3e" % (li, ed)
            ref = oracle_verify(As[li], xs[li])
            r = D.verify(xd[li])
            torch.cuda.synchronize()
            assert np.array_equal(to_np(r["ids"]), ref["ids"])
            cache.use(li, ref["ids"].reshape(-1).tolist())
            nm = int(r["n_missing"].item())
            # the scheduler's table and the kernel agree on what is missing (ascending list)
            table = cache.slot_table(li)
            assert to_np(r["missing"])[:nm].tolist() == sorted({e for e in ref["ids"].reshape(-1).tolist() if table[e] < 0})
            if nm:
                copy_stream.wait_stream(main)
                fetches = cache.on_demand(li, to_np(r["missing"])[:nm].tolist())
                total_fetch += nm
                on_demand += nm
                apply(fetches)
                D.verify(xd[li], flags=B.MOE_VERIFY_ACCUMULATE | B.MOE_VERIFY_ONLY_LISTED, y=r["y"])
                torch.cuda.synchronize()
                assert int(r["n_missing"].item()) == 0
            yv = to_np(r["y"])
            assert np.isfinite(yv).all()
            e = rel_err(yv, ref["y"])
            say("  layer %d: draft rel err %.3e, %d on demand, verify rel err %.3e" % (li, ed, nm, e))
            assert e <= TOL_VERIFY
        cache.end_window()
        elb.close()
    hits, misses = cache.stats()
    say("coverage %.1f %%, %d experts fetched (%d on demand)" % (100.0 * hits / (hits + misses), total_fetch, on_demand))
    assert total_fetch > 0 and hits > 0
    return total_fetch, on_demand


def test_scheduler_driven_cycles_match_the_oracle():
    cfg = synth.config_by_name("tiny")
    run_stack_cycles(cfg, n_layers=3, n_slots=5, residents=[[(0, 0), (1, 1)]] * 3, T=4, cycles=4, guided_budget=2)


def test_dsv2lite_stack_partial_residency_side_stream_copies():
    cfg = synth.config_by_name("dsv2lite")
    assert cfg.n_experts == 64 and cfg.n_resident == 16 and cfg.n_shared == 2 and cfg.top_k == 6
    n_layers, n_slots = 3, 52
    rng = np.random.Generator(np.random.PCG64(20251))
    residents = []
    for li in range(n_layers):
        experts = rng.permutation(cfg.n_experts)[:cfg.n_resident]
        slots = rng.permutation(n_slots)[:cfg.n_resident]
        pairs = [(int(e), int(s)) for e, s in zip(experts, slots)]
        assert any(e != s for e, s in pairs) and [s for _, s in pairs] != sorted(s for _, s in pairs)
        residents.append(pairs)
    fetched, on_demand = run_stack_cycles(cfg, n_layers, n_slots, residents, T=max(cfg.verify_tokens), cycles=2,
                                          guided_budget=8)
    # the draft saw K of the K+1 rows, so some of the last row's experts come in on demand
    assert fetched > on_demand > 0
