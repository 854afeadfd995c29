"""Parity of the HIP path (through the C ABI) with the CPU oracle on the five workloads.
Integers (ids, histogram, permutation, union, missing lists) must match bit for bit; float
outputs within max|y - y_oracle| <= tol * rms(y_oracle) with tol = 2e-2 for the bf16 verify
pass and 1e-3 for the int4 draft pass."""
import gc

import numpy as np
import pytest
import torch

import synth
from oracle import oracle as orc
from tests.common import oracle_arrays, oracle_draft, oracle_verify, rel_err, bf16_exact
from tests.gpu_common import (TOL_DRAFT, TOL_VERIFY, build_layer, say, to_np,
                              tokens_with_clear_routing)

pytestmark = pytest.mark.gpu

from paper_2511_14102_amd import binding as B          # noqa: E402
from paper_2511_14102_amd.harness import DeviceLayer   # noqa: E402


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = B.Context(0)
    yield c
    c.close()


class Case:
    """One config on the device plus its oracle-side arrays."""

    def __init__(self, ctx, cfg, layer=0, bias=None, resident=None, n_slots=None):
        say("building", cfg.name, "layer", layer, "bias", bias)
        self.cfg = cfg
        self.L = build_layer(cfg, layer, bias=bias)
        self.A = oracle_arrays(self.L)
        self.D = DeviceLayer(ctx, cfg, self.L, max_tokens=max(max(cfg.verify_tokens), 8),
                             resident=resident, n_slots=n_slots)
        torch.cuda.synchronize()
        say("  on device")


@pytest.fixture(scope="module", params=[c.name for c in synth.CONFIGS])
def case(request, ctx):
    cfg = synth.config_by_name(request.param)
    c = Case(ctx, cfg)
    yield c
    del c
    gc.collect()
    torch.cuda.empty_cache()


def check_route(case, x, r, ref_ids, ref_w, ref_conf):
    cfg = case.cfg
    assert np.array_equal(to_np(r["ids"]), ref_ids)
    np.testing.assert_allclose(to_np(r["w"]), ref_w, rtol=2e-6, atol=1e-9)
    np.testing.assert_allclose(to_np(r["conf"]), ref_conf, rtol=2e-6, atol=1e-12)
    if r.get("count") is not None:
        cnt, off, pm = orc.perm(ref_ids, cfg.n_experts)
        assert np.array_equal(to_np(r["count"]), cnt)
        assert np.array_equal(to_np(r["off"]), off)
        assert np.array_equal(to_np(r["perm"]), pm)


def test_route_topk(case):
    cfg = case.cfg
    for T in sorted(set(cfg.verify_tokens) | {1}):
        x = tokens_with_clear_routing(cfg, case.A, T, step=T)
        say("route", cfg.name, "T", T)
        r = case.D.route(x.cuda())
        torch.cuda.synchronize()
        ids, w, conf, _ = orc.route(orc.bits(x), case.A["router"], case.A["bias"], cfg.top_k,
                                    cfg.renormalize)
        check_route(case, x, r, ids, w, conf)


def test_draft_layer(case):
    cfg = case.cfg
    T = max(cfg.verify_tokens)
    x = tokens_with_clear_routing(cfg, case.A, T, step=10)
    ref = oracle_draft(case.A, x)
    # canonical use: one token per call, K+1 calls
    for t in range(T):
        say("draft", cfg.name, "token", t)
        r = case.D.draft(x[t:t + 1].cuda())
        torch.cuda.synchronize()
        assert np.array_equal(to_np(r["ids"]), ref["ids"][t:t + 1])
        np.testing.assert_allclose(to_np(r["conf"]), ref["conf"][t:t + 1], rtol=2e-6)
        e = rel_err(to_np(r["y"]), ref["y"][t:t + 1])
        say("   rel err %.3e" % e)
        assert e <= TOL_DRAFT
    # several tokens in one call (each distinct expert streamed once)
    Tm = min(T, 8)
    say("draft", cfg.name, "T", Tm, "in one call")
    r = case.D.draft(x[:Tm].cuda())
    torch.cuda.synchronize()
    assert np.array_equal(to_np(r["ids"]), ref["ids"][:Tm])
    e = rel_err(to_np(r["y"]), ref["y"][:Tm])
    say("   rel err %.3e" % e)
    assert e <= TOL_DRAFT
    # same call again: identical ids; y is summed with fp32 atomics, so only its last bits may move
    r2 = case.D.draft(x[:Tm].cuda())
    torch.cuda.synchronize()
    assert torch.equal(r["ids"], r2["ids"]) and torch.equal(r["conf"], r2["conf"])
    assert rel_err(to_np(r2["y"]), to_np(r["y"])) <= 1e-5


@pytest.mark.parametrize("name", ["tiny", "phi", "qwen3", "dsv2lite"])
def test_draft_layer_symmetric_format(ctx, name):
    # z = 8 in every group, scale blobs on the device (group sizes 32, 128, 64, 128; the last
    # with shared experts); the oracle sees the same codes and scales with an explicit z = 8
    cfg = synth.config_by_name(name)
    say("building", cfg.name, "symmetric int4")
    qdev = "cuda:0"
    L = synth.make_layer(cfg, 0, quant_device=qdev, symmetric=True)
    A = oracle_arrays(L)
    D = DeviceLayer(ctx, cfg, L, max_tokens=8, verify=False, symmetric=True)
    D2 = DeviceLayer(ctx, cfg, L, max_tokens=8, verify=False) if name in ("tiny", "qwen3") else None
    torch.cuda.synchronize()
    T = min(max(cfg.verify_tokens), 8)
    x = tokens_with_clear_routing(cfg, A, T, step=20)
    ref = oracle_draft(A, x)
    for t in range(min(T, 3)):
        say("draft (symmetric)", cfg.name, "token", t)
        r = D.draft(x[t:t + 1].cuda())
        torch.cuda.synchronize()
        assert np.array_equal(to_np(r["ids"]), ref["ids"][t:t + 1])
        e = rel_err(to_np(r["y"]), ref["y"][t:t + 1])
        say("   rel err %.3e" % e)
        assert e <= TOL_DRAFT
    for Tm in sorted({2, min(T, 4), T}):
        say("draft (symmetric)", cfg.name, "T", Tm, "in one call")
        r = D.draft(x[:Tm].cuda())
        torch.cuda.synchronize()
        assert np.array_equal(to_np(r["ids"]), ref["ids"][:Tm])
        np.testing.assert_allclose(to_np(r["conf"]), ref["conf"][:Tm], rtol=2e-6)
        e = rel_err(to_np(r["y"]), ref["y"][:Tm])
        say("   rel err %.3e" % e)
        assert e <= TOL_DRAFT
        if D2 is not None:      # the general format holding z = 8 computes the same sums
            r2 = D2.draft(x[:Tm].cuda())
            torch.cuda.synchronize()
            assert torch.equal(r["ids"], r2["ids"])
            assert rel_err(to_np(r2["y"]), to_np(r["y"])) <= 1e-5
    if name in ("tiny", "dsv2lite"):    # the prefill form reads the same scale blobs
        Tp = 37 if name == "tiny" else 20
        xp = tokens_with_clear_routing(cfg, A, Tp, step=21, kind="iid")
        refp = oracle_draft(A, xp)
        say("prefill (symmetric)", cfg.name, "T", Tp)
        rp = D.prefill(xp.cuda())
        torch.cuda.synchronize()
        assert np.array_equal(to_np(rp["ids"]), refp["ids"])
        e = rel_err(to_np(rp["y"]), refp["y"])
        say("   rel err %.3e" % e)
        assert e <= TOL_DRAFT
    del D, D2
    gc.collect()
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name,tokens", [("tiny", (1, 9, 37, 200, 1500, 4096)), ("qwen3", (40,)), ("phi", (48,)),
                                         ("dsv2lite", (5, 45))])
def test_draft_prefill(ctx, name, tokens):
    # many tokens in one call: routed first, grouped by expert, up to 64 assignments of an expert per item
    cfg = synth.config_by_name(name)
    say("building", cfg.name, "for prefill")
    L = build_layer(cfg)
    A = oracle_arrays(L)
    D = DeviceLayer(ctx, cfg, L, max_tokens=8, verify=False)
    torch.cuda.synchronize()
    for T in tokens:
        x = tokens_with_clear_routing(cfg, A, T, step=30 + T, kind="iid")
        ref = oracle_draft(A, x)
        say("prefill", cfg.name, "T", T)
        r = D.prefill(x.cuda())
        torch.cuda.synchronize()
        assert np.array_equal(to_np(r["ids"]), ref["ids"])
        np.testing.assert_allclose(to_np(r["conf"]), ref["conf"], rtol=2e-6)
        e = rel_err(to_np(r["y"]), ref["y"])
        say("   rel err %.3e" % e)
        assert e <= TOL_DRAFT
        if T <= 8:                       # the same tokens through the one-launch draft call
            r1 = D.draft(x.cuda())
            torch.cuda.synchronize()
            assert torch.equal(r1["ids"], r["ids"])
            # two kernels with different fp32 summation orders, each within TOL_DRAFT of the oracle
            assert rel_err(to_np(r1["y"]), to_np(r["y"])) <= 1e-4
    # a second call reuses the workspace (nothing is carried over) and a draft call still works after it
    r2 = D.prefill(x.cuda())
    torch.cuda.synchronize()
    assert torch.equal(r2["ids"], r["ids"]) and rel_err(to_np(r2["y"]), to_np(r["y"])) <= 1e-5
    r3 = D.draft(x[:1].cuda())
    torch.cuda.synchronize()
    assert np.array_equal(to_np(r3["ids"]), ref["ids"][:1])
    assert rel_err(to_np(r3["y"]), ref["y"][:1]) <= TOL_DRAFT
    del D
    gc.collect()
    torch.cuda.empty_cache()


def test_verify_layer(case):
    cfg = case.cfg
    for T in cfg.verify_tokens:
        x = tokens_with_clear_routing(cfg, case.A, T, step=20 + T)
        ref = oracle_verify(case.A, x)
        say("verify", cfg.name, "T", T, "unique experts", len(set(ref["ids"].reshape(-1).tolist())))
        r = case.D.verify(x.cuda())
        torch.cuda.synchronize()
        assert np.array_equal(to_np(r["ids"]), ref["ids"])
        assert int(r["n_missing"].item()) == 0
        e = rel_err(to_np(r["y"]), ref["y"])
        say("   rel err %.3e" % e)
        assert e <= TOL_VERIFY
        r2 = case.D.verify(x.cuda())
        torch.cuda.synchronize()
        assert torch.equal(r["y"], r2["y"])


def test_union_of_window(case):
    cfg = case.cfg
    E = cfg.n_experts
    rng = np.random.default_rng(cfg.index)
    slot = np.where(rng.random(E) < 0.5, np.arange(E), -1).astype(np.int32)
    saved = case.D.slot_of_expert.clone()
    case.D.slot_of_expert.copy_(torch.from_numpy(slot))
    try:
        for n in (0, 1, 7, cfg.top_k * 8, 5 * cfg.top_k * 8):
            ids = rng.integers(0, E, n).astype(np.int32)
            say("union", cfg.name, "n", n)
            r = case.D.union(torch.from_numpy(ids).cuda())
            torch.cuda.synchronize()
            mask, lst, miss = orc.union(ids, E, slot)
            assert np.array_equal(to_np(r["mask"]).view(np.uint64), mask)
            nl, nm = int(r["n_list"].item()), int(r["n_missing"].item())
            assert nl == lst.size and nm == miss.size
            assert np.array_equal(to_np(r["list"])[:nl], lst)
            assert np.array_equal(to_np(r["missing"])[:nm], miss)
            r = case.D.union(torch.from_numpy(ids).cuda(), use_slots=False)
            torch.cuda.synchronize()
            assert int(r["n_missing"].item()) == 0 and int(r["n_list"].item()) == lst.size
    finally:
        case.D.slot_of_expert.copy_(saved)


def test_mixtral_all_tokens_same_experts(case):
    cfg = case.cfg
    if cfg.name != "mixtral":
        pytest.skip("the skew case belongs to the mixtral-shaped workload")
    saved_bias, saved_A = case.D.bias, case.A["bias"]
    case.D.bias = synth.skew_bias(cfg).cuda()
    case.A["bias"] = synth.skew_bias(cfg).numpy()
    try:
        x = synth.make_tokens(cfg, 8, step=61)
        ref = oracle_verify(case.A, x)
        assert len(set(ref["ids"].reshape(-1).tolist())) == 2
        say("mixtral skew: verify T=8, 2 distinct experts")
        r = case.D.verify(x.cuda())
        torch.cuda.synchronize()
        assert np.array_equal(to_np(r["ids"]), ref["ids"])
        e = rel_err(to_np(r["y"]), ref["y"])
        say("   rel err %.3e" % e)
        assert e <= TOL_VERIFY
    finally:
        case.D.bias, case.A["bias"] = saved_bias, saved_A


# ---------------------------------------------------------------- special cases (tiny shape)

@pytest.fixture(scope="module")
def tiny(ctx):
    return Case(ctx, synth.config_by_name("tiny"))


def test_exact_ties_pick_the_lower_index(ctx, tiny):
    cfg = tiny.cfg
    L = dict(tiny.L)
    row = L["router"][2:3]
    L["router"] = row.repeat(cfg.n_experts, 1).contiguous()          # all logits exactly equal
    D = DeviceLayer(ctx, cfg, L, max_tokens=4, draft=False, verify=False)
    x = synth.make_tokens(cfg, 4, step=77)
    say("ties: duplicate router rows")
    r = D.route(x.cuda())
    torch.cuda.synchronize()
    assert np.array_equal(to_np(r["ids"]), np.tile(np.arange(cfg.top_k, dtype=np.int32), (4, 1)))
    np.testing.assert_allclose(to_np(r["w"]), 1.0 / cfg.top_k, rtol=1e-6)
    # small integers: logits exact on both sides, many ties
    rng = np.random.default_rng(5)
    xi = bf16_exact(rng.integers(-2, 3, (4, cfg.hidden)).astype(np.float64))
    L["router"] = bf16_exact(rng.integers(-1, 2, (cfg.n_experts, cfg.hidden)).astype(np.float64))
    L["router"][5] = L["router"][1]
    D = DeviceLayer(ctx, cfg, L, max_tokens=4, draft=False, verify=False)
    say("ties: small-integer logits")
    r = D.route(xi.cuda())
    torch.cuda.synchronize()
    ids, w, conf, _ = orc.route(orc.bits(xi), orc.bits(L["router"]), None, cfg.top_k, True)
    assert np.array_equal(to_np(r["ids"]), ids)
    np.testing.assert_allclose(to_np(r["w"]), w, rtol=2e-6)


def test_renormalize_off_and_bias(ctx, tiny):
    cfg = tiny.cfg
    L = dict(tiny.L)
    L["router_bias"] = torch.linspace(-1, 1, cfg.n_experts)
    D = DeviceLayer(ctx, cfg, L, max_tokens=4)
    D.desc.renormalize = 0
    A = oracle_arrays(L)
    x = synth.make_tokens(cfg, 4, step=31)
    xb = orc.bits(x)
    ids, w, conf, _ = orc.route(xb, A["router"], A["bias"], cfg.top_k, False)
    say("renormalize off + bias: route")
    r = D.route(x.cuda())
    torch.cuda.synchronize()
    assert np.array_equal(to_np(r["ids"]), ids)
    np.testing.assert_allclose(to_np(r["w"]), conf, rtol=2e-6)
    y = orc.layer_bf16(xb, A["gate"], A["up"], A["down"], cfg.n_experts, ids, w)
    say("renormalize off + bias: verify")
    rv = D.verify(x.cuda())
    torch.cuda.synchronize()
    assert rel_err(to_np(rv["y"]), y) <= TOL_VERIFY


def test_missing_experts_and_on_demand_accumulate(ctx, tiny):
    cfg = tiny.cfg
    E = cfg.n_experts
    x = tokens_with_clear_routing(cfg, tiny.A, 4, step=41)
    ref = oracle_verify(tiny.A, x)
    used = sorted(set(ref["ids"].reshape(-1).tolist()))
    absent = used[::2]                                     # every other used expert is not resident
    resident = [e for e in range(E) if e not in absent]
    D = DeviceLayer(ctx, cfg, tiny.L, max_tokens=4, resident=resident, n_slots=E, draft=False)
    present = np.ones(E, np.uint8); present[absent] = 0
    part = oracle_verify(tiny.A, x, present=present)
    say("missing: first call, absent", absent)
    r = D.verify(x.cuda())
    torch.cuda.synchronize()
    nm = int(r["n_missing"].item())
    assert nm == len(absent) and to_np(r["missing"])[:nm].tolist() == absent
    assert rel_err(to_np(r["y"]), part["y"]) <= TOL_VERIFY
    # strict mode reports it as an error
    with pytest.raises(B.MoeError) as ei:
        D.verify(x.cuda(), flags=B.MOE_VERIFY_STRICT)
    assert ei.value.status == B.MOE_ERR_MISSING_EXPERT
    # fetch the missing experts from pinned host memory on a side stream, then add their terms
    y = r["y"]
    D.verify(x.cuda(), y=y)                                # recompute the partial sum (strict call overwrote nothing else)
    copy_stream = torch.cuda.Stream()
    ev = torch.cuda.Event()
    ev.record(copy_stream)                                 # torch creates the HIP event on first record
    from paper_2511_14102_amd import pack
    for i, e in enumerate(absent):
        blob = pack.pack_bf16_expert(tiny.L["gate"][e], tiny.L["up"][e], tiny.L["down"][e]).pin_memory()
        slot = len(resident) + i
        ctx.expert_copy_async(D.slot_view(slot), blob, blob.numel(), copy_stream, ev)
        D.set_slot(e, slot)
    torch.cuda.current_stream().wait_event(ev)
    say("missing: accumulate call")
    r2 = D.verify(x.cuda(), flags=B.MOE_VERIFY_ACCUMULATE | B.MOE_VERIFY_ONLY_LISTED, y=y)
    torch.cuda.synchronize()
    assert int(r2["n_missing"].item()) == 0
    assert rel_err(to_np(y), ref["y"]) <= TOL_VERIFY
    # slot numbering is irrelevant: a fresh layer with all experts in reversed slots agrees
    D2 = DeviceLayer(ctx, cfg, tiny.L, max_tokens=4, resident=list(range(E))[::-1], draft=False)
    r3 = D2.verify(x.cuda())
    torch.cuda.synchronize()
    assert rel_err(to_np(r3["y"]), ref["y"]) <= TOL_VERIFY


def test_argument_errors_enqueue_nothing(ctx, tiny):
    D = tiny.D
    x = synth.make_tokens(tiny.cfg, 4).cuda()
    with pytest.raises(B.MoeError) as ei:                  # misaligned activations
        bad = torch.empty(4 * 256 + 8, dtype=torch.bfloat16, device="cuda")[1:1 + 4 * 256].view(4, 256)
        D.route(bad)
    assert ei.value.status == B.MOE_ERR_INVALID_ARG
    small = D.workspace
    D.workspace = small[:1024]
    try:
        with pytest.raises(B.MoeError) as ei:
            D.verify(x)
        assert ei.value.status == B.MOE_ERR_WORKSPACE
    finally:
        D.workspace = small
    with pytest.raises(B.MoeError) as ei:                  # draft takes at most 8 tokens
        D.draft(torch.zeros((9, 256), dtype=torch.bfloat16, device="cuda"))
    assert ei.value.status == B.MOE_ERR_INVALID_ARG
    # a hidden size whose token copy does not fit into LDS for 8 tokens (it does for 4): rejected on
    # the host, nothing is read (the buffers here are far too small for the shape)
    big = B.LayerDesc(16384, 4, 128, 1, 0, 128, 1)
    assert B.validate_desc(big) == 0
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    ws = torch.zeros(B.workspace_bytes(big, 8), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.MoeError) as ei:
        ctx.draft_layer_int4(big, buf, buf, None, buf, buf, B.int4_expert_q_bytes(big),
                             B.int4_expert_sz_bytes(big), None, 8, buf, buf, None, ws)
    assert ei.value.status == B.MOE_ERR_INVALID_ARG
    # the call over a long run of tokens (no LDS limit; real buffers of the tiny layer): too many
    # tokens, then a workspace that is too small
    xp = synth.make_tokens(tiny.cfg, 19).cuda()
    yp = torch.empty((19, 256), dtype=torch.float32, device="cuda")
    idp = torch.empty((19, tiny.cfg.top_k), dtype=torch.int32, device="cuda")
    pws = torch.zeros(B.prefill_workspace_bytes(D.desc, 19), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.MoeError) as ei:
        B.prefill_workspace_bytes(D.desc, B.MOE_MAX_PREFILL_TOKENS + 1)
    assert ei.value.status == B.MOE_ERR_INVALID_ARG
    for T, w, status in ((B.MOE_MAX_PREFILL_TOKENS + 1, pws, B.MOE_ERR_INVALID_ARG), (0, pws, B.MOE_ERR_INVALID_ARG),
                         (19, pws[:4096], B.MOE_ERR_WORKSPACE)):
        with pytest.raises(B.MoeError) as ei:
            ctx.draft_prefill_int4(D.desc, xp, D.router, D.bias, D.q_blob, D.sz_blob, D.q_bytes, D.sz_bytes,
                                   D.shared, T, yp, idp, None, w)
        assert ei.value.status == status, (T, status)
    torch.cuda.synchronize()


def test_skew_all_tokens_same_experts(ctx):
    cfg = synth.config_by_name("tiny")
    c = Case(ctx, cfg, bias="skew")
    x = synth.make_tokens(cfg, 4, step=51)
    ref = oracle_verify(c.A, x)
    assert len(set(map(tuple, ref["ids"].tolist()))) == 1
    say("skew: verify")
    r = c.D.verify(x.cuda())
    torch.cuda.synchronize()
    assert np.array_equal(to_np(r["ids"]), ref["ids"])
    assert rel_err(to_np(r["y"]), ref["y"]) <= TOL_VERIFY
    refd = oracle_draft(c.A, x)
    say("skew: draft T=4")
    rd = c.D.draft(x.cuda())
    torch.cuda.synchronize()
    assert rel_err(to_np(rd["y"]), refd["y"]) <= TOL_DRAFT


def test_graph_replays_match_eager_calls(ctx, tiny):
    """A captured draft + union + verify step, replayed several times with new activations in
    the static input buffer and eager work in between, must give what eager calls give."""
    cfg = tiny.cfg
    D = tiny.D
    T, k, H = 4, cfg.top_k, cfg.hidden
    xbuf = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
    yd = torch.empty((1, H), dtype=torch.float32, device="cuda")
    idd = torch.empty((1, k), dtype=torch.int32, device="cuda")
    cfd = torch.empty((1, k), dtype=torch.float32, device="cuda")
    yv = torch.empty((T, H), dtype=torch.bfloat16, device="cuda")
    idv = torch.empty((T, k), dtype=torch.int32, device="cuda")
    xbuf.copy_(synth.make_tokens(cfg, T, step=90).cuda())
    D.draft(xbuf[:1], y=yd, ids=idd, conf=cfd)             # warm up outside capture
    D.verify(xbuf, y=yv, ids=idv)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    say("graph: capture")
    with torch.cuda.graph(g, stream=side):
        D.draft(xbuf[:1], y=yd, ids=idd, conf=cfd)
        D.verify(xbuf, y=yv, ids=idv)
    torch.cuda.synchronize()
    for rep in range(4):
        x = synth.make_tokens(cfg, T, step=91 + rep)
        xbuf.copy_(x.cuda())
        say("graph: replay", rep)
        g.replay()
        torch.cuda.synchronize()
        got = (yd.clone(), idd.clone(), yv.clone(), idv.clone())
        e_d = D.draft(x[:1].cuda())                        # eager work between replays
        e_v = D.verify(x.cuda())
        torch.cuda.synchronize()
        assert torch.equal(got[1], e_d["ids"]) and torch.equal(got[3], e_v["ids"])
        assert rel_err(to_np(got[0]), to_np(e_d["y"])) <= 1e-5
        assert torch.equal(got[2], e_v["y"])
        ref = oracle_draft(tiny.A, x[:1])
        assert np.array_equal(to_np(got[1]), ref["ids"]) and rel_err(to_np(got[0]), ref["y"]) <= TOL_DRAFT


def test_eight_tokens_on_a_small_hidden_size(ctx, tiny):
    # with 5 to 8 tokens the partial gate/up sums reuse the LDS of the x copy, which is smaller than
    # they are when H is small: the launch must size the buffer for both
    cfg, D = tiny.cfg, tiny.D
    for T in (5, 8):
        x = tokens_with_clear_routing(cfg, tiny.A, T, step=500 + T)
        ref = oracle_draft(tiny.A, x)
        r = D.draft(x.cuda())
        torch.cuda.synchronize()
        assert np.array_equal(to_np(r["ids"]), ref["ids"])
        assert rel_err(to_np(r["y"]), ref["y"]) <= TOL_DRAFT


def test_mixed_token_counts_share_one_workspace(ctx, tiny):
    """Draft and verify calls of changing token counts on one layer / one workspace: the counters
    the kernels leave in the workspace (tickets, arrivals, tagged slots) must be back in their idle
    state after every call whatever the grid of the previous one was."""
    cfg, D = tiny.cfg, tiny.D
    rng = np.random.default_rng(7)
    for it in range(24):
        T = int(rng.integers(1, 9))
        x = tokens_with_clear_routing(cfg, tiny.A, T, step=300 + it)
        if it % 3 != 2:
            ref = oracle_draft(tiny.A, x)
            r = D.draft(x.cuda())
            torch.cuda.synchronize()
            assert np.array_equal(to_np(r["ids"]), ref["ids"]), (it, T)
            assert rel_err(to_np(r["y"]), ref["y"]) <= TOL_DRAFT, (it, T)
        else:
            ref = oracle_verify(tiny.A, x)
            r = D.verify(x.cuda())
            torch.cuda.synchronize()
            assert np.array_equal(to_np(r["ids"]), ref["ids"]), (it, T)
            assert rel_err(to_np(r["y"]), ref["y"]) <= TOL_VERIFY, (it, T)


def test_workspace_is_idle_again_after_every_call(ctx, tiny):
    """The contract of moe_workspace_init: counters, status word and the tags of the exchange slots are
    zero whenever no call runs, after draft calls of every launch shape and after verify calls."""
    D, cfg = tiny.D, tiny.cfg
    n = B.workspace_idle_bytes(D.desc)
    assert 512 < n < D.workspace.numel()
    x = tokens_with_clear_routing(cfg, tiny.A, 8, step=77)

    def idle():
        head = int(D.workspace[:512].count_nonzero().item())
        tags = D.workspace[512:n].view(torch.int64).reshape(-1, 2)[:, 1]      # 16-byte slots: {logit, tag}
        return head == 0 and int(tags.count_nonzero().item()) == 0
    for T in (1, 2, 5, 8):
        D.draft(x[:T].cuda())
        torch.cuda.synchronize()
        assert idle(), ("draft", T)
        D.verify(x[:T].cuda())
        torch.cuda.synchronize()
        assert idle(), ("verify", T)
    assert ctx.draft_status(D.workspace) == B.MOE_DRAFT_OK


@pytest.mark.parametrize("name", ["tiny", "qwen3"])
def test_draft_wait_that_runs_out_is_reported(ctx, name):
    """The bounded wait for the router result, forced to give up from the host (one poll allowed, and
    the loop tests the limit before it polls): every kernel still ends, ids are -1, the status word says
    so, and after moe_workspace_init the workspace serves correct calls again."""
    cfg = synth.config_by_name(name)
    L = build_layer(cfg)
    A = oracle_arrays(L)
    D = DeviceLayer(ctx, cfg, L, max_tokens=8, verify=False)
    x = tokens_with_clear_routing(cfg, A, 4, step=31)
    try:
        for T in (1, 4):
            ctx.set_draft_spin_limit(1)
            say("forced time-out", name, "T", T)
            r = D.draft(x[:T].cuda())
            torch.cuda.synchronize()                                   # the launch ended by itself
            assert ctx.draft_status(D.workspace) == B.MOE_DRAFT_TIMED_OUT
            assert bool((r["ids"] == -1).all()) and bool((r["conf"] == 0).all())
            ctx.set_draft_spin_limit(1 << 22)
            ctx.workspace_init(D.workspace)
            assert ctx.draft_status(D.workspace) == B.MOE_DRAFT_OK
            ref = oracle_draft(A, x[:T])
            r = D.draft(x[:T].cuda())
            torch.cuda.synchronize()
            assert np.array_equal(to_np(r["ids"]), ref["ids"])
            assert rel_err(to_np(r["y"]), ref["y"]) <= TOL_DRAFT
            assert ctx.draft_status(D.workspace) == B.MOE_DRAFT_OK
    finally:
        ctx.set_draft_spin_limit(1 << 22)
    with pytest.raises(B.MoeError):
        ctx.set_draft_spin_limit(0)


class Guarded:
    """A device buffer with canary bytes before and after the part handed to the library."""
    PAD = 4096

    def __init__(self, nbytes, dtype=torch.uint8, shape=None):
        self.raw = torch.full((nbytes + 2 * self.PAD,), 0xA5, dtype=torch.uint8, device="cuda")
        self.view = self.raw[self.PAD:self.PAD + nbytes].view(dtype)
        if shape is not None:
            self.view = self.view.reshape(shape)

    def intact(self):
        n = self.raw.numel()
        return bool((self.raw[:self.PAD] == 0xA5).all()) and bool((self.raw[n - self.PAD:] == 0xA5).all())


@pytest.mark.parametrize("name", ["tiny", "s192"])
def test_no_entry_point_writes_outside_its_outputs_or_workspace(ctx, name):
    """Canary bytes around every output and around the workspace survive one call of every entry point
    (a shape with a shared expert exercises the plan, intermediate and partial-output scratch)."""
    from synth.configs import LayerConfig
    cfg = synth.config_by_name("tiny") if name == "tiny" else LayerConfig(52, "s192", 192, 5, 128, 2, 64, 1, 1)
    L = build_layer(cfg)
    A = oracle_arrays(L)
    D = DeviceLayer(ctx, cfg, L, max_tokens=8)
    H, k, E = cfg.hidden, cfg.top_k, cfg.n_experts
    ws = Guarded(D.workspace.numel())
    ctx.workspace_init(ws.view)
    D.workspace = ws.view
    x = tokens_with_clear_routing(cfg, A, 8, step=5)
    guards = [ws]

    def out(T, cols, dtype):
        g = Guarded(T * cols * torch.empty((), dtype=dtype).element_size(), dtype, (T, cols))
        guards.append(g)
        return g.view
    for T in (1, 3, 8):
        xd = x[:T].cuda()
        ref_d, ref_v = oracle_draft(A, x[:T]), oracle_verify(A, x[:T])
        r = D.draft(xd, y=out(T, H, torch.float32), ids=out(T, k, torch.int32), conf=out(T, k, torch.float32))
        torch.cuda.synchronize()
        assert np.array_equal(to_np(r["ids"]), ref_d["ids"]) and rel_err(to_np(r["y"]), ref_d["y"]) <= TOL_DRAFT
        r = D.prefill(xd, y=out(T, H, torch.float32), ids=out(T, k, torch.int32), conf=out(T, k, torch.float32))
        torch.cuda.synchronize()
        assert rel_err(to_np(r["y"]), ref_d["y"]) <= TOL_DRAFT
        D.missing, D.n_missing = out(1, E, torch.int32).reshape(-1), out(1, 1, torch.int32).reshape(-1)
        r = D.verify(xd, y=out(T, H, torch.bfloat16), ids=out(T, k, torch.int32))
        torch.cuda.synchronize()
        assert np.array_equal(to_np(r["ids"]), ref_v["ids"]) and rel_err(to_np(r["y"]), ref_v["y"]) <= TOL_VERIFY
        ids, w, conf = out(T, k, torch.int32), out(T, k, torch.float32), out(T, k, torch.float32)
        cnt, off, pm = out(1, E, torch.int32).reshape(-1), out(1, E + 1, torch.int32).reshape(-1), out(1, T * k, torch.int32).reshape(-1)
        ctx.route_topk(D.desc, xd, D.router, D.bias, T, ids, w, conf, cnt, off, pm)
        mask, lst, miss = out(1, (E + 63) // 64, torch.int64).reshape(-1), out(1, E, torch.int32).reshape(-1), out(1, E, torch.int32).reshape(-1)
        nl, nm = out(1, 1, torch.int32).reshape(-1), out(1, 1, torch.int32).reshape(-1)
        ctx.expert_union(ids.reshape(-1), T * k, E, D.slot_of_expert, mask, lst, nl, miss, nm)
        torch.cuda.synchronize()
        assert np.array_equal(to_np(ids), ref_v["ids"])
    # the prefill workspace is allocated by the harness; give it canaries too
    pw = Guarded(B.prefill_workspace_bytes(D.desc, 40))
    guards.append(pw)
    D._prefill_ws = pw.view
    xp = tokens_with_clear_routing(cfg, A, 40, step=6, kind="iid")
    r = D.prefill(xp.cuda(), y=out(40, H, torch.float32), ids=out(40, k, torch.int32), conf=out(40, k, torch.float32))
    torch.cuda.synchronize()
    assert rel_err(to_np(r["y"]), oracle_draft(A, xp)["y"]) <= TOL_DRAFT
    assert all(g.intact() for g in guards), [i for i, g in enumerate(guards) if not g.intact()]
