"""The synthetic-input recipe: determinism, the RTN quantiser's contract, and the routing
statistics each workload is supposed to have (measured with the oracle's router)."""
import numpy as np
import torch

import synth
from oracle import oracle as orc


def test_generators_are_deterministic_and_order_independent():
    cfg = synth.config_by_name("tiny")
    a = synth.make_experts_bf16(cfg)
    b = synth.make_experts_bf16(cfg, experts=[3, 1])
    assert torch.equal(a["gate"][3], b["gate"][0]) and torch.equal(a["down"][1], b["down"][1])
    assert torch.equal(synth.make_tokens(cfg, 4), synth.make_tokens(cfg, 4))
    assert not torch.equal(synth.make_tokens(cfg, 4, step=0), synth.make_tokens(cfg, 4, step=1))
    assert synth.layer_seed(synth.config_by_name("phi"), 7) == 2007
    w = a["gate"].float()
    assert abs(float(w.std()) - 0.02) < 5e-4 and abs(float(w.mean())) < 2e-4


def test_rtn_quantiser_contract():
    rng = np.random.default_rng(0)
    for g in (32, 64, 128):
        w = torch.from_numpy((0.02 * rng.standard_normal((48, 4 * g))).astype(np.float32)) \
            .to(torch.bfloat16)
        w[0, :g] = 0                                   # a dead group
        w[1, :g] = w[1, :g].abs()                      # one-sided groups still contain 0
        w[2, :g] = -w[2, :g].abs()
        q, s, z = synth.quantize_rtn_int4(w, g)
        assert q.dtype == torch.uint8 and s.dtype == torch.float16 and z.dtype == torch.float16
        assert q.shape == w.shape and s.shape == (48, 4) and z.shape == (48, 4)
        assert int(q.max()) <= 15
        zf = z.double()
        assert torch.equal(zf, zf.round()) and float(zf.min()) >= 0 and float(zf.max()) <= 15
        assert float(s[0, 0]) == 1.0 and float(z[0, 0]) == 0.0 and int(q[0, :g].max()) == 0
        assert float(z[1, 0]) == 0.0 and float(z[2, 0]) == 15.0
        deq = (q.double().reshape(48, 4, g) - zf.unsqueeze(-1)) * s.double().unsqueeze(-1)
        err = (deq.reshape(48, -1) - w.double()).abs().reshape(48, 4, g)
        # inside the clamp range the error is at most half a step (fp16 rounding of the scale
        # can push the extreme value of a group just outside it: allow one step there)
        assert bool((err <= 0.5 * s.double().unsqueeze(-1) * 1.0001).float().mean() > 0.99)
        assert bool((err <= 1.0 * s.double().unsqueeze(-1) * 1.0001).all())
        q2, s2, z2 = synth.quantize_rtn_int4(w, g)
        assert torch.equal(q, q2) and torch.equal(s, s2) and torch.equal(z, z2)


def test_symmetric_rtn_quantiser_contract():
    rng = np.random.default_rng(1)
    for g in (32, 128):
        w = torch.from_numpy((0.02 * rng.standard_normal((16, 4 * g))).astype(np.float32)).to(torch.bfloat16)
        w[0, :g] = 0
        q, s, z = synth.quantize_rtn_int4_symmetric(w, g)
        assert q.dtype == torch.uint8 and s.dtype == torch.float16 and z.dtype == torch.float16
        assert bool((z == 8).all()) and int(q.max()) <= 15
        assert float(s[0, 0]) == 1.0 and bool((q[0, :g] == 8).all())
        deq = (q.double().reshape(16, 4, g) - 8.0) * s.double().unsqueeze(-1)
        err = (deq.reshape(16, -1) - w.double()).abs().reshape(16, 4, g)
        assert bool((err <= 0.5 * s.double().unsqueeze(-1) * 1.01).all())   # |w| <= 7 s up to fp16 rounding of s
        # the largest magnitude of a live group lands on code 1 or 15 (-7 or +7)
        top = (q.reshape(16, 4, g).to(torch.int32) - 8).abs().amax(-1)
        assert bool((top[1:] == 7).all())


def test_qwen3_tokens_repeat_about_30_percent_of_experts():
    cfg = synth.config_by_name("qwen3")
    wr = orc.bits(synth.make_router(cfg))
    ov = []
    for step in range(8):
        x = synth.make_tokens(cfg, 64, step=step)
        ids, _, _, _ = orc.route(orc.bits(x), wr, None, cfg.top_k)
        ov += [len(set(ids[t]) & set(ids[t - 1])) / cfg.top_k for t in range(1, 64)]
    assert 0.27 <= float(np.mean(ov)) <= 0.33


def test_phi_bias_gives_zipf_like_popularity():
    cfg = synth.config_by_name("phi")
    wr = orc.bits(synth.make_router(cfg))
    b = synth.zipf_bias(cfg).numpy()
    hits = np.zeros(cfg.n_experts)
    for step in range(8):
        x = synth.make_tokens(cfg, 64, step=step)
        ids, _, _, _ = orc.route(orc.bits(x), wr, b, cfg.top_k)
        hits += np.bincount(ids.reshape(-1), minlength=cfg.n_experts)
    order = np.argsort(-b)
    top4 = hits[order[:4]].sum() / hits.sum()
    assert top4 > 0.45                                # 4 of 16 experts take about half
    assert hits[order[0]] > 3 * hits[order[-1]]
    assert np.isclose(np.exp(b.astype(np.float64)).sum(), 1.0, atol=1e-5)


def test_skew_bias_sends_every_token_to_the_same_pair():
    cfg = synth.config_by_name("mixtral")
    wr = orc.bits(synth.make_router(cfg))
    x = synth.make_tokens(cfg, 8)
    ids, w, _, _ = orc.route(orc.bits(x), wr, synth.skew_bias(cfg).numpy(), cfg.top_k)
    assert np.array_equal(ids, np.tile(np.array([1, 5], np.int32), (8, 1)))
