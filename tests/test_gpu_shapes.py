"""Parity on small layers of unusual shape: group counts that do not divide by the number of waves,
fewer row tiles than waves, more than 64 and more than 128 experts, k = 1 and k = E, shared
experts, no renormalisation.  Every entry point against the oracle, same tolerances as the
workload tests."""
import gc

import numpy as np
import pytest
import torch

import synth
from oracle import oracle as orc
from synth.configs import LayerConfig
from tests.common import oracle_arrays, oracle_draft, oracle_verify, rel_err
from tests.gpu_common import TOL_DRAFT, TOL_VERIFY, say, to_np, tokens_with_clear_routing

pytestmark = pytest.mark.gpu

from paper_2511_14102_amd import binding as B          # noqa: E402
from paper_2511_14102_amd.harness import DeviceLayer   # noqa: E402

SHAPES = [
    #            idx  name    H    E   I   k   g  S  renorm
    LayerConfig(51, "s64", 64, 4, 64, 1, 32, 0, 1),
    LayerConfig(52, "s192", 192, 5, 128, 2, 64, 1, 1),
    LayerConfig(53, "s320", 320, 70, 192, 3, 32, 0, 1),
    LayerConfig(54, "s384", 384, 130, 128, 4, 128, 2, 1),
    LayerConfig(55, "s512", 512, 9, 320, 2, 64, 0, 0),
    LayerConfig(56, "s1024", 1024, 16, 128, 16, 128, 0, 1),
]


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = B.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("cfg", SHAPES, ids=[c.name for c in SHAPES])
def test_unusual_shape(ctx, cfg):
    d = B.LayerDesc.from_config(cfg)
    assert B.validate_desc(d) == 0
    k = cfg.top_k
    say("shape", cfg.name)
    L = synth.make_layer(cfg, 0)
    A = oracle_arrays(L)
    Tv = min(16, 128 // k)
    D = DeviceLayer(ctx, cfg, L, max_tokens=Tv)
    torch.cuda.synchronize()
    # router + histogram + permutation
    x = tokens_with_clear_routing(cfg, A, Tv, step=1)
    r = D.route(x.cuda())
    torch.cuda.synchronize()
    ids, w, conf, _ = orc.route(orc.bits(x), A["router"], A["bias"], k, cfg.renormalize)
    assert np.array_equal(to_np(r["ids"]), ids)
    np.testing.assert_allclose(to_np(r["w"]), w, rtol=2e-6, atol=1e-9)
    cnt, off, pm = orc.perm(ids, cfg.n_experts)
    assert np.array_equal(to_np(r["count"]), cnt) and np.array_equal(to_np(r["off"]), off)
    assert np.array_equal(to_np(r["perm"]), pm)
    # verify pass: 1 token, a ragged count, the largest call
    for T in sorted({1, min(7, Tv), Tv}):
        ref = oracle_verify(A, x[:T])
        say("  verify T", T)
        rv = D.verify(x[:T].cuda())
        torch.cuda.synchronize()
        assert np.array_equal(to_np(rv["ids"]), ref["ids"])
        assert int(rv["n_missing"].item()) == 0
        assert rel_err(to_np(rv["y"]), ref["y"]) <= TOL_VERIFY
    # draft pass: every token capacity of the kernel
    Td = min(8, 128 // k)
    for T in sorted({1, 2, min(3, Td), min(5, Td), Td}):
        ref = oracle_draft(A, x[:T])
        say("  draft T", T)
        rd = D.draft(x[:T].cuda())
        torch.cuda.synchronize()
        assert np.array_equal(to_np(rd["ids"]), ref["ids"])
        np.testing.assert_allclose(to_np(rd["conf"]), ref["conf"], rtol=2e-6)
        e = rel_err(to_np(rd["y"]), ref["y"])
        assert e <= TOL_DRAFT, (T, e)
    # prefill form
    xp = tokens_with_clear_routing(cfg, A, 19, step=2, kind="iid")
    ref = oracle_draft(A, xp)
    say("  prefill T 19")
    rp = D.prefill(xp.cuda())
    torch.cuda.synchronize()
    assert np.array_equal(to_np(rp["ids"]), ref["ids"])
    assert rel_err(to_np(rp["y"]), ref["y"]) <= TOL_DRAFT
    # symmetric format where the shape allows it
    if B.int4_expert_scale_bytes(d) > 0:
        Ls = synth.make_layer(cfg, 0, symmetric=True)
        As = oracle_arrays(Ls)
        Ds = DeviceLayer(ctx, cfg, Ls, max_tokens=8, verify=False, symmetric=True)
        for T in sorted({1, Td}):
            ref = oracle_draft(As, x[:T])
            say("  draft (symmetric) T", T)
            rs = Ds.draft(x[:T].cuda())
            torch.cuda.synchronize()
            assert np.array_equal(to_np(rs["ids"]), ref["ids"])
            assert rel_err(to_np(rs["y"]), ref["y"]) <= TOL_DRAFT
        del Ds
    del D
    gc.collect()
    torch.cuda.empty_cache()
