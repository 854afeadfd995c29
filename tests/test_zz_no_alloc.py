"""moe_draft_layer_int4_noalloc (scratch in a static device array, nothing allocated by the call)
against moe_draft_layer_int4 (caller workspace) and the oracle: two calls in a row on each shape,
the second with fewer tokens, so that the second call meets the first call's leftovers in the
shared array.  Shapes with and without shared experts and with more than 64 experts (the exchange
slots, the plan and the shared experts' intermediate all live in the scratch)."""
import numpy as np
import pytest
import torch

import synth
from synth.configs import LayerConfig
from paper_2511_14102_amd import binding as B
from paper_2511_14102_amd.harness import DeviceLayer
from tests.common import oracle_arrays, oracle_draft, rel_err
from tests.gpu_common import TOL_DRAFT, say, to_np, tokens_with_clear_routing

pytestmark = pytest.mark.gpu

SHAPES = [
    synth.config_by_name("tiny"),
    LayerConfig(52, "s192", 192, 5, 128, 2, 64, 1, 1),
    LayerConfig(54, "s384", 384, 130, 128, 4, 128, 2, 1),
]


def noalloc_draft(ctx, D, x):
    T, k = x.shape[0], D.cfg.top_k
    y = torch.full((T, D.cfg.hidden), float("nan"), dtype=torch.float32, device="cuda")
    ids = torch.full((T, k), -7, dtype=torch.int32, device="cuda")
    conf = torch.full((T, k), float("nan"), dtype=torch.float32, device="cuda")
    ctx.draft_layer_int4_noalloc(D.desc, x, D.router, D.bias, D.q_blob, D.sz_blob, D.q_bytes, D.sz_bytes,
                                 D.shared, T, y, ids, conf, symmetric=D.symmetric)
    return dict(y=y, ids=ids, conf=conf)


def test_noalloc_draft_matches_workspace_draft():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    ctx = B.Context(0)
    assert B.noalloc_scratch_bytes() == 2 << 20
    for cfg in SHAPES:
        L = synth.make_layer(cfg, 0)
        A = oracle_arrays(L)
        D = DeviceLayer(ctx, cfg, L, max_tokens=8, verify=False)
        assert B.workspace_bytes(D.desc, 8) <= B.noalloc_scratch_bytes()
        x = tokens_with_clear_routing(cfg, A, 8, step=3)
        for T in (8, 3, 1):                       # back to back, each smaller than the one before
            say("noalloc", cfg.name, "T", T)
            xd = x[:T].cuda()
            ref = oracle_draft(A, x[:T])
            r = noalloc_draft(ctx, D, xd)
            torch.cuda.synchronize()
            w = D.draft(xd)
            torch.cuda.synchronize()
            assert np.array_equal(to_np(r["ids"]), ref["ids"]) and torch.equal(r["ids"], w["ids"])
            assert torch.equal(r["conf"], w["conf"])
            e = rel_err(to_np(r["y"]), ref["y"])
            assert e <= TOL_DRAFT, (cfg.name, T, e)
            # both entry points run the same kernels; y is summed with atomics, so last bits may move
            assert rel_err(to_np(r["y"]), to_np(w["y"])) <= 1e-5
        del D
    # a shape whose workspace does not fit the static array is refused, nothing enqueued
    big = LayerConfig(57, "big", 4096, 256, 8192, 16, 128, 4, 1)
    d = B.LayerDesc.from_config(big)
    assert B.validate_desc(d) == 0 and B.workspace_bytes(d, 8) > B.noalloc_scratch_bytes()
    dummy = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.MoeError) as ei:
        ctx.draft_layer_int4_noalloc(d, dummy, dummy, None, dummy, dummy, B.int4_expert_q_bytes(d),
                                     B.int4_expert_sz_bytes(d), dummy, 8, dummy, dummy, None)
    assert ei.value.status == B.MOE_ERR_WORKSPACE
    ctx.close()
