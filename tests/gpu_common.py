"""Shared pieces of the GPU parity tests: build a synthetic layer (quantising on the GPU when
one is there -- same fp64 elementwise arithmetic, much faster), put it on the device, and the
two tolerances."""
import sys

import numpy as np
import torch

import synth
from tests.common import oracle_arrays, routing_gap

TOL_VERIFY = 2e-2     # max |y - oracle| <= 2e-2 * rms(oracle), bf16 verify pass
TOL_DRAFT = 1e-3      # ... <= 1e-3 * rms(oracle), int4 draft pass (fp32 accumulation, fp32 y)
MIN_GAP = 1e-9        # routing is well defined when neighbouring top logits differ by more


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def build_layer(cfg, layer=0, bias=None, quantize=True):
    """synth.make_layer on the CPU streams, with the RTN quantiser run on the GPU if available."""
    qdev = "cuda:0" if torch.cuda.is_available() else None
    return synth.make_layer(cfg, layer, bias=bias, quantize=quantize, quant_device=qdev)


def tokens_with_clear_routing(cfg, A, T, layer=0, step=0, kind=None):
    """Seeded tokens whose oracle routing gap exceeds MIN_GAP (bumps `step` otherwise)."""
    from oracle import oracle as orc
    for bump in range(16):
        x = synth.make_tokens(cfg, T, layer=layer, step=step + 1000 * bump, kind=kind)
        _, _, _, logits = orc.route(orc.bits(x), A["router"], A["bias"], cfg.top_k, cfg.renormalize)
        if routing_gap(logits, min(cfg.top_k, cfg.n_experts - 1)) > MIN_GAP:
            if bump:
                say("  routing gap too small, bumped token seed %d times" % bump)
            return x
    raise AssertionError("no seed with a clear routing gap")


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64) if t.is_floating_point() \
        else t.detach().cpu().numpy()
