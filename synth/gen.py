"""Seeded generators for weights, activations, router biases, and the RTN int4 quantiser.

Conventions (logical layouts; every consumer packs or widens them itself):
  router        [E, H]            bf16
  gate / up     [E + S, I, H]     bf16   (shared experts, if any, are rows E .. E+S-1)
  down          [E + S, H, I]     bf16
  int4 codes    same shape as the matrix, uint8 holding 0..15   (routed experts only)
  scale / zero  [..., in / g]     fp16, one per group of g consecutive input columns
  tokens        [T, H]            bf16

Randomness: on the CPU every tensor is drawn from numpy's PCG64 seeded with
(config index, layer, tensor tag), so tensors do not depend on the order they are made in.
With device="cuda" the draw uses torch's device generator instead (benchmark filler layers
that no oracle ever sees).
"""
import math
from typing import Dict, Optional

import numpy as np
import torch

from .configs import LayerConfig

WEIGHT_STD = 0.02
AR1_RHO = 0.56          # ~30 % adjacent-token overlap of the top-8 sets on the qwen3 shape
ZIPF_EXPONENT = 1.1
SKEW_BIAS = 30.0

_TAGS = {"router": 1, "gate": 2, "up": 3, "down": 4, "tokens": 5, "zipf": 6, "misc": 7}


def layer_seed(cfg: LayerConfig, layer: int = 0) -> int:
    """The documented seed of one layer: 1000 * config index + layer."""
    return 1000 * cfg.index + layer


def _rng(cfg: LayerConfig, layer: int, tag: str, extra: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence([layer_seed(cfg, layer), _TAGS[tag], extra])
    return np.random.Generator(np.random.PCG64(ss))


def _normal_bf16(shape, std, rng: Optional[np.random.Generator], device="cpu",
                 tgen: Optional[torch.Generator] = None) -> torch.Tensor:
    if device == "cpu":
        a = rng.standard_normal(size=shape, dtype=np.float32)
        t = torch.from_numpy(a)
        if std != 1.0:
            t.mul_(std)
        return t.to(torch.bfloat16)
    t = torch.randn(shape, dtype=torch.float32, device=device, generator=tgen)
    if std != 1.0:
        t.mul_(std)
    return t.to(torch.bfloat16)


def make_router(cfg: LayerConfig, layer: int = 0) -> torch.Tensor:
    return _normal_bf16((cfg.n_experts, cfg.hidden), WEIGHT_STD, _rng(cfg, layer, "router"))


def make_experts_bf16(cfg: LayerConfig, layer: int = 0, experts=None, device="cpu",
                      tgen=None) -> Dict[str, torch.Tensor]:
    """gate/up/down for the listed experts (default: all E + S).  Each expert has its own
    stream, so a subset equals the matching rows of the full set."""
    E = cfg.n_experts + cfg.n_shared
    experts = list(range(E)) if experts is None else list(experts)
    H, I = cfg.hidden, cfg.inter
    out = {"gate": [], "up": [], "down": []}
    for e in experts:
        for name, shape in (("gate", (I, H)), ("up", (I, H)), ("down", (H, I))):
            rng = _rng(cfg, layer, name, e) if device == "cpu" else None
            out[name].append(_normal_bf16(shape, WEIGHT_STD, rng, device, tgen))
    return {k: torch.stack(v) for k, v in out.items()}


def quantize_rtn_int4(w: torch.Tensor, group_size: int):
    """Round-to-nearest asymmetric int4 over groups of `group_size` input columns.

    The range of a group is taken over its values and 0, so 0 is representable and the zero
    point is an integer in [0, 15].  scale = fp16((max - min) / 15); a group whose scale
    rounds to 0 gets scale 1, zero 0 and all codes 0.  zero = clamp(rint(-min / scale), 0, 15)
    and code = clamp(rint(w / scale) + zero, 0, 15), both with the fp16-rounded scale, in
    fp64, rint = round-half-to-even.  Returns (codes uint8, scale fp16, zero fp16).
    """
    *lead, K = w.shape
    assert K % group_size == 0
    wg = w.to(torch.float64).reshape(*lead, K // group_size, group_size)
    zero_t = torch.zeros((), dtype=torch.float64, device=w.device)
    mn = torch.minimum(wg.amin(-1), zero_t)
    mx = torch.maximum(wg.amax(-1), zero_t)
    s16 = ((mx - mn) / 15.0).to(torch.float16)
    dead = s16 == 0
    s16 = torch.where(dead, torch.ones_like(s16), s16)
    s = s16.to(torch.float64)
    z = torch.clamp(torch.round(-mn / s), 0, 15)
    z = torch.where(dead, torch.zeros_like(z), z)
    q = torch.clamp(torch.round(wg / s.unsqueeze(-1)) + z.unsqueeze(-1), 0, 15)
    q = torch.where(dead.unsqueeze(-1), torch.zeros_like(q), q)
    return (q.to(torch.uint8).reshape(*lead, K), s16, z.to(torch.float16))


def quantize_rtn_int4_symmetric(w: torch.Tensor, group_size: int):
    """Round-to-nearest symmetric int4 (signed 4-bit weights -8..7 stored as codes 0..15 with
    zero point 8) over groups of `group_size` input columns.

    scale = fp16(max|w| / 7) over the group; a group whose scale rounds to 0 gets scale 1 and
    all codes 8.  code = clamp(rint(w / scale), -8, 7) + 8 with the fp16-rounded scale, in fp64,
    rint = round-half-to-even.  Returns (codes uint8, scale fp16, zero fp16 == 8 everywhere), the
    same triple as the asymmetric quantiser.
    """
    *lead, K = w.shape
    assert K % group_size == 0
    wg = w.to(torch.float64).reshape(*lead, K // group_size, group_size)
    s16 = (wg.abs().amax(-1) / 7.0).to(torch.float16)
    dead = s16 == 0
    s16 = torch.where(dead, torch.ones_like(s16), s16)
    s = s16.to(torch.float64)
    q = torch.clamp(torch.round(wg / s.unsqueeze(-1)), -8, 7) + 8
    q = torch.where(dead.unsqueeze(-1), torch.full_like(q, 8), q)
    return (q.to(torch.uint8).reshape(*lead, K), s16, torch.full_like(s16, 8.0))


def zipf_bias(cfg: LayerConfig, layer: int = 0) -> torch.Tensor:
    """Router-logit bias ln(pi_e) with pi_e proportional to rank(e)^-1.1 under a seeded
    random ranking of the experts."""
    rng = _rng(cfg, layer, "zipf")
    rank = rng.permutation(cfg.n_experts) + 1
    pi = rank.astype(np.float64) ** (-ZIPF_EXPONENT)
    pi /= pi.sum()
    return torch.from_numpy(np.log(pi).astype(np.float32))


def skew_bias(cfg: LayerConfig, pair=(1, 5)) -> torch.Tensor:
    """All tokens pick the same experts: a large bias on a fixed set (the first is larger,
    so the order within the set is fixed too)."""
    b = torch.zeros(cfg.n_experts, dtype=torch.float32)
    for r, e in enumerate(pair):
        b[e % cfg.n_experts] = SKEW_BIAS - r
    return b


def make_tokens(cfg: LayerConfig, T: int, layer: int = 0, step: int = 0,
                kind: Optional[str] = None) -> torch.Tensor:
    """[T, H] bf16 activations: iid N(0,1), or (kind 'ar1') a stationary AR(1) sequence over
    the token axis, x_t = rho x_{t-1} + sqrt(1 - rho^2) eps_t, so that adjacent tokens share
    part of their routing."""
    kind = kind or ("ar1" if cfg.router == "ar1" else "iid")
    rng = _rng(cfg, layer, "tokens", step)
    eps = rng.standard_normal(size=(T, cfg.hidden), dtype=np.float32)
    if kind == "ar1":
        x = np.empty_like(eps)
        x[0] = eps[0]
        c = math.sqrt(1.0 - AR1_RHO * AR1_RHO)
        for t in range(1, T):
            x[t] = AR1_RHO * x[t - 1] + c * eps[t]
        eps = x
    return torch.from_numpy(eps).to(torch.bfloat16)


def make_layer(cfg: LayerConfig, layer: int = 0, bias: Optional[str] = None,
               quantize: bool = True, device: str = "cpu",
               quant_device: Optional[str] = None, symmetric: bool = False) -> Dict[str, object]:
    """One full layer in the logical layouts listed in the module docstring.

    bias: None -> what cfg.router asks for ('zipf' -> zipf_bias, otherwise no bias);
          'skew' -> skew_bias; 'none' -> no bias.
    device: "cpu" draws every tensor from the numpy streams (what the oracle sees);
            a GPU device draws the expert weights there with torch's generator seeded with
            layer_seed (benchmark filler layers; router and bias are still the CPU ones).
    quant_device: where the RTN quantiser runs (same fp64 elementwise arithmetic, so the same
            result); results are returned on `device`.
    symmetric: quantise with quantize_rtn_int4_symmetric (every zero point is 8).
    """
    E = cfg.n_experts
    L: Dict[str, object] = {"cfg": cfg, "layer": layer}
    L["router"] = make_router(cfg, layer)
    mode = bias or ("zipf" if cfg.router == "zipf" else "none")
    L["router_bias"] = {"zipf": lambda: zipf_bias(cfg, layer),
                        "skew": lambda: skew_bias(cfg),
                        "none": lambda: None}[mode]()
    tgen = None
    if device != "cpu":
        tgen = torch.Generator(device=device)
        tgen.manual_seed(layer_seed(cfg, layer))
    w = make_experts_bf16(cfg, layer, device=device, tgen=tgen)
    L.update(w)
    if quantize:
        qdev = quant_device or device
        for name in ("gate", "up", "down"):
            qs, ss, zs = [], [], []
            for e in range(E):          # one expert at a time bounds the fp64 temporaries
                quant = quantize_rtn_int4_symmetric if symmetric else quantize_rtn_int4
                q, s, z = quant(w[name][e].to(qdev), cfg.group_size)
                qs.append(q.to(device)); ss.append(s.to(device)); zs.append(z.to(device))
            L["q_" + name] = torch.stack(qs)
            L["s_" + name] = torch.stack(ss)
            L["z_" + name] = torch.stack(zs)
        L["symmetric"] = symmetric
    return L
