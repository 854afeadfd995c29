"""Runs the oracle's router + layer on one synthetic layer given in the logical layouts (torch
tensors from synth), and the error measure both float tolerances are stated in.  Test
infrastructure like the rest of oracle/: imported by tests/, the smoke check and the checker and
cpu_baseline legs of bench.py only."""
import numpy as np

from oracle import oracle as orc


def oracle_arrays(L):
    """numpy views of one synth layer for the oracle (bit patterns for 16-bit types)."""
    cfg = L["cfg"]
    A = {"cfg": cfg}
    A["router"] = orc.bits(L["router"])
    A["bias"] = None if L["router_bias"] is None else L["router_bias"].numpy()
    for n in ("gate", "up", "down"):
        A[n] = orc.bits(L[n])
        if ("q_" + n) in L:
            A["q_" + n] = L["q_" + n].numpy()
            A["s_" + n] = orc.bits(L["s_" + n])
            A["z_" + n] = orc.bits(L["z_" + n])
    return A


def oracle_verify(A, x, present=None):
    cfg = A["cfg"]
    xb = orc.bits(x)
    ids, w, conf, logits = orc.route(xb, A["router"], A["bias"], cfg.top_k, cfg.renormalize)
    y = orc.layer_bf16(xb, A["gate"], A["up"], A["down"], cfg.n_experts, ids, w, present)
    return dict(ids=ids, w=w, conf=conf, logits=logits, y=y)


def oracle_draft(A, x):
    cfg = A["cfg"]
    E = cfg.n_experts
    xb = orc.bits(x)
    ids, w, conf, logits = orc.route(xb, A["router"], A["bias"], cfg.top_k, cfg.renormalize)
    shared = None
    if cfg.n_shared:
        shared = (A["gate"][E:], A["up"][E:], A["down"][E:])
    y = orc.layer_int4(xb, {n: A["q_" + n] for n in ("gate", "up", "down")},
                       {n: A["s_" + n] for n in ("gate", "up", "down")},
                       {n: A["z_" + n] for n in ("gate", "up", "down")},
                       cfg.group_size, ids, w, shared)
    return dict(ids=ids, w=w, conf=conf, logits=logits, y=y)


def rel_err(y, ref):
    """max |y - ref| / rms(ref): the measure both float tolerances are stated in."""
    ref = np.asarray(ref, np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    return float(np.max(np.abs(np.asarray(y, np.float64) - ref))) / max(rms, 1e-300)
