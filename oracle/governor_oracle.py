"""TEST INFRASTRUCTURE - plain Python (fp64) statement of the Speculative Governor's model,
paper section 3.2.  Only tests, smoke() and bench.py's baseline leg may import this module; the
product path never does.

Each function is the paper's definition written out; where the paper is silent the reading is
stated at the function.
"""
import math
from typing import Sequence


def k_accept(p: Sequence[float], k: int) -> float:
    """Section 3.2.2: expected accepted tokens of a draft of length k,
    sum over i = 1..k of the product of p_1..p_i (p_i conditional on the first i-1 accepted)."""
    total = 0.0
    for i in range(1, k + 1):
        prod = 1.0
        for j in range(1, i + 1):
            prod *= p[j - 1]
        total += prod
    return total


def ema_update(p: Sequence[float], drafted: int, accepted: int, alpha: float):
    """Section 3.2.2: the p_i are updated with an exponential moving average.  Reading (the paper
    gives no formula): position i was observed if tokens 1..i-1 were accepted and token i was
    drafted; its observation is 1 if accepted, else 0; p_i <- (1 - alpha) p_i + alpha * obs."""
    q = list(p)
    for i in range(1, drafted + 1):
        if i <= accepted:
            q[i - 1] = (1.0 - alpha) * q[i - 1] + alpha * 1.0
        elif i == accepted + 1:
            q[i - 1] = (1.0 - alpha) * q[i - 1] + alpha * 0.0
    return q


def t_verify(tokens_pts: Sequence[int], seconds_pts: Sequence[float], tokens: float) -> float:
    """Section 3.2.2: T_verify is profiled for several lengths and interpolated.  Reading: linear
    between neighbouring points, the first / last segment's line outside them, constant with a
    single point."""
    n = len(tokens_pts)
    if n == 1:
        return seconds_pts[0]
    seg = None
    for i in range(n - 1):
        if tokens <= tokens_pts[i + 1] or i == n - 2:
            seg = i
            break
    x0, x1 = tokens_pts[seg], tokens_pts[seg + 1]
    y0, y1 = seconds_pts[seg], seconds_pts[seg + 1]
    return y0 + (y1 - y0) * (tokens - x0) / (x1 - x0)


def t_pcie_new(cfg: dict, n_new: int) -> float:
    """Section 3.2.2: T_pcie,overhead + |E_new| S_expert / B_PCIe.  Reading: nothing to fetch
    costs nothing (no overhead either)."""
    if n_new == 0:
        return 0.0
    return cfg["t_pcie_overhead"] + n_new * cfg["s_expert"] / cfg["b_pcie"]


def t_cycle(cfg: dict, k: int, n_new: int) -> float:
    """Eq. 3: max(T_draft(k), T_pcie,init) + T_pcie,new(k) + T_verify(k+1), T_draft linear in k."""
    t_draft = cfg["t_draft_base"] + k * cfg["t_draft_token"]
    return max(t_draft, cfg["t_pcie_init"]) + t_pcie_new(cfg, n_new) + \
        t_verify(cfg["verify_tokens"], cfg["verify_seconds"], k + 1)


def theta(cfg: dict, p: Sequence[float], k: int, n_new: int) -> float:
    """Eq. 2: expected accepted tokens per second."""
    return k_accept(p, k) / t_cycle(cfg, k, n_new)


def intensity(cfg: dict, p: Sequence[float], k: int, n_new: int) -> float:
    """Eq. 1 with S_token = 1: accepted tokens per byte of synchronous I/O (|E_new| S_expert)."""
    if n_new == 0:
        return math.inf
    return k_accept(p, k) / (n_new * cfg["s_expert"])


def choose_k(cfg: dict, p: Sequence[float], n_new_by_k: Sequence[int], k_slo: int = 0):
    """Eq. 4 / 5: argmax of theta over [k_min, min(k_max, k_slo)], smallest k on ties."""
    hi = cfg["k_max"] if k_slo <= 0 else min(cfg["k_max"], k_slo)
    best, best_theta = None, None
    for k in range(cfg["k_min"], hi + 1):
        th = theta(cfg, p, k, n_new_by_k[k])
        if best is None or th > best_theta:
            best, best_theta = k, th
    return best, best_theta
