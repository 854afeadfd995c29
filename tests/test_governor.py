"""Speculative Governor (paper section 3.2): the oracle against what the mathematics fixes, then
the C-ABI implementation against the oracle.  No GPU needed (host arithmetic)."""
import math
import random

import pytest

from oracle import governor_oracle as GO
from paper_2511_14102_amd import binding as B
from paper_2511_14102_amd.sched import Governor

CFG = dict(t_draft_base=1e-3, t_draft_token=4e-3, t_pcie_init=6e-3, t_pcie_overhead=2e-4, b_pcie=50e9,
           s_expert=17.3e6, verify_tokens=[2, 4, 8], verify_seconds=[10e-3, 12e-3, 20e-3],
           ema_alpha=0.25, p_init=0.8, k_min=1, k_max=8)


# ---- pins of the oracle ------------------------------------------------------------------------
def test_k_accept_geometric_closed_form():
    for p in (0.0, 0.3, 0.9, 1.0):
        for k in range(0, 9):
            want = float(k) if p == 1.0 else p * (1 - p ** k) / (1 - p)
            assert GO.k_accept([p] * 8, k) == pytest.approx(want, rel=1e-14, abs=1e-300)


def test_k_accept_worked_example_and_bounds():
    # by hand: p = (0.9, 0.5, 0.2): 0.9 + 0.45 + 0.09 = 1.44
    assert GO.k_accept([0.9, 0.5, 0.2], 3) == pytest.approx(1.44, rel=1e-15)
    assert GO.k_accept([0.9, 0.5, 0.2], 1) == pytest.approx(0.9)
    rng = random.Random(1)
    for _ in range(50):
        p = [rng.random() for _ in range(8)]
        prev = 0.0
        for k in range(1, 9):
            v = GO.k_accept(p, k)
            assert prev <= v <= k            # monotone in k, at most k tokens
            # recurrence: k_accept(k) = p_1 (1 + k_accept of the shifted sequence at k-1)
            assert v == pytest.approx(p[0] * (1 + GO.k_accept(p[1:], k - 1)), rel=1e-13)
            prev = v


def test_ema_update_positions():
    p = [0.5] * 4
    q = GO.ema_update(p, drafted=4, accepted=2, alpha=0.25)
    assert q == [0.625, 0.625, 0.375, 0.5]          # two accepted, the third rejected, the fourth not reached
    assert GO.ema_update(p, 3, 3, 1.0) == [1.0, 1.0, 1.0, 0.5]
    assert GO.ema_update(p, 3, 0, 1.0) == [0.0, 0.5, 0.5, 0.5]
    # a constant observation stream converges to it
    q = [0.5] * 4
    for _ in range(200):
        q = GO.ema_update(q, 4, 4, 0.1)
    assert all(abs(v - 1.0) < 1e-8 for v in q)


def test_verify_interpolation_hits_points_and_lines():
    xs, ys = CFG["verify_tokens"], CFG["verify_seconds"]
    for x, y in zip(xs, ys):
        assert GO.t_verify(xs, ys, x) == pytest.approx(y, rel=1e-15)
    assert GO.t_verify(xs, ys, 3) == pytest.approx(11e-3)
    assert GO.t_verify(xs, ys, 6) == pytest.approx(16e-3)
    assert GO.t_verify(xs, ys, 1) == pytest.approx(9e-3)          # first segment's line
    assert GO.t_verify(xs, ys, 10) == pytest.approx(24e-3)        # last segment's line
    assert GO.t_verify([5], [7e-3], 9) == 7e-3


def test_cycle_time_worked_example():
    # k = 3, 5 new experts: max(1 + 12, 6) ms + (0.2 ms + 5 * 17.3e6 / 50e9 s) + T_verify(4) = 12 ms
    want = 13e-3 + (2e-4 + 5 * 17.3e6 / 50e9) + 12e-3
    assert GO.t_cycle(CFG, 3, 5) == pytest.approx(want, rel=1e-15)
    # the draft hides under the first fetch: k = 1 -> max(5 ms, 6 ms)
    assert GO.t_cycle(CFG, 1, 0) == pytest.approx(6e-3 + 10e-3, rel=1e-15)


def test_roofs_bound_the_operating_point():
    """Section 3.2.1: throughput lies under the I/O roof (slope B_PCIe) and under the compute roof."""
    rng = random.Random(2)
    for _ in range(200):
        p = [rng.random() for _ in range(8)]
        k, n_new = rng.randint(1, 8), rng.randint(0, 40)
        th = GO.theta(CFG, p, k, n_new)
        it = GO.intensity(CFG, p, k, n_new)
        compute_roof = GO.k_accept(p, k) / GO.t_cycle(CFG, k, 0)
        assert th <= compute_roof * (1 + 1e-12)
        assert th <= it * CFG["b_pcie"] * (1 + 1e-12)
        if n_new == 0:
            assert it == math.inf and th == pytest.approx(compute_roof)


def test_choose_k_brute_force_and_slo():
    rng = random.Random(3)
    for _ in range(100):
        p = [rng.random() for _ in range(8)]
        n_new = [0] + sorted(rng.randint(0, 30) for _ in range(8))
        k, th = GO.choose_k(CFG, p, n_new)
        thetas = {kk: GO.theta(CFG, p, kk, n_new[kk]) for kk in range(1, 9)}
        assert th == max(thetas.values()) and k == min(kk for kk, v in thetas.items() if v == th)
        k3, _ = GO.choose_k(CFG, p, n_new, k_slo=3)
        assert k3 <= 3 and thetas[k3] == max(thetas[kk] for kk in (1, 2, 3))
    # a falling acceptance rate favours a shorter draft
    n_new = [0] * 9
    k_hi, _ = GO.choose_k(CFG, [0.95] * 8, n_new)
    k_lo, _ = GO.choose_k(CFG, [0.2] * 8, n_new)
    assert k_lo < k_hi


# ---- the library against the oracle ----------------------------------------------------------------
def test_library_matches_oracle():
    rng = random.Random(4)
    for trial in range(30):
        cfg = dict(CFG)
        cfg["t_draft_token"] = rng.uniform(1e-4, 8e-3)
        cfg["t_pcie_init"] = rng.uniform(0, 2e-2)
        cfg["ema_alpha"] = rng.uniform(0.05, 1.0)
        cfg["p_init"] = rng.random()
        npts = rng.randint(1, 4)
        cfg["verify_tokens"] = sorted(rng.sample(range(1, 12), npts))
        cfg["verify_seconds"] = sorted(rng.uniform(1e-3, 3e-2) for _ in range(npts))
        g = Governor(cfg)
        p = [cfg["p_init"]] * cfg["k_max"]
        for _ in range(rng.randint(0, 20)):
            drafted = rng.randint(0, cfg["k_max"])
            accepted = rng.randint(0, drafted)
            g.observe(drafted, accepted)
            p = GO.ema_update(p, drafted, accepted, cfg["ema_alpha"])
        assert g.probabilities() == pytest.approx(p, rel=1e-14, abs=1e-300)
        n_new = [0] + [rng.randint(0, 40) for _ in range(cfg["k_max"])]
        for k in range(0, cfg["k_max"] + 1):
            assert g.k_accept(k) == pytest.approx(GO.k_accept(p, k), rel=1e-13, abs=1e-300)
            assert g.cycle_time(k, n_new[k]) == pytest.approx(GO.t_cycle(cfg, k, n_new[k]), rel=1e-13)
            th, it = g.evaluate(k, n_new[k])
            assert th == pytest.approx(GO.theta(cfg, p, k, n_new[k]), rel=1e-12, abs=1e-300)
            assert it == pytest.approx(GO.intensity(cfg, p, k, n_new[k]), rel=1e-12, abs=1e-300)
        for slo in (0, 2, 5):
            k_lib, th_lib = g.choose_k(n_new, slo)
            k_or, th_or = GO.choose_k(cfg, p, n_new, slo)
            assert th_lib == pytest.approx(th_or, rel=1e-12)
            # equal up to rounding: the chosen k's theta is the maximum
            assert GO.theta(cfg, p, k_lib, n_new[k_lib]) == pytest.approx(th_or, rel=1e-12)
        g.close()


def test_library_rejects_bad_arguments():
    for key, val in (("b_pcie", 0.0), ("k_min", 0), ("k_max", 65), ("ema_alpha", 0.0), ("p_init", 1.5),
                     ("verify_tokens", [4, 4, 8]), ("t_draft_base", float("nan"))):
        bad = dict(CFG)
        bad[key] = val
        with pytest.raises(B.MoeError):
            Governor(bad)
    g = Governor(CFG)
    with pytest.raises(B.MoeError):
        g.observe(3, 4)
    with pytest.raises(B.MoeError):
        g.k_accept(9)
    with pytest.raises(B.MoeError):
        g.cycle_time(2, -1)
    with pytest.raises(B.MoeError):
        g.choose_k([0, 1, -1, 0, 0, 0, 0, 0, 0])
