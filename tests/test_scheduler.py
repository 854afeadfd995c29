"""Expert Scheduler (paper section 3.3): the Python oracle against textbook / hand-worked cases,
then the C-ABI implementation against the oracle.  No GPU needed (host logic)."""
import random
from collections import OrderedDict

import pytest

from oracle import scheduler_oracle as SO
from paper_2511_14102_amd import binding as B
from paper_2511_14102_amd import sched as S


def elb_from(steps):
    """steps[step][layer] = [(expert, conf)] -> library Elb"""
    L, k = len(steps[0]), len(steps[0][0])
    elb = S.Elb(L, max(len(steps), 1), k)
    for i, st in enumerate(steps):
        elb.put_step(i, [[e for e, _ in lay] for lay in st], [[c for _, c in lay] for lay in st])
    return elb


# ---- pins of the oracle ------------------------------------------------------------------------
def test_oracle_is_textbook_lru_without_lookahead():
    """One expert per step, misses loaded on demand: hit count and contents of a classic LRU."""
    rng = random.Random(0)
    for C in (1, 2, 5):
        c = SO.Cache(1, 12, C)
        lru = OrderedDict()
        hits = 0
        for _ in range(400):
            e = rng.randrange(12) if rng.random() < 0.7 else rng.randrange(4)
            h, m = c.use(0, [e])
            if e in lru:
                hits += 1
                lru.move_to_end(e)
                assert (h, m) == (1, 0)
            else:
                assert (h, m) == (0, 1)
                if len(lru) == C:
                    lru.popitem(last=False)
                lru[e] = True
                c.on_demand(0, [e])
            assert c.resident(0) == set(lru)
        assert c.hits == hits and c.hits + c.misses == 400


def test_oracle_lookahead_beats_recency():
    """Hand example: slots hold A = 0 (old) and B = 1 (recent); the window names A and C = 2.
    Recency alone would drop A; the lookahead keeps A and drops B."""
    c = SO.Cache(1, 4, 2)
    c.place(0, 0, 0)
    c.place(0, 1, 1)
    c.use(0, [0])
    c.use(0, [1])
    out = c.plan([[[(0, 0.9), (2, 0.8)]]], 3)
    assert out == [(0, 2, 1, 1)] and c.resident(0) == {0, 2}
    # the same request on demand, no lookahead: the least recently used (A) goes
    d = SO.Cache(1, 4, 2)
    d.place(0, 0, 0)
    d.place(0, 1, 1)
    d.use(0, [0])
    d.use(0, [1])
    assert d.on_demand(0, [2]) == [(0, 2, 0, 0)]


def test_oracle_phases_by_hand():
    c = SO.Cache(2, 8, 3)
    c.place(0, 5, 0)
    window = [[[(5, 0.5), (1, 0.25)], [(2, 0.75), (3, 0.125)]],
              [[(1, 0.5), (6, 0.0625)], [(2, 0.5), (4, 0.25)]]]
    assert c.plan(window, 1) == []                                 # priming fetches nothing ...
    assert c.protected[0] == {5, 1, 6} and c.protected[1] == {2, 3, 4}
    # guided: layer 0 misses 1 (0.5), 6 (0.0625); layer 1 misses 2 (0.75), 4 (0.25), 3 (0.125);
    # threshold 0.1 drops expert 6, budget 3 keeps (0,1), (1,2), (1,4)
    assert c.plan(window, 2, max_fetch=3, min_conf=0.1) == [(0, 1, 1, -1), (1, 2, 0, -1), (1, 4, 1, -1)]
    # saturation brings the rest in expert order
    assert c.plan(window, 3) == [(0, 6, 2, -1), (1, 3, 2, -1)]
    assert c.plan(window, 3) == []
    # every slot of layer 1 now holds a named expert: a further named expert is skipped
    assert c.plan([[[(5, 1.0), (1, 1.0)], [(7, 1.0), (2, 1.0)]]], 3) == []
    c.end_window()
    assert c.plan([[[(5, 1.0), (1, 1.0)], [(7, 1.0), (2, 1.0)]]], 3) == [(1, 7, 1, 4)]   # 4 and 3 never used: lowest slot


def test_oracle_full_coverage_when_the_window_fits():
    rng = random.Random(1)
    L, E, k, K = 3, 16, 2, 4
    c = SO.Cache(L, E, K * k)
    for _ in range(50):
        window = [[[(e, 1.0) for e in rng.sample(range(E), k)] for _ in range(L)] for _ in range(K)]
        c.plan(window, 3)
        for layer in range(L):
            need = [e for st in window for e, _ in st[layer]]
            assert c.use(layer, need)[1] == 0
        c.end_window()
    assert c.misses == 0


# ---- the library against the oracle ----------------------------------------------------------------
def test_elb_round_trip_and_errors():
    elb = S.Elb(2, 3, 2)
    assert elb.steps() == 0
    elb.put_step(0, [[3, 1], [0, 7]], [[0.5, 0.25], [1.0, 0.0]])
    elb.put_step(1, [[2, 2], [5, 6]])
    assert elb.steps() == 2
    assert elb.entry(0, 1) == ([0, 7], [1.0, 0.0]) and elb.entry(1, 0) == ([2, 2], [1.0, 1.0])
    with pytest.raises(B.MoeError):
        elb.put_step(3, [[0, 0], [0, 0]])          # out of order
    with pytest.raises(B.MoeError):
        elb.entry(2, 0)                            # not filled
    elb.reset()
    assert elb.steps() == 0
    with pytest.raises(B.MoeError):
        S.Elb(0, 1, 1)


def test_library_matches_oracle_on_random_histories():
    rng = random.Random(2)
    for trial in range(25):
        L, E = rng.randint(1, 4), rng.choice([8, 16, 64])
        C, k, K = rng.randint(1, min(E, 12)), rng.randint(1, 3), rng.randint(1, 5)
        lib, orc = S.Cache(L, E, C), SO.Cache(L, E, C)
        for layer in range(L):
            for slot, e in enumerate(rng.sample(range(E), rng.randint(0, C))):
                lib.place(layer, e, slot)
                orc.place(layer, e, slot)
        for cycle in range(12):
            window = [[[(rng.randrange(E), rng.randrange(65) / 64.0) for _ in range(k)] for _ in range(L)]
                      for _ in range(K)]
            seen = rng.randint(1, K)
            for phase, upto in ((1, 1), (2, seen), (3, K)):
                part = window[:upto]
                budget, thr = rng.randint(0, 6), rng.randrange(33) / 64.0
                elb = elb_from(part)
                assert lib.plan(elb, phase, budget, thr) == orc.plan(part, phase, budget, thr)
                elb.close()
            for layer in range(L):
                need = [e for st in window for e, _ in st[layer]] + [rng.randrange(E) for _ in range(k)]
                assert lib.use(layer, need) == orc.use(layer, need)
                missing = sorted(set(need) - orc.resident(layer))[:C]
                assert lib.on_demand(layer, missing) == orc.on_demand(layer, missing)
                assert lib.slot_table(layer) == orc.slot_table(layer)
            lib.end_window()
            orc.end_window()
        assert lib.stats() == (orc.hits, orc.misses)
        lib.close()


def test_library_rejects_bad_arguments():
    c = S.Cache(1, 8, 2)
    c.place(0, 3, 0)
    with pytest.raises(B.MoeError):
        c.place(0, 4, 0)                           # slot taken
    with pytest.raises(B.MoeError):
        c.place(0, 3, 1)                           # expert already resident
    with pytest.raises(B.MoeError):
        c.use(0, [8])
    with pytest.raises(B.MoeError):
        c.on_demand(0, [3])                        # not missing
    with pytest.raises(B.MoeError) as ei:
        c.on_demand(0, [1, 2, 4])                  # more than the layer's slots
    assert ei.value.status == B.MOE_ERR_WORKSPACE
    elb = elb_from([[[(1, 1.0), (2, 1.0)]]])
    with pytest.raises(B.MoeError) as ei:
        c.plan(elb, S.PHASE_SATURATE, max_out=0)   # a fetch is due (one slot is empty) but out holds none
    assert ei.value.status == B.MOE_ERR_WORKSPACE
    assert c.slot_table(0)[1] == -1                # ... and nothing was applied
    with pytest.raises(B.MoeError):
        c.plan(elb, 7)
    with pytest.raises(B.MoeError):
        S.Cache(1, 8, 9)


def test_coverage_ordering_on_a_routed_stream():
    """The experiment of the paper's hit-rate table in small: expert ids of an AR(1) token stream
    from the oracle router, one token per step, K drafted tokens per cycle known ahead.  Looking
    ahead covers more than recency alone; the library reproduces the oracle's counts."""
    import numpy as np
    import synth
    from oracle import oracle as orc
    cfg = synth.config_by_name("tiny")
    L, N, K, k, E = 3, 160, 3, cfg.top_k, cfg.n_experts
    ids = []
    for li in range(L):
        x = synth.make_tokens(cfg, N, layer=li, kind="ar1")
        r = orc.route(orc.bits(x), orc.bits(synth.make_router(cfg, li)), None, k, True)
        ids.append(np.asarray(r[0]))
    ids = np.stack(ids)                                            # [L, N, k]

    def play(make_cache, make_window, plan, predicted):
        c = make_cache(L, E, 3)
        pos = 0
        while pos + K + 1 <= N:
            for row in range(K + 1):
                if row in predicted:
                    w = make_window([[[(int(e), 1.0) for e in ids[li, pos + row]] for li in range(L)]])
                    plan(c, w)
                for li in range(L):
                    need = [int(e) for e in ids[li, pos + row]]
                    c.use(li, need)
                    t = c.slot_table(li)
                    c.on_demand(li, sorted({e for e in need if t[e] < 0}))
                c.end_window()
            pos += K + 1
        return c

    cover = {}
    for name, predicted in (("lru", []), ("single", [0]), ("speculative", list(range(K)))):
        o = play(SO.Cache, lambda w: w, lambda c, w: c.plan(w, 3), predicted)
        lib = play(S.Cache, elb_from, lambda c, w: (c.plan(w, S.PHASE_SATURATE), w.close()), predicted)
        assert lib.stats() == (o.hits, o.misses)
        cover[name] = o.hits / (o.hits + o.misses)
    assert cover["lru"] < cover["single"] < cover["speculative"]
    assert cover["speculative"] >= K / (K + 1)                     # every predicted token's experts were in place
