"""Pins for the CPU oracle: every function of oracle/moe_oracle.c is checked against something
that does not go through it -- brute force on tiny inputs, closed forms, invariants, special
cases that reduce to a numpy / scipy / torch routine, and the one worked example the paper
gives (the reordering example of section 3.4.4).  The paper prints no numeric example of the
layer itself, so there is no golden value from the paper for the float outputs."""
import itertools
import os

import numpy as np
import pytest
import scipy.special
import torch
from hypothesis import given, settings, strategies as st

from oracle import oracle as orc
from tests.common import bf16_exact

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f16bits(a):
    return np.asarray(a, np.float16).view(np.uint16)


def bf(a):
    return orc.bits(bf16_exact(a))


def widen_bf16(t):
    return t.to(torch.float64).numpy()


# ---------------------------------------------------------------- 16-bit widening

def test_fp16_widening_all_patterns_match_numpy():
    pats = np.arange(65536, dtype=np.uint16)
    ref = pats.view(np.float16).astype(np.float64)
    got = np.array([orc.fp16_to_f64(int(p)) for p in pats])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


def test_bf16_widening_all_patterns_match_torch():
    pats = np.arange(65536, dtype=np.uint16)
    ref = torch.from_numpy(pats.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([orc.bf16_to_f64(int(p)) for p in pats])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])


# ---------------------------------------------------------------- router: logits

def test_logits_match_numpy_matmul_and_are_not_transposed():
    rng = np.random.default_rng(1)
    T, H, E = 3, 40, 7                      # all different: a transposed operand cannot pass
    x = torch.from_numpy(rng.standard_normal((T, H), dtype=np.float32)).to(torch.bfloat16)
    wr = torch.from_numpy(rng.standard_normal((E, H), dtype=np.float32)).to(torch.bfloat16)
    b = rng.standard_normal(E).astype(np.float32)
    _, _, _, logits = orc.route(orc.bits(x), orc.bits(wr), b, 2)
    ref = widen_bf16(x) @ widen_bf16(wr).T + b.astype(np.float64)
    np.testing.assert_allclose(logits, ref, rtol=0, atol=1e-12)
    _, _, _, l0 = orc.route(orc.bits(x), orc.bits(wr), None, 2)
    np.testing.assert_allclose(l0, ref - b.astype(np.float64), rtol=0, atol=1e-12)


def test_logits_exact_on_small_integers():
    rng = np.random.default_rng(2)
    x = rng.integers(-4, 5, (5, 16)).astype(np.float64)
    wr = rng.integers(-4, 5, (6, 16)).astype(np.float64)
    _, _, _, logits = orc.route(bf(x), bf(wr), None, 1)
    assert np.array_equal(logits, x @ wr.T)


# ---------------------------------------------------------------- router: top-k and ties

def route_on_logits(l, k, renorm=True):
    """Drive orc_route with chosen logits: identity router, x = logits (bf16-exact values)."""
    l = np.atleast_2d(np.asarray(l, np.float64))
    E = l.shape[1]
    return orc.route(bf(l), bf(np.eye(E)), None, k, renorm)


def brute_force_topk(row, k):
    """The size-k subset that is maximal under 'larger logit first, then lower index',
    found by enumerating every subset and comparing their sorted key lists."""
    E = len(row)
    best = None
    for sub in itertools.combinations(range(E), k):
        key = sorted((-row[e], e) for e in sub)
        if best is None or key < best[0]:
            best = (key, sub)
    return [e for _, e in best[0]]


@settings(max_examples=200, deadline=None)
@given(st.integers(2, 8).flatmap(lambda E: st.tuples(
    st.lists(st.integers(-3, 3), min_size=E, max_size=E), st.integers(1, E))))
def test_topk_matches_brute_force_with_duplicates(case):
    row, k = case
    ids, w, conf, _ = route_on_logits([float(v) / 2 for v in row], k)
    assert ids[0].tolist() == brute_force_topk([float(v) / 2 for v in row], k)


def test_topk_random_rows_match_stable_argsort():
    rng = np.random.default_rng(3)
    l = torch.from_numpy(rng.standard_normal((64, 37), dtype=np.float32)).to(torch.bfloat16)
    l = widen_bf16(l)
    ids, _, _, _ = route_on_logits(l, 5)
    ref = np.argsort(-l, axis=1, kind="stable")[:, :5]
    assert np.array_equal(ids, ref)


def test_ties_go_to_the_lower_index():
    # duplicate router rows give exactly equal logits
    rng = np.random.default_rng(4)
    H = 32
    x = torch.from_numpy(rng.standard_normal((6, H), dtype=np.float32)).to(torch.bfloat16)
    row = torch.from_numpy(rng.standard_normal((1, H), dtype=np.float32)).to(torch.bfloat16)
    wr = row.repeat(5, 1)
    ids, w, conf, logits = orc.route(orc.bits(x), orc.bits(wr), None, 3)
    assert np.all(logits == logits[:, :1])
    assert np.array_equal(ids, np.tile(np.arange(3, dtype=np.int32), (6, 1)))
    np.testing.assert_allclose(w, 1.0 / 3.0, rtol=0, atol=1e-15)
    np.testing.assert_allclose(conf, 1.0 / 5.0, rtol=0, atol=1e-15)
    # a tie between a late and an early expert, with a clear winner in the middle
    ids, _, _, _ = route_on_logits([[1.0, 0.0, 2.0, 1.0, -1.0]], 3)
    assert ids[0].tolist() == [2, 0, 3]
    ids, _, _, _ = route_on_logits([[0.5, 1.0, 1.0, 0.5]], 3)
    assert ids[0].tolist() == [1, 2, 0]


# ---------------------------------------------------------------- router: softmax weights

def test_softmax_weights_closed_forms():
    rng = np.random.default_rng(5)
    l = widen_bf16(torch.from_numpy(3 * rng.standard_normal((32, 16), dtype=np.float32))
                   .to(torch.bfloat16))
    k = 4
    ids, w, conf, logits = route_on_logits(l, k, renorm=True)
    assert np.array_equal(logits, l)
    p = scipy.special.softmax(l, axis=1)
    np.testing.assert_allclose(conf, np.take_along_axis(p, ids, 1), rtol=1e-13, atol=0)
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=0, atol=1e-15)
    # the full normaliser cancels: w is the softmax over the k selected logits alone
    sel = np.take_along_axis(l, ids, 1)
    np.testing.assert_allclose(w, scipy.special.softmax(sel, axis=1), rtol=1e-13, atol=0)
    assert np.all(conf.sum(1) <= 1.0 + 1e-15)
    # without renormalisation the weights are the probabilities themselves
    ids2, w2, conf2, _ = route_on_logits(l, k, renorm=False)
    assert np.array_equal(ids2, ids) and np.array_equal(w2, conf2)
    np.testing.assert_allclose(conf2, conf, rtol=0, atol=0)
    # weights follow rank order
    assert np.all(np.diff(w, axis=1) <= 0)


def test_softmax_shift_invariance_and_large_logits():
    rng = np.random.default_rng(6)
    H, E, T = 24, 9, 5
    x = torch.from_numpy(rng.standard_normal((T, H), dtype=np.float32)).to(torch.bfloat16)
    wr = torch.from_numpy(rng.standard_normal((E, H), dtype=np.float32)).to(torch.bfloat16)
    b = (np.round(rng.standard_normal(E) * 64) / 64).astype(np.float32)   # b + 64 exact in fp32
    a = orc.route(orc.bits(x), orc.bits(wr), b, 3)
    c = orc.route(orc.bits(x), orc.bits(wr), (b + np.float32(64.0)).astype(np.float32), 3)
    assert np.array_equal(a[0], c[0])
    np.testing.assert_allclose(a[1], c[1], rtol=1e-9)
    np.testing.assert_allclose(a[2], c[2], rtol=1e-9)
    # logits of +-600 overflow a naive exp(); the shifted form must stay finite
    ids, w, conf, _ = orc.route(bf(np.zeros((1, 4))), bf(np.zeros((3, 4))),
                                np.array([600.0, -600.0, 599.0], np.float32), 2)
    assert ids[0].tolist() == [0, 2]
    np.testing.assert_allclose(w[0], scipy.special.softmax([600.0, 599.0]), rtol=1e-13)
    assert np.all(np.isfinite(conf))


# ---------------------------------------------------------------- histogram / permutation

def test_reorder_example_of_the_paper():
    tok, exp, order = [], [], {}
    with open(os.path.join(GOLDEN, "reorder_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("order"):
                head, rest = line.split(":")
                order[int(head.split()[1])] = [int(v) for v in rest.split()]
            else:
                t, e = line.split()
                tok.append(int(t)); exp.append(int(e))
    assert tok == list(range(1, 10))
    count, off, pm = orc.perm(np.array(exp, np.int32), 3)
    got = {e: [int(a) + 1 for a in pm[off[e]:off[e + 1]]] for e in range(3)}
    assert got == order
    assert count.tolist() == [3, 3, 3]


@settings(max_examples=200, deadline=None)
@given(st.integers(1, 20).flatmap(lambda E: st.tuples(
    st.just(E), st.lists(st.integers(0, E - 1), min_size=0, max_size=64))))
def test_perm_invariants_and_stable_argsort(case):
    E, ids = case
    ids = np.array(ids, np.int32)
    count, off, pm = orc.perm(ids, E)
    n = ids.size
    assert count.sum() == n and off[0] == 0 and off[E] == n
    assert np.array_equal(np.diff(off), count)
    assert np.array_equal(count, np.bincount(ids, minlength=E))
    assert sorted(pm.tolist()) == list(range(n))
    assert np.all(np.diff(ids[pm]) >= 0)
    assert np.array_equal(pm, np.argsort(ids, kind="stable").astype(np.int32))
    for e in range(E):                      # stability: ascending assignment index per expert
        seg = pm[off[e]:off[e + 1]]
        assert np.all(np.diff(seg) > 0) and np.all(ids[seg] == e)


# ---------------------------------------------------------------- union

@settings(max_examples=200, deadline=None)
@given(st.integers(1, 200).flatmap(lambda E: st.tuples(
    st.just(E), st.lists(st.integers(0, E - 1), min_size=0, max_size=80),
    st.lists(st.booleans(), min_size=E, max_size=E))))
def test_union_matches_python_sets(case):
    E, ids, resident = case
    slot = np.full(E, -1, np.int32)
    nxt = 0
    for e in range(E):
        if resident[e]:
            slot[e] = nxt
            nxt += 1
    mask, lst, miss = orc.union(np.array(ids, np.int32), E, slot)
    want = sorted(set(ids))
    assert lst.tolist() == want
    assert miss.tolist() == [e for e in want if slot[e] < 0]
    pop = sum(bin(int(m)).count("1") for m in mask)
    assert pop == len(want)
    for e in range(E):
        assert bool((int(mask[e // 64]) >> (e % 64)) & 1) == (e in set(ids))
    _, lst2, miss2 = orc.union(np.array(ids, np.int32), E, None)
    assert lst2.tolist() == want and miss2.size == 0


# ---------------------------------------------------------------- dequantisation

def test_dequant_closed_form_all_codes():
    codes = np.arange(16, dtype=np.uint8)
    for s in (1.0, 0.5, 0.0123, 3.0e-4, 2.0):
        for z in (0.0, 8.0, 15.0, 3.0, 7.5):
            s16, z16 = np.float16(s), np.float16(z)
            q = codes.reshape(1, 16)
            got = orc.dequant(q, f16bits([[s16]]), f16bits([[z16]]), 16)
            want = (codes.astype(np.float64) - float(z16)) * float(s16)
            assert np.array_equal(got[0], want)
    # z = 8 is symmetric int4: codes 0..15 -> (-8..7) * s
    got = orc.dequant(codes.reshape(1, 16), f16bits([[0.25]]), f16bits([[8.0]]), 16)
    assert np.array_equal(got[0], np.arange(-8, 8) * 0.25)


def test_dequant_groups_run_along_the_input_dimension():
    # 2 rows, 8 columns, group 4: each (row, group) has its own scale / zero
    q = np.arange(16, dtype=np.uint8).reshape(2, 8)
    s = np.array([[1.0, 2.0], [0.5, 4.0]], np.float16)
    z = np.array([[0.0, 1.0], [2.0, 3.0]], np.float16)
    got = orc.dequant(q, f16bits(s), f16bits(z), 4)
    want = np.empty((2, 8))
    for r in range(2):
        for c in range(8):
            want[r, c] = (float(q[r, c]) - float(z[r, c // 4])) * float(s[r, c // 4])
    assert np.array_equal(got, want)
    assert got[0, 4] == (4 - 1) * 2.0 and got[1, 3] == (11 - 2) * 0.5


# ---------------------------------------------------------------- SwiGLU expert

def test_silu_special_values_through_identity_expert():
    # H = I, Wg = Wu = Wd = identity: FFN(x)[i] = silu(x_i) * x_i
    n = 16
    eye = bf(np.eye(n))
    xs = np.array([0.0, 1.0, -1.0, 2.5, -2.5, 8.0, -8.0, 0.125, -0.125, 30.0, -30.0,
                   0.5, -0.5, 3.0, -3.0, 100.0])
    out = orc.ffn_bf16(eye, eye, eye, xs)
    np.testing.assert_allclose(out, xs * scipy.special.expit(xs) * xs, rtol=1e-14, atol=0)
    assert out[0] == 0.0
    silu_vals = out[1:] / xs[1:]
    # silu(a) - silu(-a) = a
    for i in (0, 2, 4, 6, 8, 10, 12):
        np.testing.assert_allclose(silu_vals[i] - silu_vals[i + 1], xs[1 + i], rtol=1e-13)


def test_ffn_bf16_matches_numpy_and_scipy_non_square():
    rng = np.random.default_rng(7)
    H, I = 24, 40
    wg = torch.from_numpy(rng.standard_normal((I, H), dtype=np.float32)).to(torch.bfloat16)
    wu = torch.from_numpy(rng.standard_normal((I, H), dtype=np.float32)).to(torch.bfloat16)
    wd = torch.from_numpy(rng.standard_normal((H, I), dtype=np.float32)).to(torch.bfloat16)
    x = rng.standard_normal(H)
    got = orc.ffn_bf16(orc.bits(wg), orc.bits(wu), orc.bits(wd), x)
    a = widen_bf16(wg) @ x
    want = widen_bf16(wd) @ (a * scipy.special.expit(a) * (widen_bf16(wu) @ x))
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    # gate and up are not interchangeable, and a zero gate kills the output
    swapped = orc.ffn_bf16(orc.bits(wu), orc.bits(wg), orc.bits(wd), x)
    assert np.max(np.abs(swapped - want)) > 1e-3
    zero = orc.ffn_bf16(orc.bits(torch.zeros_like(wg)), orc.bits(wu), orc.bits(wd), x)
    assert np.array_equal(zero, np.zeros(H))
    # doubling Wd doubles the output exactly (a power of two)
    dbl = orc.ffn_bf16(orc.bits(wg), orc.bits(wu), orc.bits(wd * 2), x)
    assert np.array_equal(dbl, 2.0 * got)


def test_ffn_int4_integer_case_is_exact_and_equals_bf16_ffn_on_dequantised_weights():
    rng = np.random.default_rng(8)
    H, I, g = 32, 64, 16
    q = {n: rng.integers(0, 16, shp).astype(np.uint8)
         for n, shp in (("g", (I, H)), ("u", (I, H)), ("d", (H, I)))}
    # power-of-two scales and integer zeros: (q - z) * s has < 8 significant bits -> bf16-exact
    def sz(rows, groups):
        s = (2.0 ** rng.integers(-6, -2, (rows, groups))).astype(np.float16)
        z = rng.integers(0, 16, (rows, groups)).astype(np.float16)
        return s, z
    sg, zg = sz(I, H // g); su, zu = sz(I, H // g); sd, zd = sz(H, I // g)
    x = rng.integers(-3, 4, H).astype(np.float64)
    got = orc.ffn_int4(q["g"], f16bits(sg), f16bits(zg), q["u"], f16bits(su), f16bits(zu),
                       q["d"], f16bits(sd), f16bits(zd), g, x)

    def deq(qq, s, z):
        return (qq.astype(np.float64) - np.repeat(z.astype(np.float64), g, 1)) \
            * np.repeat(s.astype(np.float64), g, 1)
    Wg, Wu, Wd = deq(q["g"], sg, zg), deq(q["u"], su, zu), deq(q["d"], sd, zd)
    a = Wg @ x
    want = Wd @ (a * scipy.special.expit(a) * (Wu @ x))
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    via_bf16 = orc.ffn_bf16(bf(Wg), bf(Wu), bf(Wd), x)
    np.testing.assert_allclose(got, via_bf16, rtol=1e-13, atol=1e-13)
    # s = 1, z = 0 and integer x: the gate pre-activation is an exact integer dot product;
    # check it through an expert whose up path is 1 and whose down path picks row 0
    one = np.ones((I, H // g), np.float16); zero = np.zeros((I, H // g), np.float16)
    qu1 = np.zeros((I, H), np.uint8); qu1[:, 0] = 1
    xx = x.copy(); xx[0] = 1.0
    qd1 = np.zeros((H, I), np.uint8); qd1[0, 5] = 1
    out = orc.ffn_int4(q["g"], f16bits(one), f16bits(zero), qu1, f16bits(one), f16bits(zero),
                       qd1, f16bits(np.ones((H, I // g), np.float16)),
                       f16bits(np.zeros((H, I // g), np.float16)), g, xx)
    a5 = float(q["g"][5].astype(np.int64) @ xx.astype(np.int64))
    np.testing.assert_allclose(out[0], a5 * scipy.special.expit(a5), rtol=1e-14)
    assert np.array_equal(out[1:], np.zeros(H - 1))


# ---------------------------------------------------------------- the layer

def small_layer(seed, T=5, H=24, I=40, E=6, S=0):
    rng = np.random.default_rng(seed)
    def t(*shape, std=1.0):
        return torch.from_numpy((std * rng.standard_normal(shape)).astype(np.float32)) \
            .to(torch.bfloat16)
    return dict(x=t(T, H), wr=t(E, H, std=0.5), wg=t(E + S, I, H, std=0.3),
                wu=t(E + S, I, H, std=0.3), wd=t(E + S, H, I, std=0.3), E=E, S=S)


def numpy_ffn(wg, wu, wd, x):
    a = wg @ x
    return wd @ (a * scipy.special.expit(a) * (wu @ x))


def run_bf16(L, k, renorm=True, present=None):
    ids, w, conf, logits = orc.route(orc.bits(L["x"]), orc.bits(L["wr"]), None, k, renorm)
    y = orc.layer_bf16(orc.bits(L["x"]), orc.bits(L["wg"]), orc.bits(L["wu"]),
                       orc.bits(L["wd"]), L["E"], ids, w, present)
    return ids, w, y


def test_layer_k_equals_E_is_the_dense_softmax_mixture():
    L = small_layer(11)
    ids, w, y = run_bf16(L, L["E"], renorm=False)
    x = widen_bf16(L["x"]); wr = widen_bf16(L["wr"])
    p = scipy.special.softmax(x @ wr.T, axis=1)
    want = np.zeros_like(y)
    for t in range(x.shape[0]):
        for e in range(L["E"]):
            want[t] += p[t, e] * numpy_ffn(widen_bf16(L["wg"][e]), widen_bf16(L["wu"][e]),
                                           widen_bf16(L["wd"][e]), x[t])
    np.testing.assert_allclose(y, want, rtol=1e-11, atol=1e-11)


def test_layer_k1_is_the_argmax_expert():
    L = small_layer(12)
    ids, w, y = run_bf16(L, 1, renorm=True)
    x = widen_bf16(L["x"]); wr = widen_bf16(L["wr"])
    best = np.argmax(x @ wr.T, axis=1)
    assert np.array_equal(ids[:, 0], best)
    assert np.array_equal(w, np.ones_like(w))
    for t in range(x.shape[0]):
        e = int(best[t])
        want = numpy_ffn(widen_bf16(L["wg"][e]), widen_bf16(L["wu"][e]),
                         widen_bf16(L["wd"][e]), x[t])
        np.testing.assert_allclose(y[t], want, rtol=1e-11, atol=1e-11)


def test_layer_identical_experts_make_routing_irrelevant():
    L = small_layer(13)
    for n in ("wg", "wu", "wd"):
        L[n] = L[n][:1].repeat(L["E"], 1, 1)
    _, w, y = run_bf16(L, 3, renorm=True)
    x = widen_bf16(L["x"])
    for t in range(x.shape[0]):
        want = numpy_ffn(widen_bf16(L["wg"][0]), widen_bf16(L["wu"][0]),
                         widen_bf16(L["wd"][0]), x[t])
        np.testing.assert_allclose(y[t], want, rtol=1e-11, atol=1e-11)


def test_layer_expert_relabelling_permutes_ids_and_keeps_y():
    L = small_layer(14)
    ids, w, y = run_bf16(L, 2)
    pi = np.random.default_rng(0).permutation(L["E"])       # new index -> old index
    M = dict(L)
    for n in ("wr", "wg", "wu", "wd"):
        M[n] = L[n][torch.from_numpy(pi)]
    ids2, w2, y2 = run_bf16(M, 2)
    assert np.array_equal(pi[ids2], ids)
    np.testing.assert_allclose(w2, w, rtol=1e-14)
    np.testing.assert_allclose(y2, y, rtol=1e-12, atol=1e-13)


def test_layer_shared_experts_add_with_weight_one_and_absent_experts_drop_out():
    L = small_layer(15, S=2)
    E = L["E"]
    ids, w, y = run_bf16(L, 2)
    x = widen_bf16(L["x"])
    base = dict(L); base["S"] = 0
    for n in ("wg", "wu", "wd"):
        base[n] = L[n][:E]
    _, _, y0 = run_bf16(base, 2)
    for t in range(x.shape[0]):
        add = sum(numpy_ffn(widen_bf16(L["wg"][E + s]), widen_bf16(L["wu"][E + s]),
                            widen_bf16(L["wd"][E + s]), x[t]) for s in range(2))
        np.testing.assert_allclose(y[t] - y0[t], add, rtol=1e-9, atol=1e-11)
    # an absent expert's term is simply missing
    gone = int(ids[0, 1])
    present = np.ones(E, np.uint8); present[gone] = 0
    _, _, yp = run_bf16(base, 2, present=present)
    for t in range(x.shape[0]):
        want = y0[t].copy()
        for j in range(2):
            if ids[t, j] == gone:
                want -= w[t, j] * numpy_ffn(widen_bf16(L["wg"][gone]), widen_bf16(L["wu"][gone]),
                                            widen_bf16(L["wd"][gone]), x[t])
        np.testing.assert_allclose(yp[t], want, rtol=1e-9, atol=1e-11)


def test_draft_layer_equals_verify_layer_on_dequantised_weights():
    rng = np.random.default_rng(16)
    T, H, I, E, S, g, k = 4, 32, 64, 5, 1, 16, 2
    q, s, z, deq = {}, {}, {}, {}
    for n, (r, c) in (("gate", (I, H)), ("up", (I, H)), ("down", (H, I))):
        q[n] = rng.integers(0, 16, (E, r, c)).astype(np.uint8)
        s[n] = (2.0 ** rng.integers(-6, -3, (E, r, c // g))).astype(np.float16)
        z[n] = rng.integers(0, 16, (E, r, c // g)).astype(np.float16)
        deq[n] = (q[n].astype(np.float64) - np.repeat(z[n].astype(np.float64), g, 2)) \
            * np.repeat(s[n].astype(np.float64), g, 2)
    sh = small_layer(17, T=T, H=H, I=I, E=S)                 # S shared experts, bf16
    x = sh["x"]
    wr = torch.from_numpy(rng.standard_normal((E, H), dtype=np.float32)).to(torch.bfloat16)
    ids, w, conf, _ = orc.route(orc.bits(x), orc.bits(wr), None, k)
    y_draft = orc.layer_int4(orc.bits(x), q, {n: f16bits(s[n]) for n in s},
                             {n: f16bits(z[n]) for n in z}, g, ids, w,
                             (orc.bits(sh["wg"]), orc.bits(sh["wu"]), orc.bits(sh["wd"])))
    full = {n: np.concatenate([bf(deq[m]), orc.bits(sh[n])])
            for n, m in (("wg", "gate"), ("wu", "up"), ("wd", "down"))}
    y_verify = orc.layer_bf16(orc.bits(x), full["wg"], full["wu"], full["wd"], E, ids, w)
    np.testing.assert_allclose(y_draft, y_verify, rtol=1e-12, atol=1e-13)
    assert np.max(np.abs(y_draft)) > 1e-3
