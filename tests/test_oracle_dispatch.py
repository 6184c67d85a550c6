"""Pins of the oracle's selective-offloading statistics (top-k compression, margin score, dispatch
probabilities) against what the paper's equations and the mathematics fix."""
import math

import numpy as np
import pytest

import oracle


def test_p_conf_closed_forms_of_the_first_dispatch_equation():
    # Section 4.2: 1 at or below the threshold; just above it norm = -1/2 -> 1 / (1 + e^-5); at c = 1
    # norm = +1/2 -> 1 / (1 + e^5); k = 10
    for c_th in (0.7, 0.8, 0.95):
        assert oracle.p_conf(c_th, c_th) == 1.0
        assert oracle.p_conf(0.0, c_th) == 1.0
        assert oracle.p_conf(c_th + 1e-12, c_th) == pytest.approx(1 / (1 + math.exp(-5)), abs=1e-9)
        assert oracle.p_conf(1.0, c_th) == pytest.approx(1 / (1 + math.exp(5)), abs=1e-12)
        mid = (1 + c_th) / 2                       # norm = 0 -> 1/2
        assert oracle.p_conf(mid, c_th) == pytest.approx(0.5, abs=1e-12)
    assert 1 / (1 + math.exp(-5)) == pytest.approx(0.99331, abs=1e-5)
    assert 1 / (1 + math.exp(5)) == pytest.approx(0.00669, abs=1e-5)
    # monotone non-increasing in c, slope parameter: k = 0 flattens the sigmoid to 1/2
    cs = np.linspace(0.0, 1.0, 201)
    v = [oracle.p_conf(c, 0.7) for c in cs]
    assert all(a >= b - 1e-15 for a, b in zip(v, v[1:]))
    assert oracle.p_conf(0.9, 0.7, k=0.0) == 0.5


def test_p_imp_three_tiers_of_the_second_dispatch_equation():
    i_th = 0.4
    assert oracle.p_imp(0.0, i_th) == 0.0 and oracle.p_imp(i_th / 2, i_th) == 0.0
    assert oracle.p_imp(i_th * 1.0001, i_th) == 1.0 and oracle.p_imp(5.0, i_th) == 1.0
    # theta = -10: just above i_th/2 norm = -1/2 -> 1 / (1 + e^5); at i_th norm = +1/2 -> 1 / (1 + e^-5)
    assert oracle.p_imp(i_th / 2 + 1e-12, i_th) == pytest.approx(1 / (1 + math.exp(5)), abs=1e-9)
    assert oracle.p_imp(i_th, i_th) == pytest.approx(1 / (1 + math.exp(-5)), abs=1e-12)
    assert oracle.p_imp(0.75 * i_th, i_th) == pytest.approx(0.5, abs=1e-12)
    v = [oracle.p_imp(i, i_th) for i in np.linspace(0, 1, 301)]
    assert all(a <= b + 1e-15 for a, b in zip(v, v[1:]))          # non-decreasing in i


def test_topk_against_numpy_sort_and_the_plain_confidence_functions():
    rng = np.random.default_rng(3)
    for V, k in ((7, 3), (50, 8), (1000, 5), (4096, 1)):
        x = rng.normal(0, 3, V)
        ids, p = oracle.topk_row(x, k)
        order = np.argsort(-x, kind="stable")[:k]
        assert np.array_equal(ids, order)
        full = np.exp(x - x.max()); full /= full.sum()
        assert np.allclose(p, full[order], rtol=1e-13, atol=0)
        idx, p1, _, _ = oracle.confidence_row(x)
        assert ids[0] == idx and p[0] == pytest.approx(p1, rel=1e-13)
        assert np.all(np.diff(p) <= 0)
    # k = V: the compressed distribution is the whole one
    x = rng.normal(0, 1, 33)
    ids, p = oracle.topk_row(x, 33)
    assert sorted(ids.tolist()) == list(range(33)) and p.sum() == pytest.approx(1.0, abs=1e-13)


def test_topk_ties_go_to_the_lower_id_and_margin_closed_forms():
    ids, p = oracle.topk_row([1.0, 3.0, 3.0, 0.0, 3.0], 4)
    assert ids.tolist() == [1, 2, 4, 0]
    assert p[0] == p[1] == p[2]
    assert oracle.margin_row([1.0, 3.0, 3.0]) == 0.0
    # two-token vocabulary with logit gap d: p1 - p2 = tanh(d / 2)
    for d in (0.0, 0.3, 2.0, 9.0):
        assert oracle.margin_row([0.0, d]) == pytest.approx(math.tanh(d / 2), abs=1e-14)
    # uniform logits: every probability 1/V, margin 0; one-hot limit: margin -> 1
    ids, p, mg = oracle.topk(np.zeros((2, 64)), 4)
    assert np.allclose(p, 1 / 64) and np.all(mg == 0) and ids.tolist() == [[0, 1, 2, 3]] * 2
    x = np.zeros(100); x[17] = 60.0
    assert oracle.margin_row(x) == pytest.approx(1.0, abs=1e-20 + 1e-12)
    # the margin of topk() is top-1 minus top-2 whatever k is
    z = np.random.default_rng(2).normal(0, 2, (3, 50))
    assert np.array_equal(oracle.topk(z, 1)[2], oracle.topk(z, 5)[2])
    assert oracle.topk(z, 1)[2][0] == oracle.margin_row(z[0])
    # shift invariance
    y = np.random.default_rng(1).normal(0, 2, 300)
    a = oracle.topk_row(y, 6); b = oracle.topk_row(y + 77.0, 6)
    assert np.array_equal(a[0], b[0]) and np.allclose(a[1], b[1], rtol=1e-12)


def test_chunk_dispatch_means_and_probabilities():
    p1 = np.array([0.9, 0.8, 1.0, 0.2, 0.95, 0.95, 0.95, 0.5])
    cu = np.array([0, 3, 4, 4, 7, 8])
    mean, pc = oracle.chunk_dispatch(p1, cu, c_th=0.7)
    assert np.allclose(mean, [0.9, 0.2, 0.0, 0.95, 0.5])
    want = [oracle.p_conf(0.9, 0.7), 1.0, 1.0, oracle.p_conf(0.95, 0.7), 1.0]
    assert np.allclose(pc, want, rtol=0, atol=1e-15)
    # c = 0.9 with c_th = 0.7: norm = 2/3 - 1/2 = 1/6 -> 1 / (1 + e^(10/6))
    assert pc[0] == pytest.approx(1 / (1 + math.exp(10 / 6)), abs=1e-12)


def test_topp_count_closed_forms_and_brute_force():
    """Nucleus size: uniform over V -> ceil(p V) (binary fractions, exact in float32); one-hot -> 1; a list
    that never reaches p is kept whole; and against sorting + cumulative sums of a random distribution."""
    import math
    import oracle
    V = 64
    for p in (0.25, 0.5, 0.515625, 1.0):
        n, mass = oracle.topp_count([1.0 / V] * V, p)
        assert n == math.ceil(p * V) and abs(mass - n / V) < 1e-7
    assert oracle.topp_count([1.0, 0.0, 0.0], 0.9) == (1, 1.0)
    assert oracle.topp_count([0.5, 0.25], 0.9) == (2, 0.75)            # a top-2 window that holds 75 %: keep both
    rng = np.random.default_rng(5)
    for _ in range(50):
        x = rng.normal(0, 3, 200)
        ids, pr = oracle.topk_row(x, 200)
        pr32 = pr.astype(np.float32)
        p = float(rng.uniform(0.05, 0.999))
        n, mass = oracle.topp_count(pr32, p)
        cum = np.cumsum(np.sort(oracle.softmax_probs(x))[::-1])       # float64 reference of the definition
        n_ref = int(np.searchsorted(cum, p, side="left")) + 1
        assert abs(n - n_ref) <= (1 if np.min(np.abs(cum - p)) < 1e-5 else 0)
        assert mass >= p - 1e-6 and (n == 1 or mass - float(pr32[n - 1]) < p + 1e-6)


def test_topk_at_the_sizes_of_a_transmitted_list():
    """"Compression before transmission" cuts a 32000-entry distribution by over 99.5 %: lists of up to 160
    entries.  The same definition at k = 64, 160, 256: against numpy's stable sort, on rows with many exact ties
    (bf16-rounded logits), and the mass the list holds against the complement's."""
    rng = np.random.default_rng(8)
    for V, k in ((32000, 64), (32000, 160), (4096, 256), (300, 256)):
        x = oracle.bf16_round(rng.normal(4.0, 0.05 if V == 4096 else 3.0, V)).astype(np.float64)
        ids, p = oracle.topk_row(x, k)
        order = np.argsort(-x, kind="stable")[:k]
        assert np.array_equal(ids, order)
        assert len(set(ids.tolist())) == k and np.all(np.diff(p) <= 0)
        full = oracle.softmax_probs(x)
        rest = np.delete(full, order)
        assert p.sum() + rest.sum() == pytest.approx(1.0, abs=1e-12)
        assert rest.max() <= p[-1]


def test_nucleus_closed_forms_and_brute_force():
    """Full-vocabulary top-p: uniform over V -> ceil(p V) tokens; a geometric distribution p_i = (1 - r) r^i ->
    the smallest n with 1 - r^n >= top_p; one-hot -> 1; and against the float32 list form on a sorted vector."""
    V = 64
    for tp in (0.25, 0.5, 0.515625, 1.0):
        n, mass, cut, gap = oracle.nucleus_row(np.zeros(V), tp)
        assert n == math.ceil(tp * V) and mass == pytest.approx(n / V, abs=1e-14) and cut == 0.0
    r, V = 0.9, 400                                      # logits i ln r: p_i = r^i (1 - r) / (1 - r^V)
    x = np.arange(V) * math.log(r)
    for tp in (0.1, 0.5, 0.9, 0.99):
        n, mass, cut, gap = oracle.nucleus_row(x, tp)
        want = math.ceil(math.log(1 - tp * (1 - r ** V)) / math.log(r) - 1e-12)
        assert n == want
        assert mass == pytest.approx((1 - r ** n) / (1 - r ** V), rel=1e-12)
        assert cut == pytest.approx((n - 1) * math.log(r), rel=1e-12)
    hot = np.zeros(100); hot[17] = 50.0
    assert oracle.nucleus_row(hot, 0.999)[0] == 1
    # permuting the vocabulary changes neither the size nor the mass; ties are kept in id order
    rng = np.random.default_rng(4)
    for _ in range(30):
        x = rng.normal(0, 3, 500)
        tp = float(rng.uniform(0.05, 0.999))
        n, mass, cut, gap = oracle.nucleus_row(x, tp)
        perm = rng.permutation(500)
        n2, mass2, cut2, _ = oracle.nucleus_row(x[perm], tp)
        assert (n, cut) == (n2, cut2) and mass == pytest.approx(mass2, rel=1e-12)
        assert mass >= tp - 1e-12 and np.sum(x >= cut) == n
        _, pr = oracle.topk_row(x, 500)
        n32, _ = oracle.topp_count(pr.astype(np.float32), tp)
        assert abs(n32 - n) <= (1 if gap < 1e-5 else 0)
    t = np.array([1.0, 2.0, 2.0, 2.0, 0.0])               # three tied leaders: 2 of them reach 0.5
    assert oracle.nucleus_row(t, 0.5)[0] == 2 and oracle.nucleus_row(t, 0.5)[2] == 2.0


def test_golden_points_of_the_dispatch_curves():
    """tests/golden/dispatch_probabilities.txt: values worked by hand from the two printed equations."""
    import os
    import oracle
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "dispatch_probabilities.txt")
    n = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        fn, x, th, slope, want, tol = line.split()
        got = {"p_conf": oracle.p_conf, "p_imp": oracle.p_imp}[fn](float(x), float(th), float(slope))
        assert abs(got - float(want)) <= float(tol), line
        n += 1
    assert n == 13
