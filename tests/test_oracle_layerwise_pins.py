"""Pins for the oracle's layer-wise threshold (Section 3.4, Eq. 4): mean and variance
of a layer's gradient importance and the threshold derived from them.  CPU only;
checked against a hand-worked example, exact rational arithmetic, closed forms,
numpy's mean / var, and the threshold-mode step fed with independently computed
thresholds."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
EPS = np.float32(1e-8)


def _hand():
    rows, exp = [], {}
    for line in open(os.path.join(GOLDEN, "hand_example.txt")):
        line = line.strip()
        if line and not line.startswith("#") and not line.startswith("expect_"):
            rows.append([float(t) for t in line.split()[1:]])
    for line in open(os.path.join(GOLDEN, "hand_example_layerwise.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            tok = line.split()
            exp[tok[0].replace("expect_", "")] = tok[1:]
    return np.array(rows, np.float32), exp


def _f32_of(fr: Fraction) -> np.float32:
    return np.float32(fr.numerator / fr.denominator)


def test_hand_worked_example():
    a, exp = _hand()
    w, r0, g0, r1, g1 = [np.ascontiguousarray(a[:, c]) for c in range(5)]
    alpha, beta, c = float(exp["alpha"][0]), float(exp["beta"][0]), float(exp["C"][0])
    A0, A1 = r0 + g0, r1 + g1
    for node, acc in enumerate((A0, A1)):
        m, v = oracle.layer_stats(w, acc, 0.0)
        assert m == float(exp["mean%d" % node][0]) and v == float(exp["var%d" % node][0])
        num, den = [int(t) for t in exp["thr%d_fraction" % node]]
        assert oracle.layerwise_threshold(m, v, alpha, beta, c) == _f32_of(Fraction(num, den))
    stats, thr, mask, counts, idx, sm = oracle.step_layerwise(w, [g0, g1], [r0, r1], [(0, 8, 0, 0)],
                                                              np.array([[0, 1]], np.uint32), alpha, beta, c, 0.0, -0.5, 8)
    assert stats[0, 0].tolist() == [1.1875, 0.49609375] and stats[0, 1].tolist() == [1.1875, 2.66796875]
    assert mask.tolist() == [int(t, 0) for t in exp["mask"]]
    assert idx.tolist() == [int(t) for t in exp["idx"]] and counts.tolist() == [len(exp["idx"])]
    assert sm.tolist() == [float(t) for t in exp["sum"]]
    assert not r0[idx].any() and not r1[idx].any() and r0[1] == 2.0 and r1[1] == 1.0


def test_statistics_exact_rational():
    """Mean and population variance against exact rational arithmetic on the fp32 scores."""
    rng = np.random.default_rng(5)
    for n in (1, 2, 3, 17, 200):
        w = rng.standard_normal(n).astype(np.float32)
        r = (rng.standard_t(3, n) * 1e-2).astype(np.float32)
        s = oracle.score(w, r, float(EPS))
        fs = [Fraction(float(x)) for x in s]
        mean = sum(fs) / n
        var = sum((x - mean) ** 2 for x in fs) / n
        m, v = oracle.layer_stats(w, r, float(EPS))
        assert abs(Fraction(m) - mean) <= abs(mean) * Fraction(1, 10 ** 14)
        assert abs(Fraction(v) - var) <= var * Fraction(1, 10 ** 13) + Fraction(1, 10 ** 300)


def test_statistics_closed_forms():
    one = np.float32(1.0)                                  # |w| + 1e-8 rounds to 1 in binary32: score = |r|
    for n in (2, 10, 4097, 100_001):
        r = np.arange(1, n + 1, dtype=np.float32) * np.where(np.arange(n) % 2, -1, 1).astype(np.float32)
        m, v = oracle.layer_stats(np.full(n, one), r, float(EPS))
        assert m == (n + 1) / 2                            # arithmetic progression 1..n
        assert v == pytest.approx((n * n - 1) / 12, rel=1e-14)
    # population, not sample, variance: {1, 3} -> 1 (the sample variance would be 2)
    assert oracle.layer_stats(np.full(2, one), np.array([1, -3], np.float32), float(EPS)) == (2.0, 1.0)
    # constant importance: variance 0 exactly
    m, v = oracle.layer_stats(np.full(1000, np.float32(0.5)), np.full(1000, np.float32(0.25)), 0.0)
    assert (m, v) == (0.5, 0.0)
    # a large common offset does not cost the variance its digits
    r = (np.float32(2 ** 20) + (np.arange(4096) % 2)).astype(np.float32)
    m, v = oracle.layer_stats(np.full(4096, one), r, float(EPS))
    assert (m, v) == (2 ** 20 + 0.5, 0.25)
    # |.| on both operands and eps in the denominator
    m, v = oracle.layer_stats(np.array([-2.0, 0.0], np.float32), np.array([-4.0, 1.0], np.float32), 0.5)
    assert m == pytest.approx(1.8, rel=1e-7) and v == pytest.approx(0.04, rel=1e-6)
    assert oracle.layer_stats(np.zeros(0, np.float32), np.zeros(0, np.float32), 0.5) == (0.0, 0.0)


def test_statistics_against_numpy():
    rng = np.random.default_rng(6)
    for n in (1000, 65_537, 1_000_000):
        w = (rng.standard_normal(n) * 0.05).astype(np.float32)
        w[rng.random(n) < 0.001] = 0.0
        r = (rng.standard_t(3, n) * 1e-3).astype(np.float32)
        s = oracle.score(w, r, float(EPS)).astype(np.float64)
        m, v = oracle.layer_stats(w, r, float(EPS))
        assert m == pytest.approx(np.mean(s), rel=1e-12)
        assert v == pytest.approx(np.var(s), rel=1e-11)


def test_threshold_rule():
    """Eq. 4 as read: plus branch strictly above C, minus branch otherwise."""
    f = oracle.layerwise_threshold
    assert f(2.0, 6.0, 0.5, 0.25, 1.0) == np.float32(0.5 + 0.25 * 3.0)        # ratio 3 > C
    assert f(2.0, 6.0, 0.5, 0.25, 3.0) == np.float32(0.5 - 0.25 * 3.0)        # ratio == C: not above
    assert f(2.0, 6.0, 0.5, 0.25, 5.0) == np.float32(0.5 - 0.25 * 3.0)
    assert f(4.0, 1.0, 0.1, 0.0, 0.0) == np.float32(0.1)                       # beta = 0: alpha on both branches
    assert f(4.0, 0.0, 0.1, 7.0, 0.0) == np.float32(0.1)                       # no spread: alpha
    assert np.isnan(f(0.0, 0.0, 0.1, 1.0, 1.0))                                # all-zero importance: no threshold ...
    # rounded once from binary64
    assert f(3.0, 1.0, 0.1, 0.1, 0.0) == np.float32(0.1 + 0.1 * (1.0 / 3.0))
    rng = np.random.default_rng(8)
    for _ in range(200):
        mean, var = rng.random() + 0.01, rng.random() * 3
        alpha, beta, c = rng.random(), rng.random(), rng.random() * 3
        ratio = var / mean
        want = alpha + beta * ratio if ratio > c else alpha - beta * ratio
        assert f(mean, var, alpha, beta, c) == np.float32(want)
    # both branches are monotone in the ratio, in opposite directions
    assert f(1.0, 2.0, 1.0, 0.5, 0.0) < f(1.0, 3.0, 1.0, 0.5, 0.0)
    assert f(1.0, 2.0, 1.0, 0.5, 9.0) > f(1.0, 3.0, 1.0, 0.5, 9.0)


def test_nan_threshold_sends_nothing():
    w = np.ones(64, np.float32)
    r = [np.zeros(64, np.float32), np.ones(64, np.float32)]
    g = [np.zeros(64, np.float32)] * 2
    stats, thr, mask, counts, idx, sm = oracle.step_layerwise(w, g, r, [(0, 64, 0, 0)], np.array([[0]], np.uint32),
                                                              0.1, 1.0, 1.0, 1e-8, -1.0, 64)
    assert np.isnan(thr[0, 0]) and counts.tolist() == [0] and not mask.any() and r[1].all()


def test_step_equals_threshold_step_with_independent_thresholds():
    """The whole layer-wise step against numpy-computed statistics and thresholds handed
    to the fixed-threshold step, each chosen node with its own threshold."""
    rng = np.random.default_rng(9)
    sizes = [100, 4097, 33, 20_000]
    rows, off = [], 0
    for n in sizes:
        rows.append((off, n, 0, 0))
        off += n + 5
    W, n_lead = 4, 2
    w = (rng.standard_normal(off) * 0.05).astype(np.float32)
    g = [(rng.standard_t(3, off) * 1e-3).astype(np.float32) for _ in range(W)]
    r = [(rng.standard_t(3, off) * 1e-3).astype(np.float32) for _ in range(W)]
    leaders = rng.integers(0, W, (len(sizes), n_lead)).astype(np.uint32)
    alpha, beta, c = 0.02, 0.001, 30.0
    w1, r1 = w.copy(), [x.copy() for x in r]
    stats, thr, mask, counts, idx, sm = oracle.step_layerwise(w1, g, r1, rows, leaders, alpha, beta, c, float(EPS),
                                                              -0.01, off)
    thr_np = np.zeros((len(sizes), n_lead), np.float32)
    branches = set()
    for j, (o, n, _, _) in enumerate(rows):
        for q in range(n_lead):
            p = leaders[j, q]
            acc = r[p][o:o + n] + g[p][o:o + n]
            s = (np.abs(acc) / (np.abs(w[o:o + n]) + EPS)).astype(np.float64)
            mean, var = s.mean(), s.var()
            assert stats[j, q, 0] == pytest.approx(mean, rel=1e-12) and stats[j, q, 1] == pytest.approx(var, rel=1e-11)
            ratio = stats[j, q, 1] / stats[j, q, 0]
            branches.add(bool(ratio > c))
            thr_np[j, q] = np.float32(alpha + beta * ratio if ratio > c else alpha - beta * ratio)
    assert branches == {True, False}, "the example must exercise both branches of the rule"
    assert np.array_equal(thr, thr_np)
    w2, r2 = w.copy(), [x.copy() for x in r]
    mask2, counts2, idx2, sm2 = oracle.step_threshold(w2, g, r2, rows, leaders, thr_np, float(EPS), -0.01, off)
    assert np.array_equal(mask, mask2) and np.array_equal(counts, counts2) and np.array_equal(idx, idx2)
    assert np.array_equal(sm.view(np.uint32), sm2.view(np.uint32)) and np.array_equal(w1.view(np.uint32), w2.view(np.uint32))
    for a, b in zip(r1, r2):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert 0 < counts.sum() < sum(sizes)


def test_per_node_thresholds_in_threshold_step():
    """Each chosen node compares against its own threshold; the masks are then OR-ed."""
    rng = np.random.default_rng(10)
    n = 5000
    w = (rng.standard_normal(n) * 0.05).astype(np.float32)
    r = [(rng.standard_t(3, n) * 1e-3).astype(np.float32) for _ in range(3)]
    g = [np.zeros(n, np.float32)] * 3
    thr = np.array([[0.05, 0.2]], np.float32)
    leaders = np.array([[2, 0]], np.uint32)
    s2 = np.abs(r[2]) / (np.abs(w) + EPS)
    s0 = np.abs(r[0]) / (np.abs(w) + EPS)
    want = np.nonzero((s2 > thr[0, 0]) | (s0 > thr[0, 1]))[0]
    swapped = np.nonzero((s2 > thr[0, 1]) | (s0 > thr[0, 0]))[0]
    assert not np.array_equal(want, swapped)
    mask, counts, idx, sm = oracle.step_threshold(w.copy(), g, [x.copy() for x in r], [(0, n, 0, 0)], leaders, thr,
                                                  float(EPS), -0.01, n)
    assert np.array_equal(idx, want)
