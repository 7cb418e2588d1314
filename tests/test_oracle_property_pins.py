"""Property-based pins of the oracle (hypothesis): small adversarial layers -- ties,
zeros, signed zeros, denormals, infinities, k anywhere in [1, n] -- against the plain
definitions written with numpy's sort / comparison routines and exact rationals."""
from fractions import Fraction

import numpy as np
from hypothesis import given, settings, strategies as st

import oracle

EPS = np.float32(1e-8)
PALETTE = np.array([0.0, -0.0, 1.0, -1.0, 0.5, 2.0, 1e-3, -1e-3, 1e-45, -1e-45, 3e38, -3e38, 0.25, 7.0, 1e-20],
                   np.float32)
small_f32 = st.one_of(st.sampled_from(PALETTE.tolist()),
                      st.floats(min_value=-10, max_value=10, width=32, allow_nan=False))


@st.composite
def layers(draw, max_n=40):
    n = draw(st.integers(1, max_n))
    w = np.array(draw(st.lists(small_f32, min_size=n, max_size=n)), np.float32)
    r = np.array(draw(st.lists(small_f32, min_size=n, max_size=n)), np.float32)
    return w, r


@settings(max_examples=300, deadline=None, derandomize=True)
@given(layers(), st.data())
def test_select_is_the_sorted_prefix(layer, data):
    """O3/O4: the k first under (score descending, index ascending), returned ascending."""
    w, r = layer
    n = r.size
    k = data.draw(st.integers(1, n))
    with np.errstate(all="ignore"):
        s = oracle.score(w, r, float(EPS))
        want_s = (np.abs(r) / (np.abs(w) + EPS)).astype(np.float32)
    assert np.array_equal(s.view(np.uint32), want_s.view(np.uint32))
    order = np.lexsort((np.arange(n), -s.astype(np.float64)))          # stable: score desc, then index asc
    want = np.sort(order[:k]).astype(np.uint32)
    idx, thr = oracle.select(s, k)
    assert np.array_equal(idx, want)
    key, n_gt, n_eq = thr
    kth = s[order[k - 1]]
    assert key == int(np.float32(kth).view(np.uint32)) & 0x7FFFFFFF
    assert n_gt == int((s > kth).sum()) and n_eq == k - n_gt and 1 <= n_eq <= int((s == kth).sum())
    for i in range(n):                                                   # rank by counting, element by element
        rank = int((s > s[i]).sum() + (s[:i] == s[i]).sum())
        assert oracle.rank_of(s, i) == rank and (rank < k) == bool(i in set(want.tolist()))


@settings(max_examples=200, deadline=None, derandomize=True)
@given(layers(), st.sampled_from([0.0, 0.005, 0.5, 1.0, 1e-30, 3e38, float("inf")]))
def test_threshold_mask_is_the_strict_comparison(layer, thr):
    w, r = layer
    n = r.size
    with np.errstate(all="ignore"):
        s = (np.abs(r) / (np.abs(w) + EPS)).astype(np.float32)
    want = s > np.float32(thr)
    mask = oracle.mask_threshold(w, r, float(EPS), thr)
    assert mask.size == oracle.mask_bytes(n) == 4 * ((n + 31) // 32)
    assert np.array_equal(np.unpackbits(mask, bitorder="little")[:n].astype(bool), want)
    assert not np.unpackbits(mask, bitorder="little")[n:].any()
    assert np.array_equal(oracle.mask_indices(mask, n), np.nonzero(want)[0].astype(np.uint32))


@settings(max_examples=150, deadline=None, derandomize=True)
@given(st.lists(st.floats(min_value=0, max_value=100, width=32), min_size=1, max_size=30))
def test_layer_statistics_are_exact_rationals_rounded(scores):
    """L1 with |w| + eps = 1 (score = |r|): mean and population variance against exact arithmetic."""
    r = np.array(scores, np.float32)
    w = np.ones(r.size, np.float32)                                      # 1 + 1e-8 rounds to 1 in binary32
    fs = [Fraction(float(x)) for x in r]
    mean = sum(fs) / len(fs)
    var = sum((x - mean) ** 2 for x in fs) / len(fs)
    m, v = oracle.layer_stats(w, r, float(EPS))
    assert abs(Fraction(m) - mean) <= abs(mean) * Fraction(1, 10 ** 14)
    assert abs(Fraction(v) - var) <= var * Fraction(1, 10 ** 12) + Fraction(1, 10 ** 40)


@settings(max_examples=150, deadline=None, derandomize=True)
@given(layers(max_n=24), st.sampled_from([1.0, 0.5, 0.9, 0.0]),
       st.lists(small_f32, min_size=24, max_size=24))
def test_conservation_through_a_step(layer, m, gs):
    """One worker, one layer: what is sent plus what stays equals the accumulated value, exactly."""
    w, r = layer
    n = r.size
    g = np.array(gs[:n], np.float32)
    ok = np.isfinite(r) & np.isfinite(g) & (np.abs(r) < 1e30) & (np.abs(g) < 1e30)
    r, g, w = r[ok].copy(), g[ok].copy(), w[ok].copy()
    n = r.size
    if n == 0:
        return
    k = max(1, n // 3)
    acc = r.copy()
    oracle.accumulate_momentum(acc, g, m)
    r1, w1 = r.copy(), w.copy()
    idx, val, sm, _ = oracle.step(w1, [g], [r1], [(0, n, k, 0)], np.zeros(1, np.uint32), float(EPS), -0.5, momentum=m)
    assert idx.size == k and np.array_equal(val.view(np.uint32), acc[idx].view(np.uint32))
    assert np.array_equal(sm.view(np.uint32), val.view(np.uint32))
    kept = acc.copy()
    kept[idx] = 0.0
    assert np.array_equal(r1.view(np.uint32), kept.view(np.uint32))
    rest = np.ones(n, bool)
    rest[idx] = False
    assert np.array_equal(w1[rest].view(np.uint32), w[rest].view(np.uint32))
    with np.errstate(all="ignore"):
        assert np.array_equal(w1[idx].view(np.uint32), (w[idx] + np.float32(-0.5) * val).astype(np.float32).view(np.uint32))
