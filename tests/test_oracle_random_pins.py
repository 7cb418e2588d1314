"""Pins for the oracle's random gradient selection (Section 3.3, P(update) =
importance / threshold) and the counter-based generator behind it.  CPU only:
published known-answer vectors of the generator, a hand-worked example built on
them, exactness of the uniform mapping, frequency = probability, independence across
positions / layers / steps / seeds, and the relation to the plain threshold mask."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
EPS = np.float32(1e-8)


def _unpack(mask, n):
    return np.unpackbits(mask, bitorder="little")[:n].astype(bool)


def test_generator_known_answers():
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(t, 16) for t in line.split()]
        assert oracle.philox4x32_10(v[0:4], v[4:6]).tolist() == v[6:10]


def _hand():
    d = {}
    for line in open(os.path.join(GOLDEN, "hand_example_random.txt")):
        if line.startswith("#") or not line.strip():
            continue
        t = line.split()
        d[t[0]] = t[1:]
    return d


def test_hand_worked_example():
    d = _hand()
    for i, tok in enumerate(d["u24"]):
        assert oracle.uniform(0, 0, 0, i) == np.float32(int(tok, 0) / 2 ** 24)
    w = np.ones(4, np.float32)
    for case in "ABC":
        r = np.array([float(t) for t in d["case%s_r" % case]], np.float32)
        thr = float(d["case%s_thr" % case][0])
        m = oracle.mask_threshold_random(w, r, 0.0, thr, 0, 0, 0)
        assert m.tolist() == [int(d["case%s_mask" % case][0], 0), 0, 0, 0], case
    # through the whole step: one worker, one layer, step 0, seed 0
    r = np.array([float(t) for t in d["caseB_r"]], np.float32)
    w2 = w.copy()
    mask, counts, idx, sm = oracle.step_threshold(w2, [np.zeros(4, np.float32)], [r], [(0, 4, 0, 0)],
                                                  np.array([[0]], np.uint32), np.array([1.0], np.float32), 0.0, -1.0, 4,
                                                  random=(0, 0))
    assert idx.tolist() == [1, 2, 3] and np.array_equal(sm, np.array([0.9, 2.0, 0.61], np.float32))
    assert r.tolist() == [-0.25, 0.0, 0.0, 0.0]


def test_boundary_draw_equal_to_probability_is_not_sent():
    """P(update) = importance / threshold (Section 3.3): the element is sent iff u < p, strictly.  With
    |w| = 1, eps = 0, thr = 1 and |r| set to the draws themselves, p == u bit for bit and nothing is sent;
    one unit of the 24-bit grid above the draw is sent.  An element of importance 0 is never sent, not
    even where the draw is exactly 0."""
    d = _hand()
    r = np.array([int(t, 0) / 2 ** 24 for t in d["caseD_r24"]], np.float32)
    r[1] = -r[1]
    for i in range(2):
        assert np.float32(abs(r[i])) == oracle.uniform(0, 0, 0, i)          # p == u exactly
    m = oracle.mask_threshold_random(np.ones(4, np.float32), r, 0.0, float(d["caseD_thr"][0]), 0, 0, 0)
    assert m.tolist() == [int(d["caseD_mask"][0], 0), 0, 0, 0]
    # the same boundary with thr = 0.5 and |r| = u / 2 (the divide is exact)
    m = oracle.mask_threshold_random(np.ones(4, np.float32), r * np.float32(0.5), 0.0, 0.5, 0, 0, 0)
    assert m.tolist() == [int(d["caseD_mask"][0], 0), 0, 0, 0]
    # a draw of exactly zero against a probability of exactly zero
    layer, e = int(d["zero_draw_layer"][0]), int(d["zero_draw_elem"][0])
    ctr = [e // 4, layer, 0, 0]
    assert int(oracle.philox4x32_10(ctr, [0, 0])[e % 4]) == int(d["zero_draw_word"][0], 0)
    assert oracle.uniform(0, 0, layer, e) == 0.0
    n = e + 2
    rz = np.zeros(n, np.float32)
    rz[e + 1] = 1e-30                          # the neighbour has a tiny positive probability and a non-zero draw
    mz = _unpack(oracle.mask_threshold_random(np.ones(n, np.float32), rz, 0.0, 1.0, 0, 0, layer), n)
    assert not mz.any()
    rz[e] = 1e-30                              # any positive probability beats a draw of 0
    mz = _unpack(oracle.mask_threshold_random(np.ones(n, np.float32), rz, 0.0, 1.0, 0, 0, layer), n)
    assert np.nonzero(mz)[0].tolist() == [e]


def test_uniform_mapping_and_counter_layout():
    """u = (word >> 8) * 2^-24 of output word i % 4 of the block with counter
    (i / 4, layer, step low, step high) and key (seed low, seed high)."""
    rng = np.random.default_rng(1)
    for _ in range(50):
        seed = int(rng.integers(0, 2 ** 63)) * 2 + int(rng.integers(0, 2))
        step = int(rng.integers(0, 2 ** 63)) * 2 + int(rng.integers(0, 2))
        layer = int(rng.integers(0, 2 ** 32))
        i = int(rng.integers(0, 2 ** 32))
        blk = oracle.philox4x32_10([i >> 2, layer, step & 0xFFFFFFFF, step >> 32], [seed & 0xFFFFFFFF, seed >> 32])
        u = oracle.uniform(seed, step, layer, i)
        assert u == np.float32((int(blk[i & 3]) >> 8) / 2 ** 24)
        assert 0.0 <= u < 1.0 and float(u) * 2 ** 24 == int(float(u) * 2 ** 24)


def _draws(seed, step, layer, n):
    return np.array([oracle.uniform(seed, step, layer, i) for i in range(n)], np.float64)


def test_uniform_statistics():
    n = 40_000
    u = _draws(12345, 7, 3, n)
    assert abs(u.mean() - 0.5) < 4 * np.sqrt(1 / 12 / n)
    hist = np.histogram(u, bins=20, range=(0, 1))[0]
    chi2 = ((hist - n / 20) ** 2 / (n / 20)).sum()
    assert chi2 < 50                                          # 19 degrees of freedom: 99.99 % point is ~ 49
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.03       # neighbours (same and different blocks)
    assert abs(np.corrcoef(u[:-4], u[4:])[0, 1]) < 0.03
    for other in (_draws(12345, 8, 3, n), _draws(12345, 7, 4, n), _draws(12346, 7, 3, n), _draws(12345, 7 + 2 ** 32, 3, n),
                  _draws(12345 + 2 ** 32, 7, 3, n)):
        assert not np.array_equal(u, other)
        assert abs(np.corrcoef(u, other)[0, 1]) < 0.03


def test_selection_frequency_is_importance_over_threshold():
    """P(update) = importance / threshold for elements not above the threshold; always
    sent above it; never sent at zero importance."""
    n = 4096
    w = np.ones(n, np.float32)
    levels = np.array([0.0, 0.1, 0.25, 0.5, 0.9, 1.0, 1.5], np.float32)       # importance / threshold
    thr = np.float32(0.02)
    r = (np.tile(levels, n // len(levels) + 1)[:n] * thr).astype(np.float32)
    r[::2] *= -1
    lvl = (np.abs(r) / thr)
    steps = 300
    hits = np.zeros(n)
    for t in range(steps):
        hits += _unpack(oracle.mask_threshold_random(w, r, float(EPS), float(thr), 99, t, 5), n)
    for p in levels:
        sel = np.isclose(lvl, p)
        freq = hits[sel].sum() / (sel.sum() * steps)
        if p == 0.0:
            assert freq == 0.0
        elif p > 1.0:
            assert freq == 1.0
        else:
            sd = np.sqrt(max(p * (1 - p), 1e-9) / (sel.sum() * steps))
            assert abs(freq - min(p, 1.0)) < 5 * sd + 1e-12, (p, freq)


def test_superset_of_threshold_mask_and_limits():
    rng = np.random.default_rng(4)
    n = 10_000
    w = (rng.standard_normal(n) * 0.05).astype(np.float32)
    r = (rng.standard_t(3, n) * 1e-3).astype(np.float32)
    for thr in (0.005, 0.05, 0.1):
        plain = _unpack(oracle.mask_threshold(w, r, float(EPS), thr), n)
        rnd = _unpack(oracle.mask_threshold_random(w, r, float(EPS), thr, 1, 2, 3), n)
        assert np.all(rnd[plain]) and rnd.sum() > plain.sum()
        # the extra elements are exactly those whose draw is below importance / threshold
        s = oracle.score(w, r, float(EPS))
        u = np.array([oracle.uniform(1, 2, 3, i) for i in range(n)], np.float32)
        assert np.array_equal(rnd, (s > np.float32(thr)) | (u < s / np.float32(thr)))
    # an infinite threshold: probability 0; threshold 0: only the plain rule (0/0 is no probability)
    assert not oracle.mask_threshold_random(w, r, float(EPS), float("inf"), 1, 2, 3).any()
    z = r.copy()
    z[::3] = 0.0
    assert np.array_equal(_unpack(oracle.mask_threshold_random(w, z, float(EPS), 0.0, 1, 2, 3), n), z != 0)


def test_step_with_random_selection_matches_dense_formulation():
    rng = np.random.default_rng(6)
    sizes = [37, 5000, 4096]
    rows, off = [], 0
    for n in sizes:
        rows.append((off, n, 0, 0))
        off += n + 3
    W = 3
    w = (rng.standard_normal(off) * 0.05).astype(np.float32)
    g = [(rng.standard_t(3, off) * 1e-3).astype(np.float32) for _ in range(W)]
    r = [(rng.standard_t(3, off) * 1e-3).astype(np.float32) for _ in range(W)]
    for x in g:                                               # nothing accumulates between the layers
        for (o, n, _, _) in rows:
            x[o + n:o + n + 3] = 0.0
    leaders = np.array([[0, 2], [1, 1], [2, 0]], np.uint32)
    thr = np.array([0.05, 0.02, 0.1], np.float32)
    seed, step = 2 ** 40 + 17, 2 ** 33 + 5
    w1, r1 = w.copy(), [x.copy() for x in r]
    mask, counts, idx, sm = oracle.step_threshold(w1, g, r1, rows, leaders, thr, float(EPS), -0.01, off,
                                                  random=(seed, step))
    acc = [a + b for a, b in zip(r, g)]
    want_idx = []
    for j, (o, n, _, _) in enumerate(rows):
        u = np.array([oracle.uniform(seed, step, j, i) for i in range(n)], np.float32)
        m = np.zeros(n, bool)
        for q in range(2):
            a = acc[leaders[j, q]][o:o + n]
            s = np.abs(a) / (np.abs(w[o:o + n]) + EPS)
            m |= (s > thr[j]) | (u < s / thr[j])
        want_idx.append(o + np.nonzero(m)[0])
        assert counts[j] == m.sum()
    want_idx = np.concatenate(want_idx)
    assert np.array_equal(idx, want_idx)
    dense = (acc[0][idx] + acc[1][idx]) + acc[2][idx]
    assert np.array_equal(sm.view(np.uint32), dense.astype(np.float32).view(np.uint32))
    w_want = w.copy()
    w_want[idx] = w[idx] + np.float32(-0.01) * dense
    assert np.array_equal(w1.view(np.uint32), w_want.view(np.uint32))
    for p in range(W):
        keep = acc[p].copy()
        keep[idx] = 0.0
        assert np.array_equal(r1[p].view(np.uint32), keep.view(np.uint32))
