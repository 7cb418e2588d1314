"""Pins for the oracle's momentum-weighted residual (Eq. 3: the residual is accumulated
locally with momentum, r <- m * r + g).  CPU only: exact rational arithmetic with two
roundings, a case that tells a fused multiply-add apart, closed forms (geometric
series, the coefficient pattern of Eq. 2), m = 1 against plain accumulation, and the
whole steps against accumulation done by hand."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from test_oracle_pins import _round_to_f32

EPS = np.float32(1e-8)


def bits(x):
    return np.ascontiguousarray(x, np.float32).view(np.uint32)


def test_hand_values():
    r = np.array([2.0, -4.0, 0.0, -0.0, 3.0], np.float32)
    g = np.array([1.0, 1.0, 0.5, -0.0, -1.5], np.float32)
    oracle.accumulate_momentum(r, g, 0.5)
    assert r.tolist() == [2.0, -1.0, 0.5, 0.0, 0.0]
    assert np.signbit(r[3]) and not np.signbit(r[4])           # (0.5 * -0) + -0 = -0 ; 1.5 - 1.5 = +0


def test_two_roundings_exact():
    rng = np.random.default_rng(2)
    n = 400
    r = (rng.standard_t(3, n) * 1e-3).astype(np.float32)
    g = (rng.standard_t(3, n) * 1e-3).astype(np.float32)
    r[:8] = np.array([1e-38, -1e-38, 1e-45, 3e38, -3e38, 1.0, 0.0, -0.0], np.float32)
    for m in (0.9, 0.5, 0.99, 1.0, 0.0, 1e-3):
        m32 = np.float32(m)
        out = r.copy()
        oracle.accumulate_momentum(out, g, float(m32))
        for i in range(n):
            prod = _round_to_f32(Fraction(float(m32)) * Fraction(float(r[i])))
            want = _round_to_f32(Fraction(float(prod)) + Fraction(float(g[i])))
            assert bits(out[i]) == bits(want) or (out[i] == 0 and want == 0), (m, i, r[i], g[i], out[i], want)


def test_not_a_fused_multiply_add():
    """m * r = 1 + 2^-11 + 2^-24 rounds to 1 + 2^-11 (tie to even); adding -(1 + 2^-11)
    gives 0 with two roundings, 2^-24 with a fused multiply-add."""
    m = np.float32(1 + 2.0 ** -12)
    r = np.array([1 + 2.0 ** -12], np.float32)
    g = np.array([-(1 + 2.0 ** -11)], np.float32)
    assert Fraction(float(m)) * Fraction(float(r[0])) + Fraction(float(g[0])) == Fraction(1, 2 ** 24)
    oracle.accumulate_momentum(r, g, float(m))
    assert r[0] == 0.0


def test_momentum_one_is_plain_accumulation():
    rng = np.random.default_rng(3)
    pat = rng.integers(0, 2 ** 32, 200_000, dtype=np.uint64).astype(np.uint32)
    r = pat.view(np.float32).copy()
    g = rng.integers(0, 2 ** 32, 200_000, dtype=np.uint64).astype(np.uint32).view(np.float32).copy()
    ok = np.isfinite(r) & np.isfinite(g)
    r, g = r[ok].copy(), g[ok].copy()
    a, b = r.copy(), r.copy()
    with np.errstate(all="ignore"):
        oracle.accumulate(a, g)
        oracle.accumulate_momentum(b, g, 1.0)
    same = (bits(a) == bits(b)) | (np.isnan(a) & np.isnan(b))
    assert same.all()


def test_geometric_series_and_eq2_coefficients():
    # constant gradient 1, m = 1/2, r_0 = 0: r_t = 2 - 2^(1-t), exact in binary32 for t <= 24
    r = np.zeros(3, np.float32)
    g = np.ones(3, np.float32)
    for t in range(1, 25):
        oracle.accumulate_momentum(r, g, 0.5)
        assert np.all(r == np.float32(2 - 2.0 ** (1 - t)))
    # without sending, after T steps the residual is sum_tau m^tau g_{T - tau} (Eq. 2's coefficients)
    rng = np.random.default_rng(4)
    T, n, m = 30, 1000, np.float32(0.9)
    gs = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(T)]
    r = np.zeros(n, np.float32)
    for g in gs:
        oracle.accumulate_momentum(r, g, float(m))
    want = sum(float(m) ** (T - 1 - t) * gs[t].astype(np.float64) for t in range(T))
    assert np.allclose(r, want, rtol=1e-5, atol=1e-9)


@pytest.mark.parametrize("mode", ["topk", "threshold", "random", "layerwise"])
def test_whole_steps_use_momentum_accumulation(mode):
    """Every whole-step function with momentum m equals: M1 by hand on every accumulating
    worker and layer (nothing between the layers), then the same step with accumulation
    switched off."""
    rng = np.random.default_rng(5)
    sizes = [50, 4097, 1000]
    rows, off, out = [], 2, 0
    for n in sizes:
        k = max(1, n // 20)
        rows.append((off, n, k, out))
        off += n + 7
        out += k
    W, m = 3, 0.9
    w = (rng.standard_normal(off) * 0.05).astype(np.float32)
    g = [(rng.standard_t(3, off) * 1e-3).astype(np.float32) for _ in range(W)]
    r = [(rng.standard_t(3, off) * 1e-3).astype(np.float32) for _ in range(W)]
    accumulate = [1, 0, 1]
    hand = [x.copy() for x in r]
    for p in range(W):
        if accumulate[p]:
            for (o, n, _, _) in rows:
                seg = hand[p][o:o + n].copy()
                oracle.accumulate_momentum(seg, np.ascontiguousarray(g[p][o:o + n]), m)
                hand[p][o:o + n] = seg
    assert not np.array_equal(hand[0], r[0] + g[0])            # m = 0.9 differs from plain accumulation
    leaders = rng.integers(0, W, (3, 2)).astype(np.uint32)
    thr = np.array([0.05, 0.03, 0.08], np.float32)

    def run(res, acc_mask, mom):
        ww = w.copy()
        if mode == "topk":
            o = oracle.step(ww, g, res, rows, leaders[:, 0], float(EPS), -0.01, acc_mask, momentum=mom)
        elif mode == "threshold":
            o = oracle.step_threshold(ww, g, res, rows, leaders, thr, float(EPS), -0.01, off, acc_mask, momentum=mom)
        elif mode == "random":
            o = oracle.step_threshold(ww, g, res, rows, leaders, thr, float(EPS), -0.01, off, acc_mask, random=(5, 6),
                                      momentum=mom)
        else:
            o = oracle.step_layerwise(ww, g, res, rows, leaders, 0.05, 1e-4, 10.0, float(EPS), -0.01, off, acc_mask,
                                      momentum=mom)
        return o, ww

    r1 = [x.copy() for x in r]
    o1, w1 = run(r1, accumulate, m)
    r2 = [x.copy() for x in hand]
    o2, w2 = run(r2, [0, 0, 0], 1.0)
    for a, b in zip(o1, o2):
        assert np.array_equal(np.asarray(a), np.asarray(b), equal_nan=True)
    assert np.array_equal(bits(w1), bits(w2))
    for a, b in zip(r1, r2):
        assert np.array_equal(bits(a), bits(b))
