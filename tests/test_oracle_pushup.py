"""Pins for the oracle's PushUp quantities (CPU only).

Follows Sec. 3.3: "The PushUp Operation" (gradient-diversity equation, the suggestions s1, s2 and
their combination), "Dealing with Fixed-Points Limited Range" (buffer bits) and "Strategy,
Resolution and Lookback".  The paper prints no numbers for these, so the pins are closed forms
(identical, orthogonal and cancelling gradients), the triangle inequality, an independent fp64
evaluation on dequantized values, exact rational arithmetic on tiny inputs, and hand-evaluated
cases of the scalar rules.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import pushup_oracle as pu


def test_identical_gradients_have_diversity_one():
    g = np.array([3, -4, 0, 12, 5, -7], dtype=np.int64)
    for r in (1, 2, 4, 8):
        res = pu.gradient_diversity([g] * r, [5] * r)
        assert res["ds"] == pytest.approx(1.0, rel=1e-15)
        assert res["log_ds"] == pytest.approx(0.0, abs=1e-15)
        assert res["sumsq"] == [int(np.sum(g * g))] * r
        assert res["sumsq_sum"] == r * r * int(np.sum(g * g))


def test_orthogonal_gradients():
    # m one-hot gradients of equal magnitude at different positions: sum of norms m|v|, norm of the sum sqrt(m)|v|
    for m in (2, 4, 9):
        codes = []
        for k in range(m):
            c = np.zeros(16, dtype=np.int64)
            c[k] = -7 if k % 2 else 7
            codes.append(c)
        res = pu.gradient_diversity(codes, [3] * m)
        assert res["ds"] == pytest.approx(math.sqrt(m), rel=1e-15)
        assert res["log_ds"] == pytest.approx(0.5 * math.log(m), rel=1e-14)


def test_cancelling_and_zero_gradients_are_the_otherwise_case():
    g = np.array([1, -2, 3], dtype=np.int64)
    res = pu.gradient_diversity([g, -g], [4, 4])
    assert res["den"] == 0.0 and math.isinf(res["ds"]) and res["log_ds"] == 1.0
    z = np.zeros(5, dtype=np.int64)
    res = pu.gradient_diversity([z, z, z], [4, 4, 4])
    assert math.isnan(res["ds"]) and res["log_ds"] == 1.0


def test_formats_are_aligned_by_value():
    # the same real-valued gradient written on two grids: c * 2^-4 == (4c) * 2^-6
    g = np.array([5, -3, 2, 0, 7], dtype=np.int64)
    res = pu.gradient_diversity([g, 4 * g, g], [4, 6, 4])
    assert res["fl_max"] == 6
    assert res["ds"] == pytest.approx(1.0, rel=1e-15)
    assert res["sumsq_sum"] == int(np.sum((12 * g) ** 2))


def test_matches_fp64_norms_of_dequantized_values_and_exact_rationals():
    rng = np.random.default_rng(11)
    for trial in range(20):
        count = int(rng.integers(1, 7))
        n = int(rng.integers(1, 40))
        fls = [int(f) for f in rng.integers(0, 9, count)]
        codes = [rng.integers(-128, 128, n) for _ in range(count)]
        res = pu.gradient_diversity(codes, fls)
        vals = [c.astype(np.float64) * 2.0 ** -f for c, f in zip(codes, fls)]
        num = sum(np.linalg.norm(v) for v in vals)
        den = np.linalg.norm(np.sum(vals, axis=0))
        if den > 0:
            assert res["ds"] == pytest.approx(num / den, rel=1e-12)
            assert res["ds"] >= 1.0 - 1e-12                    # triangle inequality
        # squared quantities exactly, with rationals
        tot = [sum(Fraction(int(c[i]), 1 << f) for c, f in zip(codes, fls)) for i in range(n)]
        assert Fraction(res["sumsq_sum"], 1 << (2 * res["fl_max"])) == sum(t * t for t in tot)
        for q, c in zip(res["sumsq"], codes):
            assert q == sum(int(v) ** 2 for v in c)
        alt = pu.gradient_diversity_np(codes, fls)
        assert alt["sumsq"] == res["sumsq"] and alt["sumsq_sum"] == res["sumsq_sum"] and alt["ds"] == res["ds"] \
            or (math.isnan(alt["ds"]) and math.isnan(res["ds"]))


def test_large_values_do_not_overflow():
    # 64 tensors of int16 extremes on grids 0..4: the aligned sum reaches 64 * 2^15 * 2^4 < 2^31 hmm = 2^25
    codes = [np.full(1000, -32768, dtype=np.int64) for _ in range(64)]
    fls = [k % 5 for k in range(64)]
    res = pu.gradient_diversity_np(codes, fls)
    per_elem = sum(-32768 << (4 - f) for f in fls)
    assert res["sumsq_sum"] == 1000 * per_elem * per_elem
    assert res["sumsq"] == [1000 * 32768 * 32768] * 64


# ---- scalar rules, evaluated by hand ------------------------------------------------------------

def test_suggestions_by_hand():
    e = math.e
    # L = 2: s1 = ceil(1/(2-1)) = 1; s2 = min(32*4-1, 32) - 5 = 27
    assert pu.pushup_suggest(e ** 2, 6, 5, pu.ST_MIN, 0)[2:] == (1, 27, 1)
    assert pu.pushup_suggest(e ** 2, 6, 5, pu.ST_MEAN, 0)[2:] == (1, 27, 14)
    assert pu.pushup_suggest(e ** 2, 6, 5, pu.ST_MAX, 0)[2:] == (1, 27, 27)
    # new lengths: FL = min(5 + s, 32), WL = min(max(6, 5) + 1, 32) = 7; the range rule with buff = 0 then
    # lifts WL to at least FL: WL = max(min(FL + 0, 32), 7)
    assert pu.pushup_suggest(e ** 2, 6, 5, pu.ST_MIN, 0)[:2] == (7, 6)
    assert pu.pushup_suggest(e ** 2, 6, 5, pu.ST_MEAN, 0)[:2] == (19, 19)
    assert pu.pushup_suggest(e ** 2, 6, 5, pu.ST_MAX, 0)[:2] == (32, 32)
    # L = 1.5: s1 = ceil(1/0.5) = 2; s2 = min(71, 32) - 3 = 29
    assert pu.pushup_suggest(e ** 1.5, 8, 3, pu.ST_MIN, 0)[2:] == (2, 29, 2)
    # L = 0.5: 1/(L-1) = -2 -> s1 = 1; s2 = max(32*0.25 - 1 - 3, 1) = 4
    assert pu.pushup_suggest(e ** 0.5, 8, 3, pu.ST_MAX, 0)[2:] == (1, 4, 4)
    # L = 0 (ds = 1, all gradients parallel) is not > 0: s = 1
    assert pu.pushup_suggest(1.0, 8, 3, pu.ST_MAX, 0) == (9, 4, 1, 1, 1)
    # the otherwise case (ds not finite or not positive) has L = 1: s1 at its cap
    assert pu.pushup_suggest(math.inf, 8, 3, pu.ST_MIN, 0)[2:] == (32, 28, 28)
    assert pu.pushup_suggest(math.nan, 8, 3, pu.ST_MIN, 0)[2:] == (32, 28, 28)


def test_buffer_bits_and_caps():
    # FL = min(5 + 27, 32) = 32 -> min(32, 32 - 4) = 28; WL = max(min(28 + 4, 32), 7) = 32
    assert pu.pushup_suggest(math.e ** 2, 6, 5, pu.ST_MAX, 4)[:2] == (32, 28)
    # a 16-bit cap: s2 = min(27, 16) = 16, FL = min(5 + 16, 16) = 16 -> 16 - 2 = 14, WL = max(min(16, 16), 7) = 16
    assert pu.pushup_suggest(math.e ** 2, 6, 5, pu.ST_MAX, 2, wl_cap=16) == (16, 14, 1, 16, 16)
    # small suggestion, buffer widens the word only: FL = 4, WL = max(min(4 + 3, 32), 9) = 9
    assert pu.pushup_suggest(1.0, 8, 3, pu.ST_MIN, 3)[:2] == (9, 4)


def test_strategy_lookback_resolution_by_hand():
    assert pu.adapt_strategy(pu.ST_MIN, 1.0, 1.5) == pu.ST_MEAN       # no progress: escalate
    assert pu.adapt_strategy(pu.ST_MEAN, 1.0, 1.0) == pu.ST_MAX
    assert pu.adapt_strategy(pu.ST_MAX, 1.0, 2.0) == pu.ST_MAX
    assert pu.adapt_strategy(pu.ST_MAX, 2.0, 1.0) == pu.ST_MIN        # progress: back to min
    # lb_new = clamp(ceil(100 / 4), 25, 100) = 25; lb = ceil(25 * 0.5 + 0.5 * 60) = 43
    assert pu.adapt_lookback(60, 4.0, 25, 100, 0.5) == 43
    # ds = 1.2: ceil(83.33) = 84; lb = ceil(84 * 0.25 + 0.75 * 50) = ceil(58.5) = 59
    assert pu.adapt_lookback(50, 1.2, 25, 100, 0.25) == 59
    # not finite: lb_new = lb_upr
    assert pu.adapt_lookback(50, math.inf, 25, 100, 1.0) == 100
    assert pu.adapt_lookback(50, math.nan, 25, 100, 0.0) == 50
    assert pu.adapt_resolution(50, 100, 25, 100, 20, 60) == 51
    assert pu.adapt_resolution(60, 100, 25, 100, 20, 60) == 60
    assert pu.adapt_resolution(50, 25, 25, 100, 20, 60) == 49
    assert pu.adapt_resolution(20, 25, 25, 100, 20, 60) == 20
    assert pu.adapt_resolution(50, 40, 25, 100, 20, 60) == 50
