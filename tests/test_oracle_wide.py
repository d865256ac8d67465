"""Pins of the 17..32-bit oracle (oracle/wide_oracle.py): on operands that fit the narrow oracle it must give what
that oracle (pinned elsewhere, int64 / C) gives; products at the corners of the 32-bit range against hand values;
the requantize rule against exact rationals; quantize to 32 bits against closed forms."""
from fractions import Fraction

import numpy as np

from oracle import conv_oracle as co
from oracle import fxp_oracle as orc
from oracle import wide_oracle as wo


def test_contractions_agree_with_the_narrow_oracle_on_narrow_operands():
    g = np.random.default_rng(1)
    a, b = g.integers(-2000, 2000, (7, 13)), g.integers(-2000, 2000, (13, 5))
    assert np.array_equal(wo.gemm(a, b).astype(np.int64), orc.gemm(a, b))
    assert np.array_equal(wo.gemm(a.T.copy(), b.T.copy(), True, True).astype(np.int64), orc.gemm(a, b))
    x, w = g.integers(-300, 300, (2, 7, 6, 5)), g.integers(-300, 300, (4, 3, 3, 5))
    for stride, pad in ((1, 1), (2, 1), (1, 0), (2, 0)):
        y = co.conv_fwd(x, w, stride, pad)
        assert np.array_equal(wo.conv_fwd(x, w, stride, pad).astype(np.int64), y)
        dy = g.integers(-300, 300, y.shape)
        assert np.array_equal(wo.conv_dgrad(dy, w, 7, 6, stride, pad).astype(np.int64), co.conv_dgrad(dy, w, 7, 6, stride, pad))
        assert np.array_equal(wo.conv_wgrad(dy, x, 3, 3, stride, pad).astype(np.int64), co.conv_wgrad(dy, x, 3, 3, stride, pad))


def test_corner_products_do_not_wrap():
    lo, hi = -(1 << 31), (1 << 31) - 1
    a = np.array([[lo, hi, lo]], dtype=np.int64)
    b = np.array([[lo], [hi], [hi]], dtype=np.int64)
    assert int(wo.gemm(a, b)[0, 0]) == (1 << 62) + ((1 << 31) - 1) ** 2 - (1 << 31) * ((1 << 31) - 1)
    a = np.array([[lo, lo, lo]], dtype=np.int64)
    assert int(wo.gemm(a, a.T.copy())[0, 0]) == 3 << 62                # beyond int64
    x = np.full((1, 3, 3, 2), hi, dtype=np.int64)
    w = np.full((1, 3, 3, 2), hi, dtype=np.int64)
    assert int(wo.conv_fwd(x, w, 1, 1)[0, 1, 1, 0]) == 18 * hi * hi


def test_requantize_matches_the_narrow_rule_and_exact_rationals():
    g = np.random.default_rng(2)
    acc = g.integers(-(1 << 40), 1 << 40, 500)
    for shift, wl in ((0, 32), (-3, 32), (5, 32), (16, 24), (17, 32), (30, 20), (40, 8)):
        for mode in (orc.SR, orc.RN_HALF_UP):
            got = wo.requantize(acc, shift, wl, mode, 3, 4, relu=(shift == 5))
            if wl <= 16 or True:
                want = orc.requantize(acc, shift, wl, mode, 3, 4, relu=(shift == 5)) if abs(shift) < 24 else None
                if want is not None:
                    assert np.array_equal(got, want), (shift, wl, mode)
    # a 100-bit accumulator: within one step of the exact quotient, saturating at 32 bits
    big = [(-1) ** i * ((1 << 99) // (i + 1)) for i in range(40)]
    q = wo.requantize(np.array(big, dtype=object), 70, 32, orc.SR, 1, 1)
    for v, c in zip(big, q):
        exact = Fraction(v, 1 << 70)
        assert abs(Fraction(int(c)) - max(min(exact, (1 << 31) - 1), -(1 << 31))) < 1
    assert int(q[0]) == (1 << 29) and int(q[1]) == -(1 << 28)          # 2^99 / 2^70 and -2^98 / 2^70 are exact


def test_quantize_to_thirty_two_bits():
    # values on the grid are reproduced exactly whatever the rounding bits; fp32 has 24 significant bits, so codes
    # of 2^24 and more are exact integers times a power of two
    codes = np.array([0, 1, -1, (1 << 23) + 1, -(1 << 23) - 1, 1 << 30, -(1 << 31), (1 << 31) - 128], dtype=np.int64)
    x = (codes.astype(np.float64) * 2.0 ** -20).astype(np.float32)
    q, nnz, sat = orc.quantize(x, 32, 20, orc.SR, 5, 6)
    assert np.array_equal(q, codes) and nnz == 7 and sat == 0
    # saturation at both ends, NaN -> 0, infinities saturate
    x = np.array([3000.0, -3000.0, 2048.0, -2048.0, np.nan, np.inf, -np.inf], dtype=np.float32)
    q, nnz, sat = orc.quantize(x, 32, 20, orc.SR, 5, 6)
    assert q.tolist() == [(1 << 31) - 1, -(1 << 31), (1 << 31) - 1, -(1 << 31), 0, (1 << 31) - 1, -(1 << 31)] and sat == 5
    # small values still round stochastically on the 2^-31 grid: mean of many draws is the value
    x = np.full(20000, 2.0 ** -32 * 0.75, dtype=np.float32)
    q, _, _ = orc.quantize(x, 32, 31, orc.SR, 1, 2)
    assert set(np.unique(q)) <= {0, 1} and abs(q.mean() - 0.375) < 0.02
    # 17 bits: the first word length that needs int32 storage
    x = (np.random.default_rng(3).standard_normal(1000) * 0.3).astype(np.float32)
    q, _, _ = orc.quantize(x, 17, 15, orc.RN_HALF_UP, 0, 0)
    assert np.array_equal(q, np.clip(np.floor(x.astype(np.float64) * 2 ** 15 + 0.5), -(1 << 16), (1 << 16) - 1).astype(np.int64))
