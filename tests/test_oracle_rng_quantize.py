"""Pins for the oracle's random bits and quantizer (CPU only).

The quantizer follows Sec. 3.2 (SR equation) on the <WL,FL> format of Sec. 2.1.  The paper
prints no worked numbers, so the pins are closed forms, invariants and exhaustive
enumeration of the rounding bits.
"""
import math

import numpy as np
import pytest

from oracle import fxp_oracle as orc


# ---------------------------------------------------------------- random bits

def test_r16_uniform_bytes():
    r = orc.r16(7, 3, np.arange(1 << 20))
    assert r.min() >= 0 and r.max() < 65536
    for byte in (r & 0xFF, r >> 8):
        cnt = np.bincount(byte, minlength=256)
        exp = r.size / 256
        chi2 = ((cnt - exp) ** 2 / exp).sum()
        # 255 dof: mean 255, sd 22.6 -> 6 sd
        assert chi2 < 255 + 6 * 22.6


def test_r16_adjacent_lanes_independent():
    r = orc.r16(1, 0, np.arange(1 << 20)).reshape(-1, 8)
    for a in range(7):
        pair = (r[:, a] >> 12) * 16 + (r[:, a + 1] >> 12)
        cnt = np.bincount(pair, minlength=256)
        exp = pair.size / 256
        chi2 = ((cnt - exp) ** 2 / exp).sum()
        assert chi2 < 255 + 6 * 22.6
        c = np.corrcoef(r[:, a], r[:, a + 1])[0, 1]
        assert abs(c) < 6 / math.sqrt(r.shape[0])


def test_philox_is_injective_on_counters_and_depends_on_every_input():
    n = 1 << 16
    j = np.arange(n, dtype=np.uint64)
    z = np.zeros(n, dtype=np.uint64)
    base = np.stack(orc.philox4x32_10((5, 9), (j, z, z, z)), axis=-1)
    assert len({tuple(row) for row in base.tolist()}) == n
    for key, ctr in (((6, 9), (j, z, z, z)), ((5, 10), (j, z, z, z)),
                     ((5, 9), (j, z + np.uint64(1), z, z)), ((5, 9), (j, z, z + np.uint64(1), z)),
                     ((5, 9), (j, z, z, z + np.uint64(1)))):
        other = np.stack(orc.philox4x32_10(key, ctr), axis=-1)
        # every output word changes for (almost) every counter
        assert (other != base).mean() > 0.999


def test_philox_avalanche():
    n = 4096
    j = np.arange(n, dtype=np.uint64) * np.uint64(977)
    z = np.zeros(n, dtype=np.uint64)
    a = np.stack(orc.philox4x32_10((1, 2), (j, z, z, z)), axis=-1)
    for bit in (0, 7, 19, 31):
        b = np.stack(orc.philox4x32_10((1, 2), (j ^ np.uint64(1 << bit), z, z, z)), axis=-1)
        flips = np.array([bin(int(v)).count("1") for v in (a ^ b).ravel()]).reshape(n, 4).sum(1)
        assert abs(flips.mean() - 64) < 1.0          # sd of the mean = 5.66/64 = 0.09


def test_streams_and_seeds_differ():
    i = np.arange(4096)
    a = orc.r16(0, 0, i)
    assert (orc.r16(0, 1, i) != a).mean() > 0.99
    assert (orc.r16(1, 0, i) != a).mean() > 0.99
    assert (orc.r16(1 << 32, 0, i) != a).mean() > 0.99
    assert (orc.r16(0, 1 << 32, i) != a).mean() > 0.99
    assert np.array_equal(orc.r16(0, 0, i), a)


def test_r16_lane_layout():
    # 8 consecutive elements share one block; lanes are the 16-bit halves, low half first
    key = (3, 0)
    words = orc.philox4x32_10(key, (np.array([5], dtype=np.uint64), np.array([0], dtype=np.uint64),
                                    np.array([2], dtype=np.uint64), np.array([0], dtype=np.uint64)))
    words = [int(w[0]) for w in words]
    expect = []
    for w in words:
        expect += [w & 0xFFFF, w >> 16]
    assert orc.r16(3, 2, np.arange(40, 48)).tolist() == expect


# ---------------------------------------------------------------- quantizer

FORMATS = [(2, 0), (4, 2), (8, 4), (8, 6), (8, 5), (12, 9), (16, 13), (16, 0), (8, 12), (3, 31)]


@pytest.mark.parametrize("wl,fl", FORMATS)
def test_range_and_neighbours(wl, fl):
    g = np.random.default_rng(wl * 100 + fl)
    x = (g.standard_normal(20000) * 2.0 ** (wl - 1 - fl) * 0.7).astype(np.float32)
    q, nnz, sat = orc.quantize(x, wl, fl, orc.SR, seed=11, stream=4)
    qmin, qmax = -(1 << (wl - 1)), (1 << (wl - 1)) - 1
    assert q.min() >= qmin and q.max() <= qmax
    y = x.astype(np.float64) * 2.0 ** fl
    inside = (y >= qmin) & (y <= qmax)
    fl_y = np.floor(y)
    ok = (q == fl_y) | (q == fl_y + 1)
    assert ok[inside].all()
    assert (np.abs(q[inside] * 2.0 ** -fl - x[inside].astype(np.float64)) < 2.0 ** -fl).all()
    assert (q[y > qmax] == qmax).all() and (q[y < qmin] == qmin).all()
    assert nnz == int((q != 0).sum())
    assert sat == int((~inside).sum())


@pytest.mark.parametrize("wl,fl", FORMATS)
def test_grid_points_are_fixed_points(wl, fl):
    qmin, qmax = -(1 << (wl - 1)), (1 << (wl - 1)) - 1
    codes = np.unique(np.clip(np.random.default_rng(0).integers(qmin, qmax + 1, 5000), qmin, qmax))
    x = (codes * 2.0 ** -fl).astype(np.float32)
    assert np.array_equal(x.astype(np.float64) * 2.0 ** fl, codes)      # exactly representable
    for seed in range(5):
        q, _, sat = orc.quantize(x, wl, fl, orc.SR, seed=seed, stream=seed + 1)
        assert np.array_equal(q, codes) and sat == 0


@pytest.mark.parametrize("wl,fl", [(8, 4), (12, 9), (16, 13)])
def test_nearest_mode_closed_form(wl, fl):
    g = np.random.default_rng(5)
    x = (g.standard_normal(50000) * 2.0 ** (wl - 1 - fl) * 0.5).astype(np.float32)
    q, _, _ = orc.quantize(x, wl, fl, orc.RN_HALF_UP)
    y = x.astype(np.float64) * 2.0 ** fl
    qmin, qmax = -(1 << (wl - 1)), (1 << (wl - 1)) - 1
    # ties (fraction exactly 1/2) go up; fractions are resolved to 2^-16, which is exact for
    # every value whose fraction has at most 16 bits and floor-consistent otherwise
    expect = np.clip(np.floor(np.floor(y * 65536.0) / 65536.0 + 0.5), qmin, qmax)
    assert np.array_equal(q, expect.astype(np.int64))
    far = np.abs(y - np.floor(y) - 0.5) > 2.0 ** -15
    assert np.array_equal(q[far], np.clip(np.floor(y + 0.5), qmin, qmax)[far].astype(np.int64))


def test_all_rounding_bit_patterns_exhaustive():
    """For one value, enumerate all 2^16 random patterns: the number that round up equals
    floor(frac * 2^16) exactly, and the ones that do are the largest patterns."""
    wl, fl = 8, 4
    for xv in (0.3, -0.3, 1.0 / 3.0, -5.03125, 0.0, 2.0 ** -20, -2.0 ** -20, 7.9, -8.0):
        x = np.full(65536, xv, dtype=np.float32)
        q, _, _ = orc.quantize_with_bits(x, wl, fl, np.arange(65536))
        y = float(np.float32(xv)) * 16.0
        yc = min(max(y, -128.0), 127.0)
        lo = math.floor(yc)
        f16 = math.floor((yc - lo) * 65536)
        ups = int((q == lo + 1).sum())
        assert ups == f16 and int((q == lo).sum()) == 65536 - f16
        assert (np.diff(q) >= 0).all()


def test_stochastic_rounding_is_unbiased():
    wl, fl = 8, 4
    x = np.linspace(-3.9, 3.9, 64, dtype=np.float32)
    nseed = 10000
    acc = np.zeros(64)
    idx = np.arange(64)
    for seed in range(nseed):
        q, _, _ = orc.quantize_with_bits(x, wl, fl, orc.r16(seed, 1, idx))
        acc += q
    y = x.astype(np.float64) * 16
    f = y - np.floor(y)
    sigma = np.sqrt(np.maximum(f * (1 - f), 1e-12) / nseed)
    assert (np.abs(acc / nseed - y) < 4.5 * sigma + 2.0 ** -16).all()


def test_special_values():
    wl, fl = 8, 4
    den = np.float32(1e-45)
    x = np.array([np.nan, np.inf, -np.inf, -0.0, 0.0, den, -den, 3.4e38, -3.4e38], dtype=np.float32)
    for bits in (0, 65535):
        q, nnz, sat = orc.quantize_with_bits(x, wl, fl, np.full(x.size, bits))
        up = 1 if bits == 65535 else 0
        # a negative denormal has floor(y*2^16) = -1: rounds to -1 unless the random bits carry
        assert q.tolist() == [0, 127, -128, 0, 0, 0, -1 + up, 127, -128]
        assert sat == 4
        assert nnz == int((q != 0).sum())


def test_fl_not_less_than_wl():
    # FL >= WL just means |value| < 1/2
    x = np.array([0.01, -0.02, 0.4, -0.4], dtype=np.float32)
    q, _, sat = orc.quantize(x, 8, 12, orc.RN_HALF_UP)
    assert q.tolist() == [41, -82, 127, -128] and sat == 2


def test_requantize_matches_quantize_of_dyadic_value():
    """An accumulator a with F fractional bits is the real number a*2^-F; converting it with
    the accumulator rule must equal quantizing that real number with the same random bits
    whenever it is exactly an fp32 value (|a| < 2^24)."""
    g = np.random.default_rng(3)
    acc = g.integers(-(1 << 23), 1 << 23, 4096)
    F = 12
    for wl_o, fl_o in ((8, 4), (8, 2), (16, 10), (12, 12), (16, 14)):
        shift = F - fl_o
        for mode in (orc.SR, orc.RN_HALF_UP):
            got = orc.requantize(acc, shift, wl_o, mode, seed=2, stream=9)
            x = (acc * 2.0 ** -F).astype(np.float32)
            assert np.array_equal(x.astype(np.float64), acc * 2.0 ** -F)
            want, _, _ = orc.quantize(x, wl_o, fl_o, mode, seed=2, stream=9)
            if shift <= 0:
                want = np.clip(acc * (1 << -shift), -(1 << (wl_o - 1)), (1 << (wl_o - 1)) - 1)
            if 1 <= shift <= 16 and mode == orc.SR:
                # only the top `shift` random bits are used: emulate by truncating them
                bits = orc.r16(2, 9, np.arange(acc.size))
                bits = (bits >> (16 - shift)) << (16 - shift)
                want, _, _ = orc.quantize_with_bits(x, wl_o, fl_o, bits)
            assert np.array_equal(got, want)


def test_requantize_wide_shift_and_relu():
    acc = np.array([-(1 << 40), -(1 << 30) - 5, -1, 0, 1, (1 << 30) + 12345, 1 << 40])
    q = orc.requantize(acc, 20, 16, orc.RN_HALF_UP)
    t = acc >> 4
    want = np.clip((t + 32768) >> 16, -32768, 32767)
    assert np.array_equal(q, want)
    qr = orc.requantize(acc, 20, 16, orc.RN_HALF_UP, relu=True)
    assert np.array_equal(qr, np.maximum(want, 0))
    # floor semantics of the arithmetic shift: -1 >> s = -1
    assert orc.requantize(np.array([-1]), 3, 8, orc.SR, seed=0)[0] in (-1, 0)
