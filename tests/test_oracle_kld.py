"""Pins for the oracle's KL-divergence precision search (CPU only).

Follows Sec. 3.3 "The PushDown Operation" (binning / discrete KL equations) and Alg. 3.
No published numbers exist, so the pins are: a hand-enumerated example (tests/golden),
the lossless special case the paper's criterion is built on (KL = 0 iff nothing is lost),
Gibbs' inequality, count conservation, a closed form, a library routine for the unsmoothed
divergence, and a second derivation of the histograms through dequantized values.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.stats

from oracle import fxp_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "kld_hand_example.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        out[key] = [int(v) for v in vals]
    return out


def test_hand_example():
    g = _golden()
    w = np.array([-0.75, -0.5, -0.25, 0, 0.25, 0.25, 0.5, 0.75], dtype=np.float32)
    res = orc.kld_precision_search(w, 2, 4, 2, 8, 1e-9, mode=orc.RN_HALF_UP)
    assert [res["e"], res["base"], res["nb"]] == g["e"] + g["base"] + g["nb"]
    assert res["cq"].tolist() == g["cq"]
    for c, key in enumerate(("cp2", "cp3", "cp4")):
        assert res["cp"][c].tolist() == g[key]
        # KL from the definition with exact rationals: alpha = 1/nb, denominators n + 1
        nb, n = g["nb"][0], 8
        total = 0.0
        for b in range(nb):
            p = (Fraction(g[key][b]) + Fraction(1, nb)) / (n + 1)
            q = (Fraction(g["cq"][b]) + Fraction(1, nb)) / (n + 1)
            total += float(p) * math.log2(p / q)
        assert res["kld"][c] == pytest.approx(total, rel=1e-12, abs=1e-15)
    assert res["kld"][2] == 0.0 and res["kld"][0] > res["kld"][1] > 0
    assert [res["wl_sel"], res["fl_sel"]] == g["wl_sel"] + g["fl_sel"]


def test_bin_grid_closed_cases():
    assert orc.bin_grid(-1.0, 1.0, 2048) == (-9, -512, 1025)      # width 2^-10 would need 2049
    assert orc.bin_grid(0.0, 1.0, 2) == (0, 0, 2)
    assert orc.bin_grid(0.0, 1.0, 1) == (1, 0, 1)
    assert orc.bin_grid(-0.75, 0.75, 8) == (-2, -3, 7)
    # minimality and the bins/2 < nb <= bins property
    g = np.random.default_rng(0)
    for _ in range(200):
        lo, hi = np.sort(g.standard_normal(2).astype(np.float32) * 10.0 ** g.integers(-6, 6))
        if lo == hi:
            continue
        bins = int(g.integers(2, 4096))
        e, base, nb = orc.bin_grid(float(lo), float(hi), bins)
        assert nb <= bins
        assert orc._floor_scaled(float(hi), e - 1) - orc._floor_scaled(float(lo), e - 1) + 1 > bins
        assert base == math.floor(Fraction(float(lo)) / Fraction(2) ** e)


def test_bin_of_values_matches_exact_integer_binning():
    g = np.random.default_rng(1)
    w = np.concatenate([g.standard_normal(500) * 0.05, [1e-40, -1e-40, 0.0, -0.0]]).astype(np.float32)
    lo, hi = orc.finite_range(w)
    e, base, nb = orc.bin_grid(lo, hi, 100)
    got = orc.bin_of_values(w, e, base, nb)
    want = [math.floor(Fraction(float(v)) / Fraction(2) ** e) - base for v in w]
    assert got.tolist() == want and min(want) == 0 and max(want) == nb - 1


@pytest.mark.parametrize("w0,f0,il", [(6, 4, 2), (9, 6, 3), (12, 10, 2)])
def test_lossless_special_case_selects_the_grid_precision(w0, f0, il):
    """A tensor already on the <W0,F0> grid: candidates with at least F0 fractional bits
    reproduce it exactly (KL exactly 0); the selection with eps -> 0+ is W0 = F0 + il."""
    assert w0 == f0 + il
    g = np.random.default_rng(w0)
    qmax = (1 << (w0 - 1)) - 1
    codes = np.clip(np.round(g.standard_normal(20000) * qmax / 3), -qmax, qmax)
    codes[:2] = [-qmax - 1, qmax]                       # use the whole range
    codes[2] = 1                                        # an odd code: needs all F0 bits
    w = (codes * 2.0 ** -f0).astype(np.float32)
    res = orc.kld_precision_search(w, 2, 16, il, 2048, 1e-300, seed=3, stream=1)
    for c, wl in enumerate(range(2, 17)):
        if wl >= w0:
            assert res["kld"][c] == 0.0
            assert np.array_equal(res["cp"][c], res["cq"])
        else:
            assert res["kld"][c] > 0.0
    assert res["wl_sel"] == w0 and res["fl_sel"] == f0 and res["wl_bisect"] == w0


@pytest.mark.parametrize("seed", range(4))
def test_gibbs_and_count_conservation(seed):
    g = np.random.default_rng(seed)
    w = (g.standard_normal(5000) * 0.05).astype(np.float32)
    w[::97] = np.nan
    w[5] = np.inf
    bins = [50, 150, 2048, 7][seed]
    res = orc.kld_precision_search(w, 2, 16, 2, bins, 1e-3, seed=seed, stream=2)
    nfin = int(np.isfinite(w).sum())
    assert res["cq"].sum() == nfin
    assert (res["cp"].sum(axis=1) == nfin).all()
    assert (res["kld"] >= 0).all()
    assert bins / 2 < res["nb"] <= bins
    # coarser candidates lose more: the finest candidate is the closest
    assert res["kld"][-1] < res["kld"][0]


def test_two_point_closed_form():
    # P = (a, 1-a), Q = (b, 1-b): KL = a log2(a/b) + (1-a) log2((1-a)/(1-b))
    cp, cq = np.array([30, 70]), np.array([55, 45])
    a, b = 0.3, 0.55
    want = a * math.log2(a / b) + (1 - a) * math.log2((1 - a) / (1 - b))
    assert orc.kl_divergence_bits(cp, cq, 0.0) == pytest.approx(want, rel=1e-13)


def test_unsmoothed_matches_library_relative_entropy():
    g = np.random.default_rng(9)
    cq = g.integers(1, 50, 300)
    cp = g.integers(0, 50, 300)
    want = scipy.stats.entropy(cp, cq, base=2)
    assert orc.kl_divergence_bits(cp, cq, 0.0) == pytest.approx(want, rel=1e-12)
    cq[7], cp[7] = 0, 3
    assert orc.kl_divergence_bits(cp, cq, 0.0) == math.inf
    # smoothing = the library routine applied to the smoothed masses
    alpha = 1.0 / 300
    assert orc.kl_divergence_bits(cp, cq, alpha) == pytest.approx(
        scipy.stats.entropy(cp + alpha, cq + alpha, base=2), rel=1e-12)


def test_nearest_mode_is_seed_independent():
    w = (np.random.default_rng(4).standard_normal(3000) * 0.05).astype(np.float32)
    a = orc.kld_precision_search(w, 4, 12, 2, 150, 1e-3, mode=orc.RN_HALF_UP, seed=1, stream=1)
    b = orc.kld_precision_search(w, 4, 12, 2, 150, 1e-3, mode=orc.RN_HALF_UP, seed=99, stream=7)
    assert np.array_equal(a["kld"], b["kld"]) and np.array_equal(a["cp"], b["cp"])


@pytest.mark.parametrize("bins,il,scale", [(2048, 2, 0.05), (100, 3, 0.5), (64, 2, 1e-4), (300, 4, 3.0)])
def test_histograms_equal_quantize_dequantize_bin(bins, il, scale):
    """Second derivation: quantize with the public quantizer, turn the codes back into real
    numbers, bin those numbers with the value-binning rule, clamp to the end bins."""
    w = (np.random.default_rng(bins).standard_normal(4000) * scale).astype(np.float32)
    res = orc.kld_precision_search(w, 2, 16, il, bins, 1e-3, seed=5, stream=6)
    e, base, nb = res["e"], res["base"], res["nb"]
    for c, wl in enumerate(range(2, 17)):
        fl = wl - il
        q, _, _ = orc.quantize(w, wl, fl, orc.SR, seed=5, stream=6)
        vals = orc.dequantize(q, fl)
        b = np.clip(np.floor(vals / 2.0 ** e) - base, 0, nb - 1).astype(np.int64)
        assert np.array_equal(np.bincount(b, minlength=nb), res["cp"][c])


def test_degenerate_inputs():
    r = orc.kld_precision_search(np.full(10, 0.25, dtype=np.float32), 3, 8, 2, 100, 1e-3)
    assert r["wl_sel"] == 3 and (r["kld"] == 0).all()
    r = orc.kld_precision_search(np.array([np.nan, np.inf], dtype=np.float32), 3, 8, 2, 100, 1e-3)
    assert r["wl_sel"] == 3 and (r["kld"] == 0).all()
    # tiny range far from zero: codes shift left by many bits before binning
    w = (1.0 + np.arange(64) * 2.0 ** -20).astype(np.float32)
    r = orc.kld_precision_search(w, 4, 16, 2, 32, 1e-3)
    assert r["nb"] == 32 and (r["cp"].sum(axis=1) == 64).all() and (r["kld"] > 0).all()


def test_selection_rule_and_bisection():
    w = (np.random.default_rng(12).standard_normal(65536) * 0.05).astype(np.float32)
    res = orc.kld_precision_search(w, 2, 16, 2, 2048, 1e-2, seed=0, stream=0)
    k = res["kld"]
    below = [wl for wl, v in zip(range(2, 17), k) if v < 1e-2]
    assert res["wl_sel"] == (below[0] if below else 16)
    if (np.diff(k) <= 0).all():
        assert res["wl_bisect"] == res["wl_sel"]
