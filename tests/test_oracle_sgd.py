"""Pins for the oracle's fused master-weight update + re-quantization (CPU only).

Follows Alg. 1 (backward-pass line and the Quantize loop), Sec. 3.3 "Dealing with Fixed-Points
Limited Range" (gradient divided by its 2-norm) and Sec. 3.4 "Inducing Sparsity" (L1/L2 terms).
The paper prints no numbers; the pins are: the exactness of the fp32 fused multiply-add
emulation against rational arithmetic (including constructed double-rounding traps), special
cases with closed forms (no step, pure decay, unit-norm step), an fp64 evaluation of the same
formula, and the composition with the quantizer oracle.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import fxp_oracle as orc
from oracle import sgd_oracle as so


def _exact_fma(a, b, c):
    return so._round_fraction_to_f32(Fraction(float(a)) * Fraction(float(b)) + Fraction(float(c)))


def test_rounding_of_rationals_onto_fp32():
    f = so._round_fraction_to_f32
    assert f(Fraction(1, 3)) == np.float32(1.0 / 3.0)
    assert f(Fraction(1) + Fraction(1, 1 << 24)) == np.float32(1.0)                       # tie -> even
    assert f(Fraction(1) + Fraction(3, 1 << 24)) == np.float32(1.0 + 2.0 ** -22)          # tie -> even (up)
    assert f(Fraction(1) + Fraction(1, 1 << 24) + Fraction(1, 1 << 90)) == np.float32(1.0 + 2.0 ** -23)
    assert f(Fraction(1, 1 << 149)) == np.float32(2.0 ** -149)                            # smallest subnormal
    assert f(Fraction(1, 1 << 150)) == np.float32(0.0)                                    # tie -> even (zero)
    assert f(Fraction(3, 1 << 150)) == np.float32(2.0 ** -148)
    assert f(-Fraction(5, 7)) == np.float32(-5.0 / 7.0)


def test_fma_double_rounding_traps():
    a = np.float32(1.0 + 2.0 ** -12)
    # a*a = 1 + 2^-11 + 2^-24 lies exactly between two fp32 numbers; a tiny addend decides the direction
    up = so.fma32(a, a, np.float32(2.0 ** -80))
    dn = so.fma32(a, a, np.float32(-2.0 ** -80))
    tie = so.fma32(a, a, np.float32(0.0))
    assert up == np.float32(1.0 + 2.0 ** -11 + 2.0 ** -23)
    assert dn == np.float32(1.0 + 2.0 ** -11)
    assert tie == np.float32(1.0 + 2.0 ** -11)          # even mantissa
    assert up == _exact_fma(a, a, np.float32(2.0 ** -80))


def test_fma_matches_rationals_on_random_and_denormal_inputs():
    rng = np.random.default_rng(3)
    a = (rng.standard_normal(4000) * 10.0 ** rng.integers(-20, 5, 4000)).astype(np.float32)
    b = (rng.standard_normal(4000) * 10.0 ** rng.integers(-20, 5, 4000)).astype(np.float32)
    c = (rng.standard_normal(4000) * 10.0 ** rng.integers(-40, 5, 4000)).astype(np.float32)
    c[::7] = -(a[::7].astype(np.float64) * b[::7].astype(np.float64)).astype(np.float32)   # heavy cancellation
    got = so.fma32(a, b, c)
    for i in range(a.size):
        want = _exact_fma(a[i], b[i], c[i])
        assert got[i] == want or (np.isnan(got[i]) and np.isnan(want)), (a[i], b[i], c[i])


def test_no_step_is_plain_quantize():
    rng = np.random.default_rng(1)
    w = (rng.standard_normal(5000) * 0.1).astype(np.float32)
    g = rng.integers(-128, 128, 5000)
    res = so.sgd_update_quantize(w, g, 5, 0.0, 0.0, 0.0, 8, 5, orc.SR, 3, 4)
    assert np.array_equal(res["w"], w)
    q, nnz, sat = orc.quantize(w, 8, 5, orc.SR, 3, 4)
    assert np.array_equal(res["q"], q) and (res["nnz"], res["sat"]) == (nnz, sat)
    assert res["lo"] == float(w.min()) and res["hi"] == float(w.max())
    # zero gradient: normalised step is 0, not a division by zero
    res = so.sgd_update_quantize(w, np.zeros(5000, dtype=np.int64), 5, 0.1, 0.0, 0.0, 8, 5)
    assert res["step"] == 0.0 and np.array_equal(res["w"], w)


def test_normalised_step_has_length_lr():
    rng = np.random.default_rng(2)
    w = rng.standard_normal(20000).astype(np.float32)
    g = rng.integers(-2000, 2000, 20000)
    for lr in (0.5, 0.01):
        res = so.sgd_update_quantize(w, g, 9, lr, 0.0, 0.0, 12, 9)
        moved = np.linalg.norm(res["w"].astype(np.float64) - w.astype(np.float64))
        assert moved == pytest.approx(lr, rel=2e-4)
        # and it points against the gradient
        assert np.dot(res["w"].astype(np.float64) - w, g) < 0
    # without normalisation the step is lr * g
    res = so.sgd_update_quantize(w, g, 9, 0.25, 0.0, 0.0, 12, 9, normalize=False)
    assert np.allclose(res["w"], w - 0.25 * g * 2.0 ** -9, rtol=0, atol=1e-6)


def test_decay_terms():
    w = np.array([0.5, -0.25, 0.0, 2.0, -3.0], dtype=np.float32)
    z = np.zeros(5, dtype=np.int64)
    res = so.sgd_update_quantize(w, z, 4, 0.5, 0.0, 0.25, 8, 4)       # l2 only: w (1 - lr l2), exact here
    assert np.array_equal(res["w"], w * np.float32(0.875))
    res = so.sgd_update_quantize(w, z, 4, 0.5, 0.125, 0.0, 8, 4)      # l1 only: towards zero by lr l1; 0 stays
    assert np.array_equal(res["w"], np.array([0.4375, -0.1875, 0.0, 1.9375, -2.9375], dtype=np.float32))


def test_matches_fp64_formula_and_composes_with_quantize():
    rng = np.random.default_rng(4)
    w = (rng.standard_normal(30000) * 0.2).astype(np.float32)
    g = rng.integers(-128, 128, 30000)
    lr, l1, l2 = 0.05, 1e-4, 5e-3
    res = so.sgd_update_quantize(w, g, 6, lr, l1, l2, 8, 5, orc.SR, 1, 2)
    w64 = w.astype(np.float64)
    step = lr / np.sqrt(float(np.sum(g.astype(np.float64) ** 2)))
    want = w64 - step * g - lr * (l1 * np.sign(w64) + l2 * w64)
    assert np.max(np.abs(res["w"] - want)) <= 4 * np.spacing(np.float32(np.max(np.abs(w))))
    q, nnz, sat = orc.quantize(res["w"], 8, 5, orc.SR, 1, 2)
    assert np.array_equal(res["q"], q) and (res["nnz"], res["sat"]) == (nnz, sat)
    assert res["sumsq"] == int(np.sum(g.astype(object) ** 2))
    assert res["lo"] == float(res["w"].min()) and res["hi"] == float(res["w"].max())
