"""CPU oracle for the master-weight update of AdaPT-SGD fused with re-quantization
(arXiv 2107.13490).

TEST INFRASTRUCTURE ONLY.  Slow, plain reference; nothing in the product package may import it;
only tests/, the smoke check and the benchmark's cpu_baseline leg do.  It shares no code with
the HIP path.

What it follows: Alg. 1 (AdaPT-SGD), the backward-pass line and the per-layer Quantize loop
after it; Sec. 3.3 "Dealing with Fixed-Points Limited Range" (the gradient of a layer is
divided by its 2-norm); Sec. 3.4 "Inducing Sparsity" (the L1 and L2 terms of the loss, whose
derivatives are l1*sign(w) and l2*w).  The paper fixes no operation order for the fp32 master
update; the order taken here (three fused multiply-adds per element) is part of the contract:

    step = fp32( lr / sqrt(sum_i c_i^2) )                  (g / ||g||_2 = c / sqrt(sum c^2): the scale 2^-FL_g
                                                             cancels; fp64, rounded once; 0 if the sum is 0;
                                                             fp32(lr * 2^-FL_g) without normalisation)
    d    = fma(l2, w, l1 * sign(w))                          (fp32; sign(0) = 0)
    w1   = fma(-step, c, w)                                  (c = the gradient code as fp32, exact)
    w'   = fma(-lr, d, w1)
    q    = quantize(w', <WL,FL>)  (the oracle's quantizer), nnz, saturated, min/max of the finite w'

fp32 fused multiply-adds are evaluated exactly: in fp64 where that is provably the correctly
rounded result, with rationals otherwise.
"""
from __future__ import annotations

import math
from fractions import Fraction

import numpy as np

from . import fxp_oracle as orc


def _round_fraction_to_f32(x: Fraction) -> np.float32:
    """Round-to-nearest-even of an exact rational onto the fp32 grid (subnormals included)."""
    if x == 0:
        return np.float32(0.0)
    sign = -1 if x < 0 else 1
    a = abs(x)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    e = max(e, -126)                      # subnormals share the exponent of the smallest normal
    ulp = Fraction(2) ** (e - 23)
    qf = a / ulp
    q = qf.numerator // qf.denominator
    rem = qf - q
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (q & 1)):
        q += 1
    val = q * ulp
    if val >= Fraction(2) ** 128:
        return np.float32(sign * math.inf)
    return np.float32(sign * float(val))  # exact: at most 24 significant bits


def fma32(a, b, c) -> np.ndarray:
    """Correctly rounded fp32 fma(a, b, c) element-wise (finite inputs)."""
    a = np.asarray(a, dtype=np.float32)
    b = np.asarray(b, dtype=np.float32)
    c = np.asarray(c, dtype=np.float32)
    a, b, c = np.broadcast_arrays(a, b, c)
    r64 = a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)   # product exact, one rounding
    out = r64.astype(np.float32)
    # The fp64 sum is the exact value rounded to 53 bits.  Rounding it again to 24 bits can differ
    # from rounding the exact value only if the fp64 value sits exactly on a midpoint between two
    # fp32 numbers; results in the subnormal range have coarser midpoints and are all redone.
    bits = r64.view(np.uint64)
    tie = (bits & np.uint64((1 << 29) - 1)) == np.uint64(1 << 28)
    small = np.abs(r64) < 2.0 ** -125
    redo = np.flatnonzero((tie | small) & np.isfinite(r64) & (r64 != 0.0))
    if redo.size:
        flat = out.reshape(-1).copy()
        af, bf, cf = a.reshape(-1), b.reshape(-1), c.reshape(-1)
        for i in redo:
            flat[i] = _round_fraction_to_f32(Fraction(float(af[i])) * Fraction(float(bf[i])) + Fraction(float(cf[i])))
        out = flat.reshape(out.shape)
    return out


def sgd_step_size(lr: float, fl_g: int, sumsq) -> np.float32:
    """fp32 step per unit of gradient code; sumsq = sum of squared codes, or None (no normalisation)."""
    if sumsq is None:
        return np.float32(lr * 2.0 ** -fl_g)
    if sumsq == 0:
        return np.float32(0.0)
    return np.float32(lr / math.sqrt(float(sumsq)))


def sgd_update_quantize(w, g_codes, fl_g: int, lr: float, l1: float, l2: float, wl: int, fl: int,
                        mode: int = orc.SR, seed: int = 0, stream: int = 0, normalize: bool = True):
    """Returns dict(w=new master weights (fp32), q=codes, nnz, sat, lo, hi, step, sumsq)."""
    w = np.asarray(w, dtype=np.float32)
    c = np.asarray(g_codes).astype(np.int64)
    assert w.shape == c.shape
    sumsq = int(np.sum(c.astype(object) ** 2)) if c.size else 0
    step = sgd_step_size(lr, fl_g, sumsq if normalize else None)
    lr32, l1_32, l2_32 = np.float32(lr), np.float32(l1), np.float32(l2)
    sign_term = np.where(w > 0, l1_32, np.where(w < 0, -l1_32, np.float32(0.0))).astype(np.float32)
    d = fma32(l2_32, w, sign_term)
    w1 = fma32(-step, c.astype(np.float32), w)
    w_new = fma32(-lr32, d, w1)
    q, nnz, sat = orc.quantize(w_new, wl, fl, mode, seed, stream)
    fin = w_new[np.isfinite(w_new)]
    lo = float(fin.min()) if fin.size else math.inf
    hi = float(fin.max()) if fin.size else -math.inf
    return {"w": w_new, "q": q, "nnz": nnz, "sat": sat, "lo": lo, "hi": hi, "step": step, "sumsq": sumsq}
