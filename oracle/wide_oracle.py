"""CPU oracle for contractions with word lengths 17..32 (AdaPT, arXiv 2107.13490: Sec. 3.3 bounds the
precision that PushUp may ask for at 32 bits).

TEST INFRASTRUCTURE ONLY.  Slow, plain reference; nothing in the product package may import it;
only tests/, the smoke check and the benchmark's cpu_baseline leg do.  It shares no code with
the HIP path.

Also here, on the same Python integers: the fitting requantization of exact accumulators of any size
(the narrow oracle's rule, shift = max(0, bit_length(max |acc|) - (WL-1))) and the gradient-diversity sums
of windows that hold codes above 16 bits.

Codes of up to 32 bits multiply to 62 bits and a reduction adds more, so the exact sums do not fit
64 bits: everything here is Python integers (numpy arrays of dtype object), the contractions written
out from their definitions, and the accumulator -> <WL,FL> rule of the narrow oracle applied to those
integers unchanged (shift <= 0: multiply; 1..16: add the top bits of the 16 random bits and shift;
above 16: drop shift-16 bits, then the 16 guard bits; ReLU; saturation).
"""
from __future__ import annotations

import numpy as np

from . import fxp_oracle as orc


def _obj(a):
    return np.asarray(a).astype(object)


def gemm(a, b, trans_a: bool = False, trans_b: bool = False):
    a, b = _obj(a), _obj(b)
    if trans_a:
        a = a.T
    if trans_b:
        b = b.T
    return a.dot(b)


def conv_fwd(x, w, stride: int, pad: int):
    """y[n,p,q,k] = sum_{r,s,c} x[n, p*stride - pad + r, q*stride - pad + s, c] * w[k,r,s,c] (zero padding)."""
    x, w = _obj(x), _obj(w)
    n, h, wd, c = x.shape
    k, r, s, _ = w.shape
    p, q = (h + 2 * pad - r) // stride + 1, (wd + 2 * pad - s) // stride + 1
    y = np.zeros((n, p, q, k), dtype=object)
    for i in range(p):
        for j in range(q):
            for dr in range(r):
                for ds in range(s):
                    hh, ww = i * stride - pad + dr, j * stride - pad + ds
                    if 0 <= hh < h and 0 <= ww < wd:
                        y[:, i, j, :] += x[:, hh, ww, :].dot(w[:, dr, ds, :].T)
    return y


def conv_dgrad(dy, w, h: int, wd: int, stride: int, pad: int):
    """dx[n,hh,ww,c] = sum over the outputs that read it: dy[n,p,q,k] * w[k,r,s,c]."""
    dy, w = _obj(dy), _obj(w)
    n, p, q, k = dy.shape
    _, r, s, c = w.shape
    dx = np.zeros((n, h, wd, c), dtype=object)
    for i in range(p):
        for j in range(q):
            for dr in range(r):
                for ds in range(s):
                    hh, ww = i * stride - pad + dr, j * stride - pad + ds
                    if 0 <= hh < h and 0 <= ww < wd:
                        dx[:, hh, ww, :] += dy[:, i, j, :].dot(w[:, dr, ds, :])
    return dx


def conv_wgrad(dy, x, r: int, s: int, stride: int, pad: int):
    """dw[k,r,s,c] = sum_{n,p,q} dy[n,p,q,k] * x[n, p*stride - pad + r, q*stride - pad + s, c]."""
    dy, x = _obj(dy), _obj(x)
    n, p, q, k = dy.shape
    _, h, wd, c = x.shape
    dw = np.zeros((k, r, s, c), dtype=object)
    for i in range(p):
        for j in range(q):
            for dr in range(r):
                for ds in range(s):
                    hh, ww = i * stride - pad + dr, j * stride - pad + ds
                    if 0 <= hh < h and 0 <= ww < wd:
                        dw[:, dr, ds, :] += dy[:, i, j, :].T.dot(x[:, hh, ww, :])
    return dw


def requantize(acc, shift: int, wl_o: int, mode: int = orc.SR, seed: int = 0, stream: int = 0, relu: bool = False):
    """The accumulator -> <wl_o, FL_o> rule of the narrow oracle on Python integers (wl_o up to 32)."""
    a = _obj(acc)
    flat = a.ravel()
    if shift <= 0:
        q = flat * (1 << (-shift))
    else:
        bits = orc.rounding_bits(flat.size, mode, seed, stream).astype(object)
        if shift <= 16:
            q = np.array([(int(v) + (int(r) >> (16 - shift))) >> shift for v, r in zip(flat, bits)], dtype=object)
        else:
            q = np.array([((int(v) >> (shift - 16)) + int(r)) >> 16 for v, r in zip(flat, bits)], dtype=object)
    lo, hi = -(1 << (wl_o - 1)), (1 << (wl_o - 1)) - 1
    q = np.array([min(max(max(int(v), 0) if relu else int(v), lo), hi) for v in q], dtype=np.int64)
    return q.reshape(a.shape)


def fit_shift(acc, wl: int) -> int:
    """Smallest right shift after which the largest magnitude of acc has at most wl-1 bits."""
    flat = _obj(acc).ravel()
    m = max((abs(int(v)) for v in flat), default=0)
    return max(0, m.bit_length() - (wl - 1))


def requantize_fit(acc, wl: int, mode: int = orc.SR, seed: int = 0, stream: int = 0):
    """Exact accumulators of any size -> wl-bit codes (wl up to 32) with the fitting shift.
    Returns (codes int64, shift, sum of squared codes as a Python integer)."""
    sh = fit_shift(acc, wl)
    q = requantize(acc, sh, wl, mode, seed, stream, False)
    return q, sh, sum(int(v) * int(v) for v in q.ravel())


def gradient_diversity(codes, fls):
    """The gradient-diversity quantities of the PushUp oracle (Sec. 3.3 "The PushUp Operation") for windows whose
    codes or aligned sums exceed 32 bits: the same exact integer sums (numpy arrays of Python integers), the same
    fp64 norms.  codes: list of integer arrays of one shape, oldest first; fls: their FL."""
    import math
    fl_max = max(int(f) for f in fls)
    total = None
    sumsq = []
    for c, f in zip(codes, fls):
        flat = _obj(np.asarray(c).ravel())
        sumsq.append(int((flat * flat).sum()) if flat.size else 0)
        scaled = flat * (1 << (fl_max - int(f)))
        total = scaled if total is None else total + scaled
    sumsq_sum = int((total * total).sum()) if total.size else 0
    num = 0.0
    for q, f in zip(sumsq, fls):
        num += math.sqrt(q) * 2.0 ** (-int(f))
    den = math.sqrt(sumsq_sum) * 2.0 ** (-fl_max)
    if den > 0.0:
        ds = num / den
    else:
        ds = math.inf if num > 0.0 else math.nan
    log_ds = math.log(ds) if (0.0 < ds < math.inf) else 1.0
    return {"sumsq": sumsq, "fl_max": fl_max, "sumsq_sum": sumsq_sum, "num": num, "den": den, "ds": ds, "log_ds": log_ds}
