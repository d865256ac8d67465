"""CPU oracle for AdaPT's PushUp operation and switch controller (arXiv 2107.13490).

TEST INFRASTRUCTURE ONLY.  Slow, plain reference for the gradient-diversity reduction and the
scalar precision-switching rules.  Nothing in the product package may import it; only tests/,
the smoke check and the benchmark's cpu_baseline leg do.  It shares no code with the HIP path.

What each function follows (Sec. 3.3):

  gradient_diversity   "The PushUp Operation", the gradient-diversity equation: the sum of the
                       2-norms of the gradients of the last batches over the 2-norm of their
                       sum, and its logarithm with the value 1 for the degenerate cases.
                       Gradients arrive as fixed-point codes g = c * 2^-FL; all sums of codes
                       and of squares are exact Python integers, the norms fp64.
  pushup_suggest       same paragraph: the two suggestions s1, s2, their combination under the
                       strategy st, the new <WL,FL>, then "Dealing with Fixed-Points Limited
                       Range" (buffer bits).
  adapt_strategy       "Strategy, Resolution and Lookback", the strategy cases.
  adapt_lookback       same paragraph, lb_new and the momentum update.
  adapt_resolution     same paragraph, the resolution cases.

Readings taken where the text is garbled or silent are listed in the docstrings.
Integers are Python ints, floating point is fp64.
"""
from __future__ import annotations

import math

import numpy as np

ST_MIN, ST_MEAN, ST_MAX = 0, 1, 2


def gradient_diversity(codes, fls):
    """codes: list of integer arrays of one shape (the window, oldest first); fls: their FL.

    Returns a dict with
      sumsq[k]   = sum_i c_k[i]^2                      (exact int)
      fl_max     = max FL of the window
      sumsq_sum  = sum_i (sum_k c_k[i] * 2^(fl_max - FL_k))^2   (exact int; codes aligned to the finest grid)
      num        = sum_k sqrt(sumsq[k]) * 2^-FL_k      (fp64, k ascending)
      den        = sqrt(sumsq_sum) * 2^-fl_max
      ds         = num / den   (inf if den == 0 < num, nan if both are 0)
      log_ds     = ln(ds) if 0 < ds < inf else 1.0
    """
    assert len(codes) == len(fls) and len(codes) > 0
    fl_max = max(int(f) for f in fls)
    total = None
    sumsq = []
    for c, f in zip(codes, fls):
        flat = [int(v) for v in np.asarray(c).ravel()]
        sumsq.append(sum(v * v for v in flat))
        scaled = [v << (fl_max - int(f)) for v in flat]
        total = scaled if total is None else [a + b for a, b in zip(total, scaled)]
    sumsq_sum = sum(v * v for v in total)
    num = 0.0
    for q, f in zip(sumsq, fls):
        num += math.sqrt(q) * 2.0 ** (-int(f))
    den = math.sqrt(sumsq_sum) * 2.0 ** (-fl_max)
    if den > 0.0:
        ds = num / den
    else:
        ds = math.inf if num > 0.0 else math.nan
    log_ds = math.log(ds) if (0.0 < ds < math.inf) else 1.0
    return {"sumsq": sumsq, "fl_max": fl_max, "sumsq_sum": sumsq_sum, "num": num, "den": den, "ds": ds,
            "log_ds": log_ds}


def gradient_diversity_np(codes, fls):
    """The same quantities with numpy (int64 / Python-int accumulation) for larger tensors."""
    fl_max = max(int(f) for f in fls)
    total = np.zeros(np.asarray(codes[0]).size, dtype=np.int64)
    sumsq = []
    for c, f in zip(codes, fls):
        flat = np.asarray(c).ravel().astype(np.int64)
        sumsq.append(_sum_squares(flat))
        total += flat << (fl_max - int(f))
    assert np.all(np.abs(total) < (1 << 31))
    sumsq_sum = _sum_squares(total)
    num = 0.0
    for q, f in zip(sumsq, fls):
        num += math.sqrt(q) * 2.0 ** (-int(f))
    den = math.sqrt(sumsq_sum) * 2.0 ** (-fl_max)
    ds = num / den if den > 0.0 else (math.inf if num > 0.0 else math.nan)
    return {"sumsq": sumsq, "fl_max": fl_max, "sumsq_sum": sumsq_sum, "num": num, "den": den, "ds": ds,
            "log_ds": math.log(ds) if (0.0 < ds < math.inf) else 1.0}


def _sum_squares(v: np.ndarray) -> int:
    """Exact sum of squares of int64 values with |v| < 2^31: squares are split into 31-bit halves so
    that every partial sum stays below 2^63 for up to 2^31 elements."""
    sq = v * v                                   # < 2^62
    lo = int(np.sum(sq & np.int64((1 << 31) - 1)))
    hi = int(np.sum(sq >> np.int64(31)))
    return (hi << 31) + lo


def pushup_suggest(ds: float, wl_min: int, fl_min: int, strategy: int, buff: int, wl_cap: int = 32):
    """New <WL,FL> of a layer from its gradient diversity and the PushDown result <wl_min, fl_min>.

    With L = ln(ds) when 0 < ds < inf (the text writes "log"; natural logarithm taken), else 1:
      if L > 0:  s1 = max(ceil(1 / (L - 1)), 1)            (as printed; L = 1 gives the cap)
                 s2 = max(min(32 L^2 - 1, 32) - fl_min, 1)
                 s  = min(s1,s2) | ceil((s1+s2)/2) | max(s1,s2)  for st = min | mean | max
      else:      s  = 1   (the text repeats "> 0" for this branch; taken as the complement)
      s1, s2 are limited to [1, wl_cap] (the paper's bound of 32 bits on every length).
      FL = min(fl_min + s, wl_cap);  WL = min(max(wl_min, fl_min) + 1, wl_cap)
    then the buffer bits (applied to the values just computed):
      FL = min(FL, wl_cap - buff);   WL = max(min(FL + buff, wl_cap), WL)
    Returns (WL, FL, s1, s2, s).
    """
    L = math.log(ds) if (0.0 < ds < math.inf) else 1.0
    if L > 0.0:
        if L == 1.0:
            s1 = wl_cap
        else:
            s1 = max(math.ceil(1.0 / (L - 1.0)), 1)
        s1 = min(s1, wl_cap)
        s2f = max(min(32.0 * L * L - 1.0, 32.0) - fl_min, 1.0)
        s2 = min(int(math.ceil(s2f)), wl_cap)          # lengths are whole bits: round the suggestion up
        if strategy == ST_MIN:
            s = min(s1, s2)
        elif strategy == ST_MEAN:
            s = math.ceil(0.5 * (s1 + s2))
        else:
            s = max(s1, s2)
    else:
        s1 = s2 = s = 1
    fl = min(fl_min + s, wl_cap)
    wl = min(max(wl_min, fl_min) + 1, wl_cap)
    fl = min(fl, wl_cap - buff)
    wl = max(min(fl + buff, wl_cap), wl)
    return wl, fl, s1, s2, s


def adapt_strategy(strategy: int, loss_avg: float, loss_now: float) -> int:
    """|loss_avg| <= |loss_now| (no progress): min -> mean, mean -> max, max stays;
    |loss_avg| > |loss_now|: min."""
    if abs(loss_avg) > abs(loss_now):
        return ST_MIN
    return {ST_MIN: ST_MEAN, ST_MEAN: ST_MAX, ST_MAX: ST_MAX}[strategy]


def adapt_lookback(lb: int, ds: float, lb_lwr: int, lb_upr: int, gamma: float) -> int:
    """lb_new = min(max(ceil(lb_upr / ds), lb_lwr), lb_upr) if 0 < ds (finite), else lb_upr;
    lb = ceil(lb_new * gamma + (1 - gamma) * lb)."""
    if 0.0 < ds < math.inf:
        lb_new = min(max(math.ceil(lb_upr / ds), lb_lwr), lb_upr)
    else:
        lb_new = lb_upr
    return int(math.ceil(lb_new * gamma + (1.0 - gamma) * lb))


def adapt_resolution(r: int, lb: int, lb_lwr: int, lb_upr: int, r_lwr: int, r_upr: int) -> int:
    """r+1 (clamped) if lb == lb_upr; r-1 (clamped) if lb == lb_lwr; unchanged otherwise.  When
    lb_lwr == lb_upr the first case wins (the text does not order them)."""
    if lb == lb_upr:
        return min(max(r + 1, r_lwr), r_upr)
    if lb == lb_lwr:
        return min(max(r - 1, r_lwr), r_upr)
    return r
