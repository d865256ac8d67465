"""CPU oracle for AdaPT's fixed-point hot path (arXiv 2107.13490).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the HIP path is
compared against.  Nothing in the product package may import it; only tests/, the
smoke check and the benchmark's cpu_baseline leg do.  It shares no code, tables or
helpers with the HIP path.

What each function follows:

  philox4x32_10, r16      counter-based generator of Salmon et al. (SC'11).  The paper
                          (Sec. 3.2) only asks for "a random number P in [0,1]"; the
                          generator is this build's choice.  Its statistical behaviour is
                          pinned (uniformity, lane independence, bijectivity on counters);
                          agreement with the published known-answer vectors is
                          PARITY UNPINNED (the vectors are not available here).
  quantize                Sec. 3.2, the SR equation, on the <WL,FL> format of Sec. 2.1
                          ("Fixed-Point Quantization"), with two's-complement saturation.
  requantize              the same SR rule applied to an integer accumulator whose low
                          bits are the fraction (the paper is silent on this conversion).
  gemm                    the plain definition C = A.B over the integers.
  kld_precision_search    Sec. 3.3 "The PushDown Operation" (EDF/binning equation, the
                          discrete KL equation) and Alg. 3.

Integers are int64 / Python ints, floating point is fp64.
"""
from __future__ import annotations

import math
import os

import numpy as np

RN_HALF_UP = 0
SR = 1

_M0 = 0xD2511F53
_M1 = 0xCD9E8D57
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK32 = 0xFFFFFFFF


# --------------------------------------------------------------------------------------------
# random numbers
# --------------------------------------------------------------------------------------------

def philox4x32_10(key, ctr):
    """Philox-4x32 with 10 rounds.

    key: (k0, k1) Python ints < 2^32.  ctr: four uint64 numpy arrays (values < 2^32) of equal
    shape.  Returns four uint64 arrays (values < 2^32).
    One round: (c0,c1,c2,c3) -> (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0));
    the key is advanced by the Weyl constants between rounds.
    """
    k0, k1 = int(key[0]) & _MASK32, int(key[1]) & _MASK32
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) for c in ctr)
    m32 = np.uint64(_MASK32)
    s32 = np.uint64(32)
    for rnd in range(10):
        p0 = np.uint64(_M0) * c0          # < 2^64, exact in uint64
        p1 = np.uint64(_M1) * c2
        hi0, lo0 = p0 >> s32, p0 & m32
        hi1, lo1 = p1 >> s32, p1 & m32
        c0, c1, c2, c3 = hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0
        k0 = (k0 + _W0) & _MASK32
        k1 = (k1 + _W1) & _MASK32
    return c0, c1, c2, c3


def r16(seed: int, stream: int, index) -> np.ndarray:
    """16 random bits for element `index` (array of non-negative ints).

    Element i takes 16-bit lane (i mod 8) of the 128-bit block with counter
    (j lo, j hi, stream lo, stream hi), j = i // 8, key (seed lo, seed hi).
    Lane order: word (i mod 8)//2, low half first.
    """
    idx = np.asarray(index, dtype=np.uint64)
    j = idx >> np.uint64(3)
    lane = (idx & np.uint64(7)).astype(np.int64)
    key = (seed & _MASK32, (seed >> 32) & _MASK32)
    ctr = (j & np.uint64(_MASK32), j >> np.uint64(32),
           np.full(idx.shape, stream & _MASK32, dtype=np.uint64),
           np.full(idx.shape, (stream >> 32) & _MASK32, dtype=np.uint64))
    words = np.stack(philox4x32_10(key, ctr), axis=-1)          # [..., 4]
    w = np.take_along_axis(words, (lane >> 1)[..., None], axis=-1)[..., 0]
    half = (lane & 1).astype(np.uint64)
    return ((w >> (np.uint64(16) * half)) & np.uint64(0xFFFF)).astype(np.int64)


# --------------------------------------------------------------------------------------------
# quantize  (Sec. 3.2, SR equation)
# --------------------------------------------------------------------------------------------

def quantize_with_bits(x, wl: int, fl: int, rbits):
    """Quantize fp32 values to <wl,fl> given the 16 rounding bits of every element.

    Works on y = x * 2^fl (the value in units of one ulp of the format).  The SR rule
    "round down, or up with probability frac(y)" is evaluated with the fraction truncated
    to 16 bits, f16 = floor(frac(y) * 2^16), and 16 uniform random bits r: the result is
    rounded up iff f16 + r carries out of 16 bits (probability f16 / 2^16), i.e.
    q = floor((floor(y * 2^16) + r) / 2^16).
    Saturation clamps to the two's-complement range.  NaN gives 0.
    Returns (q int64, nnz, saturated).
    """
    x64 = np.asarray(x, dtype=np.float32).astype(np.float64).ravel()
    r = np.asarray(rbits, dtype=np.int64).ravel()
    qmin = -(1 << (wl - 1))
    qmax = (1 << (wl - 1)) - 1
    nan = np.isnan(x64)
    y = np.where(nan, 0.0, x64) * (2.0 ** fl)
    saturated = int(np.count_nonzero((y < qmin) | (y > qmax)))
    yc = np.minimum(np.maximum(y, float(qmin)), float(qmax))
    t = np.floor(yc * 65536.0).astype(np.int64)
    q = (t + r) >> 16
    q = np.minimum(q, qmax)
    q = np.where(nan, 0, q)
    return q, int(np.count_nonzero(q)), saturated


def rounding_bits(n: int, mode: int, seed: int, stream: int, start: int = 0) -> np.ndarray:
    if mode == SR:
        # drawn in blocks of 2^20 elements, the blocks spread over the host's cores: the same values as one call of
        # r16 over the whole index range, with temporaries that stay in the caches
        out = np.empty(n, dtype=np.int64)

        def block(a):
            b = min(n, a + (1 << 20))
            out[a:b] = r16(seed, stream, np.arange(start + a, start + b, dtype=np.uint64))

        starts = range(0, n, 1 << 20)
        if len(starts) > 1:
            from concurrent.futures import ThreadPoolExecutor
            with ThreadPoolExecutor(max_workers=min(len(starts), os.cpu_count() or 1)) as pool:
                list(pool.map(block, starts))
        else:
            for a in starts:
                block(a)
        return out
    if mode == RN_HALF_UP:
        return np.full(n, 1 << 15, dtype=np.int64)
    raise ValueError("unknown rounding mode")


def quantize(x, wl: int, fl: int, mode: int = SR, seed: int = 0, stream: int = 0):
    """Quantize(L, <WL,FL>) of Alg. 1 / Alg. 3: element i uses r16(seed, stream, i)."""
    x = np.asarray(x, dtype=np.float32)
    q, nnz, sat = quantize_with_bits(x, wl, fl, rounding_bits(x.size, mode, seed, stream))
    return q.reshape(x.shape), nnz, sat


def dequantize(q, fl: int) -> np.ndarray:
    return np.asarray(q, dtype=np.float64) * (2.0 ** -fl)


# --------------------------------------------------------------------------------------------
# contractions and the accumulator -> <WL,FL> conversion
# --------------------------------------------------------------------------------------------

def gemm(a, b, trans_a: bool = False, trans_b: bool = False) -> np.ndarray:
    """C[m,n] = sum_k A[m,k] * B[k,n], exactly, in int64."""
    a = np.asarray(a, dtype=np.int64)
    b = np.asarray(b, dtype=np.int64)
    if trans_a:
        a = a.T
    if trans_b:
        b = b.T
    return a @ b


def requantize(acc, shift: int, wl_o: int, mode: int = SR, seed: int = 0, stream: int = 0,
               relu: bool = False, start: int = 0) -> np.ndarray:
    """Exact accumulator (FL_a+FL_b fractional bits) -> <wl_o, FL_o>, shift = FL_a+FL_b-FL_o.

    shift <= 0 : multiply by 2^-shift.
    1..16      : add the top `shift` bits of the element's 16 random bits (or half an ulp),
                 arithmetic shift right.
    > 16       : drop shift-16 bits first (floor), then 16 guard bits as in `quantize`.
    ReLU (optional) and saturation come last.  Element i of the flattened output uses
    r16(seed, stream, start + i): `start` > 0 converts a slice of a larger tensor.
    """
    a = np.asarray(acc, dtype=np.int64)
    flat = a.ravel()
    if shift <= 0:
        q = flat * (1 << (-shift))
    else:
        bits = rounding_bits(flat.size, mode, seed, stream, start)
        if shift <= 16:
            r = bits >> (16 - shift)
            q = (flat + r) >> shift
        else:
            t = flat >> (shift - 16)
            q = (t + bits) >> 16
    if relu:
        q = np.maximum(q, 0)
    q = np.clip(q, -(1 << (wl_o - 1)), (1 << (wl_o - 1)) - 1)
    return q.reshape(a.shape)


# --------------------------------------------------------------------------------------------
# KL-divergence precision search  (Sec. 3.3 PushDown, Alg. 3)
# --------------------------------------------------------------------------------------------

def finite_range(w):
    w = np.asarray(w, dtype=np.float32).ravel()
    f = w[np.isfinite(w)]
    if f.size == 0:
        return None
    return float(f.min()), float(f.max())


def _floor_scaled(v: float, e: int) -> int:
    """floor(v * 2^-e) as an exact Python int (v is a finite double holding an fp32 value)."""
    m, ex = math.frexp(v)                      # v = m * 2^ex, 0.5 <= |m| < 1
    mi = int(m * (1 << 53))                    # exact: m has <= 53 significant bits
    sh = ex - 53 - e                           # v * 2^-e = mi * 2^sh
    return mi << sh if sh >= 0 else mi >> (-sh)   # >> on Python ints floors


def bin_grid(lo: float, hi: float, bins: int):
    """Power-of-two bin width 2^e, aligned to multiples of 2^e: the smallest e such that
    nb = floor(hi/2^e) - floor(lo/2^e) + 1 <= bins.  Returns (e, base, nb)."""
    e = -200
    while True:
        base = _floor_scaled(lo, e)
        nb = _floor_scaled(hi, e) - base + 1
        if nb <= bins:
            return e, base, nb
        e += 1


def bin_of_values(w, e: int, base: int, nb: int) -> np.ndarray:
    """bin(v) = floor(v * 2^-e) - base for finite fp32 values inside [lo, hi].

    Scaling an fp32 value by a power of two and flooring are exact in fp64 here (no fp32
    value times 2^-e with e >= -200 leaves the fp64 range), and so is the difference of
    two such floored values that are less than `bins` apart."""
    f = np.floor(np.ldexp(np.asarray(w, dtype=np.float64), -e))
    return (f - float(base)).astype(np.int64)


def bin_of_code(q: int, fl: int, e: int, base: int, nb: int) -> int:
    """Bin of the fixed-point value q * 2^-fl, clamped to the end bins."""
    sh = fl + e
    f = (q >> sh) if sh >= 0 else (q << (-sh))
    return min(max(f - base, 0), nb - 1)


def kl_divergence_bits(cp, cq, alpha: float) -> float:
    """KL(P||Q) in bits between two count vectors on the same nb bins, with additive
    smoothing alpha per bin.  alpha = 0 is the literal definition (0 log 0 = 0; +inf
    when P>0 where Q=0).  Summed in ascending bin order in fp64."""
    cp = np.asarray(cp, dtype=np.float64)
    cq = np.asarray(cq, dtype=np.float64)
    nb = cp.size
    dp = cp.sum() + alpha * nb
    dq = cq.sum() + alpha * nb
    total = 0.0
    for b in range(nb):
        p = (cp[b] + alpha) / dp
        q = (cq[b] + alpha) / dq
        if p == 0.0:
            continue
        if q == 0.0:
            return math.inf
        total += p * math.log2(p / q)
    return total


def kld_precision_search(w, wl_lo: int, wl_hi: int, il: int, bins: int, eps: float,
                         alpha=None, mode: int = SR, seed: int = 0, stream: int = 0):
    """PushDown by exhaustive scan over candidate word lengths wl_lo..wl_hi (FL_c = WL_c - il).

    Q = histogram of the fp32 tensor, P_c = histogram of its <WL_c,FL_c> quantization, both on
    the shared power-of-two bin grid taken from the tensor's range; every candidate uses the
    same 16 random bits per element.  Non-finite elements are left out of the range and of
    every histogram.  Returns a dict with kld[c], counts, the grid, the selected <WL,FL>
    (lowest WL with KL < eps, else wl_hi) and the result of a bisection over the same KLs.
    """
    w = np.asarray(w, dtype=np.float32).ravel()
    ncand = wl_hi - wl_lo + 1
    rng = finite_range(w)
    if rng is None or rng[0] == rng[1]:
        return dict(kld=np.zeros(ncand), wl_sel=wl_lo, fl_sel=wl_lo - il, wl_bisect=wl_lo,
                    e=None, base=None, nb=0, cq=None, cp=None, lo=rng[0] if rng else None,
                    hi=rng[1] if rng else None)
    lo, hi = rng
    e, base, nb = bin_grid(lo, hi, bins)
    finite = np.isfinite(w)
    wf = w[finite]
    if alpha is None:
        alpha = 1.0 / nb
    cq = np.bincount(bin_of_values(wf, e, base, nb), minlength=nb)
    bits = rounding_bits(w.size, mode, seed, stream)[finite]
    kld = np.zeros(ncand)
    cps = np.zeros((ncand, nb), dtype=np.int64)
    for c in range(ncand):
        wl = wl_lo + c
        fl = wl - il
        q, _, _ = quantize_with_bits(wf, wl, fl, bits)
        codes, inverse = np.unique(q, return_inverse=True)
        table = np.array([bin_of_code(int(code), fl, e, base, nb) for code in codes],
                         dtype=np.int64)
        cps[c] = np.bincount(table[inverse], minlength=nb)
        kld[c] = kl_divergence_bits(cps[c], cq, alpha)
    below = [c for c in range(ncand) if kld[c] < eps]
    wl_sel = wl_lo + below[0] if below else wl_hi
    # bisection as the paper describes it: assumes KL is non-increasing in WL
    a, b = 0, ncand - 1
    if not kld[b] < eps:
        wl_bis = wl_hi
    else:
        while a < b:
            mid = (a + b) // 2
            if kld[mid] < eps:
                b = mid
            else:
                a = mid + 1
        wl_bis = wl_lo + b
    return dict(kld=kld, wl_sel=wl_sel, fl_sel=wl_sel - il, wl_bisect=wl_bis, e=e, base=base,
                nb=nb, cq=cq, cp=cps, lo=lo, hi=hi)
