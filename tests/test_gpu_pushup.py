"""GPU parity: adapt_gradient_diversity against the CPU oracle (Sec. 3.3 "The PushUp Operation",
gradient-diversity equation).  Integer sums bit for bit; the fp64 ratio and its logarithm within
1e-12 relative (both sides take sqrt, one division and one log of the same exact integers; they
differ only in how a > 53-bit integer is rounded to fp64)."""
import math

import numpy as np
import pytest

import paper_2107_13490_amd as pkg
import workloads as wk
from oracle import fxp_oracle as orc
from oracle import pushup_oracle as pu

from gpu_util import ctx, dev, host

pytestmark = pytest.mark.gpu


def _codes(rng, n, wl, scale=0.4):
    lim = 1 << (wl - 1)
    return np.clip(np.rint(rng.standard_normal(n) * lim * scale), -lim, lim - 1).astype(np.int8 if wl <= 8 else np.int16)


def _check(codes, fmts):
    out, sums = ctx().gradient_diversity([dev(c) for c in codes], fmts)
    ref = pu.gradient_diversity_np([c.astype(np.int64) for c in codes], [f[1] for f in fmts])
    got = host(sums).view(np.uint64)
    k = len(codes)
    assert [int(v) for v in got[:k]] == ref["sumsq"]
    assert (int(got[k + 1]) << 32) + int(got[k]) == ref["sumsq_sum"]
    ds, log_ds = host(out).tolist()
    if math.isnan(ref["ds"]):
        assert math.isnan(ds)
    elif math.isinf(ref["ds"]):
        assert ds == ref["ds"]
    else:
        assert ds == pytest.approx(ref["ds"], rel=1e-12)
    assert log_ds == pytest.approx(ref["log_ds"], rel=1e-12, abs=1e-12)
    return ds


@pytest.mark.parametrize("n", [1, 15, 16, 17, 4095, 4096, 4097, 110592, (1 << 20) + 5])
@pytest.mark.parametrize("count", [1, 2, 3, 4, 5, 9, 25])
def test_sizes_and_window_lengths(n, count):
    rng = np.random.default_rng(1000 * count + n % 997)
    codes = [_codes(rng, n, 8) for _ in range(count)]
    ds = _check(codes, [(8, 5)] * count)
    assert ds >= 1.0 - 1e-12


def test_mixed_formats_and_storage_types():
    rng = np.random.default_rng(5)
    fmts = [(8, 5), (12, 9), (4, 1), (16, 13), (6, 3), (9, 6), (8, 7)]
    codes = [_codes(rng, 50001, wl) for wl, _ in fmts]
    _check(codes, fmts)


def test_closed_forms():
    g = _codes(np.random.default_rng(2), 30000, 8)
    assert _check([g] * 8, [(8, 5)] * 8) == pytest.approx(1.0, rel=1e-12)        # identical gradients
    _check([g, (-g.astype(np.int16)).clip(-128, 127).astype(np.int8)], [(8, 5)] * 2)        # (nearly) cancelling
    z = np.zeros(1000, dtype=np.int8)
    _check([z, z, z], [(8, 5)] * 3)                                                # NaN -> log term 1
    h = np.array([3, -3, 5], dtype=np.int8)
    _check([h, -h], [(8, 2), (8, 2)])                                              # +inf
    onehots = []
    for k in range(9):
        c = np.zeros(64, dtype=np.int16)
        c[7 * k] = 1000 if k % 2 else -1000
        onehots.append(c)
    assert _check(onehots, [(12, 4)] * 9) == pytest.approx(3.0, rel=1e-12)       # orthogonal: sqrt(9)


def test_extreme_codes_at_the_int32_bound():
    # 64 tensors of the most negative int16 code on grids 0..4: aligned sum 64 * 2^15 * 2^4 = 2^25 per element
    codes = [np.full(70000, -32768, dtype=np.int16) for _ in range(64)]
    fmts = [(16, k % 5) for k in range(64)]
    _check(codes, fmts)
    # the same with 8-bit codes widened by the largest shift the bound allows: 2 * 2^7 * 2^22 = 2^30 < 2^31
    c8 = [np.full(5000, -128, dtype=np.int8), np.full(5000, 127, dtype=np.int8), np.full(5000, -128, dtype=np.int8)]
    _check(c8, [(8, 0), (8, 22), (8, 0)])


def test_window_of_requantized_weight_gradients():
    # the window as the path produces it: wgrad outputs requantized to <8,5> with SR, one per batch
    L = wk.config2(batch=4)
    s = L.shape
    from paper_2107_13490_amd import ConvDesc, Epilogue
    d = ConvDesc(s.n, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad)
    qx = ctx().quantize(dev(L.x), 8, 5, pkg.SR, 0, 1)[0]
    grads, host_grads = [], []
    for b in range(6):
        dy = wk.normal(L.dy.shape, 0.25, 100 + b, 3)
        qdy = ctx().quantize(dev(dy), 8, 5, pkg.SR, 0, 3 + b)[0]
        g = ctx().conv_wgrad(d, qdy, (8, 5), qx, (8, 5), Epilogue.requant(8, 7, pkg.SR, 0, 50 + b))
        grads.append(g)
        host_grads.append(host(g).reshape(-1))
    out, sums = ctx().gradient_diversity([g.view(-1) for g in grads], [(8, 7)] * 6)
    ref = pu.gradient_diversity_np([c.astype(np.int64) for c in host_grads], [7] * 6)
    assert host(out)[0] == pytest.approx(ref["ds"], rel=1e-12)
    assert 1.0 <= ref["ds"] <= 6.0


def test_invalid_arguments():
    g = dev(np.zeros(64, dtype=np.int8))
    with pytest.raises(pkg.AdaptError):
        ctx().gradient_diversity([g], [(33, 3)])
    with pytest.raises(pkg.AdaptError):
        ctx().gradient_diversity([g] * 65, [(8, 3)] * 65)
    with pytest.raises(pkg.AdaptError):                      # 2^15 * 2^16 exceeds the 32-bit element sum
        ctx().gradient_diversity([dev(np.zeros(64, dtype=np.int16)), g], [(16, 0), (8, 16)])
    with pytest.raises(pkg.AdaptError):
        ctx().gradient_diversity([], [])
