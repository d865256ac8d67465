"""GPU parity: the element-wise steps of a chained step above 16 bits (int32 codes, 128-bit accumulators): pooling
and its gradient routing, the fitting requantization, the fused update and the gradient diversity, against the CPU
oracle, bit for bit."""
import numpy as np
import pytest
import torch

import paper_2107_13490_amd as pkg
from oracle import fxp_oracle as orc
from oracle import net_oracle as no
from oracle import wide_oracle as wo

from gpu_util import ctx, dev, host

pytestmark = pytest.mark.gpu


def _dt(wl):
    return np.int8 if wl <= 8 else np.int16 if wl <= 16 else np.int32


def _codes(g, shape, wl):
    lim = 1 << (wl - 1)
    a = g.integers(-lim, lim, shape, dtype=np.int64)
    flat = a.reshape(-1)
    if flat.size >= 4:
        flat[0], flat[1], flat[2] = lim - 1, -lim, 0
    return a


def _to_i128(values):
    """Python integers -> int64 array [n, 2] (low word, high word), two's complement."""
    out = np.empty((len(values), 2), dtype=np.int64)
    for i, v in enumerate(values):
        u = int(v) & ((1 << 128) - 1)
        lo, hi = u & ((1 << 64) - 1), u >> 64
        out[i, 0] = lo - (1 << 64) if lo >= 1 << 63 else lo
        out[i, 1] = hi - (1 << 64) if hi >= 1 << 63 else hi
    return out


def _u128(t):
    a = host(t).astype(np.int64)
    return (int(a[1]) & ((1 << 64) - 1)) * (1 << 64) + (int(a[0]) & ((1 << 64) - 1))


@pytest.mark.parametrize("wl", [17, 24, 32])
@pytest.mark.parametrize("shape", [(2, 4, 6, 8), (3, 2, 2, 5), (1, 8, 8, 3)])
def test_pooling_and_gradient_routing_of_int32_codes(wl, shape):
    g = np.random.default_rng(wl * 10 + shape[3])
    y = _codes(g, shape, wl)
    y[g.random(shape) < 0.3] = 0
    y[0, 0:2, 0:2, 0] = 12345                                  # a window of equal maxima
    n, h, w, c = shape
    a = ctx().maxpool2_fwd(dev(y.astype(np.int32)), wl)
    assert np.array_equal(host(a).astype(np.int64), no.maxpool2(y))
    for relu in (False, True):
        da = _codes(g, (n, h // 2, w // 2, c), wl)
        got = ctx().relu_pool_bwd(dev(da.astype(np.int32)), dev(y.astype(np.int32)), wl, relu, True)
        assert np.array_equal(host(got).astype(np.int64), no.relu_pool_bwd(da, y, relu, True))
        da = _codes(g, shape, wl)
        got = ctx().relu_pool_bwd(dev(da.astype(np.int32)), dev(y.astype(np.int32)), wl, relu, False)
        assert np.array_equal(host(got).astype(np.int64), no.relu_pool_bwd(da, y, relu, False))


@pytest.mark.parametrize("wl", [5, 16, 17, 23, 32])
@pytest.mark.parametrize("top", [20, 63, 90, 126])
@pytest.mark.parametrize("mode", [orc.SR, orc.RN_HALF_UP])
def test_fitting_requantization_of_128_bit_accumulators(wl, top, mode):
    g = np.random.default_rng(wl * 1000 + top)
    n = 3001
    mant = g.integers(-(1 << 62), 1 << 62, n)
    vals = [(int(m) << top) >> 62 for m in mant]               # magnitudes up to 2^top, all bit positions used
    vals[7] = (1 << top) - 1
    vals[8] = -(1 << top) + 1
    vals[9] = 0
    acc = dev(_to_i128(vals))
    q, shift, sumsq = ctx().requantize_fit(acc, wl, mode, 5, 77, acc_bits=128)
    want, sh, ss = wo.requantize_fit(np.array(vals, dtype=object), wl, mode, 5, 77)
    assert int(host(shift)[0]) == sh
    assert np.array_equal(host(q).astype(np.int64), want)
    assert (_u128(sumsq) if wl > 16 else int(host(sumsq).view(np.uint64)[0])) == ss


@pytest.mark.parametrize("wl", [17, 32])
def test_fitting_narrow_accumulators_to_wide_codes_and_empty_input(wl):
    g = np.random.default_rng(wl)
    for dt, lim in ((np.int32, 31), (np.int64, 63)):
        vals = g.integers(-(1 << lim), (1 << lim) - 1, 1025).astype(dt)
        q, shift, sumsq = ctx().requantize_fit(dev(vals), wl, orc.SR, 1, 2)
        want, sh, ss = wo.requantize_fit(vals.astype(object), wl, orc.SR, 1, 2)
        assert int(host(shift)[0]) == sh and np.array_equal(host(q).astype(np.int64), want) and _u128(sumsq) == ss
    q, shift, sumsq = ctx().requantize_fit(dev(np.zeros((0, 2), np.int64)), wl, orc.SR, 1, 2, acc_bits=128)
    assert int(host(shift)[0]) == 0 and _u128(sumsq) == 0 and q.numel() == 0


def test_sum_of_squares_beyond_64_bits():
    vals = [(1 << 31) - 1] * 5000 + [-(1 << 31)] * 5000          # 10000 squares of about 2^62
    q, shift, sumsq = ctx().requantize_fit(dev(_to_i128(vals)), 32, orc.RN_HALF_UP, 0, 0, acc_bits=128)
    assert int(host(shift)[0]) == 1                               # 2^31 needs 32 magnitude bits
    want, sh, ss = wo.requantize_fit(np.array(vals, dtype=object), 32, orc.RN_HALF_UP, 0, 0)
    assert np.array_equal(host(q).astype(np.int64), want) and _u128(sumsq) == ss
    vals = [(1 << 31) - 1] * 9000
    q, shift, sumsq = ctx().requantize_fit(dev(_to_i128(vals)), 32, orc.RN_HALF_UP, 0, 0, acc_bits=128)
    assert int(host(shift)[0]) == 0 and _u128(sumsq) == 9000 * ((1 << 31) - 1) ** 2 and _u128(sumsq) > 1 << 64


def _pair(v):
    """A non-negative Python integer below 2^128 -> device int64[2] (low word first)."""
    return dev(_to_i128([v])[0])


@pytest.mark.parametrize("n", [1, 9, 2048, 70003])
@pytest.mark.parametrize("gwl,wl,fl", [(32, 32, 28), (24, 8, 5), (8, 24, 20), (17, 17, 12), (32, 16, 12), (12, 32, 30)])
def test_fused_update_with_wide_gradient_codes_or_wide_weight_codes(n, gwl, wl, fl):
    from oracle import sgd_oracle as so
    g = np.random.default_rng(n + gwl * 100 + wl)
    w = (g.standard_normal(n) * 0.2).astype(np.float32)
    c = _codes(g, n, gwl)
    ss = sum(int(v) ** 2 for v in c)
    sumsq = _pair(ss) if gwl > 16 else dev(np.array([ss], dtype=np.uint64).view(np.int64))
    wd = dev(w.copy())
    q, cnt, rr = ctx().sgd_update_quantize(wd, dev(c.astype(_dt(gwl))), (gwl, 0), 0.05, 1e-4, 5e-3, wl, fl, g_sumsq=sumsq, seed=3, stream=n)
    ref = so.sgd_update_quantize(w, c, 0, 0.05, 1e-4, 5e-3, wl, fl, orc.SR, 3, n, True)
    assert ref["sumsq"] == ss
    assert np.array_equal(host(wd).view(np.uint32), ref["w"].view(np.uint32))
    assert np.array_equal(host(q).astype(np.int64), ref["q"])
    assert host(cnt).view(np.uint64).tolist() == [ref["nnz"], ref["sat"]]
    assert tuple(host(rr).tolist()) == (ref["lo"], ref["hi"])


def test_fused_update_wide_unnormalised_nearest_and_saturation():
    from oracle import sgd_oracle as so
    g = np.random.default_rng(5)
    n = 1000
    w = (g.standard_normal(n) * 3.0).astype(np.float32)          # <20,18> holds |w| < 2: many saturate
    c = _codes(g, n, 20)
    wd = dev(w.copy())
    q, cnt, rr = ctx().sgd_update_quantize(wd, dev(c.astype(np.int32)), (20, 22), 0.5, 0.0, 0.0, 20, 18, g_sumsq=None,
                                           mode=pkg.RN_HALF_UP)
    ref = so.sgd_update_quantize(w, c, 22, 0.5, 0.0, 0.0, 20, 18, orc.RN_HALF_UP, 0, 0, False)
    assert ref["sat"] > 100
    assert np.array_equal(host(wd).view(np.uint32), ref["w"].view(np.uint32)) and np.array_equal(host(q).astype(np.int64), ref["q"])
    assert host(cnt).view(np.uint64).tolist() == [ref["nnz"], ref["sat"]]


def test_step_from_a_sum_of_squares_that_needs_rounding_to_a_double():
    from oracle import sgd_oracle as so
    # sums just below / at / above ties of the 53-bit grid at 2^100
    c = np.array([1, -1, 0, 5], np.int64)
    w = np.array([0.5, 0.25, -1.0, 2.0], np.float32)
    for ss in ((1 << 100) + (1 << 47), (1 << 100) + (1 << 47) + 1, (1 << 100) + 3 * (1 << 47), (1 << 127) + (1 << 74) - 1, (1 << 64),
               (1 << 64) - 1, 12345):
        wd = dev(w.copy())
        ctx().sgd_update_quantize(wd, dev(c.astype(np.int32)), (32, 0), 2.0 ** 60, 0.0, 0.0, 16, 8, g_sumsq=_pair(ss), mode=pkg.RN_HALF_UP)
        step = so.sgd_step_size(2.0 ** 60, 0, ss)
        want = so.fma32(-step, c.astype(np.float32), w)
        assert np.array_equal(host(wd).view(np.uint32), want.view(np.uint32)), ss


def _pairs(t, count):
    a = host(t).astype(np.int64)
    return [(int(a[2 * k + 1]) & ((1 << 64) - 1)) * (1 << 64) + (int(a[2 * k]) & ((1 << 64) - 1)) for k in range(count)]


@pytest.mark.parametrize("n", [1, 15, 16, 17, 4095, 4096, 4097, 50021])
@pytest.mark.parametrize("fmts", [[(32, 0)], [(32, 3), (32, 0), (32, 7)], [(24, 5), (8, 2), (16, 9), (17, 0)], [(20, 0)] * 9,
                                  [(32, 0), (32, 16)], [(18, 20), (4, 0)]])
def test_gradient_diversity_of_windows_with_int32_codes(n, fmts):
    g = np.random.default_rng(n + len(fmts))
    codes = [_codes(g, n, wl) for wl, _ in fmts]
    out, sums = ctx().gradient_diversity([dev(c.astype(_dt(wl))) for c, (wl, _) in zip(codes, fmts)], fmts)
    ref = wo.gradient_diversity(codes, [f for _, f in fmts])
    got = _pairs(sums, len(fmts) + 1)
    assert got[:-1] == ref["sumsq"] and got[-1] == ref["sumsq_sum"]
    ds, log_ds = host(out).tolist()
    assert abs(ds - ref["ds"]) <= 1e-12 * abs(ref["ds"]) and abs(log_ds - ref["log_ds"]) <= 1e-12 * max(1.0, abs(ref["log_ds"]))


def test_gradient_diversity_wide_limits_and_degenerate_windows():
    z = dev(np.zeros(100, np.int32))
    out, sums = ctx().gradient_diversity([z, z], [(32, 0), (32, 0)])
    ds, log_ds = host(out).tolist()
    assert np.isnan(ds) and log_ds == 1.0 and _pairs(sums, 3) == [0, 0, 0]
    a = dev(np.full(100, 5, np.int32))
    out, _ = ctx().gradient_diversity([a, dev(np.full(100, -5, np.int32))], [(20, 0), (20, 0)])
    assert host(out).tolist() == [float("inf"), 1.0]
    with pytest.raises(pkg.AdaptError):                      # 2^31 * 2^17 reaches the 2^48 bound of the element sum
        ctx().gradient_diversity([a, a], [(32, 0), (32, 17)])
    ctx().gradient_diversity([a, a], [(32, 0), (31, 16)])     # 2^31 + 2^46 < 2^48
    with pytest.raises(pkg.AdaptError):
        ctx().gradient_diversity([a], [(33, 0)])


def test_batched_quantize_with_items_above_sixteen_bits():
    g = np.random.default_rng(77)
    fmts = [(8, 5), (24, 20), (12, 9), (32, 28), (17, 10), (4, 1), (32, 0)]
    sizes = [1000, 4099, 7, 70001, 8, 0, 513]
    xs = [(g.standard_normal(n) * (3.0 if t == 4 else 0.7)).astype(np.float32) for t, n in enumerate(sizes)]
    xs[3][5] = np.nan
    xs[3][6] = np.inf
    streams = [11 * t + 3 for t in range(len(xs))]
    dx = [dev(x) for x in xs]
    outs, counters = ctx().quantize_batched(dx, fmts, streams, seed=9)
    cnt = host(counters).view(np.uint64).reshape(-1, 2)
    for t, (x, (wl, fl)) in enumerate(zip(xs, fmts)):
        q, nnz, sat = orc.quantize(x, wl, fl, orc.SR, 9, streams[t])
        assert outs[t].dtype == (torch.int8 if wl <= 8 else torch.int16 if wl <= 16 else torch.int32)
        assert np.array_equal(host(outs[t]).astype(np.int64), q), t
        assert cnt[t].tolist() == [nnz, sat], t
    ranges = torch.empty(2 * len(xs), dtype=torch.float32, device="cuda")
    outs, counters = ctx().quantize_batched(dx, fmts, streams, seed=9, ranges=ranges, range_of=[0, 1, 3, 6])
    r = host(ranges).reshape(-1, 2)
    for t, x in enumerate(xs):
        fin = x[np.isfinite(x)]
        want = (float(fin.min()), float(fin.max())) if t in (0, 1, 3, 6) and fin.size else (np.inf, -np.inf)
        assert tuple(r[t].tolist()) == want, t
        assert np.array_equal(host(outs[t]).astype(np.int64), orc.quantize(x, fmts[t][0], fmts[t][1], orc.SR, 9, streams[t])[0]), t


@pytest.mark.parametrize("n", [1, 9, 4099])
@pytest.mark.parametrize("fa,fb,fo", [((32, 31), (32, 0), (32, 0)), ((24, 5), (12, 9), (32, 28)), ((8, 5), (32, 20), (17, 3)), ((20, 10), (20, 10), (8, 0)),
                                      ((16, 12), (8, 3), (24, 20))])
def test_residual_addition_with_int32_codes(n, fa, fb, fo):
    g = np.random.default_rng(n + fa[0] + fo[0])
    a, b = _codes(g, n, fa[0]), _codes(g, n, fb[0])
    for relu in (False, True):
        got = ctx().residual_add(dev(a.astype(_dt(fa[0]))), fa, dev(b.astype(_dt(fb[0]))), fb, fo, seed=5, stream=n, relu=relu)
        want = no.residual_add(a, fa[1], b, fb[1], fo[0], fo[1], orc.SR, 5, n, relu)
        assert got.dtype == (torch.int8 if fo[0] <= 8 else torch.int16 if fo[0] <= 16 else torch.int32)
        assert np.array_equal(host(got).astype(np.int64), want)
