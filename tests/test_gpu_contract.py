"""GPU parity: integer GEMM and convolution forward / data gradient / weight gradient against
the CPU oracle, bit for bit (exact accumulators and requantized outputs).  The contractions are
the quantized layer compute of Alg. 1; requantization applies the SR rule of Sec. 3.2 to the
accumulator."""
import numpy as np
import pytest
import torch

import paper_2107_13490_amd as pkg
import workloads as wk
from oracle import conv_oracle as co
from oracle import fxp_oracle as orc
from paper_2107_13490_amd import ConvDesc, Epilogue

from gpu_util import ctx, dev, host

pytestmark = pytest.mark.gpu


def codes(shape, wl, seed, extreme=False):
    g = np.random.default_rng(seed)
    lo, hi = -(1 << (wl - 1)), (1 << (wl - 1)) - 1
    if extreme:
        a = g.choice(np.array([lo, hi, lo + 1, hi - 1, 0, -1, 1, 127, 128, -128, -129, 255, 256, 32639, 32640]).clip(lo, hi), shape)
    else:
        a = g.integers(lo, hi + 1, shape)
    return a.astype(np.int8 if wl <= 8 else np.int16)


def to_dev(a):
    return dev(a)


# ------------------------------------------------------------------------------------ GEMM

def test_config1_gemm():
    a, b = wk.config1_gemm()
    qa, _, _ = orc.quantize(a, 8, 6, orc.SR, 0, 1)
    qb, _, _ = orc.quantize(b, 8, 6, orc.SR, 0, 2)
    c = ctx().fxp_gemm(to_dev(qa.astype(np.int8)), (8, 6), to_dev(qb.astype(np.int8)), (8, 6), Epilogue.exact())
    got = host(c)
    assert got.dtype == np.int32
    assert np.array_equal(got.astype(np.int64), co.gemm(qa, qb))
    # the whole path: quantize on the GPU, then multiply
    da, _ = ctx().quantize(dev(a), 8, 6, pkg.SR, 0, 1)
    db, _ = ctx().quantize(dev(b), 8, 6, pkg.SR, 0, 2)
    c2 = ctx().fxp_gemm(da, (8, 6), db, (8, 6), Epilogue.exact())
    assert np.array_equal(host(c2), got)


GEMM_SHAPES = [(1, 1, 1), (5, 3, 7), (77, 45, 33), (128, 64, 64), (129, 65, 65), (256, 192, 576), (300, 130, 1000),
               (64, 256, 16), (33, 500, 48), (16, 16, 0)]


@pytest.mark.parametrize("m,n,k", GEMM_SHAPES)
@pytest.mark.parametrize("wla,wlb", [(8, 8), (12, 12), (16, 16), (8, 16), (13, 4)])
def test_gemm_shapes_and_word_lengths(m, n, k, wla, wlb):
    a = codes((m, k), wla, m + k, extreme=(m % 2 == 1))
    b = codes((k, n), wlb, n + k + 1, extreme=(n % 2 == 1))
    want = orc.gemm(a, b)
    c = ctx().fxp_gemm(to_dev(a), (wla, 3), to_dev(b), (wlb, 2), Epilogue.exact())
    got = host(c)
    bits = 32 if k * 2 ** (wla + wlb - 2) <= 2 ** 31 - 1 else 64
    assert got.dtype == (np.int32 if bits == 32 else np.int64)
    assert np.array_equal(got.astype(np.int64), want)


@pytest.mark.parametrize("ta,tb", [(0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("m,n,k,wl", [(64, 64, 64, 8), (100, 36, 52, 8), (37, 29, 19, 8), (96, 160, 48, 14)])
def test_gemm_transposes(ta, tb, m, n, k, wl):
    a = codes((m, k), wl, 1)
    b = codes((k, n), wl, 2)
    want = orc.gemm(a, b)
    da = to_dev(a.T.copy() if ta else a)
    db = to_dev(b.T.copy() if tb else b)
    c = ctx().fxp_gemm(da, (wl, 0), db, (wl, 0), Epilogue.exact(), trans_a=bool(ta), trans_b=bool(tb))
    assert np.array_equal(host(c).astype(np.int64), want)


def test_gemm_leading_dimensions():
    a = codes((70, 128), 8, 3)
    b = codes((96, 80), 8, 4)
    da, db = to_dev(a)[:, :96], to_dev(b)[:, :48]        # lda = 128, ldb = 80
    out = torch.full((70, 64), 7, dtype=torch.int32, device="cuda")
    c = ctx().fxp_gemm(da, (8, 0), db, (8, 0), Epilogue.exact(), out=out[:, :48])
    want = orc.gemm(a[:, :96], b[:, :48])
    got = host(out)
    assert np.array_equal(got[:, :48].astype(np.int64), want) and (got[:, 48:] == 7).all()


def test_gemm_worst_case_accumulation():
    # every product is +2^14 (or 2^30 for 16 bit): the int32 accumulators run at their bound
    k = 4096
    a = np.full((64, k), -128, dtype=np.int8)
    b = np.full((k, 64), -128, dtype=np.int8)
    c = ctx().fxp_gemm(to_dev(a), (8, 0), to_dev(b), (8, 0), Epilogue.exact())
    assert (host(c) == k * 16384).all()
    a16 = np.full((64, k), -32768, dtype=np.int16)
    b16 = np.full((k, 64), -32768, dtype=np.int16)
    c = ctx().fxp_gemm(to_dev(a16), (16, 0), to_dev(b16), (16, 0), Epilogue.exact())
    assert host(c).dtype == np.int64 and (host(c) == k * (1 << 30)).all()
    b16[:] = 32767
    c = ctx().fxp_gemm(to_dev(a16), (16, 0), to_dev(b16), (16, 0), Epilogue.exact())
    assert (host(c) == k * (-32768 * 32767)).all()


def test_gemm_long_k_is_split():
    k = 200000
    a = codes((32, k), 8, 5)
    b = codes((k, 48), 8, 6)
    c = ctx().fxp_gemm(to_dev(a), (8, 0), to_dev(b), (8, 0), Epilogue.exact())
    assert host(c).dtype == np.int64
    assert np.array_equal(host(c), orc.gemm(a, b))


@pytest.mark.parametrize("wl_o,fl_o,mode,relu", [(8, 4, pkg.SR, False), (8, 6, pkg.RN_HALF_UP, True), (16, 10, pkg.SR, True),
                                                 (12, 12, pkg.SR, False), (8, 0, pkg.SR, False), (16, 14, pkg.SR, False),
                                                 (4, 1, pkg.SR, False)])
@pytest.mark.parametrize("m,n,k,wl", [(130, 192, 96, 8), (64, 40, 33, 8), (100, 64, 128, 12)])
def test_gemm_requantize_epilogue(wl_o, fl_o, mode, relu, m, n, k, wl):
    fa, fb = 6, 6
    a = codes((m, k), wl, 11)
    b = codes((k, n), wl, 12)
    ep = Epilogue.requant(wl_o, fl_o, mode, seed=21, stream=5, relu=relu)
    c = ctx().fxp_gemm(to_dev(a), (wl, fa), to_dev(b), (wl, fb), ep)
    want = orc.requantize(orc.gemm(a, b), fa + fb - fl_o, wl_o, mode, 21, 5, relu)
    got = host(c)
    assert got.dtype == (np.int8 if wl_o <= 8 else np.int16)
    assert np.array_equal(got.astype(np.int64), want)


def test_requantize_wide_shift():
    a = codes((64, 256), 16, 13)
    b = codes((256, 64), 16, 14)
    ep = Epilogue.requant(16, 2, pkg.SR, seed=1, stream=1)
    c = ctx().fxp_gemm(to_dev(a), (16, 12), to_dev(b), (16, 12), ep)           # shift 22
    want = orc.requantize(orc.gemm(a, b), 22, 16, orc.SR, 1, 1)
    assert np.array_equal(host(c).astype(np.int64), want)


# ------------------------------------------------------------------------------------ convolutions

CONV_CASES = [
    # n, h, w, c, k, r, s, stride, pad
    (2, 8, 8, 16, 32, 3, 3, 1, 1),
    (3, 7, 5, 32, 16, 3, 3, 1, 1),
    (2, 9, 9, 16, 48, 3, 3, 2, 1),
    (2, 6, 6, 64, 64, 1, 1, 1, 0),
    (1, 8, 8, 32, 32, 1, 1, 2, 0),
    (2, 10, 10, 16, 16, 5, 5, 1, 2),
    (2, 8, 8, 3, 8, 3, 3, 1, 1),          # Cin = 3: element-wise gather path
    (2, 5, 6, 20, 12, 3, 3, 1, 0),        # C multiple of 4 only
    (1, 4, 4, 7, 5, 2, 2, 1, 1),          # nothing aligned
    (9, 1, 1, 256, 100, 1, 1, 1, 0),      # fully connected layer
    (2, 12, 12, 16, 32, 7, 7, 2, 3),      # 49 filter taps: beyond the per-row tap masks of the vector path
    (2, 9, 9, 32, 32, 5, 5, 2, 2),        # 25 taps, stride 2
]


def _conv_all(case, wlx, wlw, wldy, extreme=False):
    n, h, w, c, k, r, s, st, pad = case
    d = ConvDesc(n, h, w, c, k, r, s, st, pad)
    x = codes((n, h, w, c), wlx, 1, extreme)
    wt = codes((k, r, s, c), wlw, 2, extreme)
    dy = codes((n, d.p, d.q, k), wldy, 3, extreme)
    y = ctx().conv_fwd(d, to_dev(x), (wlx, 4), to_dev(wt), (wlw, 5), Epilogue.exact())
    assert np.array_equal(host(y).astype(np.int64), co.conv_fwd(x, wt, st, pad))
    dx = ctx().conv_dgrad(d, to_dev(dy), (wldy, 4), to_dev(wt), (wlw, 5), Epilogue.exact())
    assert np.array_equal(host(dx).astype(np.int64), co.conv_dgrad(dy, wt, h, w, st, pad))
    dw = ctx().conv_wgrad(d, to_dev(dy), (wldy, 4), to_dev(x), (wlx, 4), Epilogue.exact())
    assert np.array_equal(host(dw).astype(np.int64), co.conv_wgrad(dy, x, r, s, st, pad))


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_one_limb(case):
    _conv_all(case, 8, 8, 8)
    _conv_all(case, 4, 6, 8, extreme=True)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_two_limb(case):
    _conv_all(case, 12, 12, 12)
    _conv_all(case, 16, 16, 16, extreme=True)


@pytest.mark.parametrize("case", CONV_CASES[:4])
def test_conv_mixed_word_lengths(case):
    _conv_all(case, 8, 12, 16)
    _conv_all(case, 16, 8, 9)


COUT_CASES = [(3, 6, 6, 32, 10, 3, 3, 1, 1), (2, 8, 8, 16, 100, 3, 3, 2, 1), (5, 1, 1, 4096, 10, 1, 1, 1, 0), (2, 5, 7, 64, 17, 1, 1, 1, 0),
              (2, 6, 6, 16, 130, 3, 3, 1, 1), (300, 1, 1, 512, 100, 1, 1, 1, 0), (2, 9, 9, 32, 24, 5, 5, 2, 2)]


@pytest.mark.parametrize("case", COUT_CASES)
@pytest.mark.parametrize("wl", [8, 12, 16])
def test_output_channels_that_are_not_a_multiple_of_sixteen(case, wl):
    """The gradient contractions read dy through a copy with zero channels appended; results and rounding indices
    are those of the plain definition."""
    n, h, w, c, k, r, s, st, pad = case
    d = ConvDesc(n, h, w, c, k, r, s, st, pad)
    x, wt, dy = codes((n, h, w, c), wl, 1, True), codes((k, r, s, c), wl, 2, True), codes((n, d.p, d.q, k), wl, 3, True)
    dx_ref, dw_ref = co.conv_dgrad(dy, wt, h, w, st, pad), co.conv_wgrad(dy, x, r, s, st, pad)
    f = (wl, 4)
    dx = ctx().conv_dgrad(d, to_dev(dy), f, to_dev(wt), f, Epilogue.exact())
    dw = ctx().conv_wgrad(d, to_dev(dy), f, to_dev(x), f, Epilogue.exact())
    assert np.array_equal(host(dx).astype(np.int64), dx_ref) and np.array_equal(host(dw).astype(np.int64), dw_ref)
    bx, bw = ctx().conv_backward(d, to_dev(dy), f, to_dev(wt), f, to_dev(x), f, Epilogue.exact(), Epilogue.exact())
    assert np.array_equal(host(bx).astype(np.int64), dx_ref) and np.array_equal(host(bw).astype(np.int64), dw_ref)
    ep1, ep2 = Epilogue.requant(wl, 2, pkg.SR, seed=4, stream=21), Epilogue.requant(wl, 0, pkg.SR, seed=4, stream=22)
    bx, bw = ctx().conv_backward(d, to_dev(dy), f, to_dev(wt), f, to_dev(x), f, ep1, ep2)
    assert np.array_equal(host(bx).astype(np.int64), orc.requantize(dx_ref, 6, wl, orc.SR, 4, 21))
    assert np.array_equal(host(bw).astype(np.int64), orc.requantize(dw_ref, 8, wl, orc.SR, 4, 22))


def _layer_codes(L):
    qx, _, _ = orc.quantize(L.x, L.wl, L.fl, orc.SR, 0, 1)
    qw, _, _ = orc.quantize(L.w, L.wl, L.fl, orc.SR, 0, 2)
    qdy, _, _ = orc.quantize(L.dy, L.wl, L.fl, orc.SR, 0, 3)
    t = np.int8 if L.wl <= 8 else np.int16
    return qx.astype(t), qw.astype(t), qdy.astype(t)


def _layer_check(L, requant):
    s = L.shape
    d = ConvDesc(s.n, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad)
    qx, qw, qdy = _layer_codes(L)
    f = (L.wl, L.fl)
    dx_, dw_, ddy_ = to_dev(qx), to_dev(qw), to_dev(qdy)
    y_ref = co.conv_fwd(qx, qw, s.stride, s.pad)
    dx_ref = co.conv_dgrad(qdy, qw, s.h, s.w, s.stride, s.pad)
    dw_ref = co.conv_wgrad(qdy, qx, s.r, s.s, s.stride, s.pad)
    y = ctx().conv_fwd(d, dx_, f, dw_, f, Epilogue.exact())
    dx = ctx().conv_dgrad(d, ddy_, f, dw_, f, Epilogue.exact())
    dw = ctx().conv_wgrad(d, ddy_, f, dx_, f, Epilogue.exact())
    assert np.array_equal(host(y).astype(np.int64), y_ref)
    assert np.array_equal(host(dx).astype(np.int64), dx_ref)
    assert np.array_equal(host(dw).astype(np.int64), dw_ref)
    if requant:
        # the configuration the benchmark times: outputs requantized to the layer format
        for stream, (fn, args, ref, relu) in enumerate((
                (ctx().conv_fwd, (dx_, f, dw_, f), y_ref, True),
                (ctx().conv_dgrad, (ddy_, f, dw_, f), dx_ref, False),
                (ctx().conv_wgrad, (ddy_, f, dx_, f), dw_ref, False))):
            ep = Epilogue.requant(L.wl, L.fl, pkg.SR, seed=0, stream=10 + stream, relu=relu)
            got = host(fn(d, *args, ep)).astype(np.int64)
            want = orc.requantize(ref, L.fl, L.wl, orc.SR, 0, 10 + stream, relu)
            assert np.array_equal(got, want)


def test_config2_full_size():
    _layer_check(wk.config2(), requant=True)


def test_config3_reduced_batch():
    _layer_check(wk.config3(batch=16), requant=True)


def test_config3_full_size_sampled():
    """Full batch 256 in the launch configuration the benchmark uses.  fwd and dgrad are
    independent per image: the oracle computes a sample of images one by one; wgrad sums over
    the whole batch and is compared in full."""
    L = wk.config3()
    s = L.shape
    d = ConvDesc(s.n, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad)
    qx, qw, qdy = _layer_codes(L)
    f = (L.wl, L.fl)
    dx_, dw_, ddy_ = to_dev(qx), to_dev(qw), to_dev(qdy)
    y = host(ctx().conv_fwd(d, dx_, f, dw_, f, Epilogue.exact()))
    dx = host(ctx().conv_dgrad(d, ddy_, f, dw_, f, Epilogue.exact()))
    dw = host(ctx().conv_wgrad(d, ddy_, f, dx_, f, Epilogue.exact()))
    for img in (0, 1, 100, 254, 255):
        assert np.array_equal(y[img:img + 1].astype(np.int64), co.conv_fwd(qx[img:img + 1], qw, 1, 1))
        assert np.array_equal(dx[img:img + 1].astype(np.int64), co.conv_dgrad(qdy[img:img + 1], qw, s.h, s.w, 1, 1))
    assert np.array_equal(dw.astype(np.int64), co.conv_wgrad(qdy, qx, 3, 3, 1, 1))


def test_invalid_arguments():
    a = torch.zeros((16, 16), dtype=torch.int8, device="cuda")
    with pytest.raises(pkg.AdaptError):
        ctx().fxp_gemm(a, (33, 0), a, (8, 0), Epilogue.exact())
    with pytest.raises(pkg.AdaptError):
        ctx().fxp_gemm(a, (8, 0), a, (8, 0), Epilogue.requant(33, 0))
    with pytest.raises(pkg.AdaptError):
        ctx().fxp_gemm(a, (8, 32), a, (8, 0), Epilogue.exact())
    d = ConvDesc(1, 2, 2, 16, 16, 5, 5, 1, 0)        # filter larger than the padded input
    with pytest.raises(pkg.AdaptError):
        ctx().conv_fwd(d, a, (8, 0), a, (8, 0), Epilogue.exact(), out=a)


# ------------------------------------------------------------------------------------ layer sweeps (configs 4 and 5)

def _sweep(specs, batch, seed):
    """Every layer of the network shape at reduced batch: quantize on the GPU with the layer's own
    <WL,FL>, then fwd / dgrad / wgrad, all against the oracle."""
    import dataclasses
    for li, spec in enumerate(specs):
        shp = dataclasses.replace(spec.shape, n=batch)
        L = wk.conv_layer(shp, spec.wl, spec.fl, seed + li, spec.zero_frac, spec.name)
        s = L.shape
        d = ConvDesc(s.n, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad)
        f = (L.wl, L.fl)
        (qx, qw, qdy), _ = ctx().quantize_batched([dev(L.x), dev(L.w), dev(L.dy)], [f, f, f], [1, 2, 3], pkg.SR, seed=0)
        hx, hw, hdy = host(qx), host(qw), host(qdy)
        for t, ref_in, stream in ((hx, L.x, 1), (hw, L.w, 2), (hdy, L.dy, 3)):
            want, _, _ = orc.quantize(ref_in, L.wl, L.fl, orc.SR, 0, stream)
            assert np.array_equal(t.astype(np.int64), want), spec.name
        y = ctx().conv_fwd(d, qx, f, qw, f, Epilogue.exact())
        dx = ctx().conv_dgrad(d, qdy, f, qw, f, Epilogue.exact())
        dw = ctx().conv_wgrad(d, qdy, f, qx, f, Epilogue.exact())
        assert np.array_equal(host(y).astype(np.int64), co.conv_fwd(hx, hw, s.stride, s.pad)), spec.name
        assert np.array_equal(host(dx).astype(np.int64), co.conv_dgrad(hdy, hw, s.h, s.w, s.stride, s.pad)), spec.name
        assert np.array_equal(host(dw).astype(np.int64), co.conv_wgrad(hdy, hx, s.r, s.s, s.stride, s.pad)), spec.name
        # requantized forward output in the layer's own format
        ep = Epilogue.requant(L.wl, L.fl, pkg.SR, seed=0, stream=20 + li, relu=True)
        yq = host(ctx().conv_fwd(d, qx, f, qw, f, ep)).astype(np.int64)
        want = orc.requantize(co.conv_fwd(hx, hw, s.stride, s.pad), L.fl, L.wl, orc.SR, 0, 20 + li, True)
        assert np.array_equal(yq, want), spec.name


def test_config4_alexnet_layer_sweep_reduced_batch():
    _sweep(wk.alexnet_cifar_layers(), batch=4, seed=40)


def test_config5_resnet18_layer_sweep_reduced_batch():
    _sweep(wk.resnet18_cifar_layers(), batch=2, seed=50)


# ---- both gradients in one call --------------------------------------------------------------------------

@pytest.mark.parametrize("shape,wl", [
    ((8, 16, 16, 64, 192, 3, 3, 1, 1), 8),      # config-2 layer, reduced batch: paired launch
    ((16, 16, 16, 128, 128, 3, 3, 1, 1), 8),    # 128-wide tiles
    ((4, 32, 32, 64, 64, 3, 3, 1, 1), 6),
    ((6, 16, 16, 64, 128, 3, 3, 2, 1), 8),      # stride 2
    ((5, 9, 7, 32, 48, 3, 3, 1, 1), 8),         # ragged tiles
    ((4, 8, 8, 256, 512, 1, 1, 2, 0), 4),       # 1x1 projection (64-deep stages: not paired)
    ((3, 12, 12, 3, 64, 3, 3, 1, 1), 8),        # 3 input channels: element-wise path, not paired
    ((4, 16, 16, 64, 64, 3, 3, 1, 1), 12),      # two limbs, 64-wide tiles: paired
    ((32, 32, 32, 128, 128, 1, 1, 1, 0), 12),   # two limbs, 128-wide data-gradient tile
    ((4, 16, 16, 64, 64, 3, 3, 1, 1), 16),
    ((2, 8, 8, 192, 384, 3, 3, 1, 1), 8),       # 192-wide data-gradient tile: not paired
])
def test_backward_equals_the_two_separate_calls(shape, wl):
    n, h, w_, c, k, r, s, stride, pad = shape
    rng = np.random.default_rng(sum(shape) + wl)
    lim = 1 << (wl - 1)
    dt = np.int8 if wl <= 8 else np.int16
    d = ConvDesc(n, h, w_, c, k, r, s, stride, pad)
    x = rng.integers(-lim, lim, (n, h, w_, c)).astype(dt)
    wt = rng.integers(-lim, lim, (k, r, s, c)).astype(dt)
    dy = rng.integers(-lim, lim, (n, d.p, d.q, k)).astype(dt)
    f = (wl, wl - 3)
    for ep_dx, ep_dw in ((Epilogue.requant(wl, wl - 3, pkg.SR, 0, 11), Epilogue.requant(wl, wl - 2, pkg.SR, 0, 12)),
                         (Epilogue.exact(), Epilogue.exact())):
        dx1 = ctx().conv_dgrad(d, dev(dy), f, dev(wt), f, ep_dx)
        dw1 = ctx().conv_wgrad(d, dev(dy), f, dev(x), f, ep_dw)
        dx2, dw2 = ctx().conv_backward(d, dev(dy), f, dev(wt), f, dev(x), f, ep_dx, ep_dw)
        assert torch.equal(dx1, dx2) and torch.equal(dw1, dw2)
    # and against the oracle directly (exact outputs)
    want_dx = co.conv_dgrad(dy.astype(np.int64), wt.astype(np.int64), h, w_, stride, pad)
    want_dw = co.conv_wgrad(dy.astype(np.int64), x.astype(np.int64), r, s, stride, pad)
    assert np.array_equal(host(dx2).astype(np.int64), want_dx) and np.array_equal(host(dw2).astype(np.int64), want_dw)


def test_backward_config2_full_size():
    L = wk.config2()
    s = L.shape
    d = ConvDesc(s.n, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad)
    f = (8, 5)
    qx, qw, qdy = (ctx().quantize(dev(t), 8, 5, pkg.SR, 0, i + 1)[0] for i, t in enumerate((L.x, L.w, L.dy)))
    ep_dx, ep_dw = Epilogue.requant(8, 5, pkg.SR, 0, 11), Epilogue.requant(8, 5, pkg.SR, 0, 12)
    dx1 = ctx().conv_dgrad(d, qdy, f, qw, f, ep_dx)
    dw1 = ctx().conv_wgrad(d, qdy, f, qx, f, ep_dw)
    for _ in range(3):
        dx2, dw2 = ctx().conv_backward(d, qdy, f, qw, f, qx, f, ep_dx, ep_dw)
        assert torch.equal(dx1, dx2) and torch.equal(dw1, dw2)


# ---- layers with fewer than 16 input channels run on zero-padded copies --------------------------------------

NARROW_CASES = [
    (3, 12, 10, 3, 64, 3, 3, 1, 1),     # the first layer of an image network
    (2, 9, 9, 1, 16, 3, 3, 1, 1),       # one channel
    (2, 8, 8, 15, 24, 3, 3, 2, 1),      # just below the vector width, stride 2
    (4, 6, 6, 5, 10, 1, 1, 1, 0),       # 1x1, nothing aligned
    (1, 16, 16, 8, 32, 5, 5, 1, 2),
]


@pytest.mark.parametrize("case", NARROW_CASES)
@pytest.mark.parametrize("wl", [8, 12])
def test_narrow_layers_exact_and_requantized(case, wl):
    n, h, w, c, k, r, s, st, pad = case
    d = ConvDesc(n, h, w, c, k, r, s, st, pad)
    x = codes((n, h, w, c), wl, 1)
    wt = codes((k, r, s, c), wl, 2)
    dy = codes((n, d.p, d.q, k), wl, 3)
    f = (wl, wl - 3)
    _conv_all(case, wl, wl, wl, extreme=True)
    # requantized outputs: the rounding bits follow the logical output index, not the padded one
    eps = [Epilogue.requant(wl, wl - 4, pkg.SR, 3, 30 + i, relu=(i == 0)) for i in range(3)]
    sh = 2 * (wl - 3) - (wl - 4)
    y = ctx().conv_fwd(d, to_dev(x), f, to_dev(wt), f, eps[0])
    assert np.array_equal(host(y).astype(np.int64), orc.requantize(co.conv_fwd(x, wt, st, pad), sh, wl, orc.SR, 3, 30, True))
    dx = ctx().conv_dgrad(d, to_dev(dy), f, to_dev(wt), f, eps[1])
    assert np.array_equal(host(dx).astype(np.int64), orc.requantize(co.conv_dgrad(dy, wt, h, w, st, pad), sh, wl, orc.SR, 3, 31))
    dw = ctx().conv_wgrad(d, to_dev(dy), f, to_dev(x), f, eps[2])
    want_dw = orc.requantize(co.conv_wgrad(dy, x, r, s, st, pad), sh, wl, orc.SR, 3, 32)
    assert np.array_equal(host(dw).astype(np.int64), want_dw)
    dx2, dw2 = ctx().conv_backward(d, to_dev(dy), f, to_dev(wt), f, to_dev(x), f, eps[1], eps[2])
    assert torch.equal(dx, dx2) and torch.equal(dw, dw2)


def test_narrow_layer_accumulator_type_follows_the_logical_reduction():
    # K = 3*3*3 = 27 fits int32 accumulators at <16,.> x <10,.>; the padded reduction (144) would not, and must not widen the output
    d = ConvDesc(2, 8, 8, 3, 16, 3, 3, 1, 1)
    fa, fb = (16, 8), (10, 5)
    assert pkg.acc_bits(27, pkg.Fmt(*fa), pkg.Fmt(*fb)) == 32 and pkg.acc_bits(144, pkg.Fmt(*fa), pkg.Fmt(*fb)) == 64
    x, wt = codes((2, 8, 8, 3), 16, 1, True), codes((16, 3, 3, 3), 10, 2, True)
    y = ctx().conv_fwd(d, to_dev(x), fa, to_dev(wt), fb, Epilogue.exact())
    assert y.dtype == torch.int32
    assert np.array_equal(host(y).astype(np.int64), co.conv_fwd(x, wt, 1, 1))


def test_narrow_layer_falls_back_when_the_workspace_is_small():
    small = pkg.Context(workspace_bytes=1 << 16)            # 60 KiB of scratch: the padded input does not fit
    n, h, w, c, k = 4, 32, 32, 3, 16
    d = ConvDesc(n, h, w, c, k, 3, 3, 1, 1)
    x, wt, dy = codes((n, h, w, c), 8, 1), codes((k, 3, 3, c), 8, 2), codes((n, h, w, k), 8, 3)
    y = small.conv_fwd(d, to_dev(x), (8, 4), to_dev(wt), (8, 5), Epilogue.exact())
    assert np.array_equal(host(y).astype(np.int64), co.conv_fwd(x, wt, 1, 1))
    dx = small.conv_dgrad(d, to_dev(dy), (8, 4), to_dev(wt), (8, 5), Epilogue.exact())
    assert np.array_equal(host(dx).astype(np.int64), co.conv_dgrad(dy, wt, h, w, 1, 1))
    small.close()


# ---- stride-2 data gradient: rows in parity-class order, stages of invisible taps skipped --------------------

STRIDE2_CASES = [
    # n, h, w, c, k, r, s, pad
    (2, 8, 8, 32, 64, 3, 3, 1),         # four classes of 32 rows: every 64-row tile straddles two classes
    (8, 8, 8, 32, 64, 3, 3, 1),         # classes of 128 rows: tiles inside one class
    (5, 12, 8, 16, 128, 3, 3, 1),       # ragged class size (120 rows): some tiles straddle
    (4, 16, 16, 64, 128, 1, 1, 0),      # 1x1 projection: three classes see no tap at all
    (3, 8, 8, 32, 64, 5, 5, 2),
    (3, 8, 8, 32, 64, 2, 2, 0),         # even filter: every class sees exactly one tap
    (4, 8, 8, 16, 64, 3, 3, 0),         # no padding
    (4, 8, 8, 48, 192, 3, 3, 1),        # one limb: 192-deep stages stay (Kout % 192 == 0)
    (4, 8, 8, 48, 256, 3, 3, 1),        # one limb: stages shortened to 64 for the skip
    (2, 6, 10, 3, 64, 3, 3, 1),         # narrow layer (padded filters) and stride 2
]


@pytest.mark.parametrize("case", STRIDE2_CASES)
@pytest.mark.parametrize("wl", [8, 13])
def test_stride2_data_gradient(case, wl):
    n, h, w, c, k, r, s, pad = case
    d = ConvDesc(n, h, w, c, k, r, s, 2, pad)
    wt = codes((k, r, s, c), wl, 2, True)
    dy = codes((n, d.p, d.q, k), wl, 3, True)
    x = codes((n, h, w, c), wl, 1)
    f = (wl, wl - 3)
    want = co.conv_dgrad(dy, wt, h, w, 2, pad)
    dx = ctx().conv_dgrad(d, to_dev(dy), f, to_dev(wt), f, Epilogue.exact())
    assert np.array_equal(host(dx).astype(np.int64), want)
    ep = Epilogue.requant(wl, wl - 5, pkg.SR, 9, 77)
    sh = 2 * (wl - 3) - (wl - 5)
    dxq = ctx().conv_dgrad(d, to_dev(dy), f, to_dev(wt), f, ep)
    assert np.array_equal(host(dxq).astype(np.int64), orc.requantize(want, sh, wl, orc.SR, 9, 77))
    # the paired backward call takes the same path
    dx2, dw2 = ctx().conv_backward(d, to_dev(dy), f, to_dev(wt), f, to_dev(x), f, ep, Epilogue.exact())
    assert torch.equal(dxq, dx2)
    assert np.array_equal(host(dw2).astype(np.int64), co.conv_wgrad(dy, x, r, s, 2, pad))


# ---- mixed word lengths: the int8 operand stays one limb inside the two-limb kernels -----------------------------

@pytest.mark.parametrize("case", CONV_CASES + NARROW_CASES[:2])
@pytest.mark.parametrize("wls", [(8, 16, 8), (16, 8, 16), (16, 8, 8), (5, 9, 13)])
def test_conv_mixed_one_and_two_limb_operands(case, wls):
    _conv_all(case, *wls, extreme=True)
    _conv_all(case, *wls)


@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("wla,wlb", [(8, 16), (16, 8)])
def test_gemm_mixed_worst_case_and_transposes(ta, tb, wla, wlb):
    m, n, k = 96, 160, 4096 + 64
    for va, vb in ((-1, -1), (-1, 1), (1, -1)):           # every product at its bound, all sign combinations
        a = np.full((m, k), -(1 << (wla - 1)) if va < 0 else (1 << (wla - 1)) - 1, dtype=np.int8 if wla <= 8 else np.int16)
        b = np.full((k, n), -(1 << (wlb - 1)) if vb < 0 else (1 << (wlb - 1)) - 1, dtype=np.int8 if wlb <= 8 else np.int16)
        da = to_dev(a.T.copy() if ta else a)
        db = to_dev(b.T.copy() if tb else b)
        c = ctx().fxp_gemm(da, (wla, 0), db, (wlb, 0), Epilogue.exact(), trans_a=bool(ta), trans_b=bool(tb))
        assert (host(c).astype(np.int64) == k * int(a[0, 0]) * int(b[0, 0])).all()
    a, b = codes((m, k), wla, 3, True), codes((k, n), wlb, 4, True)
    da = to_dev(a.T.copy() if ta else a)
    db = to_dev(b.T.copy() if tb else b)
    ep = Epilogue.requant(12, 0, pkg.SR, seed=2, stream=9)
    c = ctx().fxp_gemm(da, (wla, 7), db, (wlb, 7), ep, trans_a=bool(ta), trans_b=bool(tb))
    assert np.array_equal(host(c).astype(np.int64), orc.requantize(orc.gemm(a, b), 14, 12, orc.SR, 2, 9))


# ---- the full bench sizes (configs 4 and 5 at their own batch) against the oracle ----------------------------------

def _spread_samples(n, rows_per_sample):
    """First and last sample, and two neighbours in the middle of the batch that lie on either side of a boundary of
    the 64-, 128- and 256-row output tiles (samples smaller than a tile share tiles; larger ones span several)."""
    per_tile = max(1, 256 // rows_per_sample)
    k = max(1, (n // 2) // per_tile * per_tile)
    return sorted({0, k - 1, min(k, n - 1), n - 1})


def _full_batch_layer(spec, seed):
    """One layer at the batch the benchmark times, in the calls the benchmark makes (forward with the requantizing ReLU
    epilogue, both gradients through conv_backward), on the seeded workload tensors.  The oracle quantizes the same
    fp32 tensors (codes compared in full), computes the weight gradient in full and the forward output and data
    gradient, which treat samples independently, for samples spread over the batch."""
    from gpu_util import oracle_quantize
    L = wk.layer_inputs(spec, seed)
    s = L.shape
    d = ConvDesc(s.n, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad)
    f = (L.wl, L.fl)
    c = ctx()
    c.reserve_for_layers([(d, f, f, f)])
    (qx, qw, qdy), _ = c.quantize_batched([dev(L.x), dev(L.w), dev(L.dy)], [f, f, f], [1, 2, 3], pkg.SR, seed=0)
    hx, hw, hdy = (oracle_quantize(t, L.wl, L.fl, 0, i + 1) for i, t in enumerate((L.x, L.w, L.dy)))
    for got, want in ((qx, hx), (qw, hw), (qdy, hdy)):
        assert np.array_equal(host(got).astype(np.int64), want), spec.name
    eps = [Epilogue.requant(L.wl, L.fl, pkg.SR, 0, 10 + i, relu=(i == 0)) for i in range(3)]
    ex = Epilogue.exact()
    y, yq = host(c.conv_fwd(d, qx, f, qw, f, ex)), host(c.conv_fwd(d, qx, f, qw, f, eps[0]))
    dx, dw = (host(t) for t in c.conv_backward(d, qdy, f, qw, f, qx, f, ex, ex))
    dxq, dwq = (host(t) for t in c.conv_backward(d, qdy, f, qw, f, qx, f, eps[1], eps[2]))
    want_dw = co.conv_wgrad(hdy, hx, s.r, s.s, s.stride, s.pad)
    assert np.array_equal(dw.astype(np.int64), want_dw), spec.name
    assert np.array_equal(dwq.astype(np.int64), orc.requantize(want_dw, L.fl, L.wl, orc.SR, 0, 12)), spec.name
    per_y, per_x = s.p * s.q * s.k, s.h * s.w * s.c
    for i in _spread_samples(s.n, min(s.p * s.q, s.h * s.w)):
        want_y = co.conv_fwd(hx[i:i + 1], hw, s.stride, s.pad)
        assert np.array_equal(y[i:i + 1].astype(np.int64), want_y), (spec.name, i)
        assert np.array_equal(yq[i:i + 1].astype(np.int64), orc.requantize(want_y, L.fl, L.wl, orc.SR, 0, 10, True, start=i * per_y)), (spec.name, i)
        want_dx = co.conv_dgrad(hdy[i:i + 1], hw, s.h, s.w, s.stride, s.pad)
        assert np.array_equal(dx[i:i + 1].astype(np.int64), want_dx), (spec.name, i)
        assert np.array_equal(dxq[i:i + 1].astype(np.int64), orc.requantize(want_dx, L.fl, L.wl, orc.SR, 0, 11, False, start=i * per_x)), (spec.name, i)


@pytest.mark.parametrize("li", range(8))
def test_config4_full_batch_against_the_oracle(li):
    _full_batch_layer(wk.alexnet_cifar_layers()[li], 40 + li)


@pytest.mark.parametrize("li", range(21))
def test_config5_full_batch_against_the_oracle(li):
    _full_batch_layer(wk.resnet18_cifar_layers()[li], 50 + li)


# ---- workspace: sizing query, fewer splits when it is short, the accumulator bound ------------------------------------

def test_workspace_query_matches_what_the_calls_take():
    """A context created with exactly the bytes the query returns runs the call with its preferred plan; the result is
    the one a roomy context gives."""
    d = ConvDesc(16, 16, 16, 64, 64, 3, 3, 1, 1)
    f = (8, 5)
    x, wt, dy = codes((16, 16, 16, 64), 8, 1), codes((64, 3, 3, 64), 8, 2), codes((16, 16, 16, 64), 8, 3)
    need = ctx().workspace_bytes(pkg.CALL_CONV_BACKWARD, conv=d, fa=f, fb=f, fc=f)
    assert need > 64 * 3 * 3 * 64 * 4              # at least one slab of the weight gradient
    exact = pkg.Context(workspace_bytes=need)
    dx, dw = exact.conv_backward(d, to_dev(dy), f, to_dev(wt), f, to_dev(x), f, Epilogue.exact(), Epilogue.exact())
    assert np.array_equal(host(dw).astype(np.int64), co.conv_wgrad(dy, x, 3, 3, 1, 1))
    assert np.array_equal(host(dx).astype(np.int64), co.conv_dgrad(dy, wt, 16, 16, 1, 1))
    exact.close()
    assert ctx().workspace_bytes(pkg.CALL_KLD_SEARCH, n=65536, wl_lo=2, wl_hi=16, bins=2048) > 16 * 2048 * 4
    with pytest.raises(pkg.AdaptError):
        ctx().workspace_bytes(pkg.CALL_CONV_FWD, conv=ConvDesc(1, 2, 2, 16, 16, 5, 5, 1, 0), fa=f, fb=f)
    grown = pkg.Context(workspace_bytes=1 << 16)
    grown.reserve_workspace(need)
    _, dw2 = grown.conv_backward(d, to_dev(dy), f, to_dev(wt), f, to_dev(x), f, Epilogue.exact(), Epilogue.exact())
    assert torch.equal(dw2, dw)
    grown.close()


def test_short_workspace_takes_fewer_splits_and_long_reductions_report_the_bound():
    small = pkg.Context(workspace_bytes=1 << 16)            # 60 KiB of scratch
    d = ConvDesc(16, 16, 16, 64, 64, 3, 3, 1, 1)            # a weight gradient that would like many splits of 147 KB slabs
    x, dy = codes((16, 16, 16, 64), 8, 1), codes((16, 16, 16, 64), 8, 3)
    dw = small.conv_wgrad(d, to_dev(dy), (8, 4), to_dev(x), (8, 4), Epilogue.exact())
    assert np.array_equal(host(dw).astype(np.int64), co.conv_wgrad(dy, x, 3, 3, 1, 1))
    # K = 200,000 needs four splits of int32 partial sums whatever the workspace: 4 x 64 x 64 x 8 bytes do not fit 60 KiB
    k = 200000
    a, b = codes((64, k), 8, 5), codes((k, 64), 8, 6)
    with pytest.raises(pkg.AdaptError) as err:
        small.fxp_gemm(to_dev(a), (8, 0), to_dev(b), (8, 0), Epilogue.exact())
    assert err.value.status == -3                           # ADAPT_EBOUND
    small.close()
    c = ctx().fxp_gemm(to_dev(a), (8, 0), to_dev(b), (8, 0), Epilogue.exact())
    assert np.array_equal(host(c), orc.gemm(a, b))


# ---- the launch configurations of the full bench sizes, checked against runs that the oracle tests cover --------

def _full_batch_consistency(specs):
    """Forward and data gradient treat samples independently and the weight gradient is a sum over samples: the full
    batch (tiles, K splits and pairings of the size the benchmark times) must reproduce, exactly, what small-batch
    runs of the same layer give (those configurations are compared with the oracle in the sweeps above)."""
    c = ctx()
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    for sp in specs:
        s = sp.shape
        wl = sp.wl
        dt = torch.int8 if wl <= 8 else torch.int16
        lo, hi = -(1 << (wl - 1)), 1 << (wl - 1)
        d = ConvDesc(s.n, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad)
        c.reserve_for_layers([(d, (wl, wl - 3), (wl, wl - 3), (wl, wl - 3))])
        x = torch.randint(lo, hi, (s.n, s.h, s.w, s.c), device="cuda", generator=g, dtype=torch.int32).to(dt)
        wt = torch.randint(lo, hi, (s.k, s.r, s.s, s.c), device="cuda", generator=g, dtype=torch.int32).to(dt)
        dy = torch.randint(lo, hi, (s.n, d.p, d.q, s.k), device="cuda", generator=g, dtype=torch.int32).to(dt)
        f = (wl, wl - 3)
        ex = Epilogue.exact()
        ep = Epilogue.requant(wl, wl - 3, pkg.SR, 1, 40, relu=True)
        sub = 2
        ds = ConvDesc(sub, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad)
        y = c.conv_fwd(d, x, f, wt, f, ep)
        assert torch.equal(y[:sub], c.conv_fwd(ds, x[:sub].contiguous(), f, wt, f, ep)), sp.name
        dx, dw = c.conv_backward(d, dy, f, wt, f, x, f, ex, ex)
        assert torch.equal(dx[:sub], c.conv_dgrad(ds, dy[:sub].contiguous(), f, wt, f, ex)), sp.name
        chunk = s.n // 8
        dc = ConvDesc(chunk, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad)
        total = torch.zeros(dw.shape, dtype=torch.int64, device="cuda")
        for i in range(8):
            part = c.conv_wgrad(dc, dy[i * chunk:(i + 1) * chunk].contiguous(), f, x[i * chunk:(i + 1) * chunk].contiguous(), f, ex)
            total += part.to(torch.int64)
        assert torch.equal(dw.to(torch.int64), total), sp.name


def test_config4_full_batch_launch_configurations():
    _full_batch_consistency(wk.alexnet_cifar_layers())


def test_config5_full_batch_launch_configurations():
    _full_batch_consistency(wk.resnet18_cifar_layers())
