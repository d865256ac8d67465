"""GPU parity: word lengths 17..32 (int32 codes): quantize, and the contractions composed of 11-bit parts with
128-bit recombination, against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import paper_2107_13490_amd as pkg
from oracle import fxp_oracle as orc
from oracle import wide_oracle as wo
from paper_2107_13490_amd import ConvDesc, Epilogue

from gpu_util import ctx, dev, host

pytestmark = pytest.mark.gpu


def _dt(wl):
    return np.int8 if wl <= 8 else np.int16 if wl <= 16 else np.int32


def _codes(g, shape, wl):
    lim = 1 << (wl - 1)
    a = g.integers(-lim, lim, shape, dtype=np.int64)
    flat = a.reshape(-1)
    if flat.size >= 4:                                     # the corners of the range
        flat[0], flat[1], flat[2] = lim - 1, -lim, 0
    return a.astype(_dt(wl))


def _i128(t):
    """int64 tensor [..., 2] (low, high) -> array of Python integers."""
    a = host(t).astype(np.int64)
    lo = a[..., 0].astype(object) & ((1 << 64) - 1)
    hi = a[..., 1].astype(object)
    return hi * (1 << 64) + lo


@pytest.mark.parametrize("wl,fl", [(17, 15), (20, 12), (24, 20), (32, 31), (32, 20), (32, 0)])
@pytest.mark.parametrize("n", [1, 8, 1000, 70001])
def test_quantize_to_int32_codes(wl, fl, n):
    g = np.random.default_rng(wl * 100 + n)
    x = (g.standard_normal(n) * 2.0 ** (wl - 2 - fl)).astype(np.float32)
    if n > 6:
        x[1], x[2], x[3], x[4], x[5] = np.nan, np.inf, -np.inf, 1e30, -0.0
    for mode in (pkg.SR, pkg.RN_HALF_UP):
        q, cnt = ctx().quantize(dev(x), wl, fl, mode=mode, seed=7, stream=n)
        want, nnz, sat = orc.quantize(x, wl, fl, mode, 7, n)
        assert q.dtype == torch.int32
        assert np.array_equal(host(q).astype(np.int64), want)
        assert host(cnt).tolist() == [nnz, sat]


GEMM_CASES = [((5, 7, 9), 32, 32), ((64, 48, 130), 24, 20), ((33, 17, 64), 17, 8), ((16, 16, 16), 12, 32), ((70, 130, 300), 32, 16),
              ((128, 64, 1024), 32, 32), ((24, 40, 96), 31, 31), ((17, 9, 200), 31, 32), ((32, 32, 64), 8, 31), ((9, 33, 48), 31, 17)]


@pytest.mark.parametrize("shape,wa,wb", GEMM_CASES)
def test_wide_gemm_exact_and_requantized(shape, wa, wb):
    m, n, k = shape
    g = np.random.default_rng(m + n + k + wa)
    a, b = _codes(g, (m, k), wa), _codes(g, (k, n), wb)
    fa, fb = (wa, wa - 3), (wb, wb - 4)
    exact = wo.gemm(a, b)
    got = ctx().fxp_gemm(dev(a), fa, dev(b), fb, Epilogue.exact())
    assert got.shape == (m, n, 2) and np.array_equal(_i128(got), exact)
    for wl_o, fl_o, relu in ((32, wa + wb - 7 - 30, False), (24, wa + wb - 7 - 40, True), (16, 0, False), (8, 2, False), (32, wa + wb - 5, False)):
        fl_o = min(max(fl_o, 0), 31)
        ep = Epilogue.requant(wl_o, fl_o, pkg.SR, 3, 11, relu=relu)
        out = ctx().fxp_gemm(dev(a), fa, dev(b), fb, ep)
        want = wo.requantize(exact, fa[1] + fb[1] - fl_o, wl_o, orc.SR, 3, 11, relu)
        assert np.array_equal(host(out).astype(np.int64), want), (wl_o, fl_o)
    # transposed operands
    got = ctx().fxp_gemm(dev(a.T.copy()), fa, dev(b.T.copy()), fb, Epilogue.exact(), trans_a=True, trans_b=True)
    assert np.array_equal(_i128(got), exact)


def test_narrow_operands_with_a_wide_output():
    g = np.random.default_rng(5)
    a, b = _codes(g, (40, 96), 16), _codes(g, (96, 24), 16)
    exact = wo.gemm(a, b)
    out = ctx().fxp_gemm(dev(a), (16, 12), dev(b), (16, 13), Epilogue.requant(32, 24, pkg.SR, 1, 2))
    assert out.dtype == torch.int32
    assert np.array_equal(host(out).astype(np.int64), wo.requantize(exact, 1, 32, orc.SR, 1, 2))


CONV_CASES = [((2, 6, 6, 8, 16, 3, 3, 1, 1), 32, 32), ((3, 8, 8, 16, 8, 3, 3, 2, 1), 20, 24), ((2, 5, 7, 3, 8, 3, 3, 1, 1), 32, 8),
              ((2, 4, 4, 32, 16, 1, 1, 1, 0), 12, 32), ((1, 9, 9, 8, 8, 5, 5, 2, 2), 17, 17), ((2, 6, 6, 8, 16, 3, 3, 1, 1), 31, 31),
              ((2, 5, 5, 16, 8, 3, 3, 2, 1), 32, 31)]


@pytest.mark.parametrize("shp,wx,ww", CONV_CASES)
def test_wide_convolutions(shp, wx, ww):
    n, h, w, c, k, r, s, stride, pad = shp
    d = ConvDesc(*shp)
    g = np.random.default_rng(sum(shp) + wx)
    x, wt = _codes(g, (n, h, w, c), wx), _codes(g, (k, r, s, c), ww)
    fx, fw = (wx, wx - 4), (ww, ww - 2)
    y = wo.conv_fwd(x, wt, stride, pad)
    got = ctx().conv_fwd(d, dev(x), fx, dev(wt), fw, Epilogue.exact())
    assert np.array_equal(_i128(got), y)
    ep = Epilogue.requant(wx, 3, pkg.SR, 9, 21, relu=True)
    out = ctx().conv_fwd(d, dev(x), fx, dev(wt), fw, ep)
    assert np.array_equal(host(out).astype(np.int64), wo.requantize(y, fx[1] + fw[1] - 3, wx, orc.SR, 9, 21, True))
    dy = _codes(g, (n, d.p, d.q, k), wx)
    dx = wo.conv_dgrad(dy, wt, h, w, stride, pad)
    got = ctx().conv_dgrad(d, dev(dy), fx, dev(wt), fw, Epilogue.exact())
    assert np.array_equal(_i128(got), dx)
    dw = wo.conv_wgrad(dy, x, r, s, stride, pad)
    got = ctx().conv_wgrad(d, dev(dy), fx, dev(x), fx, Epilogue.exact())
    assert np.array_equal(_i128(got) if wx > 16 else host(got).astype(object), dw)       # two narrow operands: int32 / int64 sums
    out = ctx().conv_wgrad(d, dev(dy), fx, dev(x), fx, Epilogue.requant(32, 0, pkg.RN_HALF_UP, 0, 0))
    assert np.array_equal(host(out).astype(np.int64), wo.requantize(dw, 2 * fx[1], 32, orc.RN_HALF_UP, 0, 0))


@pytest.mark.parametrize("wdy,ww,wx", [(24, 20, 12), (12, 28, 8), (8, 8, 32), (32, 32, 32)])
def test_wide_backward_call_gives_both_gradients(wdy, ww, wx):
    shp = (2, 6, 5, 8, 16, 3, 3, 1, 1)
    n, h, w, c, k, r, s, stride, pad = shp
    d = ConvDesc(*shp)
    g = np.random.default_rng(wdy + ww + wx)
    x, wt, dy = _codes(g, (n, h, w, c), wx), _codes(g, (k, r, s, c), ww), _codes(g, (n, d.p, d.q, k), wdy)
    dx, dw = ctx().conv_backward(d, dev(dy), (wdy, 0), dev(wt), (ww, 3), dev(x), (wx, 2), Epilogue.exact(), Epilogue.exact())
    want_dx, want_dw = wo.conv_dgrad(dy, wt, h, w, stride, pad), wo.conv_wgrad(dy, x, r, s, stride, pad)
    as_int = lambda t, wide: _i128(t) if wide else host(t).astype(object)
    assert np.array_equal(as_int(dx, wdy > 16 or ww > 16), want_dx)
    assert np.array_equal(as_int(dw, wdy > 16 or wx > 16), want_dw)
    need = ctx().workspace_bytes(pkg.CALL_CONV_BACKWARD, conv=d, fa=(wdy, 0), fb=(ww, 3), fc=(wx, 2))
    one = max(ctx().workspace_bytes(pkg.CALL_CONV_DGRAD, conv=d, fa=(wdy, 0), fb=(ww, 3)),
              ctx().workspace_bytes(pkg.CALL_CONV_WGRAD, conv=d, fa=(wdy, 0), fb=(wx, 2)))
    assert need == one


def test_workspace_query_covers_a_wide_call():
    g = np.random.default_rng(8)
    m, n, k = 96, 80, 512
    a, b = _codes(g, (m, k), 32), _codes(g, (k, n), 24)
    need = ctx().workspace_bytes(pkg.CALL_GEMM, M=m, N=n, K=k, fa=(32, 20), fb=(24, 10))
    assert need > 0
    cx = pkg.Context(workspace_bytes=need)
    try:
        out = cx.fxp_gemm(dev(a), (32, 20), dev(b), (24, 10), Epilogue.requant(32, 10, pkg.SR, 1, 1))
        assert np.array_equal(host(out).astype(np.int64), wo.requantize(wo.gemm(a, b), 20, 32, orc.SR, 1, 1))
    finally:
        cx.close()
    # operands of 17..23 bits split into a byte and a part of up to 16 bits: the query covers every pair of parts
    d2 = ConvDesc(16, 16, 16, 64, 64, 3, 3, 1, 1)
    x, wt = _codes(g, (16, 16, 16, 64), 20), _codes(g, (64, 3, 3, 64), 23)
    dy = _codes(g, (16, 16, 16, 64), 20)
    calls = [(pkg.CALL_CONV_FWD, lambda c: c.conv_fwd(d2, dev(x), (20, 12), dev(wt), (23, 15), Epilogue.exact()), wo.conv_fwd(x, wt, 1, 1)),
             (pkg.CALL_CONV_DGRAD, lambda c: c.conv_dgrad(d2, dev(dy), (20, 12), dev(wt), (23, 15), Epilogue.exact()), wo.conv_dgrad(dy, wt, 16, 16, 1, 1)),
             (pkg.CALL_CONV_WGRAD, lambda c: c.conv_wgrad(d2, dev(dy), (20, 12), dev(x), (20, 12), Epilogue.exact()), wo.conv_wgrad(dy, x, 3, 3, 1, 1))]
    for call, run, want in calls:
        fb = (20, 12) if call == pkg.CALL_CONV_WGRAD else (23, 15)
        need = ctx().workspace_bytes(call, conv=d2, fa=(20, 12), fb=fb)
        cx = pkg.Context(workspace_bytes=need)
        try:
            assert np.array_equal(_i128(run(cx)), want), call
        finally:
            cx.close()
    d = ConvDesc(2, 8, 8, 16, 16, 3, 3, 1, 1)
    for call in (pkg.CALL_CONV_FWD, pkg.CALL_CONV_DGRAD, pkg.CALL_CONV_WGRAD):
        assert ctx().workspace_bytes(call, conv=d, fa=(20, 10), fb=(8, 4)) > ctx().workspace_bytes(call, conv=d, fa=(12, 10), fb=(8, 4))


def test_wide_calls_report_what_they_cannot_do():
    a = torch.zeros((8, 8), dtype=torch.int32, device="cuda")
    small = pkg.Context(workspace_bytes=1 << 20)
    try:
        with pytest.raises(pkg.AdaptError):                # the parts and the 128-bit sums need workspace
            small.fxp_gemm(a, (32, 0), a, (32, 0), Epilogue.exact())
    finally:
        small.close()
    with pytest.raises(pkg.AdaptError):
        ctx().fxp_gemm(a, (33, 0), a, (32, 0), Epilogue.exact())
    assert pkg.acc_bits(10, pkg.Fmt(17, 0), pkg.Fmt(8, 0)) == 128
