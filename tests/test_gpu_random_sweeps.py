"""GPU parity on randomly drawn cases: shapes, strides, paddings, word lengths, transposes, leading dimensions, epilogues
and value distributions are drawn from a seeded generator, so that combinations the hand-picked cases of the other
files do not list are met as well.  Every result is compared with the CPU oracle bit for bit (KL values to the bar of
test_gpu_kld).  The contractions are the quantized layer compute of Alg. 1 with the rounding rule of Sec. 3.2; the
search is PushDown of Sec. 3.3 / Alg. 3."""
import numpy as np
import pytest
import torch

import paper_2107_13490_amd as pkg
from oracle import conv_oracle as co
from oracle import fxp_oracle as orc
from paper_2107_13490_amd import ConvDesc, Epilogue

from gpu_util import ctx, dev, host
from test_gpu_kld import _compare as kld_compare

pytestmark = pytest.mark.gpu


def _codes(g, shape, wl):
    lo, hi = -(1 << (wl - 1)), (1 << (wl - 1)) - 1
    if g.integers(0, 3) == 0:                     # extremes only: the accumulators run at their bounds
        a = g.choice(np.array([lo, hi, 0, -1, 1, lo + 1]).clip(lo, hi), shape)
    else:
        a = g.integers(lo, hi + 1, shape)
    return a.astype(np.int8 if wl <= 8 else np.int16)


def _i64(t):
    return host(t).astype(np.int64)


@pytest.mark.parametrize("chunk", range(6))
def test_random_convolutions(chunk):
    for case in range(40):
        g = np.random.default_rng(7_000_000 + 1000 * chunk + case)
        r = int(g.choice([1, 1, 2, 3, 3, 5]))
        s = r if g.integers(0, 4) else int(g.choice([1, 3]))
        st = int(g.choice([1, 1, 2]))
        pad = min(int(g.integers(0, r // 2 + 2)), max(r, s) - 1) if max(r, s) > 1 else 0
        h, w = int(g.integers(r, 36)), int(g.integers(s, 36))
        c = int(g.choice([1, 3, 4, 7, 8, 16, 16, 24, 32, 48, 64, 80, 128, 200]))
        k = int(g.choice([1, 5, 8, 10, 16, 16, 17, 32, 48, 64, 100, 128, 130, 192]))
        n = int(g.choice([1, 2, 3, 5, 8, 17, 40]))
        d = ConvDesc(n, h, w, c, k, r, s, st, pad)
        if n * d.p * d.q * k * r * s * c > 3e9:   # keeps the oracle at a fraction of a second per case
            n = max(1, n // 8)
            d = ConvDesc(n, h, w, c, k, r, s, st, pad)
        wlx, wlw, wldy = (int(v) for v in g.choice([2, 4, 7, 8, 9, 12, 15, 16], 3))
        x, wt, dy = _codes(g, (n, h, w, c), wlx), _codes(g, (k, r, s, c), wlw), _codes(g, (n, d.p, d.q, k), wldy)
        tag = f"chunk {chunk} case {case}: {(n, h, w, c, k, r, s, st, pad)} wl {(wlx, wlw, wldy)}"
        C = ctx()
        fx, fw, fdy = (wlx, 4), (wlw, 5), (wldy, 4)
        wy, wdx, wdw = co.conv_fwd(x, wt, st, pad), co.conv_dgrad(dy, wt, h, w, st, pad), co.conv_wgrad(dy, x, r, s, st, pad)
        assert np.array_equal(_i64(C.conv_fwd(d, dev(x), fx, dev(wt), fw, Epilogue.exact())), wy), tag
        assert np.array_equal(_i64(C.conv_dgrad(d, dev(dy), fdy, dev(wt), fw, Epilogue.exact())), wdx), tag
        assert np.array_equal(_i64(C.conv_wgrad(d, dev(dy), fdy, dev(x), fx, Epilogue.exact())), wdw), tag
        dx2, dw2 = C.conv_backward(d, dev(dy), fdy, dev(wt), fw, dev(x), fx, Epilogue.exact(), Epilogue.exact())
        assert np.array_equal(_i64(dx2), wdx) and np.array_equal(_i64(dw2), wdw), tag
        wl_o, fl_o = int(g.choice([4, 8, 12, 16])), int(g.integers(0, 10))
        mode = pkg.SR if g.integers(0, 2) else pkg.RN_HALF_UP
        yq = C.conv_fwd(d, dev(x), fx, dev(wt), fw, Epilogue.requant(wl_o, fl_o, mode, 7, 100 + case, relu=True))
        assert np.array_equal(_i64(yq), orc.requantize(wy, 9 - fl_o, wl_o, mode, 7, 100 + case, relu=True)), tag
        dxq, dwq = C.conv_backward(d, dev(dy), fdy, dev(wt), fw, dev(x), fx, Epilogue.requant(wl_o, fl_o, mode, 8, 200 + case),
                                   Epilogue.requant(wl_o, fl_o, mode, 9, 300 + case))
        assert np.array_equal(_i64(dxq), orc.requantize(wdx, 9 - fl_o, wl_o, mode, 8, 200 + case)), tag
        assert np.array_equal(_i64(dwq), orc.requantize(wdw, 8 - fl_o, wl_o, mode, 9, 300 + case)), tag


@pytest.mark.parametrize("chunk", range(4))
def test_random_gemms(chunk):
    for case in range(50):
        g = np.random.default_rng(8_000_000 + 1000 * chunk + case)

        def dim(big):
            return int(g.choice([1, 2, 7, 16, 31, 64, 65, 100, 128, 130, 192, 256, 300, big]))
        m, n, k = dim(700), dim(520), dim(2500)
        if g.integers(0, 10) == 0:
            k = int(g.choice([0, 5000, 40000]))   # nothing to reduce; reductions long enough to be split
        if m * n * k > 4e8:
            m = max(1, m // 8)
        wla, wlb = (int(v) for v in g.choice([2, 5, 8, 8, 9, 12, 15, 16], 2))
        ta, tb = bool(g.integers(0, 2)), bool(g.integers(0, 2))
        a, b = _codes(g, (m, k), wla), _codes(g, (k, n), wlb)
        want = orc.gemm(a, b)
        pa, pb = int(g.choice([0, 16, 48])), int(g.choice([0, 16, 32]))

        def place(x, extra):                      # a slice of a wider device tensor: leading dimension > row length
            if x.size == 0:
                return dev(x)
            t = torch.zeros((x.shape[0], x.shape[1] + extra), dtype=torch.int8 if x.dtype == np.int8 else torch.int16, device="cuda")
            t[:, :x.shape[1]] = dev(x)
            return t[:, :x.shape[1]]
        da, db = place(a.T.copy() if ta else a, pa), place(b.T.copy() if tb else b, pb)
        tag = f"chunk {chunk} case {case}: {(m, n, k)} wl {(wla, wlb)} trans {(ta, tb)} extra {(pa, pb)}"
        c = ctx().fxp_gemm(da, (wla, 3), db, (wlb, 2), Epilogue.exact(), trans_a=ta, trans_b=tb)
        assert np.array_equal(_i64(c), want), tag
        wl_o, fl_o = int(g.choice([4, 8, 12, 16])), int(g.integers(0, 6))
        mode = pkg.SR if g.integers(0, 2) else pkg.RN_HALF_UP
        relu = bool(g.integers(0, 2))
        cq = ctx().fxp_gemm(da, (wla, 3), db, (wlb, 2), Epilogue.requant(wl_o, fl_o, mode, 3, case, relu=relu), trans_a=ta, trans_b=tb)
        assert np.array_equal(_i64(cq), orc.requantize(want, 5 - fl_o, wl_o, mode, 3, case, relu=relu)), tag


@pytest.mark.parametrize("chunk", range(4))
def test_random_searches_and_quantizations(chunk):
    for case in range(40):
        g = np.random.default_rng(9_000_000 + 1000 * chunk + case)
        n = int(g.choice([1, 3, 64, 1000, 4097, 30000, 70001, 200000]))
        kind = int(g.integers(0, 5))
        scale = float(10.0 ** g.uniform(-5, 2))
        if kind == 0:
            w = g.standard_normal(n) * scale
        elif kind == 1:
            w = g.laplace(size=n) * scale
        elif kind == 2:
            w = g.uniform(-1, 1, n) * scale + scale * g.uniform(-3, 3)      # a range far from zero
        elif kind == 3:
            w = np.where(g.random(n) < 0.5, 0.0, g.standard_normal(n) * scale)      # half of the weights pruned
        else:
            w = np.full(n, scale) if g.integers(0, 2) else g.choice([-scale, scale, 0.0], n)      # one or three values
        w = w.astype(np.float32)
        if g.integers(0, 6) == 0 and n > 3:
            w[:: max(n // 7, 1)] = np.nan
        lo = int(g.integers(2, 17))
        hi = int(g.integers(lo, 17))
        il = int(g.integers(1, min(lo, 5) + 1))
        bins = int(g.choice([2, 10, 100, 150, 1000, 2048, 5000, 40000]))
        eps = float(10.0 ** g.uniform(-4, -1))
        mode = pkg.SR if g.integers(0, 2) else pkg.RN_HALF_UP
        alpha = None if g.integers(0, 2) else float(10.0 ** g.uniform(-6, 0))
        kld_compare(w, lo, hi, il, bins, eps, alpha, mode, seed=case, stream=chunk)
        wl, fl = int(g.integers(2, 17)), int(g.integers(0, 20))
        q, cnt = ctx().quantize(dev(w), wl, fl, mode, seed=case, stream=5)
        rq, rn, rs = orc.quantize(w, wl, fl, mode, case, 5)
        assert np.array_equal(_i64(q), rq.astype(np.int64)) and host(cnt).tolist() == [int(rn), int(rs)], (chunk, case, wl, fl)


@pytest.mark.parametrize("chunk", range(3))
def test_random_chains_and_residual_graphs(chunk):
    """Whole training steps (every tensor against the oracle) on drawn word lengths: feed-forward chains of drawn
    shapes, the small residual network with and without the precision switch, and formats above 16 bits."""
    import test_gpu_net as tn
    g = np.random.default_rng(6_000_000 + chunk)
    for case in range(6):
        rng = np.random.default_rng(6_100_000 + 100 * chunk + case)
        layers, fmts = tn._random_net(rng)
        tn._run_chain(layers, fmts, n=int(rng.choice([2, 3, 5, 9])), seed=3000 + 100 * chunk + case)
    for case in range(6):
        fm = [(wl, wl - int(g.integers(3, 6))) for wl in (int(v) for v in g.integers(5, 17, 7))]
        tn._run_graph(tn._small_resnet(), fm, n=int(g.choice([2, 4, 6])), steps=2, seed=3200 + 100 * chunk + case)
    for case in range(3):
        fm = [(wl, wl - int(g.integers(3, 6))) for wl in (int(v) for v in g.integers(6, 17, 7))]
        kw = dict(lb_lwr=1, lb_upr=int(g.integers(2, 5)), lb_init=2, r_lwr=50, r_upr=80, r_init=60, gamma=float(g.choice([0.3, 0.5])),
                  eps=float(g.choice([1e-2, 1e-3])), buff=int(g.integers(1, 5)), wl_lo=4, wl_hi=16)
        tn._run_graph(tn._small_resnet(), fm, n=int(g.choice([2, 4])), steps=5, seed=3400 + 100 * chunk + case, switch_kw=kw)
    for case in range(3):
        fm = [(wl, wl - int(g.integers(4, 8))) for wl in (int(v) for v in g.choice([8, 12, 16, 17, 20, 23, 24, 28, 32], 7))]
        tn._run_graph(tn._tiny_resnet(), fm, n=2, steps=2, seed=3600 + 100 * chunk + case, wl_max=32)
