"""Pins for the oracle of the chained fixed-point network step (CPU only).

The step follows Alg. 1 (forward pass on quantized layers, backward pass, update, Quantize).  The
paper prints no numbers for it; the pins are library routines for the pieces that have one
(max-pooling and its gradient routing through torch, on inputs without ties), hand-worked cases
for the rules the oracle itself fixes (first maximum on ties, the mask from the stored output, the
fitting shift), exact rational arithmetic for the residual addition, and a floating-point network
with automatic differentiation that the 16-bit chain must follow closely.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import fxp_oracle as orc
from oracle import net_oracle as no


def _nchw(a):
    return torch.from_numpy(np.ascontiguousarray(np.transpose(a, (0, 3, 1, 2))))


def _nhwc(t):
    return np.transpose(t.detach().numpy(), (0, 2, 3, 1))


def test_maxpool_is_the_library_routine():
    rng = np.random.default_rng(0)
    y = rng.integers(-128, 128, (3, 6, 8, 5))
    want = _nhwc(F.max_pool2d(_nchw(y.astype(np.float64)), 2))
    assert np.array_equal(no.maxpool2(y), want.astype(np.int64))


def test_pool_and_relu_gradient_is_what_autograd_routes_without_ties():
    rng = np.random.default_rng(1)
    n, h, w, c = 2, 6, 4, 3
    # distinct values: no ties, so the routing is unique; the network stores y = relu(z)
    z = (rng.permutation(n * h * w * c).reshape(n, h, w, c) - n * h * w * c // 2).astype(np.float64)
    zt = _nchw(z).requires_grad_(True)
    out = F.max_pool2d(F.relu(zt), 2)
    up = rng.integers(-50, 50, (n, h // 2, w // 2, c)).astype(np.float64)
    out.backward(_nchw(up))
    y = np.maximum(z, 0).astype(np.int64)
    got = no.relu_pool_bwd(up.astype(np.int64), y, True, True)
    # a window whose values are all <= 0 has y = 0 everywhere: autograd sends the gradient to one of
    # the zeros and ReLU's derivative then removes it, the oracle masks it: both give 0
    assert np.array_equal(got, _nhwc(zt.grad).astype(np.int64))
    # without pooling: the plain ReLU mask
    zt2 = _nchw(z).requires_grad_(True)
    F.relu(zt2).backward(_nchw(z * 0 + 7.0))
    assert np.array_equal(no.relu_pool_bwd(np.full(z.shape, 7), y, True, False), _nhwc(zt2.grad).astype(np.int64))


def test_ties_go_to_the_first_maximum_in_scan_order_and_zero_outputs_get_nothing():
    y = np.zeros((1, 2, 4, 1), dtype=np.int64)
    y[0, :, 0:2, 0] = [[3, 5], [5, 5]]           # window 0: maximum 5 first at (0,1)
    y[0, :, 2:4, 0] = [[0, 0], [0, 0]]           # window 1: nothing positive
    da = np.array([11, 13]).reshape(1, 1, 2, 1)
    dy = no.relu_pool_bwd(da, y, True, True)
    want = np.zeros_like(y)
    want[0, 0, 1, 0] = 11
    assert np.array_equal(dy, want)
    # no ReLU: the all-zero window routes to its first element
    dy = no.relu_pool_bwd(da, y, False, True)
    want[0, 0, 2, 0] = 13
    assert np.array_equal(dy, want)
    # no pooling, no ReLU: identity
    assert np.array_equal(no.relu_pool_bwd(y + 1, y, False, False), y + 1)


def test_fitting_shift_closed_forms():
    assert no.fit_shift(np.array([0, 0]), 8) == 0
    assert no.fit_shift(np.array([127, -127]), 8) == 0
    assert no.fit_shift(np.array([128]), 8) == 1
    assert no.fit_shift(np.array([-128]), 8) == 1          # decided by the magnitude
    assert no.fit_shift(np.array([255]), 8) == 1
    assert no.fit_shift(np.array([256]), 8) == 2
    assert no.fit_shift(np.array([1 << 40]), 16) == 41 - 15
    assert no.fit_shift(np.array([5]), 2) == 2             # 5 >> 2 = 1 fits one magnitude bit
    rng = np.random.default_rng(2)
    for wl in (2, 4, 8, 12, 16):
        acc = rng.integers(-(1 << 30), 1 << 30, 1000)
        sh = no.fit_shift(acc, wl)
        m = int(np.abs(acc).max())
        assert (m >> sh) < (1 << (wl - 1)) and (sh == 0 or (m >> (sh - 1)) >= (1 << (wl - 1)))


def test_requantize_fit_keeps_values_within_one_step_and_counts_squares():
    rng = np.random.default_rng(3)
    acc = rng.integers(-(1 << 27), 1 << 27, 5000)
    for wl in (4, 8, 16):
        q, sh, ss = no.requantize_fit(acc, wl, orc.SR, 9, 4)
        lim = 1 << (wl - 1)
        assert q.min() >= -lim and q.max() <= lim - 1
        inside = np.abs(acc) < ((lim - 1) << sh)                       # not touched by saturation
        assert np.all(np.abs(q[inside] * (1 << sh) - acc[inside]) < (1 << sh))
        assert ss == sum(int(v) ** 2 for v in q)
        # round-to-nearest variant is the arithmetic definition
        qn, _, _ = no.requantize_fit(acc, wl, orc.RN_HALF_UP, 0, 0)
        want = np.clip((acc + (1 << sh >> 1)) >> sh, -lim, lim - 1) if sh else np.clip(acc, -lim, lim - 1)
        assert np.array_equal(qn, want)
    q, sh, ss = no.requantize_fit(np.zeros(7, np.int64), 8)
    assert sh == 0 and ss == 0 and not q.any()


def test_residual_add_is_the_rounded_exact_sum():
    rng = np.random.default_rng(4)
    a = rng.integers(-128, 128, 300)
    b = rng.integers(-2048, 2048, 300)
    for fl_a, fl_b, wl_o, fl_o in ((5, 9, 8, 4), (9, 5, 12, 9), (3, 3, 8, 5), (7, 2, 16, 10)):
        got = no.residual_add(a, fl_a, b, fl_b, wl_o, fl_o, orc.RN_HALF_UP)
        lim = 1 << (wl_o - 1)
        for i in range(a.size):
            v = Fraction(int(a[i]), 1 << fl_a) + Fraction(int(b[i]), 1 << fl_b)
            t = v * (1 << fl_o) + Fraction(1, 2)
            want = min(max(t.numerator // t.denominator, -lim), lim - 1)
            assert got[i] == want
        r = no.residual_add(a, fl_a, b, fl_b, wl_o, fl_o, orc.RN_HALF_UP, relu=True)
        assert np.array_equal(r, np.maximum(got, 0))
    # stochastic rounding brackets the exact value
    got = no.residual_add(a, 5, b, 9, 8, 2, orc.SR, 1, 2)
    exact = (a / 32.0 + b / 512.0) * 4.0
    ok = np.abs(exact) < 126
    assert np.all(np.abs(got[ok] - exact[ok]) < 1.0)


def _small_net():
    return [no.Layer(8, 8, 4, 8, relu=True, pool=True),
            no.Layer(4, 4, 8, 8, relu=True, pool=False),
            no.Layer(1, 1, 128, 10, 1, 1, 1, 0, relu=False, pool=False)]


def test_sixteen_bit_chain_follows_a_floating_point_network():
    rng = np.random.default_rng(5)
    layers = _small_net()
    n = 6
    fmts = [(16, 10)] * 3
    x = rng.standard_normal((n, 8, 8, 4)).astype(np.float32)
    ws = [(rng.standard_normal((L.k, L.r, L.s, L.c)) * 0.2).astype(np.float32) for L in layers]
    t = rng.standard_normal((n, 10))
    wq = no.quantize_weights(layers, fmts, ws, 1, 100)
    fwd = no.forward(layers, fmts, wq, x, 1, 100)
    dl = np.round(t * 2 ** 11).astype(np.int64).reshape(n, 1, 1, 10)       # 16-bit codes of t
    bwd = no.backward(layers, fmts, wq, fwd, dl, 1, 100)

    # the same network in fp64 with automatic differentiation (NCHW, filters KCRS); flatten in NHWC order
    tw = [torch.tensor(np.transpose(w.astype(np.float64), (0, 3, 1, 2)), requires_grad=True) for w in ws]
    h = _nchw(x.astype(np.float64))
    h = F.max_pool2d(F.relu(F.conv2d(h, tw[0], padding=1)), 2)
    h = F.relu(F.conv2d(h, tw[1], padding=1))
    flat = h.permute(0, 2, 3, 1).reshape(n, 128, 1, 1)
    logits = F.conv2d(flat, tw[2])
    (logits.reshape(n, 10) * torch.tensor(t)).sum().backward()

    got_logits = fwd["a"][2].reshape(n, 10) / 2.0 ** 10
    assert np.max(np.abs(got_logits - logits.detach().numpy().reshape(n, 10))) < 0.05
    for l in range(3):
        want = np.transpose(tw[l].grad.numpy(), (0, 2, 3, 1)).ravel()
        got = bwd["g"][l].astype(np.float64).ravel()
        cos = float(got @ want / np.sqrt((got @ got) * (want @ want)))
        assert cos > 0.999, (l, cos)
        assert bwd["sumsq"][l] == int(np.sum(bwd["g"][l].astype(object) ** 2))
    # weight-gradient codes use the available bits
    for l in range(3):
        m = int(np.abs(bwd["g"][l]).max())
        assert m >= 1 << 14 or bwd["shift_w"][l] == 0


def test_update_moves_against_the_gradient_and_requantizes():
    rng = np.random.default_rng(6)
    layers = _small_net()
    fmts = [(8, 5), (12, 8), (6, 3)]
    n = 4
    x = rng.standard_normal((n, 8, 8, 4)).astype(np.float32)
    ws = [(rng.standard_normal((L.k, L.r, L.s, L.c)) * 0.3).astype(np.float32) for L in layers]
    wq = no.quantize_weights(layers, fmts, ws, 2, 0)
    fwd = no.forward(layers, fmts, wq, x, 2, 0)
    for l, L in enumerate(layers):
        lim = 1 << (fmts[l][0] - 1)
        assert fwd["a"][l].shape == L.out_shape(n) and fwd["a"][l].min() >= -lim and fwd["a"][l].max() < lim
        if L.relu:
            assert fwd["y"][l].min() >= 0
    dl = rng.integers(-32, 32, (n, 1, 1, 10))
    bwd = no.backward(layers, fmts, wq, fwd, dl, 2, 0)
    upd = no.update(layers, fmts, ws, bwd, 0.1, 0.0, 0.0, 2, 0)
    for l in range(3):
        step = upd[l]["w"].reshape(-1) - ws[l].reshape(-1)
        g = bwd["g"][l].ravel().astype(np.float64)
        # the step is -lr * g / ||g||: length lr, direction against the gradient codes
        assert abs(np.linalg.norm(step) - 0.1) < 1e-3
        assert float(step @ g) < 0 and abs(float(step @ g) / (np.linalg.norm(step) * np.linalg.norm(g)) + 1) < 1e-3
        q2, _, _ = orc.quantize(upd[l]["w"], fmts[l][0], fmts[l][1], orc.SR, 2, no.stream_of(0, l, no.SLOT_UPD))
        assert np.array_equal(upd[l]["q"], q2)


def test_gradient_exponents_give_the_true_scale_of_the_gradient_codes():
    """codes * 2^-e must be the floating-point network's gradient, not just parallel to it."""
    rng = np.random.default_rng(7)
    layers = _small_net()
    n = 6
    fmts = [(16, 10), (16, 11), (16, 9)]
    x = rng.standard_normal((n, 8, 8, 4)).astype(np.float32)
    ws = [(rng.standard_normal((L.k, L.r, L.s, L.c)) * 0.2).astype(np.float32) for L in layers]
    t = rng.standard_normal((n, 10))
    wq = no.quantize_weights(layers, fmts, ws, 1, 100)
    fwd = no.forward(layers, fmts, wq, x, 1, 100)
    dl = np.round(t * 2 ** 11).astype(np.int64).reshape(n, 1, 1, 10)
    bwd = no.backward(layers, fmts, wq, fwd, dl, 1, 100)
    exps = no.gradient_exponents(fmts, bwd, 11)
    tw = [torch.tensor(np.transpose(w.astype(np.float64), (0, 3, 1, 2)), requires_grad=True) for w in ws]
    h = F.max_pool2d(F.relu(F.conv2d(_nchw(x.astype(np.float64)), tw[0], padding=1)), 2)
    h = F.relu(F.conv2d(h, tw[1], padding=1))
    logits = F.conv2d(h.permute(0, 2, 3, 1).reshape(n, 128, 1, 1), tw[2])
    (logits.reshape(n, 10) * torch.tensor(t)).sum().backward()
    for l in range(3):
        want = np.transpose(tw[l].grad.numpy(), (0, 2, 3, 1)).ravel()
        got = bwd["g"][l].astype(np.float64).ravel() * 2.0 ** -exps[l]
        assert abs(np.linalg.norm(got) / np.linalg.norm(want) - 1) < 0.05, (l, exps[l])     # a slip in an exponent is a factor 2
        assert np.linalg.norm(got - want) < 0.1 * np.linalg.norm(want)      # rounding noise of the 16-bit chain


def test_precision_switch_bookkeeping_over_several_batches():
    from oracle import pushup_oracle as po
    rng = np.random.default_rng(8)
    layers = _small_net()
    n = 4
    fmts = [(8, 5), (8, 5), (8, 4)]
    ws = [(rng.standard_normal((L.k, L.r, L.s, L.c)) * 0.3).astype(np.float32) for L in layers]
    st = no.SwitchState(3, lb_lwr=2, lb_upr=4, lb_init=2, r_lwr=50, r_upr=60, r_init=55, gamma=0.5, eps=1e-2, buff=2, wl_lo=2,
                        wl_hi=16)
    wq = no.quantize_weights(layers, fmts, ws, 3, 0)
    switched_any = False
    for step in range(6):
        x = rng.standard_normal((n, 8, 8, 4)).astype(np.float32)
        fwd = no.forward(layers, fmts, wq, x, 3, 100 * step)
        dl = rng.integers(-60, 60, (n, 1, 1, 10))
        bwd = no.backward(layers, fmts, wq, fwd, dl, 3, 100 * step)
        before = [len(w) for w in st.windows]
        old = list(fmts)
        rep = no.precision_switch(st, fmts, ws, bwd, 7, 2.0 - 0.1 * step, 3, 100 * step)
        assert len(st.losses) == step + 1
        for l, row in enumerate(rep):
            assert 2 <= row["lb"] <= 4 and 50 <= row["res"] <= 60
            assert row["ds"] >= 1.0 - 1e-12 or not np.isfinite(row["ds"])        # triangle inequality
            if row["switched"]:
                switched_any = True
                assert st.windows[l] == [] and before[l] + 1 >= row["lb"]
                assert row["wl_min"] <= old[l][0] and row["wl_min"] - row["fl_min"] == old[l][0] - old[l][1]
                want = po.pushup_suggest(row["ds"], row["wl_min"], row["fl_min"], st.strategy, 2, 16)
                assert fmts[l] == (want[0], want[1]) and fmts[l][0] >= fmts[l][1] + 2
            else:
                assert fmts[l] == old[l] and len(st.windows[l]) == min(before[l] + 1, 4)
        # the loss falls every batch: after the first comparison the strategy is "min"
        if step >= 1:
            assert st.strategy == po.ST_MIN
        upd = no.update(layers, fmts, ws, bwd, 0.05, 0.0, 0.0, 3, 100 * step)
        ws = [u["w"].reshape(w.shape) for u, w in zip(upd, ws)]
        wq = [u["q"].reshape(w.shape) for u, w in zip(upd, ws)]
    assert switched_any
