"""Pins of the residual / batch-norm oracle (oracle/graph_oracle.py) to what does not depend on it: the library's
fp64 batch normalisation and automatic differentiation, exact rational arithmetic on tiny inputs, closed forms."""
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import fxp_oracle as orc
from oracle import graph_oracle as go
from oracle import net_oracle as no


def _bn_case(seed, shape=(5, 4, 6, 7), wl=12, fl=8):
    g = np.random.default_rng(seed)
    lim = 1 << (wl - 1)
    y = np.clip(np.rint(g.standard_normal(shape) * (lim / 6) + g.standard_normal(shape[-1]) * (lim / 8)), -lim, lim - 1).astype(np.int64)
    gamma = (1.0 + 0.3 * g.standard_normal(shape[-1])).astype(np.float32)
    beta = (0.2 * g.standard_normal(shape[-1])).astype(np.float32)
    return g, y, gamma, beta


@pytest.mark.parametrize("seed", range(4))
def test_batch_norm_forward_is_the_library_routine_within_one_rounding(seed):
    g, y, gamma, beta = _bn_case(seed)
    fl_y, wl_o, fl_o, eps = 8, 16, 11, 1e-5
    out, st = go.bn_forward(y, fl_y, gamma, beta, eps, wl_o, fl_o, False, 1, 2, mode=orc.RN_HALF_UP)
    yt = torch.tensor(y.astype(np.float64) / 2.0 ** fl_y).permute(0, 3, 1, 2)
    want = F.batch_norm(yt, None, None, torch.tensor(gamma.astype(np.float64)), torch.tensor(beta.astype(np.float64)), True, 0.0, eps)
    want = want.permute(0, 2, 3, 1).numpy()
    # nearest rounding: half a step of the output grid, plus the 2^-30 relative error of the coefficients
    assert np.max(np.abs(out / 2.0 ** fl_o - want)) <= 0.5 / 2.0 ** fl_o + 1e-7
    # stochastic rounding: strictly inside one step, and unbiased over the tensor
    out_sr, _ = go.bn_forward(y, fl_y, gamma, beta, eps, wl_o, fl_o, False, 1, 2)
    err = out_sr / 2.0 ** fl_o - want
    assert np.max(np.abs(err)) < 1.0 / 2.0 ** fl_o + 1e-7 and abs(err.mean()) < 0.05 / 2.0 ** fl_o
    # with ReLU and a shortcut on another grid
    res = g.integers(-300, 300, y.shape)
    out_r, _ = go.bn_forward(y, fl_y, gamma, beta, eps, wl_o, fl_o, True, 1, 2, res=res, fl_res=6, mode=orc.RN_HALF_UP)
    want_r = np.maximum(want + res / 2.0 ** 6, 0.0)
    assert np.max(np.abs(out_r / 2.0 ** fl_o - want_r)) <= 0.5 / 2.0 ** fl_o + 1e-7
    # statistics
    flat = (y.astype(np.float64) / 2.0 ** fl_y).reshape(-1, y.shape[-1])
    assert np.allclose(st["mean"] / 2.0 ** fl_y, flat.mean(axis=0), rtol=1e-12, atol=1e-12)
    assert np.allclose((st["sig"] / 2.0 ** fl_y) ** 2, flat.var(axis=0) + eps, rtol=1e-10)


def test_batch_norm_coefficients_use_thirty_bits_and_saturate_gracefully():
    _, y, gamma, beta = _bn_case(9)
    st = go.bn_coeffs(y, 8, gamma, beta, 1e-5, 8)
    assert 1 << 29 <= int(np.abs(st["A"]).max()) <= 1 << 30 and 0 <= st["FA"] <= 30
    # a constant channel: variance 0, the gain is gamma / sqrt(eps) in real units and still finite
    y[..., 0] = 77
    st = go.bn_coeffs(y, 8, gamma, beta, 1e-5, 8)
    assert np.isfinite(st["alpha"]).all() and abs(st["alpha"][0] - gamma[0] * 2.0 ** 8 / np.sqrt(1e-5 * 4.0 ** 8)) < 1e-6 * abs(st["alpha"][0])
    out, _ = go.bn_forward(y, 8, gamma, beta, 1e-5, 12, 8, False, 0, 0, mode=orc.RN_HALF_UP)
    assert np.all(out[..., 0] == int(np.rint(float(beta[0]) * 256)))        # the constant channel normalises to beta
    # gamma = 0 everywhere: no gain to scale by, the output is beta
    out, st = go.bn_forward(y, 8, np.zeros_like(gamma), beta, 1e-5, 12, 8, False, 0, 0, mode=orc.RN_HALF_UP)
    assert st["FA"] == 30 and np.array_equal(out, np.broadcast_to(np.rint(beta.astype(np.float64) * 256).astype(np.int64), y.shape))


@pytest.mark.parametrize("seed", range(3))
def test_batch_norm_backward_is_what_automatic_differentiation_gives(seed):
    g, y, gamma, beta = _bn_case(10 + seed, wl=14, fl=9)
    fl_y, eps, e_dz = 9, 1e-5, 13
    st = go.bn_coeffs(y, fl_y, gamma, beta, eps, 11)                          # output grid differs from the input's
    dz = g.integers(-(1 << 13), 1 << 13, y.shape)
    r = go.bn_backward(dz, y, st, 16, 3, 4)
    yt = torch.tensor(y.astype(np.float64) / 2.0 ** fl_y, requires_grad=True)
    gt = torch.tensor(gamma.astype(np.float64), requires_grad=True)
    bt = torch.tensor(beta.astype(np.float64), requires_grad=True)
    z = F.batch_norm(yt.permute(0, 3, 1, 2), None, None, gt, bt, True, 0.0, eps).permute(0, 2, 3, 1)
    (z * torch.tensor(dz.astype(np.float64) / 2.0 ** e_dz)).sum().backward()
    want = yt.grad.numpy()
    got = r["dy"] * 2.0 ** -(e_dz + r["e_add"])
    # 16-bit codes fitted to the largest magnitude: one step of 2^-15 of it (stochastic rounding), plus coefficient rounding
    assert np.max(np.abs(got - want)) <= np.max(np.abs(want)) * 2.0 ** -14
    assert int(np.abs(r["dy"]).max()) >= 1 << 14
    assert np.allclose(r["dgamma"] * 2.0 ** -e_dz, gt.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(r["dbeta"] * 2.0 ** -e_dz, bt.grad.numpy(), rtol=1e-12, atol=1e-12)
    # the gradient of a normalised tensor sums to zero over each channel and is orthogonal to the centred input
    chan = got.reshape(-1, y.shape[-1])
    assert np.max(np.abs(chan.sum(axis=0))) <= np.max(np.abs(want)) * 2.0 ** -14 * np.sqrt(chan.shape[0]) * 4
    # zero gradient in, zero out
    z0 = go.bn_backward(np.zeros_like(dz), y, st, 16, 3, 4)
    assert not z0["dy"].any() and z0["shift"] == 0 and not z0["dgamma"].any()


def test_batch_norm_update_is_a_normalised_step():
    g = np.random.default_rng(3)
    gamma, beta = g.standard_normal(32).astype(np.float32), g.standard_normal(32).astype(np.float32)
    dg, db = g.standard_normal(32) * 1e4, g.standard_normal(32) * 1e-3
    g2, b2 = go.bn_update(gamma, beta, dg, db, 0.05)
    assert g2.dtype == np.float32 and abs(np.linalg.norm(g2 - gamma) - 0.05) < 1e-5 and abs(np.linalg.norm(b2 - beta) - 0.05) < 1e-5
    assert np.allclose(g2, gamma - 0.05 * dg / np.linalg.norm(dg), atol=1e-6)
    # any power-of-two factor of the gradient (its exponent in the chain) changes nothing, bit for bit
    g3, b3 = go.bn_update(gamma, beta, dg * 2.0 ** 17, db * 2.0 ** -9, 0.05)
    assert np.array_equal(g2, g3) and np.array_equal(b2, b3)
    # a zero gradient leaves the parameters alone
    g4, b4 = go.bn_update(gamma, beta, np.zeros(32), db, 0.05)
    assert np.array_equal(g4, gamma) and np.array_equal(b4, b2)


def test_global_average_pooling():
    g = np.random.default_rng(4)
    a = g.integers(-2000, 2000, (3, 4, 4, 5))
    out = go.gap_forward(a, 12, 0, 0, mode=orc.RN_HALF_UP)
    assert np.array_equal(out, np.floor(a.reshape(3, 16, 5).sum(axis=1) / 16.0 + 0.5).astype(np.int64))
    out_sr = go.gap_forward(a, 12, 5, 6)
    assert np.max(np.abs(out_sr - a.reshape(3, 16, 5).mean(axis=1))) < 1.0
    d, up = go.gap_backward(out, 4, 4)
    assert up == 4 and d.shape == (3, 4, 4, 5) and all(np.array_equal(d[:, i, j, :], out) for i in range(4) for j in range(4))
    # library routine: the gradient of a mean is 1/16 of the incoming gradient at every position
    t = torch.tensor(a.astype(np.float64), requires_grad=True)
    (t.mean(dim=(1, 2)) * torch.tensor(out.astype(np.float64))).sum().backward()
    assert np.array_equal(t.grad.numpy(), d * 2.0 ** -up)


def test_sum_of_two_gradient_tensors_against_exact_rationals():
    g = np.random.default_rng(5)
    for wl, e_a, e_b in ((8, 5, 9), (8, 9, 5), (6, 3, 3), (16, 0, 30), (4, 12, 2)):
        a = g.integers(-(1 << 7), 1 << 7, 40)
        b = g.integers(-(1 << 11), 1 << 11, 40)
        codes, e, shift = go.grad_add(a, e_a, b, e_b, wl, 7, 8)
        exact = [Fraction(int(x), 1 << e_a) + Fraction(int(y), 1 << e_b) for x, y in zip(a, b)]
        big = max(abs(v) for v in exact)
        step = Fraction(1, 1 << e) if e >= 0 else Fraction(1 << -e)
        assert all(abs(Fraction(int(c)) * step - v) < step for c, v in zip(codes, exact))           # one step (SR)
        assert codes.min() >= -(1 << (wl - 1)) and codes.max() < 1 << (wl - 1)
        # the shift is the smallest that fits: one bit less would overflow the largest magnitude
        assert shift == 0 or big / (step / 2) >= 1 << (wl - 1)
        assert e == max(e_a, e_b) - shift
    # one input that fits: unchanged, no rounding drawn; one that does not: refitted
    a = g.integers(-100, 100, 50)
    c, e, s = go.grad_add(a, 7, None, None, 8, 0, 0)
    assert np.array_equal(c, a) and (e, s) == (7, 0)
    c, e, s = go.grad_add(a * 64, 7, None, None, 8, 0, 0)
    assert s == no.fit_shift(a * 64, 8) and e == 7 - s and np.max(np.abs(c * 2.0 ** s - a * 64)) < 2.0 ** s
    # exponents more than 40 apart: the far smaller tensor is left out
    c, e, s = go.grad_add(a, 3, a * 3, 50, 8, 0, 0)
    assert np.array_equal(c, a) and e == 3
    c, e, s = go.grad_add(a * 3, 50, a, 3, 8, 0, 0)
    assert np.array_equal(c, a) and e == 3


def _residual_net():
    # stem conv-BN-ReLU, a basic block with identity shortcut, a down-sampling block with a 1x1 projection shortcut,
    # global average pooling, a fully connected layer
    N = go.Node
    return [N(8, 8, 3, 8, bn=True),                                              # 0 stem
            N(8, 8, 8, 8, bn=True),                                              # 1 block A conv1
            N(8, 8, 8, 8, bn=True, res=0),                                       # 2 block A conv2 + identity
            N(8, 8, 8, 16, stride=2, bn=True, src=2),                            # 3 block B conv1 (stride 2)
            N(8, 8, 8, 16, 1, 1, 2, 0, relu=False, bn=True, src=2),              # 4 block B projection 1x1 stride 2
            N(4, 4, 16, 16, bn=True, src=3, res=4, gap=True),                    # 5 block B conv2 + projection, then pooling
            N(1, 1, 16, 10, 1, 1, 1, 0, relu=False)]                             # 6 fully connected


def test_sixteen_bit_residual_chain_follows_a_floating_point_network():
    rng = np.random.default_rng(7)
    nodes = _residual_net()
    n, eps = 8, 1e-5
    fmts = [(16, 12)] * 6 + [(16, 11)]                       # range +-8: batch-normalised activations and their sums
    x = rng.standard_normal((n, 8, 8, 3)).astype(np.float32)
    ws = [(rng.standard_normal((L.k, L.r, L.s, L.c)) * (1.0 / np.sqrt(L.r * L.s * L.c))).astype(np.float32) for L in nodes]
    bn = [((1.0 + 0.2 * rng.standard_normal(L.k)).astype(np.float32), (0.1 * rng.standard_normal(L.k)).astype(np.float32)) if L.bn else None
          for L in nodes]
    t = rng.standard_normal((n, 10))
    wq = no.quantize_weights(nodes, fmts, ws, 1, 100)
    fwd = go.forward(nodes, fmts, wq, bn, x, eps, 1, 100)
    dl = np.round(t * 2 ** 11).astype(np.int64).reshape(n, 1, 1, 10)
    bwd = go.backward(nodes, fmts, wq, fwd, dl, 11, 1, 100)

    def nchw(a):
        return torch.tensor(np.transpose(a.astype(np.float64), (0, 3, 1, 2)))
    tw = [torch.tensor(np.transpose(w.astype(np.float64), (0, 3, 1, 2)), requires_grad=True) for w in ws]
    tg = [torch.tensor(p[0].astype(np.float64), requires_grad=True) if p else None for p in bn]
    tb = [torch.tensor(p[1].astype(np.float64), requires_grad=True) if p else None for p in bn]

    def cbn(h, l, stride=1, pad=1):
        return F.batch_norm(F.conv2d(h, tw[l], stride=stride, padding=pad), None, None, tg[l], tb[l], True, 0.0, eps)
    a0 = F.relu(cbn(nchw(x), 0))
    a1 = F.relu(cbn(a0, 1))
    a2 = F.relu(cbn(a1, 2) + a0)
    a3 = F.relu(cbn(a2, 3, 2))
    a4 = cbn(a2, 4, 2, 0)
    a5 = F.relu(cbn(a3, 5) + a4).mean(dim=(2, 3), keepdim=True)
    logits = F.conv2d(a5, tw[6])
    (logits.reshape(n, 10) * torch.tensor(t)).sum().backward()

    got_logits = fwd["a"][6].reshape(n, 10) / 2.0 ** 11
    assert np.max(np.abs(got_logits - logits.detach().numpy().reshape(n, 10))) < 0.02
    for l in range(7):
        want = np.transpose(tw[l].grad.numpy(), (0, 2, 3, 1)).ravel()
        got = bwd["g"][l].astype(np.float64).ravel()
        cos = float(got @ want / np.sqrt((got @ got) * (want @ want)))
        assert cos > 0.999, (l, cos)
        # the exponent gives the true scale of the codes
        scale = float(got @ want / (got @ got))
        assert abs(np.log2(scale) + bwd["e_g"][l]) < 0.05, (l, scale, bwd["e_g"][l])
        if nodes[l].bn:
            wg, wb = tg[l].grad.numpy(), tb[l].grad.numpy()
            for got_p, want_p in ((bwd["dgamma"][l], wg), (bwd["dbeta"][l], wb)):
                cosp = float(got_p @ want_p / np.sqrt((got_p @ got_p) * (want_p @ want_p)))
                assert cosp > 0.995, (l, cosp)               # 8 or 16 channels: a short vector, noisier than the weights
    # the update moves gamma and beta against their gradients by lr in 2-norm
    upd, bn_new = go.update(nodes, fmts, ws, bn, bwd, 0.01, 0.0, 0.0, 1, 100)
    for l in range(6):
        step = bn_new[l][0] - bn[l][0]
        assert abs(np.linalg.norm(step) - 0.01) < 1e-4 and float(step @ tg[l].grad.numpy()) < 0
    assert bn_new[6] is None


def test_plain_chain_through_the_graph_oracle_is_the_chain_oracle():
    rng = np.random.default_rng(8)
    layers = [no.Layer(8, 8, 4, 8, relu=True, pool=True), no.Layer(4, 4, 8, 8, relu=True, pool=False),
              no.Layer(1, 1, 128, 10, 1, 1, 1, 0, relu=False, pool=False)]
    nodes = [go.Node(L.h, L.w, L.c, L.k, L.r, L.s, L.stride, L.pad, L.relu, L.pool) for L in layers]
    fmts = [(8, 5), (12, 8), (6, 3)]
    x = rng.standard_normal((4, 8, 8, 4)).astype(np.float32)
    ws = [(rng.standard_normal((L.k, L.r, L.s, L.c)) * 0.3).astype(np.float32) for L in layers]
    wq = no.quantize_weights(layers, fmts, ws, 2, 0)
    f1, f2 = no.forward(layers, fmts, wq, x, 2, 0), go.forward(nodes, fmts, wq, [None] * 3, x, 1e-5, 2, 0)
    assert all(np.array_equal(a, b) for a, b in zip(f1["a"], f2["a"]))
    dl = rng.integers(-32, 32, (4, 1, 1, 10))
    b1, b2 = no.backward(layers, fmts, wq, f1, dl, 2, 0), go.backward(nodes, fmts, wq, f2, dl, 5, 2, 0)
    assert all(np.array_equal(a, b) for a, b in zip(b1["g"], b2["g"]))
    assert b2["e_g"] == no.gradient_exponents(fmts, b1, 5)


def test_a_fitted_gradient_that_holds_the_most_negative_code_is_stored_as_it_is():
    """The data gradient of a layer's only consumer is fitted straight into the layer's word length and stored; a
    second fitting pass over it would shift by one bit when a code equals -2^(wl-1) (its magnitude has wl bits).  On a
    plain chain the graph oracle must therefore agree with the chain oracle also in that case."""
    layers = [no.Layer(4, 4, 4, 8, relu=True, pool=False), no.Layer(4, 4, 8, 8, relu=True, pool=False),
              no.Layer(1, 1, 128, 10, 1, 1, 1, 0, relu=False, pool=False)]
    nodes = [go.Node(L.h, L.w, L.c, L.k, L.r, L.s, L.stride, L.pad, L.relu, L.pool) for L in layers]
    fmts = [(4, 1), (4, 2), (6, 3)]
    found = 0
    for seed in range(150):
        rng = np.random.default_rng(seed)
        x = rng.standard_normal((3, 4, 4, 4)).astype(np.float32)
        ws = [(rng.standard_normal((L.k, L.r, L.s, L.c)) * 0.4).astype(np.float32) for L in layers]
        wq = no.quantize_weights(layers, fmts, ws, seed, 0)
        f1, f2 = no.forward(layers, fmts, wq, x, seed, 0), go.forward(nodes, fmts, wq, [None] * 3, x, 1e-5, seed, 0)
        dl = rng.integers(-32, 32, (3, 1, 1, 10))
        b1, b2 = no.backward(layers, fmts, wq, f1, dl, seed, 0), go.backward(nodes, fmts, wq, f2, dl, 5, seed, 0)
        lowest = [int(b1["da"][l].min()) == -(1 << (fmts[l][0] - 1)) for l in range(2)]
        if any(lowest):
            found += 1
            assert all(np.array_equal(a, b) for a, b in zip(b1["g"], b2["g"])), seed
            assert all(np.array_equal(b1["da"][l].ravel(), b2["da"][l].ravel()) for l in range(2)), seed
            assert b2["e_g"] == no.gradient_exponents(fmts, b1, 5), seed
    assert found >= 3                                  # (the case needs the largest magnitude to be negative and in the top eighth of its binade)


# ---- word lengths above 16 bits -------------------------------------------------------------------------------

def _wide_bn_case(seed, shape=(3, 4, 4, 8), wl=28):
    g = np.random.default_rng(seed)
    lim = 1 << (wl - 1)
    y = np.clip(np.rint(g.standard_normal(shape) * (lim / 6) + g.standard_normal(shape[-1]) * (lim / 8)), -lim, lim - 1).astype(np.int64)
    gamma = (1.0 + 0.3 * g.standard_normal(shape[-1])).astype(np.float32)
    beta = (0.2 * g.standard_normal(shape[-1])).astype(np.float32)
    return g, y, gamma, beta


def test_python_integer_path_of_batch_norm_and_merging_equals_the_int64_path():
    g, y, gamma, beta = _bn_case(21)
    res = g.integers(-300, 300, y.shape)
    dz = g.integers(-(1 << 11), 1 << 11, y.shape)
    outs = []
    for flag in (False, True):
        no.force_wide = flag
        try:
            out, st = go.bn_forward(y, 8, gamma, beta, 1e-5, 12, 7, True, 5, 6, res=res, fl_res=5)
            r = go.bn_backward(dz, y, st, 12, 7, 8)
            m, e, sh = go.grad_add(dz, 9, res, 3, 10, 1, 2)
            p = go.gap_forward(y[:, :4, :4, :], 12, 3, 4)
        finally:
            no.force_wide = False
        outs.append((out, st, r, m, e, sh, p))
    a, b = outs
    assert np.array_equal(a[0], b[0]) and a[1]["FA"] == b[1]["FA"] and np.array_equal(a[1]["A"], b[1]["A"]) and np.array_equal(a[1]["B"], b[1]["B"])
    assert np.array_equal(a[1]["mean"], b[1]["mean"]) and np.array_equal(a[1]["sig"], b[1]["sig"])
    assert np.array_equal(a[2]["dy"], b[2]["dy"]) and a[2]["shift"] == b[2]["shift"] and np.array_equal(a[2]["dgamma"], b[2]["dgamma"])
    assert np.array_equal(a[3], b[3]) and a[4:6] == b[4:6] and np.array_equal(a[6], b[6])


@pytest.mark.parametrize("seed", range(2))
def test_batch_norm_on_twenty_eight_bit_codes_is_the_library_routine(seed):
    g, y, gamma, beta = _wide_bn_case(30 + seed)
    fl_y, wl_o, fl_o, eps = 24, 32, 27, 1e-5
    out, st = go.bn_forward(y, fl_y, gamma, beta, eps, wl_o, fl_o, False, 1, 2, mode=orc.RN_HALF_UP)
    yt = torch.tensor(y.astype(np.float64) / 2.0 ** fl_y).permute(0, 3, 1, 2)
    want = F.batch_norm(yt, None, None, torch.tensor(gamma.astype(np.float64)), torch.tensor(beta.astype(np.float64)), True, 0.0, eps)
    want = want.permute(0, 2, 3, 1).numpy()
    # half a step of the 27-bit output grid plus the 2^-30 relative error of the coefficients (values up to about 4)
    assert np.max(np.abs(out / 2.0 ** fl_o - want)) <= 0.5 / 2.0 ** fl_o + 4.0 * 2.0 ** -29
    res = g.integers(-(1 << 23), 1 << 23, y.shape)
    out_r, _ = go.bn_forward(y, fl_y, gamma, beta, eps, wl_o, fl_o, True, 1, 2, res=res, fl_res=20, mode=orc.RN_HALF_UP)
    want_r = np.maximum(want + res / 2.0 ** 20, 0.0)
    assert np.max(np.abs(out_r / 2.0 ** fl_o - want_r)) <= 0.5 / 2.0 ** fl_o + 4.0 * 2.0 ** -29
    flat = (y.astype(np.float64) / 2.0 ** fl_y).reshape(-1, y.shape[-1])
    assert np.allclose(st["mean"] / 2.0 ** fl_y, flat.mean(axis=0), rtol=1e-12, atol=1e-12)
    assert np.allclose((st["sig"] / 2.0 ** fl_y) ** 2, flat.var(axis=0) + eps, rtol=1e-10)
    # the integer totals are exact although the squares pass 64 bits
    assert [int(v) for v in st["s2"]] == [sum(int(v) ** 2 for v in y.reshape(-1, y.shape[-1])[:, k]) for k in range(y.shape[-1])]
    assert max(int(v) for v in st["s2"]) > 1 << 55

    # backward against automatic differentiation, 32-bit gradient codes
    e_dz = 30
    dz = g.integers(-(1 << 30), 1 << 30, y.shape)
    r = go.bn_backward(dz, y, st, 32, 3, 4)
    yt = torch.tensor(y.astype(np.float64) / 2.0 ** fl_y, requires_grad=True)
    gt = torch.tensor(gamma.astype(np.float64), requires_grad=True)
    bt = torch.tensor(beta.astype(np.float64), requires_grad=True)
    z = F.batch_norm(yt.permute(0, 3, 1, 2), None, None, gt, bt, True, 0.0, eps).permute(0, 2, 3, 1)
    (z * torch.tensor(dz.astype(np.float64) / 2.0 ** e_dz)).sum().backward()
    want = yt.grad.numpy()
    got = r["dy"].astype(np.float64) * 2.0 ** -(e_dz + r["e_add"])
    assert np.max(np.abs(got - want)) <= np.max(np.abs(want)) * 2.0 ** -27      # 30-bit coefficients bound the accuracy
    assert int(np.abs(r["dy"]).max()) >= 1 << 30
    assert np.allclose(r["dgamma"] * 2.0 ** -e_dz, gt.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(r["dbeta"] * 2.0 ** -e_dz, bt.grad.numpy(), rtol=1e-12, atol=1e-12)


def test_sum_of_two_wide_gradient_tensors_against_exact_rationals():
    g = np.random.default_rng(40)
    a = g.integers(-(1 << 31), 1 << 31, 50)
    b = g.integers(-(1 << 23), 1 << 23, 50)
    for e_a, e_b in ((10, 50), (50, 10), (7, 7), (0, 40)):
        codes, e, sh = go.grad_add(a, e_a, b, e_b, 32, 1, 2, mode=orc.RN_HALF_UP)
        exact = [Fraction(int(x), 1 << e_a) + Fraction(int(y), 1 << e_b) for x, y in zip(a, b)]
        step = Fraction(1, 1 << e) if e >= 0 else Fraction(1 << -e)
        assert all(abs(Fraction(int(c)) * step - v) <= step / 2 for c, v in zip(codes, exact))
        assert int(np.abs(codes).max()) >= 1 << 30 or sh == 0
    # beyond the gap of 40 the far smaller tensor is left out
    codes, e, sh = go.grad_add(a, 0, b, 41, 32, 1, 2, mode=orc.RN_HALF_UP)
    assert np.array_equal(codes, np.asarray(a)) and e == 0 and sh == 0
