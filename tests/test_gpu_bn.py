"""GPU parity: fixed-point batch normalisation (forward, backward, parameter update), global average pooling and
the merge of two gradient tensors against the CPU oracle: codes, shifts, exponents and coefficient codes bit for
bit; the fp64 statistics and parameter gradients bit for bit as well (the same correctly rounded operations in the
same order on both sides)."""
import numpy as np
import pytest
import torch

import paper_2107_13490_amd as pkg
from oracle import fxp_oracle as orc
from oracle import graph_oracle as go

from gpu_util import ctx, dev, host

pytestmark = pytest.mark.gpu


def _dt(wl):
    return np.int8 if wl <= 8 else np.int16


def _codes(g, shape, wl, scale=0.25, offset=True):
    lim = 1 << (wl - 1)
    v = g.standard_normal(shape) * (lim * scale)
    if offset:
        v = v + g.standard_normal(shape[-1]) * (lim * 0.2)
    return np.clip(np.rint(v), -lim, lim - 1).astype(_dt(wl))


def _state_fields(state, k):
    raw = host(state)
    hdr = raw[:64].view(np.int32)
    body = raw[64:]
    f64 = body[:24 * k].view(np.float64)
    i64 = body[24 * k:40 * k].view(np.int64)
    i32 = body[40 * k:52 * k].view(np.int32)
    return {"channels": int(hdr[0]), "fl_y": int(hdr[1]), "fl_o": int(hdr[2]), "FA": int(hdr[3]), "FB": int(hdr[4]),
            "mean": f64[:k], "sig": f64[k:2 * k], "alpha": f64[2 * k:3 * k], "B": i64[:k], "R": i64[k:2 * k],
            "A": i32[:k], "P": i32[k:2 * k], "Q": i32[2 * k:3 * k]}


BN_CASES = [((4, 6, 6, 8), (8, 5), (8, 5), None), ((3, 8, 8, 16), (12, 8), (12, 8), (8, 4)), ((2, 4, 4, 64), (16, 11), (6, 3), (16, 12)),
            ((5, 3, 7, 24), (8, 4), (16, 10), (12, 6)), ((16, 16, 16, 128), (14, 11), (14, 11), (14, 11)),
            ((7, 5, 5, 40), (12, 9), (12, 7), None), ((1, 1, 1, 8), (8, 5), (8, 5), None), ((2, 3, 3, 2048), (8, 6), (8, 6), (8, 6))]


@pytest.mark.parametrize("shape,fy,fo,fres", BN_CASES)
@pytest.mark.parametrize("relu", [False, True])
def test_batch_norm_forward_and_backward(shape, fy, fo, fres, relu):
    g = np.random.default_rng(sum(shape) + fy[0] + 7 * relu)
    k = shape[-1]
    y = _codes(g, shape, fy[0])
    gamma = (1.0 + 0.3 * g.standard_normal(k)).astype(np.float32)
    beta = (0.3 * g.standard_normal(k)).astype(np.float32)
    res = _codes(g, shape, fres[0], 0.2, False) if fres else None
    eps, seed, stream = 1e-5, 11, 500 + k
    out, state = ctx().bn_forward(dev(y), fy, dev(gamma), dev(beta), eps, fo, relu, dev(res) if fres else None, fres, seed=seed,
                                  stream=stream)
    want, st = go.bn_forward(y, fy[1], gamma, beta, eps, fo[0], fo[1], relu, seed, stream, res, fres[1] if fres else 0)
    got = _state_fields(state, k)
    assert (got["channels"], got["fl_y"], got["fl_o"], got["FA"]) == (k, fy[1], fo[1], st["FA"])
    for name in ("mean", "sig", "alpha"):
        assert np.array_equal(got[name].view(np.uint64), st[name].view(np.uint64)), name
    assert np.array_equal(got["A"], st["A"]) and np.array_equal(got["B"], st["B"])
    assert np.array_equal(host(out).astype(np.int64), want)

    wl_dz, wl_out = fo[0], fy[0]
    dz = _codes(g, shape, wl_dz, 0.3, False)
    e_in = torch.tensor([17], dtype=torch.int64, device="cuda")
    r = ctx().bn_backward(dev(dz), wl_dz, dev(y), fy, state, wl_out, seed=seed, stream=stream + 1, e_in=e_in)
    wb = go.bn_backward(dz, y, st, wl_out, seed, stream + 1)
    got = _state_fields(state, k)
    assert got["FB"] == wb["FB"] and int(host(r["shift"])[0]) == wb["shift"]
    assert int(host(r["e_out"])[0]) == 17 + wb["e_add"]
    assert np.array_equal(host(r["dgamma"]).view(np.uint64), wb["dgamma"].view(np.uint64))
    assert np.array_equal(host(r["dbeta"]).view(np.uint64), wb["dbeta"].view(np.uint64))
    assert np.array_equal(host(r["dy"]).astype(np.int64), wb["dy"])

    gdev, bdev = dev(gamma.copy()), dev(beta.copy())
    ctx().bn_update(gdev, bdev, r["dgamma"], r["dbeta"], 0.05)
    g2, b2 = go.bn_update(gamma, beta, wb["dgamma"], wb["dbeta"], 0.05)
    assert np.array_equal(host(gdev).view(np.uint32), g2.view(np.uint32)) and np.array_equal(host(bdev).view(np.uint32), b2.view(np.uint32))


def test_batch_norm_special_channels_and_nearest_rounding():
    g = np.random.default_rng(3)
    y = _codes(g, (4, 4, 4, 16), 12)
    y[..., 3] = 77                                  # a constant channel
    y[..., 5] = 0
    gamma = g.standard_normal(16).astype(np.float32)
    gamma[7] = 0.0
    beta = g.standard_normal(16).astype(np.float32)
    out, state = ctx().bn_forward(dev(y), (12, 8), dev(gamma), dev(beta), 1e-5, (12, 8), False, mode=pkg.RN_HALF_UP)
    want, st = go.bn_forward(y, 8, gamma, beta, 1e-5, 12, 8, False, 0, 0, mode=orc.RN_HALF_UP)
    assert np.array_equal(host(out).astype(np.int64), want)
    zero = np.zeros_like(y)
    r = ctx().bn_backward(dev(zero), 12, dev(y), (12, 8), state, 12)
    assert not host(r["dy"]).any() and int(host(r["shift"])[0]) == 0 and not host(r["dgamma"]).any()
    # all gains zero: FA = 30, the output is beta
    gz = np.zeros(16, np.float32)
    out, state = ctx().bn_forward(dev(y), (12, 8), dev(gz), dev(beta), 1e-5, (12, 8), False, mode=pkg.RN_HALF_UP)
    want, st = go.bn_forward(y, 8, gz, beta, 1e-5, 12, 8, False, 0, 0, mode=orc.RN_HALF_UP)
    assert st["FA"] == 30 and np.array_equal(host(out).astype(np.int64), want)


@pytest.mark.parametrize("channels", [1, 8, 520, 2048, 2049, 4096])
def test_batch_norm_update_alone_many_channels(channels):
    # sums of squares in channel order across the kernel's staging chunks; magnitudes spread over many binades
    g = np.random.default_rng(channels)
    gamma, beta = g.standard_normal(channels).astype(np.float32), g.standard_normal(channels).astype(np.float32)
    dgam = g.standard_normal(channels) * np.exp2(g.integers(-30, 30, channels))
    dbet = g.standard_normal(channels) * np.exp2(g.integers(-8, 8, channels))
    gdev, bdev = dev(gamma.copy()), dev(beta.copy())
    ctx().bn_update(gdev, bdev, dev(dgam), dev(dbet), 0.125)
    g2, b2 = go.bn_update(gamma, beta, dgam, dbet, 0.125)
    assert np.array_equal(host(gdev).view(np.uint32), g2.view(np.uint32)) and np.array_equal(host(bdev).view(np.uint32), b2.view(np.uint32))


def test_batch_norm_rejects_what_it_does_not_handle():
    y = torch.zeros((2, 2, 2, 12), dtype=torch.int8, device="cuda")
    p = torch.ones(12, dtype=torch.float32, device="cuda")
    with pytest.raises(pkg.AdaptError):
        ctx().bn_forward(y, (8, 4), p, p, 1e-5, (8, 4))                    # channels not a multiple of 8
    with pytest.raises(pkg.AdaptError):
        ctx().bn_forward(y[..., :8].contiguous(), (8, 4), p, p, -1.0, (8, 4))


@pytest.mark.parametrize("shape,wl", [((3, 4, 4, 8), 8), ((2, 2, 2, 16), 12), ((5, 8, 8, 64), 16), ((4, 1, 1, 8), 6), ((2, 4, 8, 24), 10)])
def test_global_average_pooling(shape, wl):
    g = np.random.default_rng(shape[-1] + wl)
    a = _codes(g, shape, wl)
    out = ctx().gap_fwd(dev(a), (wl, wl - 3), seed=4, stream=9)
    want = go.gap_forward(a, wl, 4, 9)
    assert np.array_equal(host(out).astype(np.int64), want)
    da = ctx().gap_bwd(out, wl, shape[1], shape[2])
    wd, up = go.gap_backward(want, shape[1], shape[2])
    assert np.array_equal(host(da).astype(np.int64), wd) and up == (shape[1] * shape[2]).bit_length() - 1


@pytest.mark.parametrize("n", [1, 7, 8, 1000, 70001])
@pytest.mark.parametrize("wl_a,wl_b,wl_o,e_a,e_b", [(8, 8, 8, 5, 9), (8, 12, 8, 9, 5), (16, 16, 16, 3, 3), (12, 8, 16, 0, 30),
                                                   (8, 16, 4, 12, 2), (16, 16, 12, 0, 41), (8, 8, 8, 50, 3), (8, 8, 8, -7, -2)])
def test_sum_of_two_gradient_tensors(n, wl_a, wl_b, wl_o, e_a, e_b):
    g = np.random.default_rng(n + wl_a + e_a)
    a, b = _codes(g, (n,), wl_a, 0.3, False), _codes(g, (n,), wl_b, 0.3, False)
    ea = torch.tensor([e_a], dtype=torch.int64, device="cuda")
    eb = torch.tensor([e_b], dtype=torch.int64, device="cuda")
    out, shift, e = ctx().grad_add(dev(a), wl_a, ea, dev(b), wl_b, eb, wl_o, seed=2, stream=n)
    want, we, ws = go.grad_add(a, e_a, b, e_b, wl_o, 2, n)
    assert (int(host(shift)[0]), int(host(e)[0])) == (ws, we)
    assert np.array_equal(host(out).astype(np.int64), want)
    # one tensor alone, refitted
    out, shift, e = ctx().grad_add(dev(a), wl_a, ea, None, 8, None, wl_o, seed=2, stream=n)
    want, we, ws = go.grad_add(a, e_a, None, None, wl_o, 2, n)
    assert (int(host(shift)[0]), int(host(e)[0])) == (ws, we) and np.array_equal(host(out).astype(np.int64), want)


# ---- word lengths above 16 bits --------------------------------------------------------------------------------

def _dtw(wl):
    return np.int8 if wl <= 8 else np.int16 if wl <= 16 else np.int32


def _codes_w(g, shape, wl, scale=0.25, offset=True):
    lim = 1 << (wl - 1)
    v = g.standard_normal(shape) * (lim * scale)
    if offset:
        v = v + g.standard_normal(shape[-1]) * (lim * 0.2)
    return np.clip(np.rint(v), -lim, lim - 1).astype(np.int64)


WIDE_BN_CASES = [((3, 4, 4, 8), (28, 22), (32, 26), None), ((2, 5, 3, 16), (32, 20), (24, 18), (20, 15)), ((4, 2, 2, 24), (12, 8), (20, 15), (32, 28)),
                 ((2, 3, 3, 8), (24, 20), (8, 4), (8, 5)), ((1, 1, 2, 8), (17, 10), (17, 10), None), ((9, 7, 5, 40), (32, 30), (32, 30), (32, 30)),
                 ((33, 11, 13, 16), (24, 19), (20, 14), (16, 12))]           # 4719 rows: many rows per block of the statistics pass


@pytest.mark.parametrize("shape,fy,fo,fres", WIDE_BN_CASES)
@pytest.mark.parametrize("relu", [False, True])
def test_batch_norm_above_sixteen_bits(shape, fy, fo, fres, relu):
    g = np.random.default_rng(sum(shape) + fy[0] + 7 * relu)
    k = shape[-1]
    y = _codes_w(g, shape, fy[0])
    gamma = (1.0 + 0.3 * g.standard_normal(k)).astype(np.float32)
    beta = (0.3 * g.standard_normal(k)).astype(np.float32)
    res = _codes_w(g, shape, fres[0], 0.2, False) if fres else None
    eps, seed, stream = 1e-5, 13, 900 + k
    out, state = ctx().bn_forward(dev(y.astype(_dtw(fy[0]))), fy, dev(gamma), dev(beta), eps, fo, relu,
                                  dev(res.astype(_dtw(fres[0]))) if fres else None, fres, seed=seed, stream=stream)
    want, st = go.bn_forward(y, fy[1], gamma, beta, eps, fo[0], fo[1], relu, seed, stream, res, fres[1] if fres else 0)
    got = _state_fields(state, k)
    assert (got["channels"], got["fl_y"], got["fl_o"], got["FA"]) == (k, fy[1], fo[1], st["FA"])
    for name in ("mean", "sig", "alpha"):
        assert np.array_equal(got[name].view(np.uint64), st[name].view(np.uint64)), name
    assert np.array_equal(got["A"], st["A"]) and np.array_equal(got["B"], st["B"])
    assert np.array_equal(host(out).astype(np.int64), want)

    wl_dz, wl_out = fo[0], fy[0]
    dz = _codes_w(g, shape, wl_dz, 0.3, False)
    e_in = torch.tensor([-5], dtype=torch.int64, device="cuda")
    r = ctx().bn_backward(dev(dz.astype(_dtw(wl_dz))), wl_dz, dev(y.astype(_dtw(fy[0]))), fy, state, wl_out, seed=seed, stream=stream + 1,
                          e_in=e_in)
    wb = go.bn_backward(dz, y, st, wl_out, seed, stream + 1)
    got = _state_fields(state, k)
    assert got["FB"] == wb["FB"] and int(host(r["shift"])[0]) == wb["shift"]
    assert int(host(r["e_out"])[0]) == -5 + wb["e_add"]
    assert np.array_equal(host(r["dgamma"]).view(np.uint64), wb["dgamma"].view(np.uint64))
    assert np.array_equal(host(r["dbeta"]).view(np.uint64), wb["dbeta"].view(np.uint64))
    assert np.array_equal(host(r["dy"]).astype(np.int64), wb["dy"])


@pytest.mark.parametrize("wl", [17, 24, 32])
def test_average_pooling_and_gradient_merge_above_sixteen_bits(wl):
    g = np.random.default_rng(wl)
    a = _codes_w(g, (3, 4, 4, 16), wl, 0.4)
    a.reshape(-1)[:3] = [(1 << (wl - 1)) - 1, -(1 << (wl - 1)), 0]
    out = ctx().gap_fwd(dev(a.astype(np.int32)), (wl, 3), seed=2, stream=9)
    assert np.array_equal(host(out).astype(np.int64), go.gap_forward(a, wl, 2, 9))
    one = ctx().gap_fwd(dev(a[:, :1, :1, :].astype(np.int32).copy()), (wl, 3), seed=2, stream=9)     # a single position: the codes themselves
    assert np.array_equal(host(one).astype(np.int64), a[:, 0, 0, :])
    d = _codes_w(g, (3, 16), wl, 0.4, False)
    da = ctx().gap_bwd(dev(d.astype(np.int32)), wl, 4, 4)
    assert np.array_equal(host(da).astype(np.int64), go.gap_backward(d, 4, 4)[0])
    for wl_b, e_a, e_b in ((wl, 3, 3), (12, 0, 30), (wl, 45, 5), (8, 2, 43), (32, 20, 0)):
        x = _codes_w(g, 5000, wl, 0.3, False)
        y = _codes_w(g, 5000, wl_b, 0.3, False)
        ea = torch.tensor([e_a], dtype=torch.int64, device="cuda")
        eb = torch.tensor([e_b], dtype=torch.int64, device="cuda")
        for wl_out in (wl, 10):
            codes, shift, e_out = ctx().grad_add(dev(x.astype(np.int32)), wl, ea, dev(y.astype(_dtw(wl_b))), wl_b, eb, wl_out, seed=4, stream=7)
            want, e, sh = go.grad_add(x, e_a, y, e_b, wl_out, 4, 7)
            assert int(host(shift)[0]) == sh and int(host(e_out)[0]) == e, (wl_b, e_a, e_b, wl_out)
            assert np.array_equal(host(codes).astype(np.int64), want)
    codes, shift, e_out = ctx().grad_add(dev(x.astype(np.int32)), wl, ea, None, 8, None, 12, seed=4, stream=7)        # refit alone
    want, e, sh = go.grad_add(x, e_a, None, None, 12, 4, 7)
    assert np.array_equal(host(codes).astype(np.int64), want) and int(host(e_out)[0]) == e
