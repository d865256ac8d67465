"""Pins for the oracle's integer contractions (CPU only).

The layer contractions are the plain zero-padded cross-correlation and its two adjoints
(the "ForwardPass" of Alg. 1 on quantized layers and the gradients of Sec. 3.3).  They are
pinned to library routines (numpy matmul, torch conv2d + autograd in fp64, which is exact for
these small integers), to the adjoint identity, and to special cases.
"""
import numpy as np
import pytest
import torch

from oracle import conv_oracle as co
from oracle import fxp_oracle as orc

CASES = [
    # n, h, w, c, k, r, s, stride, pad
    (2, 5, 6, 3, 4, 3, 3, 1, 1),
    (1, 8, 8, 16, 8, 3, 3, 2, 1),
    (3, 7, 5, 4, 5, 1, 1, 1, 0),
    (2, 9, 9, 2, 3, 5, 5, 2, 2),
    (2, 6, 6, 8, 8, 1, 1, 2, 0),
    (1, 4, 4, 1, 1, 3, 3, 1, 0),
]


def _rand(shape, lo, hi, seed):
    return np.random.default_rng(seed).integers(lo, hi + 1, shape)


def test_gemm_naive_loops_tiny():
    a = _rand((3, 4), -8, 7, 0)
    b = _rand((4, 2), -8, 7, 1)
    want = [[sum(int(a[m, k]) * int(b[k, n]) for k in range(4)) for n in range(2)] for m in range(3)]
    assert co.gemm(a, b).tolist() == want
    assert orc.gemm(a, b).tolist() == want


def test_gemm_matches_numpy_and_transposes():
    a = _rand((37, 129), -32768, 32767, 2)
    b = _rand((129, 23), -32768, 32767, 3)
    want = a.astype(np.int64) @ b.astype(np.int64)
    assert np.array_equal(co.gemm(a, b), want)
    assert np.array_equal(orc.gemm(a.T, b, trans_a=True), want)
    assert np.array_equal(orc.gemm(a, b.T, trans_b=True), want)


@pytest.mark.parametrize("case", CASES)
def test_conv_against_torch_fp64(case):
    n, h, w, c, k, r, s, st, pad = case
    x = _rand((n, h, w, c), -128, 127, 10)
    wt = _rand((k, r, s, c), -128, 127, 11)
    xt = torch.tensor(x.transpose(0, 3, 1, 2), dtype=torch.float64, requires_grad=True)
    wtt = torch.tensor(wt.transpose(0, 3, 1, 2), dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.conv2d(xt, wtt, stride=st, padding=pad)
    y = co.conv_fwd(x, wt, st, pad)
    assert np.array_equal(y, yt.detach().numpy().transpose(0, 2, 3, 1).astype(np.int64))
    dy = _rand(y.shape, -128, 127, 12)
    gx, gw = torch.autograd.grad(yt, (xt, wtt), torch.tensor(dy.transpose(0, 3, 1, 2), dtype=torch.float64))
    dx = co.conv_dgrad(dy, wt, h, w, st, pad)
    dw = co.conv_wgrad(dy, x, r, s, st, pad)
    assert np.array_equal(dx, gx.numpy().transpose(0, 2, 3, 1).astype(np.int64))
    assert np.array_equal(dw, gw.numpy().transpose(0, 2, 3, 1).astype(np.int64))


@pytest.mark.parametrize("case", CASES)
def test_adjoint_identity_exact(case):
    n, h, w, c, k, r, s, st, pad = case
    x = _rand((n, h, w, c), -32768, 32767, 20)
    wt = _rand((k, r, s, c), -32768, 32767, 21)
    y = co.conv_fwd(x, wt, st, pad)
    dy = _rand(y.shape, -32768, 32767, 22)
    dx = co.conv_dgrad(dy, wt, h, w, st, pad)
    dw = co.conv_wgrad(dy, x, r, s, st, pad)

    def dot(a, b):
        return sum(int(u) * int(v) for u, v in zip(a.ravel().tolist(), b.ravel().tolist()))

    lhs = dot(y, dy)
    assert lhs == dot(x, dx) == dot(wt, dw)


def test_pointwise_conv_is_gemm():
    x = _rand((2, 4, 4, 16), -128, 127, 30)
    wt = _rand((8, 1, 1, 16), -128, 127, 31)
    y = co.conv_fwd(x, wt, 1, 0)
    assert np.array_equal(y.reshape(-1, 8), x.reshape(-1, 16).astype(np.int64) @ wt.reshape(8, 16).T.astype(np.int64))


def test_one_hot_tap_shifts_the_input():
    x = _rand((1, 6, 7, 2), -100, 100, 40)
    for r in range(3):
        for s in range(3):
            wt = np.zeros((2, 3, 3, 2), dtype=np.int64)
            wt[0, r, s, 0] = 1
            wt[1, r, s, 1] = 1
            y = co.conv_fwd(x, wt, 1, 1)
            xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
            assert np.array_equal(y, xp[:, r:r + 6, s:s + 7, :])


def test_dequantized_conv_equals_float_conv_of_dequantized_operands():
    """Fixed-point semantics: the integer result carries FL_x + FL_w fractional bits."""
    g = np.random.default_rng(50)
    xf = g.standard_normal((2, 6, 6, 4)).astype(np.float32)
    wf = (g.standard_normal((3, 3, 3, 4)) * 0.2).astype(np.float32)
    qx, _, _ = orc.quantize(xf, 8, 5, seed=1, stream=1)
    qw, _, _ = orc.quantize(wf, 8, 6, seed=1, stream=2)
    y = co.conv_fwd(qx, qw, 1, 1)
    yt = torch.nn.functional.conv2d(torch.tensor(orc.dequantize(qx, 5).transpose(0, 3, 1, 2)),
                                    torch.tensor(orc.dequantize(qw, 6).transpose(0, 3, 1, 2)), padding=1)
    assert np.array_equal(orc.dequantize(y, 11), yt.numpy().transpose(0, 2, 3, 1))


def test_worst_case_operands():
    # all-minimum codes: every product is 2^30, K = 9*8 = 72 terms
    x = np.full((1, 3, 3, 8), -32768)
    wt = np.full((2, 3, 3, 8), -32768)
    y = co.conv_fwd(x, wt, 1, 1)
    assert y[0, 1, 1, 0] == 72 * (1 << 30)
    assert y[0, 0, 0, 0] == 32 * (1 << 30)
