"""Pins of the 17..32-bit oracle (oracle/wide_oracle.py): on operands that fit the narrow oracle it must give what
that oracle (pinned elsewhere, int64 / C) gives; products at the corners of the 32-bit range against hand values;
the requantize rule against exact rationals; quantize to 32 bits against closed forms."""
from fractions import Fraction

import numpy as np

from oracle import conv_oracle as co
from oracle import fxp_oracle as orc
from oracle import wide_oracle as wo


def test_contractions_agree_with_the_narrow_oracle_on_narrow_operands():
    g = np.random.default_rng(1)
    a, b = g.integers(-2000, 2000, (7, 13)), g.integers(-2000, 2000, (13, 5))
    assert np.array_equal(wo.gemm(a, b).astype(np.int64), orc.gemm(a, b))
    assert np.array_equal(wo.gemm(a.T.copy(), b.T.copy(), True, True).astype(np.int64), orc.gemm(a, b))
    x, w = g.integers(-300, 300, (2, 7, 6, 5)), g.integers(-300, 300, (4, 3, 3, 5))
    for stride, pad in ((1, 1), (2, 1), (1, 0), (2, 0)):
        y = co.conv_fwd(x, w, stride, pad)
        assert np.array_equal(wo.conv_fwd(x, w, stride, pad).astype(np.int64), y)
        dy = g.integers(-300, 300, y.shape)
        assert np.array_equal(wo.conv_dgrad(dy, w, 7, 6, stride, pad).astype(np.int64), co.conv_dgrad(dy, w, 7, 6, stride, pad))
        assert np.array_equal(wo.conv_wgrad(dy, x, 3, 3, stride, pad).astype(np.int64), co.conv_wgrad(dy, x, 3, 3, stride, pad))


def test_corner_products_do_not_wrap():
    lo, hi = -(1 << 31), (1 << 31) - 1
    a = np.array([[lo, hi, lo]], dtype=np.int64)
    b = np.array([[lo], [hi], [hi]], dtype=np.int64)
    assert int(wo.gemm(a, b)[0, 0]) == (1 << 62) + ((1 << 31) - 1) ** 2 - (1 << 31) * ((1 << 31) - 1)
    a = np.array([[lo, lo, lo]], dtype=np.int64)
    assert int(wo.gemm(a, a.T.copy())[0, 0]) == 3 << 62                # beyond int64
    x = np.full((1, 3, 3, 2), hi, dtype=np.int64)
    w = np.full((1, 3, 3, 2), hi, dtype=np.int64)
    assert int(wo.conv_fwd(x, w, 1, 1)[0, 1, 1, 0]) == 18 * hi * hi


def test_requantize_matches_the_narrow_rule_and_exact_rationals():
    g = np.random.default_rng(2)
    acc = g.integers(-(1 << 40), 1 << 40, 500)
    for shift, wl in ((0, 32), (-3, 32), (5, 32), (16, 24), (17, 32), (30, 20), (40, 8)):
        for mode in (orc.SR, orc.RN_HALF_UP):
            got = wo.requantize(acc, shift, wl, mode, 3, 4, relu=(shift == 5))
            if wl <= 16 or True:
                want = orc.requantize(acc, shift, wl, mode, 3, 4, relu=(shift == 5)) if abs(shift) < 24 else None
                if want is not None:
                    assert np.array_equal(got, want), (shift, wl, mode)
    # a 100-bit accumulator: within one step of the exact quotient, saturating at 32 bits
    big = [(-1) ** i * ((1 << 99) // (i + 1)) for i in range(40)]
    q = wo.requantize(np.array(big, dtype=object), 70, 32, orc.SR, 1, 1)
    for v, c in zip(big, q):
        exact = Fraction(v, 1 << 70)
        assert abs(Fraction(int(c)) - max(min(exact, (1 << 31) - 1), -(1 << 31))) < 1
    assert int(q[0]) == (1 << 29) and int(q[1]) == -(1 << 28)          # 2^99 / 2^70 and -2^98 / 2^70 are exact


def test_quantize_to_thirty_two_bits():
    # values on the grid are reproduced exactly whatever the rounding bits; fp32 has 24 significant bits, so codes
    # of 2^24 and more are exact integers times a power of two
    codes = np.array([0, 1, -1, (1 << 23) + 1, -(1 << 23) - 1, 1 << 30, -(1 << 31), (1 << 31) - 128], dtype=np.int64)
    x = (codes.astype(np.float64) * 2.0 ** -20).astype(np.float32)
    q, nnz, sat = orc.quantize(x, 32, 20, orc.SR, 5, 6)
    assert np.array_equal(q, codes) and nnz == 7 and sat == 0
    # saturation at both ends, NaN -> 0, infinities saturate
    x = np.array([3000.0, -3000.0, 2048.0, -2048.0, np.nan, np.inf, -np.inf], dtype=np.float32)
    q, nnz, sat = orc.quantize(x, 32, 20, orc.SR, 5, 6)
    assert q.tolist() == [(1 << 31) - 1, -(1 << 31), (1 << 31) - 1, -(1 << 31), 0, (1 << 31) - 1, -(1 << 31)] and sat == 5
    # small values still round stochastically on the 2^-31 grid: mean of many draws is the value
    x = np.full(20000, 2.0 ** -32 * 0.75, dtype=np.float32)
    q, _, _ = orc.quantize(x, 32, 31, orc.SR, 1, 2)
    assert set(np.unique(q)) <= {0, 1} and abs(q.mean() - 0.375) < 0.02
    # 17 bits: the first word length that needs int32 storage
    x = (np.random.default_rng(3).standard_normal(1000) * 0.3).astype(np.float32)
    q, _, _ = orc.quantize(x, 17, 15, orc.RN_HALF_UP, 0, 0)
    assert np.array_equal(q, np.clip(np.floor(x.astype(np.float64) * 2 ** 15 + 0.5), -(1 << 16), (1 << 16) - 1).astype(np.int64))


# ---- fitting requantization, gradient diversity and the chained step above 16 bits ---------------------------------

def test_fitting_requantization_agrees_with_the_narrow_oracle_and_with_closed_forms():
    from oracle import net_oracle as no
    g = np.random.default_rng(11)
    for wl in (4, 8, 13, 16):
        acc = g.integers(-(1 << 40), 1 << 40, 500)
        for mode in (orc.SR, orc.RN_HALF_UP):
            q0, s0, ss0 = no.requantize_fit(acc, wl, mode, 3, 9)
            q1, s1, ss1 = wo.requantize_fit(acc, wl, mode, 3, 9)
            assert s0 == s1 and ss0 == ss1 and np.array_equal(q0, q1)
    # accumulators far beyond 64 bits: the shift leaves wl - 1 magnitude bits; values on the coarse grid come out exactly
    for wl in (17, 24, 32):
        for top in (70, 100, 126):
            vals = [int(v) for v in g.integers(-(1 << 20), 1 << 20, 64)]
            sh_expect = top - (wl - 1)
            acc = np.array([v << (top - 21) for v in vals] + [(1 << top) - 1], dtype=object)
            assert wo.fit_shift(acc, wl) == sh_expect
            q, sh, ss = wo.requantize_fit(acc[:-1] - acc[:-1] % (1 << sh_expect), wl, orc.RN_HALF_UP)
            # without the largest element the maximum may have fewer bits: recompute and compare with exact division
            exact = [Fraction(int(a), 1 << sh) for a in (acc[:-1] - acc[:-1] % (1 << sh_expect))]
            assert all(abs(Fraction(int(c)) - e) <= Fraction(1, 2) for c, e in zip(q, exact))
            assert ss == sum(int(c) ** 2 for c in q)
    # largest magnitude 2^(wl-1) - 1 needs no shift, 2^(wl-1) needs one
    for wl in (17, 32):
        assert wo.fit_shift(np.array([(1 << (wl - 1)) - 1, -5], dtype=object), wl) == 0
        assert wo.fit_shift(np.array([-(1 << (wl - 1)), 3], dtype=object), wl) == 1
    q, sh, _ = wo.requantize_fit(np.array([(1 << 31) - 1, -(1 << 31) + 1, 12345], dtype=object), 32, orc.SR, 1, 2)
    assert sh == 0 and [int(v) for v in q] == [(1 << 31) - 1, -(1 << 31) + 1, 12345]


def test_gradient_diversity_on_wide_codes():
    from oracle import pushup_oracle as po
    g = np.random.default_rng(12)
    codes = [g.integers(-100, 100, 40) for _ in range(5)]
    fls = [3, 0, 2, 2, 1]
    a, b = po.gradient_diversity(codes, fls), wo.gradient_diversity(codes, fls)
    assert a["sumsq"] == b["sumsq"] and a["sumsq_sum"] == b["sumsq_sum"] and a["ds"] == b["ds"] and a["log_ds"] == b["log_ds"]
    # a common factor of 2^20 on every tensor scales the integer sums by 2^40 and leaves the ratio alone
    big = [c.astype(object) * (1 << 20) for c in codes]
    c2 = wo.gradient_diversity(big, fls)
    assert c2["sumsq"] == [s << 40 for s in a["sumsq"]] and c2["sumsq_sum"] == a["sumsq_sum"] << 40
    assert abs(c2["ds"] - a["ds"]) <= 1e-14 * a["ds"]
    # equal tensors: ds = 1; tensors with disjoint supports and equal norms: ds = sqrt(k)
    t = np.array([(1 << 31) - 1, -(1 << 31), 7, 0], dtype=object)
    assert abs(wo.gradient_diversity([t, t, t], [0, 0, 0])["ds"] - 1.0) < 1e-15
    e = [np.array([(1 << 30) if i == k else 0 for i in range(4)], dtype=object) for k in range(4)]
    assert abs(wo.gradient_diversity(e, [0] * 4)["ds"] - 2.0) < 1e-15
    # one tensor on a coarser grid: value = code * 2^-fl, so halving fl while doubling nothing changes the norms' ratio
    r = wo.gradient_diversity([t, t], [4, 0])
    num = float(np.sqrt(float(sum(int(v) ** 2 for v in t)))) * (1 + 2.0 ** -4)
    den = float(np.sqrt(float(sum((int(v) + (int(v) << 4)) ** 2 for v in t)))) * 2.0 ** -4
    assert abs(r["ds"] - num / den) < 1e-15


def test_chain_oracle_on_python_integers_equals_the_int64_chain():
    from oracle import net_oracle as no
    rng = np.random.default_rng(13)
    layers = [no.Layer(6, 6, 3, 8, pool=True), no.Layer(3, 3, 8, 8, 3, 3, 1, 1), no.Layer(1, 1, 72, 5, 1, 1, 1, 0, relu=False)]
    fmts = [(9, 5), (16, 11), (6, 3)]
    n = 3
    x = rng.standard_normal((n, 6, 6, 3)).astype(np.float32)
    ws = [(rng.standard_normal((L.k, L.r, L.s, L.c)) * 0.3).astype(np.float32) for L in layers]
    dl = rng.integers(-20, 20, (n, 1, 1, 5))
    out = []
    for flag in (False, True):
        no.force_wide = flag
        try:
            wq = no.quantize_weights(layers, fmts, ws, 2, 50)
            fwd = no.forward(layers, fmts, wq, x, 2, 50)
            bwd = no.backward(layers, fmts, wq, fwd, dl, 2, 50)
            upd = no.update(layers, fmts, ws, bwd, 0.05, 0.0, 1e-3, 2, 50)
        finally:
            no.force_wide = False
        out.append((fwd, bwd, upd))
    (f0, b0, u0), (f1, b1, u1) = out
    for l in range(3):
        assert np.array_equal(f0["y"][l], f1["y"][l]) and np.array_equal(f0["a"][l], f1["a"][l])
        assert np.array_equal(b0["g"][l], b1["g"][l]) and b0["shift_w"][l] == b1["shift_w"][l] and b0["sumsq"][l] == b1["sumsq"][l]
        assert b0["shift_a"][l] == b1["shift_a"][l]
        assert np.array_equal(u0[l]["q"], u1[l]["q"]) and np.array_equal(u0[l]["w"].view(np.uint32), u1[l]["w"].view(np.uint32))


def test_wide_chain_follows_a_floating_point_network_closely():
    import torch
    import torch.nn.functional as F
    from oracle import net_oracle as no
    rng = np.random.default_rng(14)
    layers = [no.Layer(4, 4, 3, 4, pool=True), no.Layer(2, 2, 4, 4, 3, 3, 1, 1), no.Layer(1, 1, 16, 5, 1, 1, 1, 0, relu=False)]
    n = 2
    fmts = [(28, 22), (32, 24), (24, 18)]
    x = rng.standard_normal((n, 4, 4, 3)).astype(np.float32)
    ws = [(rng.standard_normal((L.k, L.r, L.s, L.c)) * 0.3).astype(np.float32) for L in layers]
    t = rng.standard_normal((n, 5))
    wq = no.quantize_weights(layers, fmts, ws, 1, 100)
    fwd = no.forward(layers, fmts, wq, x, 1, 100)
    dl = np.round(t * 2 ** 20).astype(np.int64).reshape(n, 1, 1, 5)        # 24-bit codes of t
    bwd = no.backward(layers, fmts, wq, fwd, dl, 1, 100)
    tw = [torch.tensor(np.transpose(w.astype(np.float64), (0, 3, 1, 2)), requires_grad=True) for w in ws]
    h = torch.tensor(np.transpose(x.astype(np.float64), (0, 3, 1, 2)))
    h = F.max_pool2d(F.relu(F.conv2d(h, tw[0], padding=1)), 2)
    h = F.relu(F.conv2d(h, tw[1], padding=1))
    logits = F.conv2d(h.permute(0, 2, 3, 1).reshape(n, 16, 1, 1), tw[2])
    (logits.reshape(n, 5) * torch.tensor(t)).sum().backward()
    got = fwd["a"][2].reshape(n, 5) / 2.0 ** 18
    assert np.max(np.abs(got - logits.detach().numpy().reshape(n, 5))) < 2e-5      # a few steps of the 18-bit output grid
    for l in range(3):
        want = np.transpose(tw[l].grad.numpy(), (0, 2, 3, 1)).ravel()
        g = bwd["g"][l].astype(np.float64).ravel()
        cos = float(g @ want / np.sqrt((g @ g) * (want @ want)))
        assert cos > 1 - 1e-9, (l, cos)
        assert int(np.abs(bwd["g"][l]).max()) >= 1 << (fmts[l][0] - 2) or bwd["shift_w"][l] == 0
        assert bwd["sumsq"][l] == sum(int(v) ** 2 for v in bwd["g"][l].ravel())


def test_update_with_wide_gradient_codes_and_wide_weights_closed_form():
    from oracle import sgd_oracle as so
    # one non-zero gradient code: its normalised value is +-1, so w' = w -+ lr exactly when all are powers of two
    w = np.array([0.5, -0.25, 0.0, 1.0], np.float32)
    c = np.array([0, 0, -(1 << 31), 0], np.int64)
    r = so.sgd_update_quantize(w, c, 0, 0.125, 0.0, 0.0, 32, 28, orc.RN_HALF_UP)
    assert r["sumsq"] == 1 << 62 and float(r["step"]) == 0.125 / 2.0 ** 31
    assert list(r["w"]) == [0.5, -0.25, 0.125, 1.0]
    assert [int(v) for v in r["q"]] == [1 << 27, -(1 << 26), 1 << 25, 1 << 28]
    # a sum of squares beyond 64 bits: 8 codes of magnitude 2^31 - 1
    c = np.full(8, (1 << 31) - 1, np.int64)
    r = so.sgd_update_quantize(np.zeros(8, np.float32), c, 0, 1.0, 0.0, 0.0, 24, 20, orc.RN_HALF_UP)
    assert r["sumsq"] == 8 * ((1 << 31) - 1) ** 2 and r["sumsq"] > 1 << 64
    want = -np.float32(np.float32(1.0 / np.sqrt(float(r["sumsq"]))) * np.float32(2.0 ** 31))     # fp32(code) = 2^31
    assert np.all(r["w"] == want) and abs(float(want) + 1.0 / np.sqrt(8.0)) < 1e-7


def test_residual_addition_of_wide_codes_is_the_rounded_exact_sum():
    from oracle import net_oracle as no
    g = np.random.default_rng(15)
    a = g.integers(-(1 << 31), 1 << 31, 200)
    b = g.integers(-(1 << 23), 1 << 23, 200)
    for (fl_a, fl_b, wl_o, fl_o) in ((31, 0, 32, 0), (5, 20, 32, 28), (20, 5, 17, 3), (10, 10, 8, 0)):
        got = no.residual_add(a, fl_a, b, fl_b, wl_o, fl_o, orc.RN_HALF_UP)
        lo, hi = -(1 << (wl_o - 1)), (1 << (wl_o - 1)) - 1
        for x, y, c in zip(a, b, got):
            v = (Fraction(int(x), 1 << fl_a) + Fraction(int(y), 1 << fl_b)) * (1 << fl_o)
            want = min(max((v + Fraction(1, 2)).__floor__(), lo), hi)
            # above 16 dropped bits the rule floors once before the 16 guard bits: at most one step below the exact rounding
            assert int(c) == want or (max(fl_a, fl_b) - fl_o > 16 and int(c) == max(want - 1, lo)), (x, y, c, want)
    # narrow inputs: identical to the int64 path
    a8, b8 = g.integers(-128, 128, 300), g.integers(-2000, 2000, 300)
    no.force_wide = True
    try:
        w = no.residual_add(a8, 5, b8, 9, 12, 7, orc.SR, 3, 4, True)
    finally:
        no.force_wide = False
    assert np.array_equal(w, no.residual_add(a8, 5, b8, 9, 12, 7, orc.SR, 3, 4, True))
