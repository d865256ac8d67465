"""GPU parity: adapt_sgd_update_quantize and adapt_kld_precision_search_ranged against the CPU
oracle (Alg. 1 backward-pass line + Quantize loop; Sec. 3.3 gradient normalisation; Sec. 3.4
L1/L2 terms).  The fp32 master weights, the codes, the counters and the range are compared bit
for bit: the update is three explicit fused multiply-adds on both sides."""
import numpy as np
import pytest
import torch

import paper_2107_13490_amd as pkg
import workloads as wk
from oracle import fxp_oracle as orc
from oracle import sgd_oracle as so

from gpu_util import ctx, dev, host, u64

pytestmark = pytest.mark.gpu


def _grad_codes(rng, n, wl):
    lim = 1 << (wl - 1)
    return np.clip(np.rint(rng.standard_normal(n) * lim * 0.3), -lim, lim - 1).astype(np.int8 if wl <= 8 else np.int16)


def _run(w, g, fg, lr, l1, l2, wl, fl, normalize=True, mode=pkg.SR, seed=0, stream=0):
    wd = dev(w.copy())
    gd = dev(g)
    sumsq = None
    if normalize:
        _, sums = ctx().gradient_diversity([gd.view(-1)], [fg])
        sumsq = sums[0:1]
    q, cnt, rr = ctx().sgd_update_quantize(wd, gd, fg, lr, l1, l2, wl, fl, g_sumsq=sumsq, mode=mode, seed=seed, stream=stream)
    ref = so.sgd_update_quantize(w, g, fg[1], lr, l1, l2, wl, fl, mode, seed, stream, normalize)
    got_w = host(wd)
    assert np.array_equal(got_w.view(np.uint32), ref["w"].view(np.uint32))
    assert np.array_equal(host(q).astype(np.int64), ref["q"])
    assert u64(cnt).tolist() == [ref["nnz"], ref["sat"]]
    lo, hi = host(rr).tolist()
    assert (lo, hi) == (ref["lo"], ref["hi"])
    return wd, rr, ref


@pytest.mark.parametrize("n", [1, 7, 8, 9, 2047, 2048, 110592, (1 << 20) + 3])
@pytest.mark.parametrize("gwl,wl,fl", [(8, 8, 5), (12, 8, 4), (8, 12, 9), (16, 16, 13)])
def test_sizes_and_formats(n, gwl, wl, fl):
    rng = np.random.default_rng(n + wl)
    w = (rng.standard_normal(n) * 0.2).astype(np.float32)
    g = _grad_codes(rng, n, gwl)
    _run(w, g, (gwl, gwl - 3), 0.05, 1e-4, 5e-3, wl, fl, seed=7, stream=n)


@pytest.mark.parametrize("normalize", [True, False])
@pytest.mark.parametrize("mode", [pkg.SR, pkg.RN_HALF_UP])
def test_modes_and_plain_step(normalize, mode):
    rng = np.random.default_rng(5)
    w = (rng.standard_normal(50001) * 0.5).astype(np.float32)
    g = _grad_codes(rng, 50001, 8)
    _run(w, g, (8, 6), 0.1, 0.0, 0.0, 8, 4, normalize=normalize, mode=mode)
    _run(w, g, (8, 6), 0.0, 0.0, 0.0, 8, 4, normalize=normalize, mode=mode)      # no step: plain quantize
    _run(w, g, (8, 6), 0.3, 2e-3, 0.25, 8, 4, normalize=normalize, mode=mode)    # strong decay


def test_zero_gradient_and_special_weights():
    w = np.array([0.0, -0.0, 1e-40, -1e-40, 3.9, -4.2, 100.0, 1e-3, 0.5, -0.5, 2.0 ** -20, 7.0], dtype=np.float32)
    z = np.zeros(12, dtype=np.int8)
    _run(w, z, (8, 5), 0.1, 1e-3, 1e-2, 8, 5)           # sumsq = 0: step 0, only the decay terms act
    g = np.array([127, -128, 1, -1, 0, 5, -7, 64, -64, 3, 2, 1], dtype=np.int8)
    _run(w, g, (8, 5), 0.25, 0.0, 0.0, 8, 5)


def test_repeated_steps_track_the_oracle():
    # several AdaPT-SGD steps on the config-2 weight tensor: the master copy stays bit-identical
    L = wk.config2(batch=1)
    rng = np.random.default_rng(9)
    w = L.w.reshape(-1).copy()
    wd = dev(w.copy())
    for it in range(4):
        g = _grad_codes(rng, w.size, 8)
        gd = dev(g)
        _, sums = ctx().gradient_diversity([gd], [(8, 7)])
        q, cnt, rr = ctx().sgd_update_quantize(wd, gd, (8, 7), 0.02, 1e-5, 1e-4, 8, 5, g_sumsq=sums[0:1], seed=1, stream=it)
        ref = so.sgd_update_quantize(w, g, 7, 0.02, 1e-5, 1e-4, 8, 5, orc.SR, 1, it)
        w = ref["w"]
        assert np.array_equal(host(wd).view(np.uint32), w.view(np.uint32))
        assert np.array_equal(host(q).astype(np.int64), ref["q"])


def test_range_feeds_the_precision_search():
    rng = np.random.default_rng(3)
    w = (rng.standard_normal(110592) * 0.059).astype(np.float32)
    g = _grad_codes(rng, w.size, 8)
    wd, rr, ref = _run(w, g, (8, 7), 0.05, 1e-5, 1e-4, 8, 5, stream=2)
    res = ctx().kld_precision_search_ranged(wd, rr, 4, 16, 3, 2048, 1e-2, stream=2, want_hist=True)
    full = ctx().kld_precision_search(wd, 4, 16, 3, 2048, 1e-2, stream=2, want_hist=True)
    want = orc.kld_precision_search(ref["w"], 4, 16, 3, 2048, 1e-2, None, orc.SR, 0, 2)
    for r in (res, full):
        assert host(r["sel"]).tolist() == [want["wl_sel"], want["fl_sel"]]
        assert host(r["grid"]).tolist() == [want["e"], want["base"], want["nb"]]
        assert np.allclose(host(r["kld"]), want["kld"], rtol=1e-5, atol=1e-12)
    assert torch.equal(res["hist"], full["hist"])


def test_range_that_does_not_bound_the_tensor_is_clamped_not_trusted():
    w = dev(np.linspace(-1.0, 1.0, 4096, dtype=np.float32))
    narrow = dev(np.array([-0.5, 0.5], dtype=np.float32))
    res = ctx().kld_precision_search_ranged(w, narrow, 4, 8, 2, 64, 1e-2, mode=pkg.RN_HALF_UP, want_hist=True)
    hist = host(res["hist"])
    assert int(hist[0].sum()) == 4096                     # every element lands in some bin
    assert hist[0, 0] > 900 and hist[0].max() > 900       # the out-of-range quarters pile up at the ends


def test_invalid_arguments():
    w = dev(np.zeros(64, dtype=np.float32))
    g = dev(np.zeros(64, dtype=np.int8))
    with pytest.raises(pkg.AdaptError):
        ctx().sgd_update_quantize(w, g, (33, 3), 0.1, 0, 0, 8, 5)
    with pytest.raises(pkg.AdaptError):
        ctx().sgd_update_quantize(w, g, (8, 3), float("nan"), 0, 0, 8, 5)
    with pytest.raises(pkg.AdaptError):
        ctx().sgd_update_quantize(w, g, (8, 3), 0.1, 0, 0, 1, 0)
