"""The paper's performance model (Sec. 4.1 "Performance Model"): the oracle against closed forms that
follow from the printed formulas, and the library's host functions against the oracle (no GPU)."""
import math

import numpy as np
import pytest

import paper_2107_13490_amd as pkg
from oracle import perf_oracle as po

LAYERS = [(7.25e9, 0.61, 110592, 8, 25, 50), (1.9e10, 0.5, 147456, 12, 100, 150), (4.2e6, 1.0, 5120, 16, 40, 77)]


def test_closed_forms():
    # a dense float32 network without accumulation costs 64 bit-operations per multiply-add: 32 forward + 32 backward
    f32 = [(ops, 1.0, numel, 32, lb, r) for ops, sp, numel, wl, lb, r in LAYERS]
    assert po.step_cost(f32) == pytest.approx(64.0 * sum(l[0] for l in LAYERS), rel=1e-15)
    # identical runs have speed-up 1; halving every word length of a dense net with a free backward pass (accs -> inf) doubles it
    assert po.speedup(128, 5.0, 128, 5.0) == 1.0
    big = 10 ** 9
    half = [(ops, 1.0, numel, 16, lb, r) for ops, sp, numel, wl, lb, r in LAYERS]
    assert po.speedup(1, po.step_cost(f32, big), 1, po.step_cost(half, big)) == pytest.approx(2.0, rel=1e-6)
    # the PushDown bound: 2 log2(24) r 3 numel; the PushUp bound: (lb + 1) numel + 1
    assert po.pushdown_ops(50, 1000) == pytest.approx(6.0 * math.log2(24.0) * 50 * 1000)
    assert po.pushup_ops(25, 1000) == 26001.0
    # size and memory of a dense 8-bit net with L layers: 8 L and 40 L
    d8 = [(1.0, 1.0, 10, 8, 25, 50)] * 7
    assert po.model_size(d8) == 56.0 and po.step_memory(d8) == 280.0
    # overhead of one layer by hand: 32 (sp pd + pu) / (accs lb)
    ops, sp, numel, wl, lb, r = LAYERS[0]
    want = 32.0 * (sp * 6.0 * math.log2(24.0) * r * numel + (lb + 1) * numel + 1) / (2 * lb)
    assert po.step_overhead([LAYERS[0]], accs=2) == pytest.approx(want, rel=1e-15)


def test_library_matches_oracle():
    rng = np.random.default_rng(0)
    for trial in range(50):
        n = int(rng.integers(0, 9))
        layers = [(float(rng.uniform(1e3, 1e10)), float(rng.uniform(0, 1)), float(rng.integers(1, 10 ** 7)), int(rng.integers(2, 33)),
                   int(rng.integers(1, 101)), int(rng.integers(1, 151))) for _ in range(n)]
        accs = int(rng.integers(1, 9))
        assert pkg.perf_step_cost(layers, accs) == pytest.approx(po.step_cost(layers, accs), rel=1e-14, abs=0)
        assert pkg.perf_step_overhead(layers, accs) == pytest.approx(po.step_overhead(layers, accs), rel=1e-14, abs=0)
        assert pkg.perf_model_size(layers) == pytest.approx(po.model_size(layers), rel=1e-14, abs=0)
        assert pkg.perf_step_memory(layers) == pytest.approx(po.step_memory(layers), rel=1e-14, abs=0)
    lib = pkg.load_library()
    assert lib.adapt_perf_pushdown_ops(50, 1000.0) == pytest.approx(po.pushdown_ops(50, 1000), rel=1e-15)
    assert lib.adapt_perf_pushup_ops(25, 1000.0) == po.pushup_ops(25, 1000)
    assert lib.adapt_perf_speedup(128.0, 3.0, 512.0, 1.5) == po.speedup(128, 3.0, 512, 1.5)
    assert math.isnan(pkg.perf_step_cost(LAYERS, 0))
    assert math.isnan(pkg.perf_step_overhead([(1.0, 1.0, 10.0, 8, 0, 50)], 1))
