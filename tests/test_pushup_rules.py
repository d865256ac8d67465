"""The switch controller's scalar rules in the library (host functions, no GPU needed) against
the oracle's, over a grid of arguments (Sec. 3.3 "The PushUp Operation", "Dealing with
Fixed-Points Limited Range", "Strategy, Resolution and Lookback")."""
import itertools
import math

import pytest

import paper_2107_13490_amd as pkg
from oracle import pushup_oracle as pu

DS = [1.0, 1.0000001, 1.2, math.e ** 0.5, 2.0, math.e, math.e ** 1.5, 5.0, math.e ** 2, 40.0, 1e6, 0.5, 0.0, -1.0,
      math.inf, math.nan]


def test_suggest_matches_oracle():
    for ds, wl_min, fl_min, st, buff, cap in itertools.product(DS, (2, 6, 9, 16), (0, 3, 8, 15), (0, 1, 2), (0, 2, 4),
                                                               (16, 32)):
        assert pkg.pushup_suggest(ds, wl_min, fl_min, st, buff, cap) == pu.pushup_suggest(ds, wl_min, fl_min, st, buff, cap), \
            (ds, wl_min, fl_min, st, buff, cap)


def test_suggest_rejects_bad_arguments():
    for args in ((2.0, 6, 5, 3, 0, 32), (2.0, 6, 5, 0, -1, 32), (2.0, 6, 5, 0, 0, 33), (2.0, 0, 5, 0, 0, 32), (2.0, 6, -1, 0, 0, 32)):
        with pytest.raises(pkg.AdaptError):
            pkg.pushup_suggest(*args)


def test_strategy_lookback_resolution_match_oracle():
    for st, a, b in itertools.product((0, 1, 2), (-2.0, 0.5, 1.0, 3.0), (-1.0, 0.5, 1.0, 2.5)):
        assert pkg.strategy_next(st, a, b) == pu.adapt_strategy(st, a, b)
    for lb, ds, gamma in itertools.product((25, 50, 77, 100), DS, (0.0, 0.25, 0.5, 1.0)):
        assert pkg.lookback_next(lb, ds, 25, 100, gamma) == pu.adapt_lookback(lb, ds, 25, 100, gamma), (lb, ds, gamma)
    for r, lb in itertools.product((20, 21, 50, 59, 60), (25, 26, 99, 100)):
        assert pkg.resolution_next(r, lb, 25, 100, 20, 60) == pu.adapt_resolution(r, lb, 25, 100, 20, 60)
    assert pkg.resolution_next(50, 30, 30, 30, 20, 60) == pu.adapt_resolution(50, 30, 30, 30, 20, 60) == 51
