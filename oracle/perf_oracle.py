"""CPU oracle for the paper's analytical performance model (arXiv 2107.13490, Sec. 4.1
"Performance Model").

TEST INFRASTRUCTURE ONLY; nothing in the product package may import it.  Every function is the
printed formula written out: the PushDown / PushUp operation bounds, the training-cost and
overhead bounds (summed over steps by the caller), model size, memory and the speed-up quotient.
A layer at a step is a tuple (ops, sp, numel, wl, lookback, resolution).
"""
from __future__ import annotations

import math


def pushdown_ops(resolution: int, numel: float) -> float:
    return 2.0 * math.log2(32 - 8) * resolution * 3.0 * numel


def pushup_ops(lookback: int, numel: float) -> float:
    return (lookback + 1) * numel + 1.0


def step_cost(layers, accs: int = 1) -> float:
    return sum(ops * (sp * wl + 32.0 / accs) for ops, sp, numel, wl, lb, r in layers)


def step_overhead(layers, accs: int = 1) -> float:
    return sum(32.0 * (sp * pushdown_ops(r, numel) + pushup_ops(lb, numel)) / (accs * lb) for ops, sp, numel, wl, lb, r in layers)


def model_size(layers) -> float:
    return sum(sp * wl for ops, sp, numel, wl, lb, r in layers)


def step_memory(layers) -> float:
    return sum(sp * wl + 32.0 for ops, sp, numel, wl, lb, r in layers)


def speedup(bs_other, costs_other, bs_ours, costs_ours) -> float:
    return bs_other * costs_other / (bs_ours * costs_ours)
