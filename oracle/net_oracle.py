"""CPU oracle for one chained fixed-point training step of a feed-forward network (AdaPT,
arXiv 2107.13490).

TEST INFRASTRUCTURE ONLY.  Slow, plain reference; nothing in the product package may import it;
only tests/, the smoke check and the benchmark's cpu_baseline leg do.  It shares no code with
the HIP path.

What it follows: Alg. 1 (AdaPT-SGD) for one batch -- ForwardPass on the quantized layers, the
backward pass, the update of the master weights and the Quantize loop -- with every tensor that
crosses a layer held as fixed-point codes (Sec. 2.1 "Fixed-Point Quantization", Sec. 3.2).  The
paper states the training loop but not how a fixed-point backward pass keeps its gradients in
range, nor the integer form of ReLU and max-pooling; the rules taken here:

  layer l        z_l = conv(a_{l-1}, W^_l)   exact integer accumulator (FC = 1x1 conv on 1x1 maps)
                 y_l = requantize(ReLU(z_l)) to the layer's own <WL_l,FL_l>, SR (ReLU optional)
                 a_l = 2x2/2 max-pool of y_l (optional); max of codes = max of values
  input          a_{-1} = quantize(x, <WL_0,FL_0>)
  backward       dy_l = da_l routed through the pool to the FIRST maximum of each window in
                 scan order (dh,dw) = (0,0),(0,1),(1,0),(1,1), and zeroed where y_l <= 0 (ReLU; the
                 requantized output is what is stored, so it decides the mask)
                 dW_l = wgrad(dy_l, a_{l-1}), da_{l-1} = dgrad(dy_l, W^_l), exact accumulators
  gradient range back-propagation is linear in the incoming gradient and the weight update divides
                 each layer's gradient by its 2-norm (Sec. 3.3 "Dealing with Fixed-Points Limited
                 Range"), so a common power-of-two factor of a gradient tensor changes nothing but
                 the rounding.  An exact accumulator tensor is therefore stored in WL bits with the
                 smallest right shift that makes its largest magnitude fit:
                 shift = max(0, bit_length(max|acc|) - (WL-1)), rounded by the requantize rule
                 (SR), saturated.  da_{l-1} is stored in WL_{l-1} bits, dW_l in WL_l bits.
  update         per layer the fused SGD update + Quantize of the sgd oracle, with the gradient
                 codes and their sum of squares.

Random streams: the step is given (seed, stream0); layer l uses stream0 + 8 l + slot with slot
0 = forward output, 1 = data gradient it hands down, 2 = weight gradient, 3 = re-quantized weights,
4 = network input (l = 0 only), 5 = first quantization of the weights.

Word lengths 17..32 (Sec. 3.3 lets PushUp ask for up to 32 bits): a contraction with an operand above 16 bits, and
the fitting of its accumulators, run on Python integers (the wide oracle); every rule above is unchanged.  The
element-wise sum of a window that holds codes above 16 bits is kept in 64-bit integers, and the bound below which
the oldest entries are left out is 2^48 instead of 2^31.

Also here: the residual addition of two fixed-point tensors (exact sum on the finer grid, then the
requantize rule).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import conv_oracle as co
from . import fxp_oracle as orc
from . import sgd_oracle as so
from . import wide_oracle as wo

SLOT_FWD, SLOT_DA, SLOT_DW, SLOT_UPD, SLOT_IN, SLOT_WQ = 0, 1, 2, 3, 4, 5


def stream_of(stream0: int, layer: int, slot: int) -> int:
    return stream0 + 8 * layer + slot


# ---- element-wise pieces ---------------------------------------------------------------------------------

def maxpool2(y) -> np.ndarray:
    """(n,h,w,c) codes -> (n,h/2,w/2,c): maximum of every 2x2 window (h, w even)."""
    y = np.asarray(y)
    n, h, w, c = y.shape
    assert h % 2 == 0 and w % 2 == 0
    out = np.empty((n, h // 2, w // 2, c), dtype=np.int64)
    for i in range(h // 2):
        for j in range(w // 2):
            win = y[:, 2 * i:2 * i + 2, 2 * j:2 * j + 2, :].reshape(n, 4, c)
            out[:, i, j, :] = win.max(axis=1)
    return out


def relu_pool_bwd(da, y, relu: bool, pool: bool) -> np.ndarray:
    """Gradient w.r.t. the contraction output from the gradient w.r.t. the layer output.

    y = the stored (requantized, post-ReLU) output before pooling, da = gradient of the pooled
    tensor (or of y itself without pooling)."""
    y = np.asarray(y).astype(np.int64)
    da = np.asarray(da).astype(np.int64)
    dy = np.zeros_like(y)
    n, h, w, c = y.shape
    if pool:
        assert da.shape == (n, h // 2, w // 2, c)
        for i in range(h // 2):
            for j in range(w // 2):
                win = y[:, 2 * i:2 * i + 2, 2 * j:2 * j + 2, :].reshape(n, 4, c)
                first = win.argmax(axis=1)                      # numpy: index of the first maximum
                for t in range(4):
                    dy[:, 2 * i + t // 2, 2 * j + t % 2, :] = np.where(first == t, da[:, i, j, :], 0)
    else:
        assert da.shape == y.shape
        dy[...] = da
    if relu:
        dy[y <= 0] = 0
    return dy


def fit_shift(acc, wl: int) -> int:
    """Smallest right shift after which the largest magnitude of acc has at most wl-1 bits."""
    a = np.asarray(acc, dtype=np.int64)
    m = int(np.abs(a).max()) if a.size else 0
    return max(0, m.bit_length() - (wl - 1))


def requantize_fit(acc, wl: int, mode: int = orc.SR, seed: int = 0, stream: int = 0):
    """Exact accumulators -> wl-bit codes with the fitting shift.  Returns (codes, shift, sum of squared codes)."""
    sh = fit_shift(acc, wl)
    q = orc.requantize(acc, sh, wl, mode, seed, stream, False)
    return q, sh, int(np.sum(q.astype(object) ** 2)) if q.size else 0


def residual_add(a, fl_a: int, b, fl_b: int, wl_o: int, fl_o: int, mode: int = orc.SR, seed: int = 0,
                 stream: int = 0, relu: bool = False) -> np.ndarray:
    """codes of a*2^-fl_a + b*2^-fl_b in <wl_o,fl_o>: exact sum with max(fl_a,fl_b) fractional bits, requantized."""
    f = max(fl_a, fl_b)
    a, b = np.asarray(a, dtype=np.int64), np.asarray(b, dtype=np.int64)
    if force_wide or wl_o > 16 or (a.size and max(int(np.abs(a).max()), int(np.abs(b).max())) >= 1 << 15):
        a, b = a.astype(object), b.astype(object)            # codes above 16 bits: the aligned sum can pass 64 bits
    s = a * (1 << (f - fl_a)) + b * (1 << (f - fl_b))
    return _requantize(s, f - fl_o, wl_o, mode, seed, stream, relu)


# ---- contractions and fitting by word length -------------------------------------------------------------
# force_wide: tests run formats of at most 16 bits through the Python-integer path as well, which pins that path
# to the int64 one.
force_wide = False


def _wide(*wls) -> bool:
    return force_wide or any(w > 16 for w in wls)


def _conv_fwd(x, wl_x, w, wl_w, stride, pad):
    return wo.conv_fwd(x, w, stride, pad) if _wide(wl_x, wl_w) else co.conv_fwd(x, w, stride, pad)


def _conv_dgrad(dy, wl_dy, w, wl_w, h, wd, stride, pad):
    return wo.conv_dgrad(dy, w, h, wd, stride, pad) if _wide(wl_dy, wl_w) else co.conv_dgrad(dy, w, h, wd, stride, pad)


def _conv_wgrad(dy, wl_dy, x, wl_x, r, s, stride, pad):
    return wo.conv_wgrad(dy, x, r, s, stride, pad) if _wide(wl_dy, wl_x) else co.conv_wgrad(dy, x, r, s, stride, pad)


def _requantize(acc, shift, wl, mode, seed, stream, relu):
    if np.asarray(acc).dtype == object or wl > 16:
        return wo.requantize(acc, shift, wl, mode, seed, stream, relu)
    return orc.requantize(acc, shift, wl, mode, seed, stream, relu)


def _requantize_fit(acc, wl, mode, seed, stream):
    if np.asarray(acc).dtype == object or wl > 16:
        return wo.requantize_fit(acc, wl, mode, seed, stream)
    return requantize_fit(acc, wl, mode, seed, stream)


# ---- the chained step ------------------------------------------------------------------------------------

@dataclass
class Layer:
    """Convolution (n,h,w,c) -> k filters r x s, or a fully connected layer (h = w = r = s = 1, pad 0)."""
    h: int
    w: int
    c: int
    k: int
    r: int = 3
    s: int = 3
    stride: int = 1
    pad: int = 1
    relu: bool = True
    pool: bool = False

    @property
    def p(self) -> int:
        return (self.h + 2 * self.pad - self.r) // self.stride + 1

    @property
    def q(self) -> int:
        return (self.w + 2 * self.pad - self.s) // self.stride + 1

    def out_shape(self, n: int):
        p, q = (self.p // 2, self.q // 2) if self.pool else (self.p, self.q)
        return (n, p, q, self.k)


def quantize_weights(layers, fmts, weights, seed: int, stream0: int):
    """First Quantize of every layer's master weights (KRSC fp32) -> list of code arrays."""
    return [orc.quantize(np.asarray(w, np.float32), wl, fl, orc.SR, seed, stream_of(stream0, l, SLOT_WQ))[0]
            .reshape(L.k, L.r, L.s, L.c)
            for l, (L, (wl, fl), w) in enumerate(zip(layers, fmts, weights))]


def forward(layers, fmts, wq, x, seed: int, stream0: int):
    """x: fp32 (n,h,w,c).  Returns dict(a_in, y[], a[]) of code arrays; a[-1] are the logits' codes."""
    n = x.shape[0]
    wl0, fl0 = fmts[0]
    a_in = orc.quantize(np.asarray(x, np.float32), wl0, fl0, orc.SR, seed, stream_of(stream0, 0, SLOT_IN))[0].reshape(x.shape)
    ys, acts = [], []
    cur, fl_cur, wl_cur = a_in, fl0, wl0
    for l, (L, (wl, fl)) in enumerate(zip(layers, fmts)):
        cur = cur.reshape(n, L.h, L.w, L.c)                       # flatten / unflatten between conv and FC
        z = _conv_fwd(cur, wl_cur, wq[l], wl, L.stride, L.pad)
        shift = fl_cur + fl - fl                                   # FL of the activations + FL of the weights - FL of the output
        y = _requantize(z, shift, wl, orc.SR, seed, stream_of(stream0, l, SLOT_FWD), L.relu)
        ys.append(y)
        cur = maxpool2(y) if L.pool else y
        acts.append(cur)
        fl_cur, wl_cur = fl, wl
    return {"a_in": a_in, "y": ys, "a": acts}


def backward(layers, fmts, wq, fwd, dlogits, seed: int, stream0: int):
    """dlogits: codes of the gradient w.r.t. the last layer's output (same shape).

    Returns dict(g[] = weight-gradient codes, sumsq[], shift_w[], da[] = gradient codes handed to
    layer l (da[L-1] = dlogits), dy[], shift_a[])."""
    nl = len(layers)
    n = fwd["a_in"].shape[0]
    g, sumsq, shift_w = [None] * nl, [0] * nl, [0] * nl
    da, dy, shift_a = [None] * nl, [None] * nl, [0] * nl
    da[nl - 1] = np.asarray(dlogits).astype(np.int64).reshape(fwd["a"][nl - 1].shape)
    for l in range(nl - 1, -1, -1):
        L = layers[l]
        wl, _ = fmts[l]
        dy[l] = relu_pool_bwd(da[l], fwd["y"][l], L.relu, L.pool)
        a_prev = (fwd["a"][l - 1] if l > 0 else fwd["a_in"]).reshape(n, L.h, L.w, L.c)
        wl_prev = fmts[l - 1][0] if l > 0 else fmts[0][0]
        acc_w = _conv_wgrad(dy[l], wl, a_prev, wl_prev, L.r, L.s, L.stride, L.pad)
        g[l], shift_w[l], sumsq[l] = _requantize_fit(acc_w, wl, orc.SR, seed, stream_of(stream0, l, SLOT_DW))
        if l > 0:
            acc_a = _conv_dgrad(dy[l], wl, wq[l], wl, L.h, L.w, L.stride, L.pad)
            q, shift_a[l], _ = _requantize_fit(acc_a, fmts[l - 1][0], orc.SR, seed, stream_of(stream0, l, SLOT_DA))
            da[l - 1] = q.reshape(fwd["a"][l - 1].shape)
    return {"g": g, "sumsq": sumsq, "shift_w": shift_w, "da": da, "dy": dy, "shift_a": shift_a}


def update(layers, fmts, weights, bwd, lr: float, l1: float, l2: float, seed: int, stream0: int):
    """Fused SGD update + Quantize per layer.  Returns list of sgd-oracle result dicts (w, q, nnz, sat, lo, hi)."""
    out = []
    for l, ((wl, fl), w) in enumerate(zip(fmts, weights)):
        out.append(so.sgd_update_quantize(np.asarray(w, np.float32).ravel(), bwd["g"][l].ravel(), 0, lr, l1, l2, wl, fl,
                                          orc.SR, seed, stream_of(stream0, l, SLOT_UPD), normalize=True))
    return out


# ---- the precision switch inside the chain (Alg. 2) ------------------------------------------------------
#
# Alg. 2 runs between the pass that produces the quantized gradients and the update.  The text leaves the
# bookkeeping open; taken here:
#   * the loss history excludes the current batch; L_avg is the mean of its last ceil(mean_l lb^l) entries
#     (all of them if fewer; with an empty history the strategy is left alone)
#   * a layer's window keeps at most lb_upr gradients (oldest dropped); the diversity of the batch uses its
#     most recent min(len, lb^l) entries, lb^l before this batch's adaptation
#   * a gradient tensor of the chain is codes * 2^-e with an exponent e that follows from the fitting shifts:
#         e(dy_last) = FL of the loss gradient handed in
#         e(g_l)     = e(dy_l) + FL(a_{l-1}) - shift_w(l)
#         e(dy_{l-1}) = e(dy_l) + FL(W^_l) - shift_a(l)
#     only differences inside a window matter (the diversity is a ratio): FL_k = e_k - min_k e_k
#   * when len(window) >= lb^l (after adaptation): PushDown = the KL search on the master weights over
#     WL_c = max(wl_lo, il) .. wl_hi with il = WL - FL integer bits kept and `resolution` bins, never above
#     the current WL; PushUp = the closed-form suggestion; the window is emptied
# --------------------------------------------------------------------------------------------------------
from . import pushup_oracle as po  # noqa: E402

SLOT_KLD = 6


class SwitchState:
    def __init__(self, nl: int, lb_lwr: int, lb_upr: int, lb_init: int, r_lwr: int, r_upr: int, r_init: int, gamma: float,
                 eps: float, buff: int, wl_lo: int, wl_hi: int, strategy: int = po.ST_MIN, wl_cap: int = 16):
        self.p = dict(lb_lwr=lb_lwr, lb_upr=lb_upr, r_lwr=r_lwr, r_upr=r_upr, gamma=gamma, eps=eps, buff=buff, wl_lo=wl_lo,
                      wl_hi=wl_hi, wl_cap=wl_cap)
        self.lb = [lb_init] * nl
        self.res = [r_init] * nl
        self.windows = [[] for _ in range(nl)]            # entries (codes, wl, exponent)
        self.strategy = strategy
        self.losses = []


def gradient_exponents(fmts, bwd, dlogits_fl: int):
    """Fractional-bit count e(g_l) of every layer's weight-gradient codes for one backward pass."""
    nl = len(fmts)
    e_dy = dlogits_fl
    out = [0] * nl
    for l in range(nl - 1, -1, -1):
        fl_in = fmts[l - 1][1] if l > 0 else fmts[0][1]
        out[l] = e_dy + fl_in - bwd["shift_w"][l]
        if l > 0:
            e_dy = e_dy + fmts[l][1] - bwd["shift_a"][l]
    return out


def precision_switch(st: SwitchState, fmts, weights, bwd, dlogits_fl: int, loss: float, seed: int, stream0: int):
    """One call of Alg. 2.  fmts is updated in place (list of (WL, FL)); returns a report per layer."""
    import math
    p = st.p
    if st.losses:
        k = min(len(st.losses), int(math.ceil(sum(st.lb) / len(st.lb))))
        l_avg = sum(st.losses[-k:]) / k
        st.strategy = po.adapt_strategy(st.strategy, l_avg, loss)
    st.losses.append(loss)
    exps = bwd["e_g"] if "e_g" in bwd else gradient_exponents(fmts, bwd, dlogits_fl)    # a graph's backward pass gives them itself
    report = []
    for l, (wl, fl) in enumerate(fmts):
        win = st.windows[l]
        win.append((np.asarray(bwd["g"][l]).ravel().copy(), wl, exps[l]))
        if len(win) > p["lb_upr"]:
            win.pop(0)
        use = win[-min(len(win), st.lb[l]):]
        # The element-wise sum of the window, aligned to its finest grid, is held in 32-bit integers (64-bit ones if
        # the window holds codes above 16 bits): while the bound sum_k 2^(wl_k - 1 + e_max - e_k) reaches 2^31 (2^48)
        # the oldest entry is left out (the newest always stays).
        wide = any(w > 16 for _, w, _ in use)
        limit = 2 ** 48 if wide else 2 ** 31
        while len(use) > 1 and sum(2 ** (w - 1 + max(e for _, _, e in use) - e) for _, w, e in use) >= limit:
            use = use[1:]
        e_min = min(e for _, _, e in use)
        gd_fn = wo.gradient_diversity if wide else po.gradient_diversity_np
        gd = gd_fn([c for c, _, _ in use], [e - e_min for _, _, e in use])
        ds = gd["ds"]
        st.lb[l] = po.adapt_lookback(st.lb[l], ds, p["lb_lwr"], p["lb_upr"], p["gamma"])
        st.res[l] = po.adapt_resolution(st.res[l], st.lb[l], p["lb_lwr"], p["lb_upr"], p["r_lwr"], p["r_upr"])
        row = {"ds": ds, "lb": st.lb[l], "res": st.res[l], "switched": False, "wl_min": 0, "fl_min": 0, "used": len(use)}
        if len(win) >= st.lb[l]:
            il = wl - fl
            lo = max(p["wl_lo"], il)
            wl_min = wl
            if lo <= p["wl_hi"]:
                r = orc.kld_precision_search(np.asarray(weights[l], np.float32).ravel(), lo, p["wl_hi"], il, st.res[l], p["eps"],
                                             seed=seed, stream=stream_of(stream0, l, SLOT_KLD))
                wl_min = min(int(r["wl_sel"]), wl)
            fl_min = wl_min - il
            nw, nf, _, _, _ = po.pushup_suggest(ds, wl_min, fl_min, st.strategy, p["buff"], p["wl_cap"])
            fmts[l] = (nw, nf)
            win.clear()
            row.update(switched=True, wl_min=wl_min, fl_min=fl_min)
        row.update(wl=fmts[l][0], fl=fmts[l][1])
        report.append(row)
    return report
