"""CPU oracle for the chained fixed-point training step of a residual network with batch
normalisation (AdaPT, arXiv 2107.13490: Alg. 1 on the ResNets of Sec. 4.1).

TEST INFRASTRUCTURE ONLY.  Slow, plain reference; nothing in the product package may import it;
only tests/, the smoke check and the benchmark's cpu_baseline leg do.  It shares no code with
the HIP path.

The paper trains ResNets in fixed point but says nothing of how batch normalisation, the residual
addition, global average pooling or the merging of two gradient tensors are done on fixed-point
codes.  The rules taken here (every tensor that crosses a layer is codes * 2^-FL):

  batch norm, forward (training mode, statistics of the batch, per channel k over the m = N*P*Q
  codes y of the convolution output, which is stored in the layer's <WL,FL> without ReLU)
      S1 = sum y, S2 = sum y^2                               exact integers
      mean = S1/m, var = max(S2/m - mean*mean, 0), sig = sqrt(var + eps * 4^FL)      fp64, one rounding per operation
      alpha = gamma * 2^FL_o / sig, off = beta * 2^FL_o - mean * alpha                (gamma, beta: fp32 masters)
      FA = clamp(30 - E, 0, 30) with max_k |alpha_k| = f * 2^E, 1/2 <= f < 1
      A_k = rint(alpha_k 2^FA) (|A| <= 2^30), B_k = rint(off_k 2^FA) (|B| <= 2^61)   31- and 62-bit fixed-point coefficients
      out = requantize(A_k y + B_k [+ shortcut aligned to that grid], FA) to <WL_o,FL_o>, SR, optional ReLU
  batch norm, backward, from the codes dz of the gradient at its output
      D1 = sum dz, D2 = sum dz*y                             exact integers
      dgamma = (D2 - mean*D1)/sig, dbeta = D1                in units of the gradient's scale
      c1 = D1/m, c2 = dgamma/(m*sig); P = alpha, Q = -(alpha*c2), R = alpha*(mean*c2 - c1)
      FB from max(|P|,|Q|) as FA above; codes P^, Q^, R^ = rint(. 2^FB)
      acc = P^ dz + Q^ y + R^ (exact), stored in WL bits with the fitting shift (SR): exponent e + FB - shift + FL_o - FL_y
  update of gamma, beta: each divided by its own 2-norm over the channels (sum in channel order, fp64), one fp32 fused
      multiply-add per parameter (the rule of Sec. 3.3 "Dealing with Fixed-Points Limited Range" for weights)
  residual addition: inside the batch-norm output above (exact on the common grid, one rounding)
  global average pooling: sum over the h*w (a power of two) positions, requantize by log2(h*w); backward: the
      gradient codes are copied to every position and the exponent grows by log2(h*w)
  a tensor with two consumers: its gradient is the exact sum of the two contributions on the finer grid, stored
      with the fitting shift; if the exponents differ by more than 40 the contribution with the larger exponent
      (the far smaller values) is left out

Word lengths 17..32: the same rules on Python integers wherever a sum or product can pass 64 bits (S2 and D2 reach
85 bits, A y + B + shortcut more); an integer total enters the fp64 formulas as its nearest double (ties to even).

Random streams of the new steps: stream0 + 2^20 + 8 l + slot, slot 0 = batch-norm output, 1 = batch-norm data
gradient, 2 = average pooling, 3.. = the k-th contribution merged into the gradient of layer l's output.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

from . import conv_oracle as co
from . import fxp_oracle as orc
from . import net_oracle as no
from . import sgd_oracle as so
from . import wide_oracle as wo

X_BN, X_BNB, X_GAP, X_MERGE = 0, 1, 2, 3


def stream_x(stream0: int, layer: int, slot: int) -> int:
    return stream0 + (1 << 20) + 8 * layer + slot


# ---- batch normalisation ----------------------------------------------------------------------------------

def _coef_exponent(vmax: float) -> int:
    """clamp(30 - E, 0, 30) for vmax = f * 2^E, 1/2 <= f < 1 (E = 0 for vmax = 0 or a non-finite vmax)."""
    if not (vmax > 0.0) or math.isinf(vmax):
        return 30
    _, e = math.frexp(vmax)
    return min(max(30 - e, 0), 30)


def _big(*arrays) -> bool:
    """True when some code needs more than 16 bits (or the chain oracle is told to use Python integers throughout)."""
    return no.force_wide or any(a is not None and np.size(a) and int(np.abs(np.asarray(a, dtype=np.int64)).max()) >= (1 << 15)
                                for a in arrays)


def _ints(a, big: bool):
    a = np.asarray(a, dtype=np.int64)
    return a.astype(object) if big else a


def _f64(v) -> np.ndarray:
    """Integer totals (int64 or Python integers) as their nearest doubles."""
    return np.array([float(int(x)) for x in np.asarray(v).ravel()], dtype=np.float64).reshape(np.shape(v))


def bn_coeffs(y, fl_y: int, gamma, beta, eps: float, fl_o: int):
    """Per-channel statistics and fixed-point coefficients.  y: (..., K) codes."""
    y2 = _ints(y, _big(y)).reshape(-1, np.shape(y)[-1])
    m = y2.shape[0]
    s1 = y2.sum(axis=0)
    s2 = (y2 * y2).sum(axis=0)
    mean = _f64(s1) / np.float64(m)
    ex2 = _f64(s2) / np.float64(m)
    var = np.maximum(ex2 - mean * mean, 0.0)
    sig = np.sqrt(var + math.ldexp(float(eps), 2 * fl_y))
    g64 = np.asarray(gamma, np.float32).astype(np.float64)
    b64 = np.asarray(beta, np.float32).astype(np.float64)
    alpha = np.ldexp(g64, fl_o) / sig
    off = np.ldexp(b64, fl_o) - mean * alpha
    fa = _coef_exponent(float(np.max(np.abs(alpha))) if alpha.size else 0.0)
    a = np.clip(np.rint(np.ldexp(alpha, fa)), -float(1 << 30), float(1 << 30)).astype(np.int64)
    b = np.clip(np.rint(np.ldexp(off, fa)), -float(1 << 61), float(1 << 61)).astype(np.int64)
    return {"m": m, "s1": s1, "s2": s2, "mean": mean, "sig": sig, "alpha": alpha, "A": a, "B": b, "FA": fa, "fl_y": fl_y, "fl_o": fl_o}


def bn_forward(y, fl_y: int, gamma, beta, eps: float, wl_o: int, fl_o: int, relu: bool, seed: int, stream: int,
               res=None, fl_res: int = 0, mode: int = orc.SR):
    """Returns (codes of the normalised output [+ shortcut], state)."""
    st = bn_coeffs(y, fl_y, gamma, beta, eps, fl_o)
    big = _big(y, res) or wl_o > 16
    yi = _ints(y, big)
    acc = yi * _ints(st["A"], big) + _ints(st["B"], big)   # broadcast over the channel (last) axis
    if res is not None:
        sh = fl_o + st["FA"] - fl_res
        r = _ints(res, big).reshape(yi.shape)
        acc = acc + (r * (1 << sh) if sh >= 0 else r >> (-sh))
    out = no._requantize(acc, st["FA"], wl_o, mode, seed, stream, relu)
    return out, st


def bn_backward(dz, y, st, wl_out: int, seed: int, stream: int, mode: int = orc.SR):
    """dz: codes of the gradient at the batch-norm output; y: the codes it normalised; st: bn_coeffs' result.
    Returns dict(dy codes, shift, FB, e_add, dgamma, dbeta): for a gradient dz * 2^-e the gradient with respect to the
    normalised values is dy * 2^-(e + e_add), e_add = FB - shift + FL_o - FL_y (alpha carries 2^FL_o where the chain
    rule has 2^FL_y); dgamma and dbeta are in units of 2^-e."""
    k = np.shape(y)[-1]
    big = _big(dz, y) or wl_out > 16
    d2 = _ints(dz, big).reshape(-1, k)
    y2 = _ints(y, big).reshape(-1, k)
    m = np.float64(y2.shape[0])
    dd1 = _f64(d2.sum(axis=0))
    dd2 = _f64((d2 * y2).sum(axis=0))
    mean, sig, alpha = st["mean"], st["sig"], st["alpha"]
    dg = (dd2 - mean * dd1) / sig
    c1 = dd1 / m
    c2 = dg / (m * sig)
    p = alpha
    q = -(alpha * c2)
    r = alpha * (mean * c2 - c1)
    fb = _coef_exponent(float(max(np.max(np.abs(p)), np.max(np.abs(q)))) if p.size else 0.0)
    pc = np.clip(np.rint(np.ldexp(p, fb)), -float(1 << 30), float(1 << 30)).astype(np.int64)
    qc = np.clip(np.rint(np.ldexp(q, fb)), -float(1 << 30), float(1 << 30)).astype(np.int64)
    rc = np.clip(np.rint(np.ldexp(r, fb)), -float(1 << 61), float(1 << 61)).astype(np.int64)
    acc = d2 * _ints(pc, big) + y2 * _ints(qc, big) + _ints(rc, big)
    codes, shift, _ = no._requantize_fit(acc, wl_out, mode, seed, stream)
    return {"dy": codes.reshape(np.shape(y)), "shift": shift, "FB": fb, "e_add": fb - shift + st["fl_o"] - st["fl_y"],
            "dgamma": dg, "dbeta": dd1}


def _norm_seq(v) -> float:
    t = 0.0
    for x in np.asarray(v, dtype=np.float64):
        t = t + float(x) * float(x)
    return math.sqrt(t)


def bn_update(gamma, beta, dgamma, dbeta, lr: float):
    """gamma, beta fp32; each gradient divided by its 2-norm over the channels; p <- fma(-lr, g, p) in fp32."""
    out = []
    for p, d in ((gamma, dgamma), (beta, dbeta)):
        p = np.asarray(p, np.float32)
        nrm = _norm_seq(d)
        if nrm > 0.0 and math.isfinite(nrm):
            g32 = (np.asarray(d, np.float64) / np.float64(nrm)).astype(np.float32)
            p = so.fma32(np.float32(-np.float32(lr)), g32, p)
        out.append(p)
    return out[0], out[1]


# ---- global average pooling ---------------------------------------------------------------------------------

def gap_forward(a, wl: int, seed: int, stream: int, mode: int = orc.SR):
    """(n,h,w,c) codes -> (n,c) codes of the mean over the h*w positions, same <WL,FL>."""
    a = np.asarray(a, dtype=np.int64)
    n, h, w, c = a.shape
    hw = h * w
    assert hw & (hw - 1) == 0
    s = a.reshape(n, hw, c).sum(axis=1)
    return orc.requantize(s, hw.bit_length() - 1, wl, mode, seed, stream, False)


def gap_backward(dout, h: int, w: int):
    """Gradient codes of the pooled tensor -> codes at every position; the exponent grows by log2(h*w)."""
    d = np.asarray(dout, dtype=np.int64)
    n, c = d.shape
    return np.broadcast_to(d[:, None, None, :], (n, h, w, c)).copy(), (h * w).bit_length() - 1


# ---- sum of two gradient tensors ---------------------------------------------------------------------------

MERGE_MAX_GAP = 40


def grad_add(a, e_a: int, b, e_b, wl: int, seed: int, stream: int, mode: int = orc.SR):
    """a * 2^-e_a [+ b * 2^-e_b] as wl-bit codes with the fitting shift.  Returns (codes, exponent, shift)."""
    big = _big(a, b) or wl > 16
    ai = _ints(a, big)
    if b is None:
        acc, e = ai, e_a
    else:
        bi = _ints(b, big).reshape(ai.shape)
        if e_a - e_b > MERGE_MAX_GAP:
            acc, e = bi, e_b
        elif e_b - e_a > MERGE_MAX_GAP:
            acc, e = ai, e_a
        else:
            e = max(e_a, e_b)
            acc = ai * (1 << (e - e_a)) + bi * (1 << (e - e_b))
    codes, shift, _ = no._requantize_fit(acc, wl, mode, seed, stream)
    return codes, e - shift, shift


# ---- the chained step on a graph of layers -------------------------------------------------------------------

@dataclass
class Node(no.Layer):
    """A layer of the graph: convolution [+ batch norm [+ shortcut]] [+ ReLU] [+ 2x2 max-pool | global average pool].
    src: the layer whose output feeds the convolution (-1: the layer before, or the network input for layer 0);
    res: the layer whose output is added inside the batch norm (-1: none)."""
    bn: bool = False
    src: int = -1
    res: int = -1
    gap: bool = False

    def out_shape(self, n: int):
        if self.gap:
            return (n, 1, 1, self.k)
        return super().out_shape(n)


def _src(l: int, node) -> int:
    return node.src if node.src >= 0 else l - 1              # -1: the network input


def forward(nodes, fmts, wq, bn_params, x, eps: float, seed: int, stream0: int):
    """bn_params[l] = (gamma, beta) fp32 or None.  Returns dict(a_in, yc[], y[], a[], bn[] states)."""
    n = x.shape[0]
    wl0, fl0 = fmts[0]
    a_in = orc.quantize(np.asarray(x, np.float32), wl0, fl0, orc.SR, seed, no.stream_of(stream0, 0, no.SLOT_IN))[0].reshape(x.shape)
    yc, ys, acts, states = [], [], [], []
    for l, (L, (wl, fl)) in enumerate(zip(nodes, fmts)):
        s = _src(l, L)
        cur, fl_cur, wl_cur = (a_in, fl0, wl0) if s < 0 else (acts[s], fmts[s][1], fmts[s][0])
        cur = cur.reshape(n, L.h, L.w, L.c)
        z = no._conv_fwd(cur, wl_cur, wq[l], wl, L.stride, L.pad)
        if L.bn:
            c = no._requantize(z, fl_cur, wl, orc.SR, seed, no.stream_of(stream0, l, no.SLOT_FWD), False)
            res, fl_res = (acts[L.res], fmts[L.res][1]) if L.res >= 0 else (None, 0)
            y, st = bn_forward(c, fl, bn_params[l][0], bn_params[l][1], eps, wl, fl, L.relu, seed, stream_x(stream0, l, X_BN),
                               res, fl_res)
        else:
            assert L.res < 0
            c, st = None, None
            y = no._requantize(z, fl_cur, wl, orc.SR, seed, no.stream_of(stream0, l, no.SLOT_FWD), L.relu)
        yc.append(c)
        ys.append(y)
        states.append(st)
        if L.pool:
            cur = no.maxpool2(y)
        elif L.gap:
            cur = gap_forward(y, wl, seed, stream_x(stream0, l, X_GAP)).reshape(n, 1, 1, L.k)
        else:
            cur = y
        acts.append(cur)
    return {"a_in": a_in, "yc": yc, "y": ys, "a": acts, "bn": states}


def backward(nodes, fmts, wq, fwd, dlogits, dlogits_fl: int, seed: int, stream0: int):
    """Returns dict(g[], sumsq[], e_g[] exponents of the weight gradients, dgamma[], dbeta[], da[], e_da[], dyc[])."""
    nl = len(nodes)
    n = fwd["a_in"].shape[0]
    g, sumsq, e_g = [None] * nl, [0] * nl, [0] * nl
    dgam, dbet, dyc = [None] * nl, [None] * nl, [None] * nl
    da, e_da, ncontrib = [None] * nl, [0] * nl, [0] * nl
    da[nl - 1] = np.asarray(dlogits).astype(np.int64).reshape(fwd["a"][nl - 1].shape)
    e_da[nl - 1] = dlogits_fl

    def contribute(j: int, codes, e: int, fitted: bool = False):
        """Adds codes * 2^-e to the gradient of layer j's output (stored in layer j's word length).  fitted: the codes
        are a data gradient that the fitting rule has just stored in layer j's word length; as the first contribution
        they are kept as they are (a second fitting pass would not be the identity when a code is -2^(wl-1), whose
        magnitude has wl bits).  Codes of another tensor (a shortcut's gradient) pass through grad_add alone."""
        k = ncontrib[j]
        wl_j = fmts[j][0]
        st = stream_x(stream0, j, X_MERGE + k)
        if k == 0 and fitted:
            da[j], e_da[j] = codes.reshape(fwd["a"][j].shape), e
        elif k == 0:
            da[j], e_da[j], _ = grad_add(codes.reshape(fwd["a"][j].shape), e, None, None, wl_j, seed, st)
        else:
            da[j], e_da[j], _ = grad_add(da[j], e_da[j], codes.reshape(fwd["a"][j].shape), e, wl_j, seed, st)
        ncontrib[j] = k + 1

    for l in range(nl - 1, -1, -1):
        L = nodes[l]
        wl, fl = fmts[l]
        d, e = da[l], e_da[l]
        assert d is not None, f"layer {l} has no consumer"
        if L.gap:
            d, up = gap_backward(d.reshape(n, L.k), L.p, L.q)
            e += up
        dz = no.relu_pool_bwd(d, fwd["y"][l], L.relu, L.pool)
        if L.res >= 0:
            contribute(L.res, dz, e)
        if L.bn:
            r = bn_backward(dz, fwd["yc"][l], fwd["bn"][l], wl, seed, stream_x(stream0, l, X_BNB))
            dyc[l], e = r["dy"], e + r["e_add"]
            dgam[l], dbet[l] = r["dgamma"], r["dbeta"]
        else:
            dyc[l] = dz
        s = _src(l, L)
        a_prev, fl_in, wl_in = (fwd["a_in"], fmts[0][1], fmts[0][0]) if s < 0 else (fwd["a"][s], fmts[s][1], fmts[s][0])
        a_prev = a_prev.reshape(n, L.h, L.w, L.c)
        acc_w = no._conv_wgrad(dyc[l], wl, a_prev, wl_in, L.r, L.s, L.stride, L.pad)
        g[l], sh_w, sumsq[l] = no._requantize_fit(acc_w, wl, orc.SR, seed, no.stream_of(stream0, l, no.SLOT_DW))
        e_g[l] = e + fl_in - sh_w
        if s >= 0:
            acc_a = no._conv_dgrad(dyc[l], wl, wq[l], wl, L.h, L.w, L.stride, L.pad)
            q, sh_a, _ = no._requantize_fit(acc_a, fmts[s][0], orc.SR, seed, no.stream_of(stream0, l, no.SLOT_DA))
            contribute(s, q, e + fl - sh_a, fitted=True)
    return {"g": g, "sumsq": sumsq, "e_g": e_g, "dgamma": dgam, "dbeta": dbet, "da": da, "e_da": e_da, "dyc": dyc}


def update(nodes, fmts, weights, bn_params, bwd, lr: float, l1: float, l2: float, seed: int, stream0: int):
    """Weights as in the plain chain; gamma and beta by bn_update.  Returns (list of sgd results, list of (gamma, beta) or None)."""
    upd = no.update(nodes, fmts, weights, bwd, lr, l1, l2, seed, stream0)
    bn_new = [bn_update(p[0], p[1], bwd["dgamma"][l], bwd["dbeta"][l], lr) if nodes[l].bn else None for l, p in enumerate(bn_params)]
    return upd, bn_new
