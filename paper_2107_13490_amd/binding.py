"""ctypes binding of include/adapt_fxp.h: argument marshalling only.

Tensors are torch CUDA (HIP) tensors; the binding passes their data pointers and the current
torch stream to the library.  Names mirror the C entry points.
"""
from __future__ import annotations

import ctypes as C
import os

RN_HALF_UP = 0
SR = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
# ADAPT_FXP_LIB selects another build of the same library (e.g. an instrumented one)
_LIB_PATH = os.environ.get("ADAPT_FXP_LIB") or os.path.join(_HERE, "libadapt_fxp.so")
_lib = None


class AdaptError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load_library().adapt_error_string(status).decode()
        super().__init__(f"{where}: {msg} (status {status})")


class Fmt(C.Structure):
    _fields_ = [("wl", C.c_int), ("fl", C.c_int)]


class Rng(C.Structure):
    _fields_ = [("mode", C.c_int), ("seed", C.c_uint64), ("stream", C.c_uint64)]


class ConvDesc(C.Structure):
    _fields_ = [(f, C.c_int) for f in ("n", "h", "w", "c", "k", "r", "s", "stride", "pad")]

    @property
    def p(self):
        return (self.h + 2 * self.pad - self.r) // self.stride + 1

    @property
    def q(self):
        return (self.w + 2 * self.pad - self.s) // self.stride + 1


class Epilogue(C.Structure):
    _fields_ = [("raw", C.c_int), ("fmt", Fmt), ("rng", Rng), ("relu", C.c_int)]

    @staticmethod
    def exact():
        return Epilogue(1, Fmt(8, 0), Rng(RN_HALF_UP, 0, 0), 0)

    @staticmethod
    def requant(wl, fl, mode=SR, seed=0, stream=0, relu=False):
        return Epilogue(0, Fmt(wl, fl), Rng(mode, seed, stream), int(relu))


class QuantizeItem(C.Structure):
    _fields_ = [("x", C.c_void_p), ("q", C.c_void_p), ("n", C.c_uint64), ("wl", C.c_int32),
                ("fl", C.c_int32), ("stream", C.c_uint64)]


class KldItem(C.Structure):
    _fields_ = [("w", C.c_void_p), ("n", C.c_uint64), ("il", C.c_int32), ("bins", C.c_int32),
                ("stream", C.c_uint64)]


class WorkspaceQuery(C.Structure):
    _fields_ = [("call", C.c_int), ("n", C.c_uint64), ("count", C.c_int), ("transA", C.c_int), ("transB", C.c_int),
                ("M", C.c_int), ("N", C.c_int), ("K", C.c_int), ("lda", C.c_int), ("ldb", C.c_int), ("conv", ConvDesc),
                ("fa", Fmt), ("fb", Fmt), ("fc", Fmt), ("wl_lo", C.c_int), ("wl_hi", C.c_int), ("bins", C.c_int),
                ("kld_items", C.POINTER(KldItem))]


(CALL_QUANTIZE, CALL_QUANTIZE_BATCHED, CALL_GEMM, CALL_CONV_FWD, CALL_CONV_DGRAD, CALL_CONV_WGRAD, CALL_CONV_BACKWARD,
 CALL_KLD_SEARCH, CALL_KLD_SEARCH_BATCHED, CALL_SGD_UPDATE, CALL_GRADIENT_DIVERSITY, CALL_REQUANTIZE_FIT) = range(12)


class GradItem(C.Structure):
    _fields_ = [("g", C.c_void_p), ("wl", C.c_int32), ("fl", C.c_int32)]


class SgdParams(C.Structure):
    _fields_ = [("lr", C.c_double), ("l1", C.c_double), ("l2", C.c_double)]


class PerfLayer(C.Structure):
    _fields_ = [("ops", C.c_double), ("sp", C.c_double), ("numel", C.c_double), ("wl", C.c_int), ("lookback", C.c_int),
                ("resolution", C.c_int)]


class LayerDesc(C.Structure):
    """One layer of a chain: a ConvDesc (FC: h = w = r = s = 1, pad 0), ReLU and 2x2/2 max-pool flags."""
    _fields_ = [("conv", ConvDesc), ("relu", C.c_int), ("pool", C.c_int)]


class NodeDesc(C.Structure):
    """One layer of a network graph: a LayerDesc plus batch norm (bn), the layer that feeds the convolution (src, -1: the
    one before), the layer whose output is added inside the batch norm (res, -1: none), global average pooling (gap)."""
    _fields_ = [("conv", ConvDesc), ("relu", C.c_int), ("pool", C.c_int), ("bn", C.c_int), ("src", C.c_int), ("res", C.c_int),
                ("gap", C.c_int)]


class NetStats(C.Structure):
    _fields_ = [("g_sumsq", C.c_uint64), ("g_sumsq_hi", C.c_uint64), ("nnz", C.c_uint64), ("saturated", C.c_uint64),
                ("range_lo", C.c_float), ("range_hi", C.c_float), ("shift_w", C.c_int32), ("shift_a", C.c_int32),
                ("reserved", C.c_int32 * 4)]


NT_INPUT, NT_Y, NT_A, NT_DY, NT_DA, NT_QW, NT_G, NT_STATS, NT_YC, NT_DYC, NT_BN, NT_EXP, NT_DGAMMA, NT_DBETA = range(14)


class SwitchParams(C.Structure):
    """Hyper-parameters of the precision switch (bounds and start values of lookback and resolution, lookback
    momentum, KL threshold, buffer bits, PushDown candidates, start strategy)."""
    _fields_ = [("lb_lwr", C.c_int), ("lb_upr", C.c_int), ("lb_init", C.c_int), ("r_lwr", C.c_int), ("r_upr", C.c_int),
                ("r_init", C.c_int), ("gamma", C.c_double), ("eps", C.c_double), ("buff", C.c_int), ("wl_lo", C.c_int),
                ("wl_hi", C.c_int), ("strategy_init", C.c_int)]


class SwitchReport(C.Structure):
    _fields_ = [("ds", C.c_double), ("wl", C.c_int32), ("fl", C.c_int32), ("lb", C.c_int32), ("res", C.c_int32),
                ("switched", C.c_int32), ("wl_min", C.c_int32), ("fl_min", C.c_int32), ("used", C.c_int32)]


class PushupResult(C.Structure):
    _fields_ = [("wl", C.c_int), ("fl", C.c_int), ("s1", C.c_int), ("s2", C.c_int), ("s", C.c_int)]


ST_MIN, ST_MEAN, ST_MAX = 0, 1, 2


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Opens the HIP library.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(_LIB_PATH)
    vp, sz, i, u64, i64, dbl = C.c_void_p, C.c_size_t, C.c_int, C.c_uint64, C.c_int64, C.c_double
    lib.adapt_error_string.restype = C.c_char_p
    lib.adapt_error_string.argtypes = [i]
    lib.adapt_version.restype = i
    lib.adapt_create.argtypes = [C.POINTER(vp), vp, sz]
    lib.adapt_destroy.argtypes = [vp]
    lib.adapt_set_stream.argtypes = [vp, vp]
    lib.adapt_acc_bits.argtypes = [i64, Fmt, Fmt]
    lib.adapt_workspace_bytes.argtypes = [vp, C.POINTER(WorkspaceQuery)]
    lib.adapt_workspace_bytes.restype = sz
    lib.adapt_reserve_workspace.argtypes = [vp, sz]
    lib.adapt_quantize.argtypes = [vp, vp, sz, Fmt, Rng, vp, vp, vp]
    lib.adapt_quantize_noalloc.argtypes = [vp, vp, sz, Fmt, Rng, vp, vp, vp]
    lib.adapt_quantize_batched.argtypes = [vp, C.POINTER(QuantizeItem), i, i, u64, vp]
    lib.adapt_quantize_batched_ranges.argtypes = [vp, C.POINTER(QuantizeItem), i, i, u64, vp, vp, u64]
    lib.adapt_fxp_gemm.argtypes = [vp, i, i, i, i, i, vp, Fmt, i, vp, Fmt, i, vp, i, Epilogue]
    for f in (lib.adapt_conv_fwd, lib.adapt_conv_dgrad, lib.adapt_conv_wgrad):
        f.argtypes = [vp, ConvDesc, vp, Fmt, vp, Fmt, vp, Epilogue]
    lib.adapt_conv_backward.argtypes = [vp, ConvDesc, vp, Fmt, vp, Fmt, vp, Fmt, vp, Epilogue, vp, Epilogue]
    lib.adapt_kld_precision_search.argtypes = [vp, vp, sz, i, i, i, i, dbl, dbl, Rng, vp, vp, vp, vp]
    lib.adapt_kld_precision_search_batched.argtypes = [vp, C.POINTER(KldItem), i, i, i, dbl, dbl, i, u64, vp, vp]
    lib.adapt_kld_precision_search_batched_ranged.argtypes = [vp, C.POINTER(KldItem), C.POINTER(C.c_void_p), i, i, i, dbl, dbl, i, u64,
                                                              vp, vp]
    lib.adapt_kld_precision_search_ranged.argtypes = [vp, vp, sz, vp, i, i, i, i, dbl, dbl, Rng, vp, vp, vp, vp]
    lib.adapt_sgd_update_quantize.argtypes = [vp, vp, sz, vp, Fmt, vp, SgdParams, Fmt, Rng, vp, vp, vp]
    lib.adapt_perf_pushdown_ops.argtypes = [i, dbl]
    lib.adapt_perf_pushup_ops.argtypes = [i, dbl]
    lib.adapt_perf_speedup.argtypes = [dbl, dbl, dbl, dbl]
    for f in (lib.adapt_perf_step_cost, lib.adapt_perf_step_overhead):
        f.argtypes = [C.POINTER(PerfLayer), i, i]
    for f in (lib.adapt_perf_model_size, lib.adapt_perf_step_memory):
        f.argtypes = [C.POINTER(PerfLayer), i]
    for f in (lib.adapt_perf_pushdown_ops, lib.adapt_perf_pushup_ops, lib.adapt_perf_speedup, lib.adapt_perf_step_cost,
              lib.adapt_perf_step_overhead, lib.adapt_perf_model_size, lib.adapt_perf_step_memory):
        f.restype = dbl
    lib.adapt_maxpool2_fwd.argtypes = [vp, vp, Fmt, i, i, i, i, vp]
    lib.adapt_relu_pool_bwd.argtypes = [vp, vp, vp, Fmt, i, i, i, i, i, i, vp]
    lib.adapt_requantize_fit.argtypes = [vp, vp, i, sz, i, Rng, vp, vp, vp]
    lib.adapt_residual_add.argtypes = [vp, vp, Fmt, vp, Fmt, sz, Fmt, Rng, i, vp]
    lib.adapt_bn_state_bytes.argtypes = [i]
    lib.adapt_bn_state_bytes.restype = sz
    lib.adapt_bn_forward.argtypes = [vp, vp, Fmt, sz, i, vp, vp, dbl, vp, Fmt, Fmt, Rng, i, vp, vp]
    lib.adapt_bn_backward.argtypes = [vp, vp, i, vp, Fmt, sz, i, vp, i, Rng, vp, vp, vp, vp, vp, vp]
    lib.adapt_bn_update.argtypes = [vp, vp, vp, vp, vp, i, dbl]
    lib.adapt_gap_fwd.argtypes = [vp, vp, Fmt, i, i, i, Rng, vp]
    lib.adapt_gap_bwd.argtypes = [vp, vp, i, i, i, i, vp]
    lib.adapt_grad_add.argtypes = [vp, vp, i, vp, vp, i, vp, sz, i, Rng, vp, vp, vp]
    lib.adapt_net_workspace_bytes.argtypes = [C.POINTER(LayerDesc), i, i]
    lib.adapt_net_workspace_bytes.restype = sz
    lib.adapt_net_create.argtypes = [vp, C.POINTER(LayerDesc), i, C.POINTER(vp), C.POINTER(SwitchParams), vp, sz, C.POINTER(vp)]
    lib.adapt_net_workspace_bytes_wide.argtypes = [C.POINTER(LayerDesc), i, i, i]
    lib.adapt_net_workspace_bytes_wide.restype = sz
    lib.adapt_net_create_wide.argtypes = [vp, C.POINTER(LayerDesc), i, C.POINTER(vp), C.POINTER(SwitchParams), i, vp, sz, C.POINTER(vp)]
    lib.adapt_graph_workspace_bytes_wide.argtypes = [C.POINTER(NodeDesc), i, i, i]
    lib.adapt_graph_workspace_bytes_wide.restype = sz
    lib.adapt_graph_create_wide.argtypes = [vp, C.POINTER(NodeDesc), i, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), dbl,
                                            C.POINTER(SwitchParams), i, vp, sz, C.POINTER(vp)]
    lib.adapt_graph_workspace_bytes.argtypes = [C.POINTER(NodeDesc), i, i]
    lib.adapt_graph_workspace_bytes.restype = sz
    lib.adapt_graph_create.argtypes = [vp, C.POINTER(NodeDesc), i, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), dbl,
                                       C.POINTER(SwitchParams), vp, sz, C.POINTER(vp)]
    lib.adapt_net_precision_switch.argtypes = [vp, dbl, Rng, C.POINTER(SwitchReport), C.POINTER(i)]
    lib.adapt_net_destroy.argtypes = [vp]
    lib.adapt_net_set_format.argtypes = [vp, i, Fmt]
    lib.adapt_net_tensor.argtypes = [vp, i, i, C.POINTER(sz), C.POINTER(sz), C.POINTER(i)]
    lib.adapt_net_quantize_weights.argtypes = [vp, Rng]
    lib.adapt_net_forward.argtypes = [vp, vp, Rng]
    lib.adapt_net_backward.argtypes = [vp, vp, i, Rng]
    lib.adapt_net_update.argtypes = [vp, SgdParams, Rng]
    lib.adapt_gradient_diversity.argtypes = [vp, C.POINTER(GradItem), i, sz, vp, vp]
    lib.adapt_pushup_suggest.argtypes = [dbl, i, i, i, i, i, C.POINTER(PushupResult)]
    lib.adapt_strategy_next.argtypes = [i, dbl, dbl]
    lib.adapt_lookback_next.argtypes = [i, dbl, i, i, dbl]
    lib.adapt_resolution_next.argtypes = [i, i, i, i, i, i]
    _lib = lib
    return lib


def acc_bits(k: int, fa: Fmt, fb: Fmt) -> int:
    return load_library().adapt_acc_bits(k, fa, fb)


# -- the scalar rules of the switch controller (host functions of the library) -----------------
def pushup_suggest(ds: float, wl_min: int, fl_min: int, strategy: int, buff: int, wl_cap: int = 32):
    """Returns (WL, FL, s1, s2, s)."""
    res = PushupResult()
    _check(load_library().adapt_pushup_suggest(ds, wl_min, fl_min, strategy, buff, wl_cap, C.byref(res)),
           "adapt_pushup_suggest")
    return res.wl, res.fl, res.s1, res.s2, res.s


def strategy_next(strategy: int, loss_avg: float, loss_now: float) -> int:
    return load_library().adapt_strategy_next(strategy, loss_avg, loss_now)


def lookback_next(lb: int, ds: float, lb_lwr: int, lb_upr: int, gamma: float) -> int:
    return load_library().adapt_lookback_next(lb, ds, lb_lwr, lb_upr, gamma)


def resolution_next(r: int, lb: int, lb_lwr: int, lb_upr: int, r_lwr: int, r_upr: int) -> int:
    return load_library().adapt_resolution_next(r, lb, lb_lwr, lb_upr, r_lwr, r_upr)


# -- the paper's performance model (host functions of the library) ------------------------------
def perf_layers(rows):
    """rows: iterable of (ops, sp, numel, wl, lookback, resolution) -> ctypes array for the perf_* calls."""
    rows = list(rows)
    arr = (PerfLayer * max(len(rows), 1))()
    for k, r in enumerate(rows):
        arr[k] = PerfLayer(*r)
    return arr, len(rows)


def perf_step_cost(rows, accs=1):
    arr, n = perf_layers(rows)
    return load_library().adapt_perf_step_cost(arr, n, accs)


def perf_step_overhead(rows, accs=1):
    arr, n = perf_layers(rows)
    return load_library().adapt_perf_step_overhead(arr, n, accs)


def perf_model_size(rows):
    arr, n = perf_layers(rows)
    return load_library().adapt_perf_model_size(arr, n)


def perf_step_memory(rows):
    arr, n = perf_layers(rows)
    return load_library().adapt_perf_step_memory(arr, n)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _check(status: int, where: str):
    if status != 0:
        raise AdaptError(status, where)


class Context:
    """Owns an adapt_ctx bound to the current torch device and stream."""

    def __init__(self, workspace_bytes: int = 0, stream=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("paper_2107_13490_amd needs a HIP device; there is no CPU path")
        self._lib = load_library()
        self._torch = torch
        s = stream if stream is not None else torch.cuda.current_stream()
        self._stream = s
        h = C.c_void_p()
        _check(self._lib.adapt_create(C.byref(h), C.c_void_p(s.cuda_stream), workspace_bytes), "adapt_create")
        self._h = h

    def set_stream(self, stream):
        """Later calls launch on `stream` (a torch.cuda.Stream); the caller orders it against the old one."""
        _check(self._lib.adapt_set_stream(self._h, C.c_void_p(stream.cuda_stream)), "adapt_set_stream")
        self._stream = stream

    def close(self):
        if getattr(self, "_h", None):
            self._lib.adapt_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h

    def workspace_bytes(self, call, **fields) -> int:
        """adapt_workspace_bytes for one call: `call` is a CALL_* constant, `fields` the query fields that call reads
        (formats as (wl, fl) pairs, `conv` a ConvDesc, `kld_items` a list of (n, bins))."""
        q = WorkspaceQuery()
        q.call = call
        keep = None
        for k, v in fields.items():
            if k in ("fa", "fb", "fc"):
                v = Fmt(*v) if not isinstance(v, Fmt) else v
            if k == "kld_items":
                keep = (KldItem * max(len(v), 1))()
                for t, (n, bins) in enumerate(v):
                    keep[t] = KldItem(None, n, 1, bins, 0)
                q.count = len(v)
                v = keep
            setattr(q, k, v)
        need = self._lib.adapt_workspace_bytes(self._h, C.byref(q))
        if need == 0:
            raise AdaptError(-1, "adapt_workspace_bytes")
        return need

    def reserve_workspace(self, nbytes: int):
        _check(self._lib.adapt_reserve_workspace(self._h, nbytes), "adapt_reserve_workspace")

    def reserve_for_layers(self, layers, kld_bins=None, wl_lo=2, wl_hi=16):
        """Grows the workspace to what the forward and backward calls of the given layers need, and, with `kld_bins`, one
        batched precision search over their weight tensors.  layers: iterable of (ConvDesc, fx, fw, fdy) with (wl, fl) pairs."""
        need = 0
        items = []
        for d, fx, fw, fdy in layers:
            need = max(need, self.workspace_bytes(CALL_CONV_FWD, conv=d, fa=fx, fb=fw),
                       self.workspace_bytes(CALL_CONV_BACKWARD, conv=d, fa=fdy, fb=fw, fc=fx))
            items.append((d.k * d.r * d.s * d.c, kld_bins))
        if kld_bins:
            need = max(need, self.workspace_bytes(CALL_KLD_SEARCH_BATCHED, kld_items=items, wl_lo=wl_lo, wl_hi=wl_hi))
        need = max(need, self.workspace_bytes(CALL_QUANTIZE_BATCHED, count=64))
        self.reserve_workspace(need)
        return need

    @staticmethod
    def storage_dtype(wl: int):
        import torch
        return torch.int8 if wl <= 8 else torch.int16 if wl <= 16 else torch.int32

    # -- quantize -----------------------------------------------------------------------------
    def quantize(self, x, wl, fl, mode=SR, seed=0, stream=0, out=None, counters=None):
        """x: fp32 device tensor.  Returns (q, counters) with counters = uint64-as-int64[2] on the
        device holding nnz and saturated."""
        torch = self._torch
        if out is None:
            out = torch.empty(x.shape, dtype=self.storage_dtype(wl), device=x.device)
        if counters is None:
            counters = torch.empty(2, dtype=torch.int64, device=x.device)
        _check(self._lib.adapt_quantize(self._h, _ptr(x), x.numel(), Fmt(wl, fl), Rng(mode, seed, stream), _ptr(out),
                                        C.c_void_p(counters.data_ptr()), C.c_void_p(counters.data_ptr() + 8)),
               "adapt_quantize")
        return out, counters

    def quantize_noalloc(self, x, wl, fl, mode, seed, stream, out, counters):
        """adapt_quantize_noalloc: every buffer is the caller's (nothing is allocated here either)."""
        _check(self._lib.adapt_quantize_noalloc(self._h, _ptr(x), x.numel(), Fmt(wl, fl), Rng(mode, seed, stream), _ptr(out),
                                                C.c_void_p(counters.data_ptr()), C.c_void_p(counters.data_ptr() + 8)),
               "adapt_quantize_noalloc")
        return out, counters

    def quantize_batched(self, xs, fmts, streams, mode=SR, seed=0, outs=None, counters=None, ranges=None,
                         range_of=None):
        """One launch for all tensors.  `ranges`: optional float32[2 * len(xs)] device tensor that receives
        (min, max) of the finite elements of the inputs whose indices are listed in `range_of` (default:
        all); returns (outs, counters)."""
        torch = self._torch
        n = len(xs)
        if outs is None:
            outs = [torch.empty(x.shape, dtype=self.storage_dtype(f[0]), device=x.device) for x, f in zip(xs, fmts)]
        if counters is None:
            counters = torch.empty(2 * max(n, 1), dtype=torch.int64, device=xs[0].device if n else "cuda")
        items = (QuantizeItem * max(n, 1))()
        for t in range(n):
            items[t] = QuantizeItem(xs[t].data_ptr(), outs[t].data_ptr(), xs[t].numel(), fmts[t][0], fmts[t][1],
                                    streams[t])
        if ranges is None:
            _check(self._lib.adapt_quantize_batched(self._h, items, n, mode, seed, _ptr(counters)),
                   "adapt_quantize_batched")
        else:
            mask = sum(1 << t for t in (range(n) if range_of is None else range_of))
            _check(self._lib.adapt_quantize_batched_ranges(self._h, items, n, mode, seed, _ptr(counters), _ptr(ranges), mask),
                   "adapt_quantize_batched_ranges")
        return outs, counters

    # -- contractions -------------------------------------------------------------------------
    def _out_dtype(self, k_total, fa, fb, ep):
        torch = self._torch
        if ep.raw:
            return torch.int32 if self._lib.adapt_acc_bits(k_total, fa, fb) == 32 else torch.int64
        return self.storage_dtype(ep.fmt.wl)

    def _out_tensor(self, shape, k_total, fa, fb, ep, device):
        """Exact sums of operands above 16 bits are 128-bit integers: an int64 tensor with a last axis (low, high)."""
        torch = self._torch
        if ep.raw and self._lib.adapt_acc_bits(k_total, fa, fb) == 128:
            return torch.empty(tuple(shape) + (2,), dtype=torch.int64, device=device)
        return torch.empty(tuple(shape), dtype=self._out_dtype(k_total, fa, fb, ep), device=device)

    def fxp_gemm(self, a, fa, b, fb, ep, trans_a=False, trans_b=False, out=None):
        torch = self._torch
        m, k = (a.shape[1], a.shape[0]) if trans_a else a.shape
        k2, n = (b.shape[1], b.shape[0]) if trans_b else b.shape
        assert k == k2
        fa, fb = Fmt(*fa), Fmt(*fb)
        if out is None:
            out = self._out_tensor((m, n), k, fa, fb, ep, a.device)
        lda = a.stride(0) if a.numel() else max(a.shape[1], 1)      # empty tensors report stride 0
        ldb = b.stride(0) if b.numel() else max(b.shape[1], 1)
        ldc = n if out.dim() == 3 else out.stride(0)
        _check(self._lib.adapt_fxp_gemm(self._h, int(trans_a), int(trans_b), m, n, k, _ptr(a), fa, lda,
                                        _ptr(b), fb, ldb, _ptr(out), ldc, ep), "adapt_fxp_gemm")
        return out

    def conv_fwd(self, d: ConvDesc, x, fx, w, fw, ep, out=None):
        torch = self._torch
        fx, fw = Fmt(*fx), Fmt(*fw)
        if out is None:
            out = self._out_tensor((d.n, d.p, d.q, d.k), d.r * d.s * d.c, fx, fw, ep, x.device)
        _check(self._lib.adapt_conv_fwd(self._h, d, _ptr(x), fx, _ptr(w), fw, _ptr(out), ep), "adapt_conv_fwd")
        return out

    def conv_dgrad(self, d: ConvDesc, dy, fdy, w, fw, ep, out=None):
        torch = self._torch
        fdy, fw = Fmt(*fdy), Fmt(*fw)
        if out is None:
            out = self._out_tensor((d.n, d.h, d.w, d.c), d.r * d.s * d.k, fdy, fw, ep, dy.device)
        _check(self._lib.adapt_conv_dgrad(self._h, d, _ptr(dy), fdy, _ptr(w), fw, _ptr(out), ep), "adapt_conv_dgrad")
        return out

    def conv_wgrad(self, d: ConvDesc, dy, fdy, x, fx, ep, out=None):
        torch = self._torch
        fdy, fx = Fmt(*fdy), Fmt(*fx)
        if out is None:
            out = self._out_tensor((d.k, d.r, d.s, d.c), d.n * d.p * d.q, fdy, fx, ep, dy.device)
        _check(self._lib.adapt_conv_wgrad(self._h, d, _ptr(dy), fdy, _ptr(x), fx, _ptr(out), ep), "adapt_conv_wgrad")
        return out

    def conv_backward(self, d: ConvDesc, dy, fdy, w, fw, x, fx, ep_dx, ep_dw, out_dx=None, out_dw=None):
        """Both gradients of a layer in one call; returns (dx, dw)."""
        torch = self._torch
        fdy, fw, fx = Fmt(*fdy), Fmt(*fw), Fmt(*fx)
        if out_dx is None:
            out_dx = self._out_tensor((d.n, d.h, d.w, d.c), d.r * d.s * d.k, fdy, fw, ep_dx, dy.device)
        if out_dw is None:
            out_dw = self._out_tensor((d.k, d.r, d.s, d.c), d.n * d.p * d.q, fdy, fx, ep_dw, dy.device)
        _check(self._lib.adapt_conv_backward(self._h, d, _ptr(dy), fdy, _ptr(w), fw, _ptr(x), fx, _ptr(out_dx), ep_dx,
                                             _ptr(out_dw), ep_dw), "adapt_conv_backward")
        return out_dx, out_dw

    # -- KLD precision search -----------------------------------------------------------------
    def kld_precision_search(self, w, wl_lo, wl_hi, il, bins, eps, alpha=-1.0, mode=SR, seed=0, stream=0,
                             want_hist=False):
        """Returns dict(kld=f64[ncand], sel=int32[2], hist=uint32-as-int32[(ncand+1), bins] or None,
        grid=int64[3]) of device tensors."""
        torch = self._torch
        ncand = wl_hi - wl_lo + 1
        dev = w.device
        kld = torch.empty(max(ncand, 1), dtype=torch.float64, device=dev)
        sel = torch.empty(2, dtype=torch.int32, device=dev)
        grid = torch.empty(3, dtype=torch.int64, device=dev)
        hist = torch.empty((max(ncand, 0) + 1, bins), dtype=torch.int32, device=dev) if want_hist else None
        _check(self._lib.adapt_kld_precision_search(self._h, _ptr(w), w.numel(), wl_lo, wl_hi, il, bins, eps, alpha,
                                                    Rng(mode, seed, stream), _ptr(kld), _ptr(sel), _ptr(hist),
                                                    _ptr(grid)), "adapt_kld_precision_search")
        return dict(kld=kld, sel=sel, hist=hist, grid=grid)

    def kld_precision_search_ranged(self, w, rng_range, wl_lo, wl_hi, il, bins, eps, alpha=-1.0, mode=SR, seed=0,
                                    stream=0, want_hist=False, kld=None, sel=None, grid=None):
        """As kld_precision_search, with the tensor's (min, max) given as a device float32[2]."""
        torch = self._torch
        dev = w.device
        ncand = wl_hi - wl_lo + 1
        if kld is None:
            kld = torch.empty(max(ncand, 1), dtype=torch.float64, device=dev)
        if sel is None:
            sel = torch.empty(2, dtype=torch.int32, device=dev)
        if grid is None:
            grid = torch.empty(3, dtype=torch.int64, device=dev)
        hist = torch.empty((max(ncand, 0) + 1, bins), dtype=torch.int32, device=dev) if want_hist else None
        _check(self._lib.adapt_kld_precision_search_ranged(self._h, _ptr(w), w.numel(), _ptr(rng_range), wl_lo, wl_hi, il,
                                                           bins, eps, alpha, Rng(mode, seed, stream), _ptr(kld), _ptr(sel),
                                                           _ptr(hist), _ptr(grid)), "adapt_kld_precision_search_ranged")
        return dict(kld=kld, sel=sel, hist=hist, grid=grid)

    def kld_precision_search_batched(self, ws, ils, bins, streams, wl_lo, wl_hi, eps, alpha=-1.0, mode=SR, seed=0,
                                     kld=None, sel=None, ranges=None):
        """ranges: optional list with, per tensor, a device float32[2] tensor (min, max of its finite elements) or None."""
        torch = self._torch
        n = len(ws)
        ncand = wl_hi - wl_lo + 1
        dev = ws[0].device if n else "cuda"
        if kld is None:
            kld = torch.empty((max(n, 1), ncand), dtype=torch.float64, device=dev)
        if sel is None:
            sel = torch.empty((max(n, 1), 2), dtype=torch.int32, device=dev)
        items = (KldItem * max(n, 1))()
        for t in range(n):
            items[t] = KldItem(ws[t].data_ptr(), ws[t].numel(), ils[t], bins[t], streams[t])
        if ranges is None:
            _check(self._lib.adapt_kld_precision_search_batched(self._h, items, n, wl_lo, wl_hi, eps, alpha, mode, seed,
                                                                _ptr(kld), _ptr(sel)), "adapt_kld_precision_search_batched")
        else:
            rp = (C.c_void_p * max(n, 1))()
            for t in range(n):
                rp[t] = ranges[t].data_ptr() if ranges[t] is not None else None
            _check(self._lib.adapt_kld_precision_search_batched_ranged(self._h, items, rp, n, wl_lo, wl_hi, eps, alpha, mode, seed,
                                                                       _ptr(kld), _ptr(sel)),
                   "adapt_kld_precision_search_batched_ranged")
        return kld, sel

    # -- PushUp ---------------------------------------------------------------------------------
    def gradient_diversity(self, gs, fmts, out=None, sums=None, want_sums=True):
        """gs: device code tensors of one size (int8 for wl <= 8, int16 for wl <= 16, else int32), oldest first; fmts:
        their (wl, fl).  Returns (out, sums): out = float64[2] (ds, log ds or 1), sums = int64 view of the
        uint64[count + 2] integer sums, or of the uint64[2 (count + 1)] 128-bit sums (low word first) when a word
        length of the window exceeds 16 (None unless asked for)."""
        torch = self._torch
        count = len(gs)
        n = gs[0].numel() if count else 0
        dev = gs[0].device if count else "cuda"
        if out is None:
            out = torch.empty(2, dtype=torch.float64, device=dev)
        if sums is None and want_sums:
            wide = any(f[0] > 16 for f in fmts)
            sums = torch.empty(2 * (count + 1) if wide else count + 2, dtype=torch.int64, device=dev)
        items = (GradItem * max(count, 1))()
        for k in range(count):
            if gs[k].numel() != n:
                raise ValueError("all gradients of a window have the same number of elements")
            items[k] = GradItem(gs[k].data_ptr(), fmts[k][0], fmts[k][1])
        _check(self._lib.adapt_gradient_diversity(self._h, items, count, n, _ptr(sums), _ptr(out)),
               "adapt_gradient_diversity")
        return out, sums

    # -- master-weight update + re-quantization ---------------------------------------------------
    def sgd_update_quantize(self, w, g, fg, lr, l1, l2, wl, fl, g_sumsq=None, mode=SR, seed=0, stream=0, out=None,
                            counters=None, rng_range=None):
        """w: fp32 master weights (updated in place); g: gradient codes with format fg = (wl, fl);
        g_sumsq: device int64/uint64 scalar tensor (sum of squared codes) or None for an unnormalised
        step.  Returns (q, counters, range)."""
        torch = self._torch
        if out is None:
            out = torch.empty(w.shape, dtype=self.storage_dtype(wl), device=w.device)
        if counters is None:
            counters = torch.empty(2, dtype=torch.int64, device=w.device)
        if rng_range is None:
            rng_range = torch.empty(2, dtype=torch.float32, device=w.device)
        _check(self._lib.adapt_sgd_update_quantize(self._h, _ptr(w), w.numel(), _ptr(g), Fmt(*fg), _ptr(g_sumsq),
                                                   SgdParams(lr, l1, l2), Fmt(wl, fl), Rng(mode, seed, stream), _ptr(out),
                                                   _ptr(counters), _ptr(rng_range)), "adapt_sgd_update_quantize")
        return out, counters, rng_range

    # -- element-wise integer operations of a chained step ------------------------------------------
    def maxpool2_fwd(self, y, wl, out=None):
        """y: codes (n,h,w,c), h and w even.  Returns the 2x2/2 max-pooled codes."""
        n, h, w, c = y.shape
        if out is None:
            out = self._torch.empty((n, h // 2, w // 2, c), dtype=y.dtype, device=y.device)
        _check(self._lib.adapt_maxpool2_fwd(self._h, _ptr(y), Fmt(wl, 0), n, h, w, c, _ptr(out)), "adapt_maxpool2_fwd")
        return out

    def relu_pool_bwd(self, da, y, wl, relu, pool, out=None):
        """Gradient w.r.t. the contraction output; y = stored output before pooling (n,h,w,c)."""
        n, h, w, c = y.shape
        if out is None:
            out = self._torch.empty_like(y)
        _check(self._lib.adapt_relu_pool_bwd(self._h, _ptr(da), _ptr(y), Fmt(wl, 0), n, h, w, c, int(relu), int(pool),
                                             _ptr(out)), "adapt_relu_pool_bwd")
        return out

    def requantize_fit(self, acc, wl, mode=SR, seed=0, stream=0, out=None, want_sumsq=True, acc_bits=None):
        """acc: int32 / int64 exact accumulators, or 128-bit ones as int64[..., 2] (low word first) with acc_bits=128.
        Returns (codes, shift int32[1], sumsq or None); sumsq is int64[1], or for wl > 16 the 128-bit sum as int64[2]."""
        torch = self._torch
        bits = acc_bits if acc_bits is not None else (32 if acc.dtype == torch.int32 else 64)
        shape = acc.shape[:-1] if bits == 128 else acc.shape
        count = acc.numel() // 2 if bits == 128 else acc.numel()
        if out is None:
            out = torch.empty(shape, dtype=self.storage_dtype(wl), device=acc.device)
        shift = torch.empty(1, dtype=torch.int32, device=acc.device)
        sumsq = torch.empty(2 if wl > 16 else 1, dtype=torch.int64, device=acc.device) if want_sumsq else None
        _check(self._lib.adapt_requantize_fit(self._h, _ptr(acc), bits, count, wl, Rng(mode, seed, stream), _ptr(out),
                                              _ptr(shift), _ptr(sumsq)), "adapt_requantize_fit")
        return out, shift, sumsq

    def residual_add(self, a, fa, b, fb, fo, mode=SR, seed=0, stream=0, relu=False, out=None):
        """Codes of a + b in format fo = (wl, fl)."""
        if out is None:
            out = self._torch.empty(a.shape, dtype=self.storage_dtype(fo[0]), device=a.device)
        _check(self._lib.adapt_residual_add(self._h, _ptr(a), Fmt(*fa), _ptr(b), Fmt(*fb), a.numel(), Fmt(*fo),
                                            Rng(mode, seed, stream), int(relu), _ptr(out)), "adapt_residual_add")
        return out


    # -- batch normalisation, pooling, gradient merging -------------------------------------------
    def bn_forward(self, y, fy, gamma, beta, eps, fo, relu=False, res=None, fres=None, mode=SR, seed=0, stream=0, out=None,
                   state=None):
        """y: codes (..., channels).  Returns (out codes in format fo, state: uint8 device tensor for bn_backward)."""
        torch = self._torch
        k = y.shape[-1]
        rows = y.numel() // k
        if out is None:
            out = torch.empty(y.shape, dtype=self.storage_dtype(fo[0]), device=y.device)
        if state is None:
            state = torch.empty(max(self._lib.adapt_bn_state_bytes(k), 64), dtype=torch.uint8, device=y.device)
        _check(self._lib.adapt_bn_forward(self._h, _ptr(y), Fmt(*fy), rows, k, _ptr(gamma), _ptr(beta), float(eps),
                                          _ptr(res) if res is not None else None, Fmt(*(fres or (8, 0))), Fmt(*fo),
                                          Rng(mode, seed, stream), int(relu), _ptr(out), _ptr(state)), "adapt_bn_forward")
        return out, state

    def bn_backward(self, dz, wl_dz, y, fy, state, wl_out, mode=SR, seed=0, stream=0, e_in=None):
        """Returns dict(dy, dgamma, dbeta (float64), shift (int32[1]), e_out (int64[1]))."""
        torch = self._torch
        k = y.shape[-1]
        rows = y.numel() // k
        dy = torch.empty(y.shape, dtype=self.storage_dtype(wl_out), device=y.device)
        dg = torch.empty(k, dtype=torch.float64, device=y.device)
        db = torch.empty(k, dtype=torch.float64, device=y.device)
        shift = torch.empty(1, dtype=torch.int32, device=y.device)
        e_out = torch.empty(1, dtype=torch.int64, device=y.device)
        _check(self._lib.adapt_bn_backward(self._h, _ptr(dz), wl_dz, _ptr(y), Fmt(*fy), rows, k, _ptr(state), wl_out,
                                           Rng(mode, seed, stream), _ptr(dy), _ptr(dg), _ptr(db), _ptr(shift),
                                           _ptr(e_in) if e_in is not None else None, _ptr(e_out)), "adapt_bn_backward")
        return {"dy": dy, "dgamma": dg, "dbeta": db, "shift": shift, "e_out": e_out}

    def bn_update(self, gamma, beta, dgamma, dbeta, lr):
        _check(self._lib.adapt_bn_update(self._h, _ptr(gamma), _ptr(beta), _ptr(dgamma), _ptr(dbeta), gamma.numel(), float(lr)),
               "adapt_bn_update")

    def gap_fwd(self, a, fmt, mode=SR, seed=0, stream=0):
        """a: (n, h, w, c) codes -> (n, c) codes of the mean over the positions."""
        n, h, w, c = a.shape
        out = self._torch.empty((n, c), dtype=a.dtype, device=a.device)
        _check(self._lib.adapt_gap_fwd(self._h, _ptr(a), Fmt(*fmt), n, h * w, c, Rng(mode, seed, stream), _ptr(out)), "adapt_gap_fwd")
        return out

    def gap_bwd(self, dout, wl, h, w):
        n, c = dout.shape
        da = self._torch.empty((n, h, w, c), dtype=dout.dtype, device=dout.device)
        _check(self._lib.adapt_gap_bwd(self._h, _ptr(dout), wl, n, h * w, c, _ptr(da)), "adapt_gap_bwd")
        return da

    def grad_add(self, a, wl_a, e_a, b, wl_b, e_b, wl_out, mode=SR, seed=0, stream=0, out=None):
        """e_a, e_b: int64[1] device tensors (or None = 0); b may be None.  Returns (codes, shift int32[1], e_out int64[1])."""
        torch = self._torch
        if out is None:
            out = torch.empty(a.shape, dtype=self.storage_dtype(wl_out), device=a.device)
        shift = torch.empty(1, dtype=torch.int32, device=a.device)
        e_out = torch.empty(1, dtype=torch.int64, device=a.device)
        _check(self._lib.adapt_grad_add(self._h, _ptr(a), wl_a, _ptr(e_a) if e_a is not None else None,
                                        _ptr(b) if b is not None else None, wl_b, _ptr(e_b) if e_b is not None else None,
                                        a.numel(), wl_out, Rng(mode, seed, stream), _ptr(out), _ptr(shift), _ptr(e_out)),
               "adapt_grad_add")
        return out, shift, e_out


class Net:
    """A chained fixed-point training step (adapt_net_*).  Holds the workspace tensor and the master
    weights (fp32 device tensors, KRSC, updated in place by update())."""

    def __init__(self, ctx: Context, layers, weights, switch: "SwitchParams | None" = None, bn=None, bn_eps: float = 1e-5,
                 wl_max: int = 16):
        """layers: LayerDesc entries (a plain chain) or NodeDesc entries (a graph; bn = list with, per layer, a
        (gamma, beta) pair of device fp32 tensors or None).  wl_max = 32 lays a plain chain out for word lengths up
        to 32 (int32 codes, 128-bit accumulators)."""
        import torch
        self._ctx, self._lib, self._torch = ctx, ctx._lib, torch
        self.layers = list(layers)
        self.weights = list(weights)
        self.bn = list(bn) if bn is not None else None
        n = len(self.layers)
        graph = any(isinstance(d, NodeDesc) for d in self.layers)
        lb_upr = switch.lb_upr if switch is not None else 0
        if graph:
            descs = (NodeDesc * n)(*self.layers)
            need = (self._lib.adapt_graph_workspace_bytes(descs, n, lb_upr) if wl_max == 16 else
                    self._lib.adapt_graph_workspace_bytes_wide(descs, n, lb_upr, wl_max))
        elif wl_max != 16:
            descs = (LayerDesc * n)(*self.layers)
            need = self._lib.adapt_net_workspace_bytes_wide(descs, n, lb_upr, wl_max)
        else:
            descs = (LayerDesc * n)(*self.layers)
            need = self._lib.adapt_net_workspace_bytes(descs, n, lb_upr)
        if need == 0:
            raise AdaptError(-1, "adapt_net_workspace_bytes")
        self.workspace = torch.zeros(need, dtype=torch.uint8, device=self.weights[0].device)
        wptrs = (C.c_void_p * n)(*[w.data_ptr() for w in self.weights])
        h = C.c_void_p()
        sw = C.byref(switch) if switch is not None else None
        if graph:
            gp = (C.c_void_p * n)(*[(p[0].data_ptr() if p is not None else None) for p in (self.bn or [None] * n)])
            bp = (C.c_void_p * n)(*[(p[1].data_ptr() if p is not None else None) for p in (self.bn or [None] * n)])
            if wl_max == 16:
                _check(self._lib.adapt_graph_create(ctx.handle, descs, n, wptrs, gp, bp, float(bn_eps), sw, _ptr(self.workspace), need,
                                                    C.byref(h)), "adapt_graph_create")
            else:
                _check(self._lib.adapt_graph_create_wide(ctx.handle, descs, n, wptrs, gp, bp, float(bn_eps), sw, wl_max,
                                                         _ptr(self.workspace), need, C.byref(h)), "adapt_graph_create_wide")
        elif wl_max != 16:
            _check(self._lib.adapt_net_create_wide(ctx.handle, descs, n, wptrs, sw, wl_max, _ptr(self.workspace), need, C.byref(h)),
                   "adapt_net_create_wide")
        else:
            _check(self._lib.adapt_net_create(ctx.handle, descs, n, wptrs, sw, _ptr(self.workspace), need, C.byref(h)),
                   "adapt_net_create")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self._lib.adapt_net_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_format(self, layer, wl, fl):
        _check(self._lib.adapt_net_set_format(self._h, layer, Fmt(wl, fl)), "adapt_net_set_format")

    def tensor(self, layer, which):
        """View of one of the chain's tensors inside the workspace (flat int8 / int16; NT_STATS: a NetStats copy)."""
        torch = self._torch
        off, cnt, es = C.c_size_t(), C.c_size_t(), C.c_int()
        _check(self._lib.adapt_net_tensor(self._h, layer, which, C.byref(off), C.byref(cnt), C.byref(es)), "adapt_net_tensor")
        raw = self.workspace[off.value:off.value + cnt.value * es.value]
        if which == NT_STATS:
            return NetStats.from_buffer_copy(bytes(raw.cpu().numpy()))
        if which == NT_BN:
            return raw
        if which == NT_EXP:
            return raw.view(torch.int64)
        if which in (NT_DGAMMA, NT_DBETA):
            return raw.view(torch.float64)
        return raw.view(torch.int8 if es.value == 1 else torch.int16 if es.value == 2 else torch.int32)

    def quantize_weights(self, mode=SR, seed=0, stream=0):
        _check(self._lib.adapt_net_quantize_weights(self._h, Rng(mode, seed, stream)), "adapt_net_quantize_weights")

    def forward(self, x, mode=SR, seed=0, stream=0):
        _check(self._lib.adapt_net_forward(self._h, _ptr(x), Rng(mode, seed, stream)), "adapt_net_forward")

    def backward(self, dlogits, dlogits_fl=0, mode=SR, seed=0, stream=0):
        _check(self._lib.adapt_net_backward(self._h, _ptr(dlogits), dlogits_fl, Rng(mode, seed, stream)), "adapt_net_backward")

    def precision_switch(self, loss, mode=SR, seed=0, stream=0):
        """Alg. 2 between backward() and update().  Returns (list of SwitchReport per layer, strategy)."""
        n = len(self.layers)
        rep = (SwitchReport * n)()
        st = C.c_int()
        _check(self._lib.adapt_net_precision_switch(self._h, float(loss), Rng(mode, seed, stream), rep, C.byref(st)),
               "adapt_net_precision_switch")
        return list(rep), st.value

    def update(self, lr, l1=0.0, l2=0.0, mode=SR, seed=0, stream=0):
        _check(self._lib.adapt_net_update(self._h, SgdParams(lr, l1, l2), Rng(mode, seed, stream)), "adapt_net_update")
