#!/usr/bin/env python3
"""Benchmark of the fixed-point hot path on one MI355X.

The headline workload is the largest single-GPU configuration: the ResNet-18-CIFAR layer sweep at batch 256
(configs[4]: 21 layers, 11.2 M weights, a word length of 4..16 bits per layer).  A step is one pass of the
whole path over one synthetic batch:

    ONE batched quantize call over the X, W and dY of every layer (it also returns the range of every W)
    -> per layer: conv fwd (+ReLU) and conv backward (dgrad + wgrad), outputs requantized with SR
    -> ONE batched KL-divergence precision search over all weight tensors (WL 4..16, 2048 bins)

All inputs are resident in HBM before the timed region.  `value` is useful conv/GEMM tera-ops (2*M*N*K per
contraction, three contractions per layer) divided by the whole step time.  The other configurations run as
shorter sub-records of the same JSON line (`--config N` makes N the headline instead).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0      # dense int8 MFMA, 256 CU x 8192 op/clk x 2.4 GHz
PEAK_HBM_GBPS = 8000.0
METRIC = "fxp conv/GEMM TOPS (% int8 MFMA peak) + KLD precision-search GB/s"

# HBM bytes per step of the contraction kernels on the headline workload, from two rocprofv3 --pmc runs (FETCH_SIZE,
# then WRITE_SIZE, KiB per dispatch summed over the contraction launches of one step) scaled by what a plain 256 MiB
# device copy reads on the same counters.  Counters cannot be read from inside this process; the summary with the
# commands is the file named here, and tests/test_bench_constants.py checks that the numbers agree with it.
TRAFFIC = {
    "profile": "profiles/bench_config5_hbm_traffic.md",
    "contractions_read_bytes": 1776614211,
    "contractions_written_bytes": 840604806,
    # from the kernel trace of the same workload (profiles/bench_config5_kernel_stats.md): device time of the contraction
    # kernels per step and their launches per step; the HIP-event figure measured live (roofline.avg_launch_ms) also
    # holds the dispatch gaps between the launches of a call and the channel-padding copies
    "stats_profile": "profiles/bench_config5_kernel_stats.md",
    "contractions_us_per_step": 2425.7,
    "contraction_launches_per_step": 73,
}

WORKLOADS = {
    1: "configs[0]: GEMM 256^3 <8,6> (exact int32 output) + KLD on 65,536 values (WL 2..16, 2048 bins)",
    2: "configs[1]: AlexNet-CIFAR conv 64->192 3x3 @16x16, batch 128, <8,5>",
    3: "configs[2]: conv 128->128 3x3 @16x16, batch 256, <12,9> (two limbs), 50% zero weights",
    4: "configs[3]: AlexNet-CIFAR layer sweep (5 conv + 3 FC), batch 128, WL per layer from {4,6,8,12,16}",
    5: "configs[4]: ResNet-18-CIFAR layer sweep (21 layers, 11.2 M weights, 30% zeros), batch 256, WL per layer 4..16",
}


def _stats(ms):
    s = sorted(ms)
    return {"mean": sum(s) / len(s), "median": s[len(s) // 2], "min": s[0], "n": len(s)}


def _layers_of(cfg):
    import workloads as wk
    if cfg == 2:
        return [wk.config2()]
    if cfg == 3:
        return [wk.config3()]
    if cfg == 4:
        return [wk.layer_inputs(sp, 40 + i) for i, sp in enumerate(wk.alexnet_cifar_layers())]
    return [wk.layer_inputs(sp, 50 + i) for i, sp in enumerate(wk.resnet18_cifar_layers())]


def run_config(cfg, steps, warmup, ctx, pkg, torch, per_layer=False, plain=False):
    """Builds the device tensors of configuration `cfg`, runs `warmup` + `steps` steps and returns the measurements.
    The timed region is bracketed by synchronisations; inside it HIP events on the library's stream mark every step
    boundary (median / min) and, on every tenth step, bracket each contraction call (roofline of the contractions)."""
    import workloads as wk
    from paper_2107_13490_amd import ConvDesc, Epilogue

    calls = []            # (kind, tag, fn)
    useful = issued = q_bytes = 0.0
    kld_ws = []
    layer_rows = []
    if cfg == 1:
        a_h, b_h = wk.config1_gemm()
        a, b = torch.from_numpy(a_h).cuda(), torch.from_numpy(b_h).cuda()
        qa, qb = torch.empty(a.shape, dtype=torch.int8, device="cuda"), torch.empty(b.shape, dtype=torch.int8, device="cuda")
        c = torch.empty((256, 256), dtype=torch.int32, device="cuda")
        cnt = torch.empty(4, dtype=torch.int64, device="cuda")
        calls.append(("quantize", "A,B", lambda: ctx.quantize_batched([a, b], [(8, 6)] * 2, [1, 2], pkg.SR, 0, outs=[qa, qb], counters=cnt)))
        calls.append(("fwd", "gemm", lambda: ctx.fxp_gemm(qa, (8, 6), qb, (8, 6), Epilogue.exact(), out=c)))
        useful = issued = 2.0 * 256 ** 3
        q_bytes = 5.0 * 2 * 65536
        kld_ws = [torch.from_numpy(wk.config1_kld_tensor()).cuda()]
        kld_args = dict(ils=[2], wl_lo=2, wl_hi=16)
        layer_rows.append({"name": "gemm256", "issued_ops": issued, "idx": [1]})
        ranges = None
    else:
        layers = _layers_of(cfg)
        q_in, q_out, q_fmt, w_slots, reserve = [], [], [], [], []
        for L in layers:
            s = L.shape
            d = ConvDesc(s.n, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad)
            f = (L.wl, L.fl)
            dt = torch.int8 if L.wl <= 8 else torch.int16
            x, w, dy = (torch.from_numpy(t).cuda() for t in (L.x, L.w, L.dy))
            qx, qw, qdy = (torch.empty(t.shape, dtype=dt, device="cuda") for t in (x, w, dy))
            y, dx, dw = torch.empty(dy.shape, dtype=dt, device="cuda"), torch.empty_like(qx), torch.empty_like(qw)
            eps = [Epilogue.requant(L.wl, L.fl, pkg.SR, 0, 10 + i, relu=(i == 0)) for i in range(3)]
            ops = 2.0 * s.macs
            mult = 4 if L.wl > 8 else 1
            row = {"name": L.name, "shape": [s.n, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad], "wl": L.wl,
                   "issued_ops": 3 * ops * mult, "idx": [len(calls), len(calls) + 1]}
            layer_rows.append(row)

            def mk(d=d, f=f, qx=qx, qw=qw, qdy=qdy, y=y, dx=dx, dw=dw, eps=eps, name=L.name):
                return [("fwd", name, lambda: ctx.conv_fwd(d, qx, f, qw, f, eps[0], out=y)),
                        ("backward", name, lambda: ctx.conv_backward(d, qdy, f, qw, f, qx, f, eps[1], eps[2], out_dx=dx, out_dw=dw))]
            calls += mk()
            w_slots.append(len(q_in) + 1)
            q_in += [x, w, dy]
            q_out += [qx, qw, qdy]
            q_fmt += [f] * 3
            reserve.append((d, f, f, f))
            useful += 3 * ops
            issued += 3 * ops * mult
            q_bytes += (4.0 + (1 if L.wl <= 8 else 2)) * (x.numel() + w.numel() + dy.numel())
            kld_ws.append(w.view(-1))
        ctx.reserve_for_layers(reserve, kld_bins=2048, wl_lo=4, wl_hi=16)
        kld_args = dict(ils=[3] * len(kld_ws), wl_lo=4, wl_hi=16)
        # Quantize of the whole network: one call (the per-layer loop of Alg. 1); the ranges of the weight tensors
        # are a by-product of the pass that reads them
        q_cnt = torch.empty(2 * len(q_in), dtype=torch.int64, device="cuda")
        ranges = torch.empty(2 * len(q_in), dtype=torch.float32, device="cuda")
        q_streams = list(range(1, len(q_in) + 1))
        for r in layer_rows:
            r["idx"] = [i + 1 for i in r["idx"]]
        calls.insert(0, ("quantize", "all", lambda: ctx.quantize_batched(q_in, q_fmt, q_streams, pkg.SR, 0, outs=q_out, counters=q_cnt,
                                                                          ranges=ranges, range_of=w_slots)))
    ncand = kld_args["wl_hi"] - kld_args["wl_lo"] + 1
    kld = torch.empty((len(kld_ws), ncand), dtype=torch.float64, device="cuda")
    sel = torch.empty((len(kld_ws), 2), dtype=torch.int32, device="cuda")
    if ranges is not None and len(kld_ws) == 1:
        # one tensor: the search takes W's range from the quantize pass (no range pass of its own)
        calls.append(("kld", "W", lambda: ctx.kld_precision_search_ranged(kld_ws[0], ranges[2:4], kld_args["wl_lo"], kld_args["wl_hi"],
                                                                           kld_args["ils"][0], 2048, 1e-2, stream=2, kld=kld[0], sel=sel[0])))
        kld_bytes = 4.0 * kld_ws[0].numel()
    else:
        # the search takes every W's range from the quantize pass (no range pass of its own) where that pass ran
        kld_ranges = [ranges[2 * i:2 * i + 2] for i in w_slots] if ranges is not None else None
        calls.append(("kld", "all W", lambda: ctx.kld_precision_search_batched(kld_ws, kld_args["ils"], [2048] * len(kld_ws),
                                                                               list(range(2, 2 + len(kld_ws))), kld_args["wl_lo"],
                                                                               kld_args["wl_hi"], 1e-2, kld=kld, sel=sel,
                                                                               ranges=kld_ranges)))
        kld_bytes = (4.0 if kld_ranges else 8.0) * sum(t.numel() for t in kld_ws)      # histogram pass (+ range pass)

    EV_EVERY = 10
    conv_idx = [i for i, (k, _, _) in enumerate(calls) if k in ("fwd", "backward")]

    def step(ev=None):
        for i, (_, _, fn) in enumerate(calls):
            if ev is not None and i in ev:
                ev[i][0].record()
                fn()
                ev[i][1].record()
            else:
                fn()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    if plain:                                   # profiler runs: whole steps only, so that launches divide by the step count
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        return {"workload": WORKLOADS[cfg], "steps_run": steps + warmup, "calls_per_step": len(calls)}
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    brackets = [{i: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for i in conv_idx}
                if s % EV_EVERY == 0 else None for s in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for s in range(steps):
        step(brackets[s])
        marks[s + 1].record()
    t_enq = time.perf_counter() - t0
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_step = dt / steps * 1e3
    step_ms = [marks[s].elapsed_time(marks[s + 1]) for s in range(steps)]
    # contraction calls: device time between the events around each call, per call averaged over the sampled steps
    per_call = {i: [] for i in conv_idx}
    for br in brackets:
        if br:
            for i, (e0, e1) in br.items():
                per_call[i].append(e0.elapsed_time(e1))
    call_ms = {i: sum(v) / len(v) for i, v in per_call.items() if v}
    conv_ms = sum(call_ms.values())

    # per-kind device time outside the timed region: each call repeated back to back between two events
    kind_ms = {}
    for kind, _, fn in calls:
        reps = 20
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        kind_ms[kind] = kind_ms.get(kind, 0.0) + e0.elapsed_time(e1) / reps

    out = {
        "workload": WORKLOADS[cfg], "steps": steps, "warmup": warmup,
        "ms_per_step": ms_step, "step_ms_device": _stats(step_ms), "host_enqueue_ms_per_step": t_enq / steps * 1e3,
        "useful_ops_per_step": useful, "issued_int8_ops_per_step": issued,
        "useful_TOPS": useful / (ms_step * 1e-3) / 1e12,
        "contractions": {"calls_per_step": len(conv_idx), "ms_per_step_in_timed_region": conv_ms,
                         "useful_TOPS": useful / (conv_ms * 1e-3) / 1e12, "issued_TOPS": issued / (conv_ms * 1e-3) / 1e12,
                         "frac_int8_peak": issued / (conv_ms * 1e-3) / 1e12 / PEAK_INT8_TOPS,
                         "note": "HIP events around every conv_fwd / conv_backward / gemm call on every 10th step of the timed region, "
                                 "on the stream the library launches on; includes the dispatch gaps inside a call"},
        "calls_ms_back_to_back": kind_ms,
        "quantize": {"bytes": q_bytes, "GBps": q_bytes / (kind_ms["quantize"] * 1e-3) / 1e9,
                     "frac_hbm": q_bytes / (kind_ms["quantize"] * 1e-3) / 1e9 / PEAK_HBM_GBPS, "cache": "warm"},
        "kld": {"bytes": kld_bytes, "GBps": kld_bytes / (kind_ms["kld"] * 1e-3) / 1e9,
                "frac_hbm": kld_bytes / (kind_ms["kld"] * 1e-3) / 1e9 / PEAK_HBM_GBPS,
                "tensors": len(kld_ws), "elements": int(sum(t.numel() for t in kld_ws))},
    }
    if per_layer:
        rows = []
        for r in layer_rows:
            ms = sum(call_ms.get(i, 0.0) for i in r["idx"])
            rows.append({"name": r["name"], "shape_nhwc_krs_stride_pad": r.get("shape"), "wl": r.get("wl"), "ms": ms,
                         "issued_TOPS": r["issued_ops"] / (ms * 1e-3) / 1e12 if ms else None})
        out["layers"] = rows
        heavy = max(rows, key=lambda r: r["ms"])
        out["heaviest_layer"] = heavy
    return out


def cold_quantize(ctx, pkg, torch, cfg=2):
    """Cold-cache rate of the HBM-bound quantize call: distinct sets of configs[1]'s three tensors (340 MB of inputs and
    outputs in all, more than the 256 MB of last-level cache) used in turn."""
    import workloads as wk
    L = wk.config2()
    f = (L.wl, L.fl)
    x, w, dy = (torch.from_numpy(t).cuda() for t in (L.x, L.w, L.dy))
    counters = torch.empty(6, dtype=torch.int64, device="cuda")
    q_bytes = 5.0 * (x.numel() + w.numel() + dy.numel())
    sets = [([t.clone() for t in (x, w, dy)], [torch.empty(t.shape, dtype=torch.int8, device="cuda") for t in (x, w, dy)]) for _ in range(8)]
    for ins, outs in sets:
        ctx.quantize_batched(ins, [f, f, f], [1, 2, 3], pkg.SR, 0, outs=outs, counters=counters)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        for ins, outs in sets:
            ctx.quantize_batched(ins, [f, f, f], [1, 2, 3], pkg.SR, 0, outs=outs, counters=counters)
    e1.record()
    torch.cuda.synchronize()
    cold_ms = e0.elapsed_time(e1) / 40
    return {"workload": "configs[1] tensors, 8 sets in rotation", "ms": cold_ms, "GBps": q_bytes / (cold_ms * 1e-3) / 1e9,
            "frac_hbm": q_bytes / (cold_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS}


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg):
    """The oracle, as it stands, on a bounded sample of the headline workload: its largest layer at reduced batch
    (quantize + fwd + dgrad + wgrad + requantize), once on one thread and once on all host cores, plus the precision
    search on that layer's weight tensor."""
    import ctypes
    import workloads as wk
    from oracle import conv_oracle as co
    from oracle import fxp_oracle as orc

    if cfg == 1:
        cfg = 2
    spec = max(_specs_of(cfg), key=lambda sp: sp.shape.macs)
    s = spec.shape
    co.load()
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
    except OSError:
        gomp = None
    cores = co.num_threads()

    def run(batch, threads):
        if gomp is not None:
            gomp.omp_set_num_threads(threads)
        small = wk.conv_layer(wk.ConvShape(batch, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad), spec.wl, spec.fl, 99, spec.zero_frac, spec.name)
        t0 = time.perf_counter()
        qx, _, _ = orc.quantize(small.x, spec.wl, spec.fl, orc.SR, 0, 1)
        qw, _, _ = orc.quantize(small.w, spec.wl, spec.fl, orc.SR, 0, 2)
        qdy, _, _ = orc.quantize(small.dy, spec.wl, spec.fl, orc.SR, 0, 3)
        y = co.conv_fwd(qx, qw, s.stride, s.pad)
        dx = co.conv_dgrad(qdy, qw, s.h, s.w, s.stride, s.pad)
        dw = co.conv_wgrad(qdy, qx, s.r, s.s, s.stride, s.pad)
        orc.requantize(y, spec.fl, spec.wl, orc.SR, 0, 10, True)
        orc.requantize(dx, spec.fl, spec.wl, orc.SR, 0, 11)
        orc.requantize(dw, spec.fl, spec.wl, orc.SR, 0, 12)
        dt = time.perf_counter() - t0
        return 3 * 2.0 * small.shape.macs / dt / 1e12, dt, small

    one_tops, one_s, one = run(max(2, s.n // 4), 1)
    all_tops, all_s, small = run(s.n, cores)
    if gomp is not None:
        gomp.omp_set_num_threads(cores)
    t0 = time.perf_counter()
    orc.kld_precision_search(small.w.ravel(), 4, 16, 3, 2048, 1e-2, None, orc.SR, 0, 2)
    kld_s = time.perf_counter() - t0
    return {"value": all_tops, "unit": "TOPS", "cores": cores, "kind": "oracle", "cpu_model": cpu_model(),
            "single_thread": {"value": one_tops, "unit": "TOPS", "cores": 1, "seconds": one_s,
                              "sample": f"layer {spec.name} at batch {one.shape.n} (of {s.n}); the contractions run on one OpenMP thread, "
                                        "the rounding bits of quantize / requantize are still drawn on all cores"},
            "kld_search": {"GBps": 8.0 * small.w.size / kld_s / 1e9, "seconds": kld_s,
                           "sample": f"weight tensor of {spec.name}, {small.w.size} elements, WL 4..16, 2048 bins"},
            "sample": f"largest layer of the workload ({spec.name}, <{spec.wl},{spec.fl}>) at batch {small.shape.n} (of {s.n}): "
                      f"quantize + fwd + dgrad + wgrad + requantize, {all_s:.2f} s on {cores} threads"}


def _specs_of(cfg):
    import workloads as wk
    if cfg == 2:
        return [wk.LayerSpec("alexnet_conv2", wk.ConvShape(128, 16, 16, 64, 192), 8, 5)]
    if cfg == 3:
        return [wk.LayerSpec("resnet_block_conv", wk.ConvShape(256, 16, 16, 128, 128), 12, 9, 0.5)]
    if cfg == 4:
        return wk.alexnet_cifar_layers()
    return wk.resnet18_cifar_layers()


def next_rows(ctx, pkg, torch, n_small):
    """Per-call device time of the steps beyond the timed path (PushUp's gradient diversity, the fused
    master-weight update + re-quantization), on a weight tensor of configs[1]'s size and on a 16 M element one.
    Algorithmic bytes: diversity = window x n x 1 B of int8 codes; update = 4 + 1 B read, 4 + 1 B written."""
    def timed(fn, reps):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    res = {}
    for tag, n, window, reps in (("config2_W", n_small, 25, 50), ("16M", 1 << 24, 25, 5)):
        gs = [torch.randint(-128, 128, (n,), dtype=torch.int8, device="cuda") for _ in range(window)]
        master = torch.randn(n, device="cuda") * 0.06
        q = torch.empty(n, dtype=torch.int8, device="cuda")
        out = torch.empty(2, dtype=torch.float64, device="cuda")
        sums = torch.empty(window + 2, dtype=torch.int64, device="cuda")
        cnt = torch.empty(2, dtype=torch.int64, device="cuda")
        rr = torch.empty(2, dtype=torch.float32, device="cuda")
        fm = [(8, 7)] * window
        ms_gd = timed(lambda: ctx.gradient_diversity(gs, fm, out=out, sums=sums), reps)
        ms_up = timed(lambda: ctx.sgd_update_quantize(master, gs[0], (8, 7), 0.01, 1e-5, 1e-4, 8, 5, g_sumsq=sums[0:1],
                                                      out=q, counters=cnt, rng_range=rr), reps)
        res[tag] = {"n": n, "window": window,
                    "gradient_diversity_ms": ms_gd, "gradient_diversity_GBps": window * n / (ms_gd * 1e-3) / 1e9,
                    "sgd_update_quantize_ms": ms_up, "sgd_update_quantize_GBps": 10.0 * n / (ms_up * 1e-3) / 1e9}
        del gs, master, q
    return res


def elementwise_rows(ctx, pkg, torch):
    """Device time and algorithmic HBM rate of the chained step's element-wise kernels on tensors of the size
    AlexNet-CIFAR's first layer produces at batch 128 (128 x 32 x 32 x 64 = 8.4 M elements).  Algorithmic bytes per
    element: max-pool 1 read + 1/4 written (int8); pool/ReLU gradient 1 + 1/4 read, 1 written; fitting
    requantization int32 -> int8: 4 read twice + 1 written; residual addition 1 + 1 read, 1 written."""
    def timed(fn, reps=30):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    n, h, w, c = 128, 32, 32, 64
    ne = n * h * w * c
    y = torch.randint(0, 128, (n, h, w, c), dtype=torch.int8, device="cuda")
    a = torch.empty((n, h // 2, w // 2, c), dtype=torch.int8, device="cuda")
    da = torch.randint(-128, 128, a.shape, dtype=torch.int8, device="cuda")
    dy = torch.empty_like(y)
    acc = torch.randint(-(1 << 20), 1 << 20, (ne,), dtype=torch.int32, device="cuda")
    q = torch.empty(ne, dtype=torch.int8, device="cuda")
    b2 = torch.randint(-128, 128, (ne,), dtype=torch.int8, device="cuda")
    rows = {}
    for name, fn, bytes_per_call in (
            ("maxpool2_fwd", lambda: ctx.maxpool2_fwd(y, 8, out=a), 1.25 * ne),
            ("relu_pool_bwd", lambda: ctx.relu_pool_bwd(da, y, 8, True, True, out=dy), 2.25 * ne),
            ("requantize_fit", lambda: ctx.requantize_fit(acc, 8, out=q), 9.0 * ne),
            ("residual_add", lambda: ctx.residual_add(y.view(-1), (8, 5), b2, (8, 4), (8, 4), out=q), 3.0 * ne)):
        ms = timed(fn)
        rows[name] = {"ms": ms, "GBps": bytes_per_call / (ms * 1e-3) / 1e9, "frac_hbm": bytes_per_call / (ms * 1e-3) / 1e9 / PEAK_HBM_GBPS}
    rows["elements"] = ne
    return rows


def wide_rows(ctx, pkg, torch):
    """Word lengths 17..32 (int32 codes, contractions composed of narrower parts with 128-bit recombination): device time
    of quantize on 16 M elements and of the forward / backward calls of configs[2]'s layer shape with <20,16>, <24,20>
    and <32,28> operands (the three ways an operand is split).  TOPS are useful ops (2 M N K); these calls are exact,
    not fast."""
    from paper_2107_13490_amd import ConvDesc, Epilogue

    def timed(fn, reps=5):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    rows = {}
    n = 1 << 24
    x = torch.randn(n, device="cuda")
    q = torch.empty(n, dtype=torch.int32, device="cuda")
    ms = timed(lambda: ctx.quantize(x, 24, 20, pkg.SR, seed=1, stream=2, out=q), 20)
    rows["quantize_24bit_16M"] = {"ms": ms, "GBps": 8.0 * n / (ms * 1e-3) / 1e9, "frac_hbm": 8.0 * n / (ms * 1e-3) / 1e9 / PEAK_HBM_GBPS}
    d = ConvDesc(128, 16, 16, 64, 192, 3, 3, 1, 1)
    ops = 2.0 * d.n * d.p * d.q * d.k * d.r * d.s * d.c
    for wl, fl in ((20, 16), (24, 20), (32, 28)):
        lim = 1 << (wl - 2)
        xq = torch.randint(-lim, lim, (d.n, d.h, d.w, d.c), dtype=torch.int32, device="cuda")
        wq = torch.randint(-lim, lim, (d.k, d.r, d.s, d.c), dtype=torch.int32, device="cuda")
        dy = torch.randint(-lim, lim, (d.n, d.p, d.q, d.k), dtype=torch.int32, device="cuda")
        need = max(ctx.workspace_bytes(pkg.CALL_CONV_FWD, conv=d, fa=(wl, fl), fb=(wl, fl)),
                   ctx.workspace_bytes(pkg.CALL_CONV_BACKWARD, conv=d, fa=(wl, 0), fb=(wl, fl), fc=(wl, fl)))
        ctx.reserve_workspace(need + 2 * 9 * 8 * max(xq.numel(), dy.numel()))      # room for one exact buffer per pair of parts
        ep = Epilogue.requant(wl, fl, pkg.SR, 0, 10, relu=True)
        y = ctx.conv_fwd(d, xq, (wl, fl), wq, (wl, fl), ep)
        f_ms = timed(lambda: ctx.conv_fwd(d, xq, (wl, fl), wq, (wl, fl), ep, out=y))
        dx, dw = ctx.conv_backward(d, dy, (wl, 0), wq, (wl, fl), xq, (wl, fl), Epilogue.exact(), Epilogue.exact())
        b_ms = timed(lambda: ctx.conv_backward(d, dy, (wl, 0), wq, (wl, fl), xq, (wl, fl), Epilogue.exact(), Epilogue.exact(),
                                               out_dx=dx, out_dw=dw))
        rows[f"conv_config2_shape_wl{wl}"] = {"forward_ms": f_ms, "forward_useful_TOPS": ops / (f_ms * 1e-3) / 1e12,
                                              "backward_ms": b_ms, "backward_useful_TOPS": 2 * ops / (b_ms * 1e-3) / 1e12}
    return rows


def chained_step(ctx, pkg, torch, batch=128):
    """The AlexNet-CIFAR layers of configs[3] as one chained fixed-point training step (forward pass, backward
    pass with fitted gradient codes, update + re-quantization), formats of configs[3]; device time per phase."""
    import numpy as np
    import workloads as wk
    from paper_2107_13490_amd import ConvDesc, LayerDesc
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4)
    descs, ws, fmts, macs = [], [], [], 0
    for sp, relu, pool in wk.alexnet_cifar_chain(batch):
        s = sp.shape
        descs.append(LayerDesc(ConvDesc(s.n, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad), int(relu), int(pool)))
        ws.append(torch.randn((s.k, s.r, s.s, s.c), device="cuda", generator=gen) * (1.5 / np.sqrt(s.r * s.s * s.c)))
        fmts.append((sp.wl, sp.fl))
        macs += s.macs
    ctx.reserve_for_layers([(d.conv, f, f, f) for d in descs for f in ((8, 5), (16, 13))], kld_bins=150, wl_lo=4, wl_hi=16)
    # Alg. 2 with wide bounds on the formats so that the timing loop below keeps its layer formats close to
    # configs[3]'s (a switch changes a layer's word length by a bit or two)
    sp = pkg.SwitchParams(lb_lwr=2, lb_upr=4, lb_init=2, r_lwr=100, r_upr=150, r_init=128, gamma=0.5, eps=1e-3, buff=3,
                          wl_lo=4, wl_hi=16, strategy_init=pkg.ST_MIN)
    net = pkg.Net(ctx, descs, ws, switch=sp)
    for l, (wl, fl) in enumerate(fmts):
        net.set_format(l, wl, fl)
    x = torch.randn((batch, 32, 32, 3), device="cuda", generator=gen)
    dl = torch.randint(-4, 4, (batch, 10), device="cuda", dtype=torch.int32, generator=gen).to(
        torch.int8 if fmts[-1][0] <= 8 else torch.int16)
    net.quantize_weights()

    def timed(fn, reps=20):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def fwd():
        net.forward(x)

    def fwd_bwd():
        net.forward(x)
        net.backward(dl, 0)

    def full():
        net.forward(x)
        net.backward(dl, 0)
        net.update(0.01, 1e-5, 1e-4)
    t_f, t_fb, t_all = timed(fwd), timed(fwd_bwd), timed(full)

    # the precision switch between backward pass and update: wall time of the call, over a few real steps so that
    # windows fill and switches occur
    sw_ms, quiet_ms, switched = [], [], 0
    for step in range(8):
        net.forward(x)
        net.backward(dl, 0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rep, _ = net.precision_switch(2.0 - 0.1 * step, stream=100 * step)
        sw_ms.append((time.perf_counter() - t0) * 1e3)
        if not any(r.switched for r in rep):
            quiet_ms.append(sw_ms[-1])             # no layer switched: diversities, lookback and resolution only
        switched += sum(r.switched for r in rep)
        net.update(0.01, 1e-5, 1e-4, stream=100 * step)
    torch.cuda.synchronize()
    ops = 2.0 * macs * 3 - 2.0 * wk.alexnet_cifar_layers(batch)[0].shape.macs       # no data gradient below the first layer
    res = {"workload": f"AlexNet-CIFAR chain, batch {batch}, formats of configs[3]", "formats": fmts,
           "forward_ms": t_f, "forward_backward_ms": t_fb, "step_ms": t_all, "useful_TOPS": ops / (t_all * 1e-3) / 1e12,
           "precision_switch_ms_median": sorted(sw_ms)[len(sw_ms) // 2], "precision_switch_ms_max": max(sw_ms),
           "precision_switch_ms_when_no_layer_switches": (sorted(quiet_ms)[len(quiet_ms) // 2] if quiet_ms else None),
           "layers_switched_in_8_steps": int(switched),
           "formats_after": [(r.wl, r.fl) for r in rep]}
    net.close()
    return res


def chained_resnet18(ctx, pkg, torch, batch=256):
    """The ResNet-18-CIFAR layers of configs[4] as one chained fixed-point training step: convolutions, fixed-point batch
    normalisation with the shortcuts fused in, global average pooling, backward pass with merged gradients, update of
    weights, gamma and beta + re-quantization; formats of configs[4] (word lengths below 6 raised to 6: a chain
    feeds each layer's output to the next, and 4-bit activations saturate); device time per phase."""
    import numpy as np
    import workloads as wk
    from paper_2107_13490_amd import ConvDesc, NodeDesc
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    nodes, ws, bn, fmts, macs = [], [], [], [], 0
    graph = wk.resnet18_cifar_graph(batch)
    for sp, relu, has_bn, src, res, gap in graph:
        s = sp.shape
        nodes.append(NodeDesc(ConvDesc(s.n, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad), int(relu), 0, int(has_bn), src, res, int(gap)))
        ws.append(torch.randn((s.k, s.r, s.s, s.c), device="cuda", generator=gen) * (1.4 / np.sqrt(s.r * s.s * s.c)))
        bn.append((torch.ones(s.k, device="cuda"), torch.zeros(s.k, device="cuda")) if has_bn else None)
        wl = max(sp.wl, 6)
        fmts.append((wl, wl - 4))
        macs += s.macs
    ctx.reserve_for_layers([(d.conv, f, f, f) for d in nodes for f in ((8, 4), (16, 12))], kld_bins=150, wl_lo=4, wl_hi=16)
    net = pkg.Net(ctx, nodes, ws, bn=bn)
    for l, (wl, fl) in enumerate(fmts):
        net.set_format(l, wl, fl)
    x = torch.randn((batch, 32, 32, 3), device="cuda", generator=gen)
    dl = torch.randint(-4, 4, (batch, 100), device="cuda", dtype=torch.int32, generator=gen).to(
        torch.int8 if fmts[-1][0] <= 8 else torch.int16)
    net.quantize_weights()

    def timed(fn, reps=10):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def fwd():
        net.forward(x)

    def fwd_bwd():
        net.forward(x)
        net.backward(dl, 0)

    def full():
        net.forward(x)
        net.backward(dl, 0)
        net.update(0.01, 1e-5, 1e-4)
    t_f, t_fb, t_all = timed(fwd), timed(fwd_bwd), timed(full)
    # host time to enqueue a step with an idle queue (the device works behind it): below step_ms, the step is bound by the device
    enq = []
    for _ in range(5):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        full()
        enq.append((time.perf_counter() - t0) * 1e3)
    torch.cuda.synchronize()
    ops = 2.0 * macs * 3 - 2.0 * graph[0][0].shape.macs               # no data gradient below the first layer
    net.close()
    return {"workload": f"ResNet-18-CIFAR chain (batch norm, shortcuts, average pooling), batch {batch}, formats of configs[4] (WL >= 6)",
            "formats": fmts, "forward_ms": t_f, "forward_backward_ms": t_fb, "step_ms": t_all,
            "host_enqueue_ms": sorted(enq)[len(enq) // 2], "useful_TOPS": ops / (t_all * 1e-3) / 1e12}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-next-rows", action="store_true",
                    help="skip everything beyond the headline configuration's timed steps (sub-records of the other "
                         "configurations, PushUp, fused update, chained step): for profiler runs")
    ap.add_argument("--steps-only", action="store_true",
                    help="run warmup + steps whole steps of --config and nothing else (no per-call timing loops): every kernel's "
                         "launch count is then a multiple of the step count, which the rocprofv3 summaries under profiles/ rely on")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain device copy of 256 MiB (20 times): the known-size kernel that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters of rocprofv3 --pmc")
    ap.add_argument("--chained-step", action="store_true",
                    help="run only the chained AlexNet-CIFAR training step measurement (supplementary; for profiler runs)")
    ap.add_argument("--config", type=int, default=5, choices=[1, 2, 3, 4, 5],
                    help="the headline configuration (default 5, the largest that fits one GPU)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (use --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2107_13490_amd as pkg

    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4, "launches": 20}))
        return
    ctx = pkg.Context()
    if args.chained_step:
        print(json.dumps({"chained_step": chained_step(ctx, pkg, torch, batch=128),
                          "chained_step_resnet18": chained_resnet18(ctx, pkg, torch, batch=256)}))
        return
    if args.steps_only:
        print(json.dumps(run_config(args.config, args.steps, args.warmup, ctx, pkg, torch, plain=True)))
        return

    head = run_config(args.config, args.steps, args.warmup, ctx, pkg, torch, per_layer=True)
    con = head["contractions"]
    traffic = None
    if args.config == 5 and TRAFFIC["contractions_read_bytes"] is not None:
        traffic = TRAFFIC["contractions_read_bytes"] + TRAFFIC["contractions_written_bytes"]
    out = {
        "metric": METRIC, "value": head["useful_TOPS"], "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "ms_per_step_device": head["step_ms_device"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": head["workload"], "useful_ops_per_step": head["useful_ops_per_step"],
                   "issued_int8_ops_per_step": head["issued_int8_ops_per_step"]},
        "roofline": {"bound": "mfma",
                     "kernel": "the contraction kernels of one step (contract_kernel<...> instances, contract_pair_kernel, finish_kernel): "
                               f"{con['calls_per_step']} conv_fwd / conv_backward calls",
                     "units_per_launch": "issued int8 MFMA ops of one step (useful 2*M*N*K x 4 for layers above 8 bits) over the "
                                         "summed device time of these calls",
                     "achieved": con["issued_TOPS"], "peak": PEAK_INT8_TOPS, "unit": "TFLOP/s", "frac": con["frac_int8_peak"],
                     "avg_launch_ms": con["ms_per_step_in_timed_region"], "avg_launch_ms_note": con["note"],
                     "traffic": traffic, "traffic_profile": TRAFFIC["profile"] if traffic else None,
                     "rocprof_us_per_step": TRAFFIC["contractions_us_per_step"] if args.config == 5 else None,
                     "rocprof_launches_per_step": TRAFFIC["contraction_launches_per_step"] if args.config == 5 else None,
                     "rocprof_profile": TRAFFIC["stats_profile"] if args.config == 5 else None,
                     "useful_TOPS": con["useful_TOPS"], "heaviest_layer": head.get("heaviest_layer")},
        "quantize": head["quantize"], "kld": head["kld"], "calls_ms_back_to_back": head["calls_ms_back_to_back"],
        "host_enqueue_ms_per_step": head["host_enqueue_ms_per_step"],
        "layers": head.get("layers"),
    }
    out["quantize_cold"] = cold_quantize(ctx, pkg, torch)
    if not args.no_next_rows:
        subs = {}
        for cfg in (1, 2, 3, 4):
            if cfg == args.config:
                continue
            torch.cuda.empty_cache()
            r = run_config(cfg, 30, 5, ctx, pkg, torch)
            subs[f"configs[{cfg - 1}]"] = r
        out["other_configs"] = subs
        torch.cuda.empty_cache()
        out["next_rows"] = next_rows(ctx, pkg, torch, 110592)
        out["next_rows"]["chained_step"] = chained_step(ctx, pkg, torch, batch=128)
        torch.cuda.empty_cache()
        out["next_rows"]["chained_step_resnet18"] = chained_resnet18(ctx, pkg, torch, batch=256)
        out["next_rows"]["chained_step_elementwise"] = elementwise_rows(ctx, pkg, torch)
        out["next_rows"]["wide_17_32_bits"] = wide_rows(ctx, pkg, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
