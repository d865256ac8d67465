#!/usr/bin/env python3
"""Benchmark of the fixed-point hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch of the AlexNet-CIFAR-style
conv layer (batch 128, 64ch 16x16 -> 192ch 3x3, all tensors <8,5>):

    quantize(X, W, dY)  ->  conv fwd (+ReLU)  ->  backward: dgrad + wgrad   (outputs requantized, SR)
    ->  KL-divergence precision search on W (WL 4..16, 2048 bins)

All inputs are resident in HBM before the timed region.  `value` is useful conv/GEMM
tera-ops (2*M*N*K per contraction, three contractions) divided by the whole step time.
Prints ONE JSON line.
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
# HBM bytes per launch on this workload, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE (KiB per
# dispatch, scaled by what a plain 256 MiB device copy reads on the same counters: x2.0 and x1.0);
# the summary with the commands is profiles/bench_config2_hbm_traffic.md.  Counters cannot be read
# from inside this process.  Backward = the paired dgrad + wgrad kernel plus the slab-sum kernel.
FWD_TRAFFIC_BYTES = {"read": 3171 * 1024, "written": 6144 * 1024}
BWD_TRAFFIC_BYTES = {"read": (12695 + 7856) * 1024, "written": (9824 + 108) * 1024}

def cpu_baseline(batch: int):
    """The oracle, as it stands, on a bounded sample (reduced batch) of the same layer."""
    import numpy as np
    import workloads as wk
    from oracle import conv_oracle as co
    from oracle import fxp_oracle as orc

    L = wk.config2(batch=batch)
    s = L.shape
    co.load()
    t0 = time.perf_counter()
    qx, _, _ = orc.quantize(L.x, L.wl, L.fl, orc.SR, 0, 1)
    qw, _, _ = orc.quantize(L.w, L.wl, L.fl, orc.SR, 0, 2)
    qdy, _, _ = orc.quantize(L.dy, L.wl, L.fl, orc.SR, 0, 3)
    y = co.conv_fwd(qx, qw, s.stride, s.pad)
    dx = co.conv_dgrad(qdy, qw, s.h, s.w, s.stride, s.pad)
    dw = co.conv_wgrad(qdy, qx, s.r, s.s, s.stride, s.pad)
    orc.requantize(y, L.fl, L.wl, orc.SR, 0, 10, True)
    orc.requantize(dx, L.fl, L.wl, orc.SR, 0, 11)
    orc.requantize(dw, L.fl, L.wl, orc.SR, 0, 12)
    orc.kld_precision_search(L.w.ravel(), 4, 16, 3, 2048, 1e-2, None, orc.SR, 0, 2)
    dt = time.perf_counter() - t0
    ops = 3 * 2.0 * s.macs
    return {"value": ops / dt / 1e12, "unit": "TOPS", "cores": co.num_threads(), "kind": "oracle",
            "sample": f"same layer at batch {batch} (of 128): quantize + fwd + dgrad + wgrad + requantize + KLD, "
                      f"{dt:.2f} s"}


def next_rows(ctx, pkg, torch, w):
    """Per-call device time of the steps beyond the timed path (PushUp's gradient diversity, the fused
    master-weight update + re-quantization), on the config-2 weight tensor and on a 16 M element one.
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
    for tag, n, window, reps in (("config2_W", w.numel(), 25, 50), ("16M", 1 << 24, 25, 5)):
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


def chained_step(ctx, pkg, torch, batch=128):
    """The AlexNet-CIFAR layers of config 4 as one chained fixed-point training step (forward pass, backward
    pass with fitted gradient codes, update + re-quantization), formats of config 4; device time per phase."""
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
    ctx = pkg.Context(workspace_bytes=1 << 30)          # split-K partial sums of the larger layers
    # Alg. 2 with wide bounds on the formats so that the timing loop below keeps its layer formats close to
    # config 4's (a switch changes a layer's word length by a bit or two)
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

    # the precision switch between backward pass and update: wall time of the call (it synchronises three
    # times and runs the diversity and KL kernels), over a few real steps so that windows fill and switches occur
    import time
    sw_ms, switched = [], 0
    for step in range(8):
        net.forward(x)
        net.backward(dl, 0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rep, _ = net.precision_switch(2.0 - 0.1 * step, stream=100 * step)
        sw_ms.append((time.perf_counter() - t0) * 1e3)
        switched += sum(r.switched for r in rep)
        net.update(0.01, 1e-5, 1e-4, stream=100 * step)
    torch.cuda.synchronize()
    ops = 2.0 * macs * 3 - 2.0 * wk.alexnet_cifar_layers(batch)[0].shape.macs       # no data gradient below the first layer
    res = {"workload": f"AlexNet-CIFAR chain, batch {batch}, formats of configs[3]", "formats": fmts,
           "forward_ms": t_f, "forward_backward_ms": t_fb, "step_ms": t_all, "useful_TOPS": ops / (t_all * 1e-3) / 1e12,
           "precision_switch_ms_median": sorted(sw_ms)[len(sw_ms) // 2], "precision_switch_ms_max": max(sw_ms),
           "layers_switched_in_8_steps": int(switched),
           "formats_after": [(r.wl, r.fl) for r in rep]}
    net.close()
    ctx.close()
    return res


def other_config(args, cfg):
    """Configs 1, 3, 4 and 5 (supplementary lines; the default run is config 2).  A step is ONE batched quantize
    call over the X, W and dY of every layer of the config, then for every layer fwd + backward (dgrad + wgrad;
    requantized with SR), then ONE batched KLD call over all weight tensors.  Config 1 is a GEMM instead of a layer."""
    import numpy as np
    import torch
    import paper_2107_13490_amd as pkg
    import workloads as wk
    from paper_2107_13490_amd import ConvDesc, Epilogue

    torch.cuda.set_device(0)
    ctx = pkg.Context(workspace_bytes=1 << 30)
    calls = []            # (kind, fn)
    useful = issued = 0.0
    q_bytes = 0.0
    kld_ws, kld_bytes = [], 0.0
    if cfg == 1:
        a_h, b_h = wk.config1_gemm()
        a, b = torch.from_numpy(a_h).cuda(), torch.from_numpy(b_h).cuda()
        qa, qb = torch.empty(a.shape, dtype=torch.int8, device="cuda"), torch.empty(b.shape, dtype=torch.int8, device="cuda")
        c = torch.empty((256, 256), dtype=torch.int32, device="cuda")
        cnt = torch.empty(4, dtype=torch.int64, device="cuda")
        calls.append(("quantize", lambda: ctx.quantize_batched([a, b], [(8, 6)] * 2, [1, 2], pkg.SR, 0, outs=[qa, qb], counters=cnt)))
        calls.append(("fwd", lambda: ctx.fxp_gemm(qa, (8, 6), qb, (8, 6), Epilogue.exact(), out=c)))
        useful = issued = 2.0 * 256 ** 3
        q_bytes = 5.0 * 2 * 65536
        kld_ws = [torch.from_numpy(wk.config1_kld_tensor()).cuda()]
        kld_args = dict(ils=[2], wl_lo=2, wl_hi=16)
        workload = "configs[0]: GEMM 256^3 <8,6> (exact int32 output) + KLD on 65,536 values (WL 2..16, 2048 bins)"
        sample_layer = None
    else:
        if cfg == 3:
            layers = [wk.config3()]
            workload = "configs[2]: conv 128->128 3x3 @16x16, batch 256, <12,9> (two limbs), 50% zero weights"
        elif cfg == 4:
            layers = [wk.layer_inputs(sp, 40 + i) for i, sp in enumerate(wk.alexnet_cifar_layers())]
            workload = "configs[3]: AlexNet-CIFAR layer sweep (5 conv + 3 FC), batch 128, WL per layer from {4,6,8,12,16}"
        else:
            layers = [wk.layer_inputs(sp, 50 + i) for i, sp in enumerate(wk.resnet18_cifar_layers())]
            workload = "configs[4]: ResNet-18-CIFAR layer sweep (21 layers, 11.2 M weights), batch 256, WL per layer 4..16"
        sample_layer = max(layers, key=lambda L: L.shape.macs)
        q_in, q_out, q_fmt = [], [], []
        for L in layers:
            s = L.shape
            d = ConvDesc(s.n, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad)
            f = (L.wl, L.fl)
            dt = torch.int8 if L.wl <= 8 else torch.int16
            x, w, dy = (torch.from_numpy(t).cuda() for t in (L.x, L.w, L.dy))
            qx, qw, qdy = (torch.empty(t.shape, dtype=dt, device="cuda") for t in (x, w, dy))
            y, dx, dw = torch.empty(dy.shape, dtype=dt, device="cuda"), torch.empty_like(qx), torch.empty_like(qw)
            eps = [Epilogue.requant(L.wl, L.fl, pkg.SR, 0, 10 + i, relu=(i == 0)) for i in range(3)]

            def mk(d=d, f=f, qx=qx, qw=qw, qdy=qdy, y=y, dx=dx, dw=dw, eps=eps):
                return [("fwd", lambda: ctx.conv_fwd(d, qx, f, qw, f, eps[0], out=y)),
                        ("backward", lambda: ctx.conv_backward(d, qdy, f, qw, f, qx, f, eps[1], eps[2], out_dx=dx, out_dw=dw))]
            calls += mk()
            q_in += [x, w, dy]
            q_out += [qx, qw, qdy]
            q_fmt += [f] * 3
            ops = 3 * 2.0 * s.macs
            useful += ops
            issued += ops * (4 if L.wl > 8 else 1)
            q_bytes += (4.0 + (1 if L.wl <= 8 else 2)) * (x.numel() + w.numel() + dy.numel())
            kld_ws.append(w.view(-1))
        kld_args = dict(ils=[3] * len(kld_ws), wl_lo=4, wl_hi=16)
        # Quantize of the whole network: one call, one launch per 64 tensors (the per-layer loop of Alg. 1)
        q_cnt = torch.empty(2 * len(q_in), dtype=torch.int64, device="cuda")
        q_streams = list(range(1, len(q_in) + 1))
        calls.insert(0, ("quantize", lambda: ctx.quantize_batched(q_in, q_fmt, q_streams, pkg.SR, 0, outs=q_out, counters=q_cnt)))
    ncand = kld_args["wl_hi"] - kld_args["wl_lo"] + 1
    kld = torch.empty((len(kld_ws), ncand), dtype=torch.float64, device="cuda")
    sel = torch.empty((len(kld_ws), 2), dtype=torch.int32, device="cuda")
    calls.append(("kld", lambda: ctx.kld_precision_search_batched(kld_ws, kld_args["ils"], [2048] * len(kld_ws),
                                                                   list(range(2, 2 + len(kld_ws))), kld_args["wl_lo"],
                                                                   kld_args["wl_hi"], 1e-2, kld=kld, sel=sel)))
    kld_bytes = 8.0 * sum(t.numel() for t in kld_ws)

    def step():
        for _, fn in calls:
            fn()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) / args.steps * 1e3
    kind_ms = {}
    for kind, fn in calls:           # per-call device time, each call back to back
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
    conv_ms = sum(kind_ms.get(k, 0.0) for k in ("fwd", "backward"))
    out = {
        "metric": "fxp conv/GEMM TOPS (% int8 MFMA peak) + KLD precision-search GB/s",
        "value": useful / (ms_step * 1e-3) / 1e12, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": workload, "useful_ops_per_step": useful, "issued_int8_ops_per_step": issued},
        "roofline": {"bound": "mfma", "kernel": "contract_kernel, all contraction calls of the step",
                     "achieved": issued / (conv_ms * 1e-3) / 1e12, "peak": PEAK_INT8_TOPS, "unit": "TFLOP/s",
                     "frac": issued / (conv_ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, "traffic": None,
                     "note": "issued int8 MFMA ops (useful x 4 for two-limb layers) over the summed back-to-back device "
                             "time of the contraction calls"},
        "calls_ms_back_to_back": kind_ms,
        "useful_conv_TOPS": useful / (conv_ms * 1e-3) / 1e12,
        "quantize_GBps": q_bytes / (kind_ms["quantize"] * 1e-3) / 1e9,
        "quantize_frac_hbm": q_bytes / (kind_ms["quantize"] * 1e-3) / 1e9 / PEAK_HBM_GBPS,
        "kld_GBps": kld_bytes / (kind_ms["kld"] * 1e-3) / 1e9,
        "kld_frac_hbm": kld_bytes / (kind_ms["kld"] * 1e-3) / 1e9 / PEAK_HBM_GBPS,
    }
    if cfg == 4:
        out["chained_step"] = chained_step(ctx, pkg, torch, batch=128)
    if not args.no_cpu_baseline and sample_layer is not None:
        out["cpu_baseline"] = cpu_baseline_layer(sample_layer, args.cpu_batch)
    print(json.dumps(out))


def cpu_baseline_layer(L, batch):
    """The oracle on the config's largest layer at a reduced batch (contractions only)."""
    import workloads as wk
    from oracle import conv_oracle as co
    from oracle import fxp_oracle as orc
    s = L.shape
    small = wk.conv_layer(wk.ConvShape(min(batch, s.n), s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad), L.wl, L.fl, 99, 0.0, L.name)
    co.load()
    t0 = time.perf_counter()
    qx, _, _ = orc.quantize(small.x, L.wl, L.fl, orc.SR, 0, 1)
    qw, _, _ = orc.quantize(small.w, L.wl, L.fl, orc.SR, 0, 2)
    qdy, _, _ = orc.quantize(small.dy, L.wl, L.fl, orc.SR, 0, 3)
    co.conv_fwd(qx, qw, s.stride, s.pad)
    co.conv_dgrad(qdy, qw, s.h, s.w, s.stride, s.pad)
    co.conv_wgrad(qdy, qx, s.r, s.s, s.stride, s.pad)
    dt = time.perf_counter() - t0
    return {"value": 3 * 2.0 * small.shape.macs / dt / 1e12, "unit": "TOPS", "cores": co.num_threads(), "kind": "oracle",
            "sample": f"layer {L.name} at batch {small.shape.n} (of {s.n}): quantize + fwd + dgrad + wgrad, {dt:.2f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-next-rows", action="store_true",
                    help="skip the measurements beyond the timed step (PushUp, fused update, chained step): for profiler runs")
    ap.add_argument("--cpu-batch", type=int, default=16)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain device copy of 256 MiB (20 times): the known-size kernel that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters of rocprofv3 --pmc")
    ap.add_argument("--chained-step", action="store_true",
                    help="run only the chained AlexNet-CIFAR training step measurement (supplementary; for profiler runs)")
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5],
                    help="which of the five workload configurations to run (default 2, the one the metric is quoted on)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (use --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if args.chained_step:
        import torch
        import paper_2107_13490_amd as pkg
        torch.cuda.set_device(0)
        print(json.dumps({"chained_step": chained_step(None, pkg, torch, batch=128)}))
        return
    if args.config != 2 and not args.copy_calibration:
        other_config(args, args.config)
        return

    import torch
    import paper_2107_13490_amd as pkg
    import workloads as wk
    from paper_2107_13490_amd import ConvDesc, Epilogue

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
    L = wk.config2()
    s = L.shape
    d = ConvDesc(s.n, s.h, s.w, s.c, s.k, s.r, s.s, s.stride, s.pad)
    f = (L.wl, L.fl)
    x, w, dy = (torch.from_numpy(t).cuda() for t in (L.x, L.w, L.dy))
    qx = torch.empty(x.shape, dtype=torch.int8, device="cuda")
    qw = torch.empty(w.shape, dtype=torch.int8, device="cuda")
    qdy = torch.empty(dy.shape, dtype=torch.int8, device="cuda")
    y = torch.empty((s.n, s.p, s.q, s.k), dtype=torch.int8, device="cuda")
    dx = torch.empty(x.shape, dtype=torch.int8, device="cuda")
    dw = torch.empty(w.shape, dtype=torch.int8, device="cuda")
    counters = torch.empty(6, dtype=torch.int64, device="cuda")
    kld = torch.empty(13, dtype=torch.float64, device="cuda")
    sel = torch.empty(2, dtype=torch.int32, device="cuda")
    grid = torch.empty(3, dtype=torch.int64, device="cuda")
    ranges = torch.empty(6, dtype=torch.float32, device="cuda")
    ep_y = Epilogue.requant(L.wl, L.fl, pkg.SR, 0, 10, relu=True)
    ep_dx = Epilogue.requant(L.wl, L.fl, pkg.SR, 0, 11)
    ep_dw = Epilogue.requant(L.wl, L.fl, pkg.SR, 0, 12)

    calls = {
        # one launch quantizes the three tensors and, as a by-product of reading it, finds the range of W
        "quantize": lambda: ctx.quantize_batched([x, w, dy], [f, f, f], [1, 2, 3], pkg.SR, 0, outs=[qx, qw, qdy],
                                                 counters=counters, ranges=ranges, range_of=[1]),
        "conv_fwd": lambda: ctx.conv_fwd(d, qx, f, qw, f, ep_y, out=y),
        "conv_backward": lambda: ctx.conv_backward(d, qdy, f, qw, f, qx, f, ep_dx, ep_dw, out_dx=dx, out_dw=dw),
        # the search takes W's range from the quantize pass (no range pass of its own)
        "kld_search": lambda: ctx.kld_precision_search_ranged(w.view(-1), ranges[2:4], 4, 16, 3, 2048, 1e-2, stream=2,
                                                              kld=kld, sel=sel, grid=grid),
    }
    EV_EVERY = 10    # on every 10th step of the timed region events bracket the backward call (the dominant
                     # kernel), on every 10th + 5 the forward call

    def step(ev=None, which=None):
        calls["quantize"]()
        if which == "fwd":
            ev[0].record()
        calls["conv_fwd"]()
        if which == "fwd":
            ev[1].record()
        if which == "bwd":
            ev[0].record()
        calls["conv_backward"]()      # dgrad + wgrad of the layer, one call
        if which == "bwd":
            ev[1].record()
        calls["kld_search"]()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    kinds = ["bwd" if i % EV_EVERY == 0 else "fwd" if i % EV_EVERY == EV_EVERY // 2 else None for i in range(args.steps)]
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] if k else None for k in kinds]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i], kinds[i])
    t_enq = time.perf_counter() - t0
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_step = dt / args.steps * 1e3

    def mean_ms(kind):
        ts = [ev[0].elapsed_time(ev[1]) for ev, k in zip(events, kinds) if k == kind]
        return sum(ts) / len(ts) if ts else float("nan")
    fwd_ms, bwd_ms = mean_ms("fwd"), mean_ms("bwd")

    # per-call device time outside the timed region: each call repeated back to back between two events
    reps = 50
    call_ms = {}
    for name, fn in calls.items():
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        call_ms[name] = e0.elapsed_time(e1) / reps

    conv_ops = 2.0 * s.macs
    value = 3 * conv_ops / (ms_step * 1e-3) / 1e12
    # dominant kernel: the paired dgrad + wgrad launch of the backward call (its slab-sum kernel is inside the
    # bracket too); the forward convolution, one launch of the same contraction code, is reported beside it
    fwd_tops = conv_ops / (fwd_ms * 1e-3) / 1e12
    bwd_tops = 2 * conv_ops / (bwd_ms * 1e-3) / 1e12
    q_bytes = 5.0 * (x.numel() + w.numel() + dy.numel())
    kld_bytes = 4.0 * w.numel()      # one read of W: the range comes from the quantize pass
    note = ("HIP events around the call inside the timed region; includes the dispatch gaps that rocprofv3's kernel "
            "durations exclude (about 2-4 us per launch)")
    out = {
        "metric": "fxp conv/GEMM TOPS (% int8 MFMA peak) + KLD precision-search GB/s",
        "value": value, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "configs[1]: AlexNet-CIFAR conv 64->192 3x3 @16x16, batch 128, <8,5>; quantize(X,W,dY) "
                               "+ fwd + backward (dgrad + wgrad) (requantized, SR) + KLD search on W (WL 4..16, 2048 bins)",
                   "useful_ops_per_step": 3 * conv_ops},
        "roofline": {"bound": "mfma",
                     "kernel": "contract_pair_kernel<dgrad 64x64 | wgrad 64x64> + finish_kernel (the conv_backward call)",
                     "achieved": bwd_tops, "peak": PEAK_INT8_TOPS, "unit": "TFLOP/s", "frac": bwd_tops / PEAK_INT8_TOPS,
                     "traffic": BWD_TRAFFIC_BYTES["read"] + BWD_TRAFFIC_BYTES["written"],
                     "traffic_unit": "bytes of HBM per call (rocprofv3 --pmc, see profiles/)",
                     "algorithmic_bytes": dy.numel() + w.numel() + x.numel() + dx.numel() + dw.numel(),
                     "avg_launch_ms": bwd_ms, "avg_launch_ms_note": note},
        "roofline_fwd": {"bound": "mfma", "kernel": "contract_kernel<fwd 128x64> (the conv_fwd call is this one launch)",
                         "achieved": fwd_tops, "peak": PEAK_INT8_TOPS, "unit": "TFLOP/s", "frac": fwd_tops / PEAK_INT8_TOPS,
                         "traffic": FWD_TRAFFIC_BYTES["read"] + FWD_TRAFFIC_BYTES["written"],
                         "algorithmic_bytes": x.numel() + w.numel() + y.numel(), "avg_launch_ms": fwd_ms},
        "host_enqueue_ms_per_step": t_enq / args.steps * 1e3,
        "calls_ms_back_to_back": call_ms,
        "conv_TOPS": {"fwd": conv_ops / (call_ms["conv_fwd"] * 1e-3) / 1e12,
                      "backward (dgrad + wgrad)": 2 * conv_ops / (call_ms["conv_backward"] * 1e-3) / 1e12},
        "quantize_GBps": q_bytes / (call_ms["quantize"] * 1e-3) / 1e9,
        "quantize_frac_hbm": q_bytes / (call_ms["quantize"] * 1e-3) / 1e9 / PEAK_HBM_GBPS,
        "kld_GBps": kld_bytes / (call_ms["kld_search"] * 1e-3) / 1e9,
        "kld_frac_hbm": kld_bytes / (call_ms["kld_search"] * 1e-3) / 1e9 / PEAK_HBM_GBPS,
    }
    # cold-cache rate of the HBM-bound quantize call: 8 distinct sets of the three tensors (340 MB of
    # inputs and outputs, more than the 256 MB of last-level cache) used in turn
    sets = [([t.clone() for t in (x, w, dy)], [torch.empty_like(t) for t in (qx, qw, qdy)]) for _ in range(8)]
    for ins, outs in sets:
        ctx.quantize_batched(ins, [f, f, f], [1, 2, 3], pkg.SR, 0, outs=outs, counters=counters)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for rep in range(5):
        for ins, outs in sets:
            ctx.quantize_batched(ins, [f, f, f], [1, 2, 3], pkg.SR, 0, outs=outs, counters=counters)
    e1.record()
    torch.cuda.synchronize()
    cold_ms = e0.elapsed_time(e1) / 40
    out["quantize_cold_GBps"] = q_bytes / (cold_ms * 1e-3) / 1e9
    out["quantize_cold_frac_hbm"] = out["quantize_cold_GBps"] / PEAK_HBM_GBPS
    del sets
    if not args.no_next_rows:
        out["next_rows"] = next_rows(ctx, pkg, torch, w)
        out["next_rows"]["chained_step"] = chained_step(ctx, pkg, torch, batch=128)
        out["next_rows"]["chained_step_elementwise"] = elementwise_rows(ctx, pkg, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.cpu_batch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
