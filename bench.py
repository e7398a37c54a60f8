#!/usr/bin/env python3
"""Benchmark of the hot path: ResNet-152 fp32 training steps under an 8 GiB device-memory
budget on one MI355X (benchmark configs[3]), synthetic ImageNet-shaped data.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--k auto|N] [--budget-gib 8]

Prints ONE JSON line.  `value` = images/s over exactly K timed steps at the headline
minibatch, inputs resident in HBM (`pcie_inclusive` gives the same run with the batch handed
over in pinned host memory, the first layer's prefetch of Algorithm 1).  `roofline` prices
the dominant convolution kernel (by total time in a step) against the fp32 MFMA peak;
`conv.by_shape` every distinct convolution shape and role; `swap_points` the swap engine
where it has work to do (link GB/s, hidden fraction of the copy time, no-swap reference at
the same minibatch); `cpu_baseline` times the CPU oracle on a bounded sample of the workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GiB = 1 << 30
PEAK_FP32_MFMA_TFLOPS = 157.3     # MI355X, dense fp32 matrix
PEAK_BF16_MFMA_TFLOPS = 2500.0    # dense bf16 matrix
PEAK_HBM_GBS = 8000.0
MAX_TIMED_SWAP_BYTES = 24 << 30   # the library refuses event timing of plans that swap more
MAX_TIMED_POINT_BYTES = 16 << 30  # swap points above this are not event-timed here (copy time from the calibrated rate)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--k", default="auto", help="headline minibatch, or 'auto' = best of the sweep")
    ap.add_argument("--sweep", default="32,64,128,256", help="minibatch sizes of the sweep (configs[3])")
    ap.add_argument("--swap-points", default="64,128,4x",
                    help="minibatches at which the swap engine is measured in detail after the headline "
                         "('4x' = four times the largest minibatch that needs no swap; '' = none)")
    ap.add_argument("--budget-gib", type=float, default=8.0)
    ap.add_argument("--net", default="resnet152", choices=["vgg16", "resnet18", "resnet34", "resnet50", "resnet101", "resnet152"])
    ap.add_argument("--mode", default="dynamic", choices=["dynamic", "naive", "none"])
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"],
                    help="storage of activations / gradients / kernel-side weights (bf16: configs[4])")
    ap.add_argument("--serial", action="store_true",
                    help="weight gradients on the compute stream instead of their own (every kernel runs alone: "
                         "the setting in which single kernels are timed)")
    ap.add_argument("--graph", default="auto", choices=["auto", "on", "off"],
                    help="replay iterations that swap nothing from a HIP graph (acc_set_graph); auto: whichever is "
                         "faster in two short runs at the headline minibatch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-noswap-reference", action="store_true")
    ap.add_argument("--cpu-sample-k", type=int, default=12)
    return ap.parse_args()


# HBM bytes per launch of the dominant kernel (igemm_kernel<direct>), from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs of this script, scaled by what the same counters read for sgd_kernel
# (profiles/resnet152_k41_hbm_traffic_pmc.txt).  A figure of that profile, not of this run: counters
# need the profiler.  Known for the profiled workload only.
PROFILED_TRAFFIC_BYTES = {("resnet152", 41, 8.0): 71.3e6}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    import faulthandler
    faulthandler.enable()
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path would shard by data parallelism: one plan, pool "
              "and set of streams per GPU, one all-reduce of the weight gradients per iteration); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np  # noqa: F401
    import torch
    import synth as S
    from paper_1901_06773_amd import binding as B

    net = getattr(S, args.net)()
    chw = (net.in_c, net.in_h, net.in_w)
    budget = int(args.budget_gib * GiB)
    mode = {"dynamic": B.PLAN_DYNAMIC, "naive": B.PLAN_NAIVE_ALL, "none": B.PLAN_NONE}[args.mode]
    sweep_ks = [int(x) for x in args.sweep.split(",") if x]
    if args.k != "auto":
        sweep_ks = sorted(set(sweep_ks + [int(args.k)]))

    # ---- static analysis without the GPU: which minibatches are trainable, how much host memory
    dtype = B.BF16 if args.dtype == "bf16" else B.F32
    probe = B.Context(net.as_array(), chw, dtype=dtype)
    lo, hi = 1, 4096
    while lo < hi:                                   # largest k that fits with nothing swapped
        mid = (lo + hi + 1) // 2
        try:
            probe.plan_swaps(mid, budget, B.PLAN_NONE)
            lo = mid
        except B.AccError:
            hi = mid - 1
    noswap_max_k = lo
    swap_point_ks = [4 * noswap_max_k if x == "4x" else int(x) for x in args.swap_points.split(",") if x]
    trainable, host_need = [], 256
    for k in sorted(set(sweep_ks + swap_point_ks)):
        try:
            s_all = probe.plan_swaps(k, budget, B.PLAN_NAIVE_ALL)
            if k in sweep_ks:
                trainable.append(k)
            # what the planner's own choice swaps (with the uncalibrated model; the calibrated one may differ a
            # little: 10 % on top), never more than every map; pinned memory is capped per process on the box
            s_dyn = probe.plan_swaps(k, budget, mode if mode != B.PLAN_NONE else B.PLAN_DYNAMIC)
            host_need = max(host_need, min(s_all["host_bytes"], int(s_dyn["host_bytes"] * 1.1)))
        except B.AccError as e:
            log(f"k={k}: not trainable under {args.budget_gib} GiB ({e})")
            swap_point_ks = [x for x in swap_point_ks if x != k]
    if args.k == "auto" and noswap_max_k not in trainable:
        trainable = sorted(trainable + [noswap_max_k])     # the largest minibatch that needs no swap
    probe.close()
    if not trainable:
        print("bench.py: no minibatch of the sweep is trainable under the budget", file=sys.stderr)
        sys.exit(1)

    torch.cuda.set_device(0)
    # pinned staging for the headline's batches, taken before the large arena (pinned memory is capped per process)
    k_stage = noswap_max_k if args.k == "auto" else int(args.k)
    pin_stage = torch.empty((2, max(k_stage, 1)) + chw, dtype=torch.float32).pin_memory()
    t0 = time.time()
    ctx = B.Context(net.as_array(), chw, pool_bytes=budget, host_bytes=host_need + (64 << 20), dtype=dtype)
    ctx.set_weights(S.init_params(net))
    if args.serial:
        ctx.set_wgrad_overlap(False)
    log(f"context ready in {time.time() - t0:.1f}s: pool {budget / GiB:.2f} GiB, pinned host {host_need / GiB:.2f} GiB")

    # ---- dynamic information: per-step times at the sweep's minibatches, link bandwidth
    t0 = time.time()
    fine = list(range(max(1, noswap_max_k - 15), noswap_max_k + 1)) if args.k == "auto" else []
    ctx.calibrate(sorted(set(trainable + fine)))
    cal = ctx.get_calibration()
    log(f"calibrated at k={cal['ks']} (asked for {trainable}) in {time.time() - t0:.1f}s; "
        f"link {cal['link'][0] / 1e9:.1f} / {cal['link'][1] / 1e9:.1f} GB/s")

    # ---- Algorithm 2 / Eq. 7: the minibatch the performance model expects to be fastest
    tuner = None
    if args.k == "auto":
        tuner, _ = ctx.tune_minibatch(budget, 1, max(sweep_ks))
        log("tuner", tuner)
        if tuner["k_best"] not in trainable:
            trainable = sorted(trainable + [tuner["k_best"]])

    cache = {}

    def batch(k, step, pinned=False):
        key = (k, step, pinned)
        if key not in cache:
            img, lab = S.make_batch(net, k, step)
            t = torch.from_numpy(img)
            if pinned:
                slot = pin_stage[step % 2][:k]
                slot.copy_(t)
                cache[key] = (slot, lab)
            else:
                cache[key] = (t.cuda(), lab)
        return cache[key]

    def forget(k):
        for key in [key for key in cache if key[0] == k]:
            del cache[key]

    def run(c_, k, steps, warmup, first_step=0, pinned=False):
        imgs = [batch(k, first_step + i, pinned) for i in range(min(2, steps + warmup))]
        for i in range(warmup):
            c_.train_step(*imgs[i % len(imgs)], 0.1)
        torch.cuda.synchronize()
        t = time.perf_counter()
        loss = 0.0
        for i in range(steps):
            loss = c_.train_step(*imgs[i % len(imgs)], 0.1)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / steps, loss

    # ---- sweep (configs[3]): short runs, to find the throughput-optimal minibatch
    sweep = []
    for k in trainable:
        try:
            summ = ctx.plan_swaps(k, budget, mode)
        except B.AccError as e:
            log(f"sweep: k={k} skipped ({e})")
            continue
        sec, loss = run(ctx, k, 3, 1)
        sweep.append(dict(k=k, images_per_s=k / sec, ms_per_step=sec * 1e3, n_swapped=summ["n_swapped"],
                          n_maps=summ["n_maps"], gib_swapped_each_way=summ["bytes_swapped"] / GiB,
                          peak_gib=summ["peak_bytes"] / GiB, predicted_ms=summ["t_iter"] * 1e3,
                          predicted_stall_ms=summ["t_stall"] * 1e3, plan_ms=summ["plan_ms"]))
        log("sweep", sweep[-1])
        forget(k)
    best = max(sweep, key=lambda r: r["images_per_s"])
    k = best["k"] if args.k == "auto" else int(args.k)

    # ---- headline: W warm-up steps, then exactly K timed steps, inputs resident in HBM
    summ = ctx.plan_swaps(k, budget, mode)
    graph_choice = dict(requested=args.graph, used=False)
    if summ["n_swapped"] == 0 and args.graph != "off":
        if args.graph == "auto":
            sec_eager, _ = run(ctx, k, 5, 2)
            ctx.set_graph(True)
            sec_graph, _ = run(ctx, k, 5, 2)
            graph_choice.update(eager_ms=sec_eager * 1e3, graph_ms=sec_graph * 1e3)
            graph_choice["used"] = sec_graph < sec_eager
        else:
            graph_choice["used"] = True
        ctx.set_graph(graph_choice["used"])
    sec, loss = run(ctx, k, args.steps, args.warmup)
    value = k / sec
    stats = ctx.stats()
    # the same with the batch in pinned host memory: its copy to the device is the first layer's prefetch
    pcie_inclusive = None
    if k <= pin_stage.shape[1]:
        sec_host, _ = run(ctx, k, args.steps, 1, pinned=True)
        pcie_inclusive = dict(images_per_s=k / sec_host, ms_per_step=sec_host * 1e3,
                              note="same plan and steps, the batch handed over in pinned host memory "
                                   f"({k * chw[0] * chw[1] * chw[2] * 4 / 1e6:.1f} MB per step over the host link, on the swap-in stream)")

    # ---- roofline of the dominant kernel: events directly around every convolution launch,
    # and per-step / per-copy times.  The library refuses event timing for plans that swap
    # more than 24 GiB per iteration; then the kernels are timed in the uncapped no-swap
    # context below (same kernels, same shapes) and the copies are not timed one by one.
    def profiled(c_, kk):
        c_.set_profiling(3)
        c_.train_step(*batch(kk, 0), 0.1)
        c_.train_step(*batch(kk, 1), 0.1)
        r = (c_.kernel_profile(), c_.step_times_ms(), c_.stats(), c_.launch_profile())
        c_.set_profiling(0)
        return r

    timed_swaps = summ["host_bytes"] <= MAX_TIMED_SWAP_BYTES
    if timed_swaps:
        kp, step_ms, pstats, launches = profiled(ctx, k)
    names = [ctx.step_info(j)["name"] for j in range(ctx.step_count())]
    # bytes of the tensors every step reads and writes (the headline plan is the installed one)
    step_bytes = []
    for j in range(ctx.step_count()):
        reads, writes = ctx.step_io(j)
        step_bytes.append(sum(ctx.tensor_info(t)["bytes"] for t in set(reads) | set(writes)))

    # ---- the swap engine at work: minibatches above the no-swap maximum, same context
    swap_points = []
    for ks in swap_point_ks:
        try:
            sp_summ = ctx.plan_swaps(ks, budget, B.PLAN_DYNAMIC)
        except B.AccError as e:
            log(f"swap point: k={ks} skipped ({e})")
            continue
        if sp_summ["n_swapped"] == 0:
            continue
        sp_sec, _ = run(ctx, ks, 3, 1)
        pt = dict(k=ks, times_noswap_max=ks / noswap_max_k, images_per_s=ks / sp_sec, ms_per_step=sp_sec * 1e3,
                  predicted_ms=sp_summ["t_iter"] * 1e3, predicted_stall_ms=sp_summ["t_stall"] * 1e3,
                  n_swapped=sp_summ["n_swapped"], n_maps=sp_summ["n_maps"],
                  gib_each_way=sp_summ["bytes_swapped"] / GiB, peak_gib=sp_summ["peak_bytes"] / GiB,
                  noswap_peak_gib=sp_summ["noswap_peak_bytes"] / GiB)
        if sp_summ["host_bytes"] <= MAX_TIMED_POINT_BYTES:
            ctx.set_profiling(1)
            ctx.train_step(*batch(ks, 0), 0.1)
            ps = ctx.stats()
            ctx.set_profiling(0)
            pt.update(d2h_ms=ps["d2h_ms"], h2d_ms=ps["h2d_ms"],
                      d2h_gbs=ps["bytes_out"] / 1e9 / (ps["d2h_ms"] * 1e-3), h2d_gbs=ps["bytes_in"] / 1e9 / (ps["h2d_ms"] * 1e-3),
                      copy_times="events around every copy, one profiled step")
        else:
            pt.update(d2h_ms=sp_summ["bytes_swapped"] / cal["link"][0] * 1e3, h2d_ms=sp_summ["bytes_swapped"] / cal["link"][1] * 1e3,
                      d2h_gbs=cal["link"][0] / 1e9, h2d_gbs=cal["link"][1] / 1e9,
                      copy_times="bytes / calibrated link rate (copies are event-timed only up to 16 GiB per iteration here)")
        swap_points.append(pt)
        log("swap point", pt)
        forget(ks)
    ctx.close()
    del ctx
    torch.cuda.empty_cache()

    # ---- the same minibatches with nothing swapped in an uncapped pool: what the swaps cost
    def noswap_run(kk, peak_bytes, want_profile=False):
        big = int(peak_bytes * 1.03) + (64 << 20)
        c2 = B.Context(net.as_array(), chw, pool_bytes=big, host_bytes=256, dtype=dtype)
        c2.set_weights(S.init_params(net))
        if args.serial:
            c2.set_wgrad_overlap(False)
        c2.plan_swaps(kk, big, B.PLAN_NONE)
        s0, _ = run(c2, kk, 4, 1)
        prof = profiled(c2, kk) if want_profile else None
        c2.close()
        del c2
        torch.cuda.empty_cache()
        return s0, big, prof

    noswap = None
    sec0 = None
    if (not args.no_noswap_reference and summ["n_swapped"] > 0) or not timed_swaps:
        sec0, big, prof = noswap_run(k, summ["noswap_peak_bytes"], want_profile=not timed_swaps)
        if not timed_swaps:
            kp, step_ms, _, launches = prof
            pstats = dict(stats, d2h_ms=stats["bytes_out"] / cal["link"][0] * 1e3,
                          h2d_ms=stats["bytes_in"] / cal["link"][1] * 1e3)
    forget(k)
    if not args.no_noswap_reference:
        for pt in swap_points:
            s0, big_pt, _ = noswap_run(pt["k"], int(pt["noswap_peak_gib"] * GiB))
            copy_s = (pt["d2h_ms"] + pt["h2d_ms"]) * 1e-3
            pt.update(noswap_ms_per_step=s0 * 1e3, noswap_images_per_s=pt["k"] / s0, noswap_pool_gib=big_pt / GiB,
                      hidden_fraction=1.0 - (pt["ms_per_step"] * 1e-3 - s0) / copy_s)
            forget(pt["k"])
            log("swap point, no-swap reference", pt)

    dom = max(kp, key=lambda r: r["ms"])
    conv_flops = sum(r["flops"] for r in kp)
    conv_ms = sum(r["ms"] for r in kp)
    ach = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
    # bf16 storage: both convolution kernels multiply bf16 on the matrix cores (dense peak 2.5 PFLOP/s)
    peak = PEAK_BF16_MFMA_TFLOPS if args.dtype == "bf16" else PEAK_FP32_MFMA_TFLOPS
    traffic = PROFILED_TRAFFIC_BYTES.get((args.net, k, args.budget_gib)) if args.dtype == "f32" else None
    roofline = dict(bound="mfma", kernel=dom["name"], achieved=ach, peak=peak, unit="TFLOP/s",
                    frac=ach / peak, traffic=traffic,
                    traffic_source=("rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command "
                                    "(profiles/resnet152_k41_hbm_traffic_pmc.txt), not measured in this run") if traffic else None,
                    launches_per_step=dom["launches"],
                    avg_launch_us=dom["ms"] * 1e3 / dom["launches"],
                    flop_per_launch=dom["flops"] / dom["launches"],
                    timed_in=("two extra steps of the headline context" if timed_swaps else "the no-swap run of the same minibatch") +
                             ", weight gradients on the compute stream so that every kernel is timed alone")
    # every distinct convolution shape, per role (forward product, data gradient, weight gradient)
    by_shape = {}
    for l in launches:
        lay = net.layers[l["layer"]]
        if lay.kind != S.CONV:
            continue
        key = (lay.cin, lay.cout, lay.r, lay.stride, l["role"])
        e = by_shape.setdefault(key, dict(cin=lay.cin, cout=lay.cout, r=lay.r, stride=lay.stride, role=l["role"],
                                          launches=0, ms=0.0, flops=0.0))
        e["launches"] += 1
        e["ms"] += l["ms"]
        e["flops"] += l["flops"]
    shape_rows = []
    for e in sorted(by_shape.values(), key=lambda r: -r["flops"]):
        tf = e["flops"] / (e["ms"] * 1e-3) / 1e12 if e["ms"] > 0 else None
        shape_rows.append(dict(shape=f"{e['cin']}->{e['cout']} {e['r']}x{e['r']}/{e['stride']}", role=e["role"],
                               launches=e["launches"], ms=round(e["ms"], 4), tflops=tf,
                               frac_of_peak=tf / peak if tf else None,
                               share_of_conv_flops=e["flops"] / conv_flops))
    # step-level view: BN / pooling / update steps against the HBM roofline
    by_kind, bytes_by_kind = {}, {}
    for n_, ms, nb in zip(names, step_ms, step_bytes):
        by_kind[n_] = by_kind.get(n_, 0.0) + float(ms)
        bytes_by_kind[n_] = bytes_by_kind.get(n_, 0) + nb
    # batch norm (+ReLU, +add) against the HBM roofline: bytes of the tensors the steps touch
    # (each counted once per step, although backward reads x and dy twice) over their time
    hbm = {n_: dict(gb_per_step=bytes_by_kind[n_] / 1e9, ms_per_step=by_kind[n_],
                    gbs=bytes_by_kind[n_] / 1e9 / (by_kind[n_] * 1e-3), frac_of_hbm_peak=bytes_by_kind[n_] / 1e9 /
                    (by_kind[n_] * 1e-3) / PEAK_HBM_GBS)
           for n_ in ("bn_fwd", "bn_bwd", "maxpool_fwd", "maxpool_bwd") if by_kind.get(n_, 0) > 0}
    conv = dict(tflops=conv_flops / (conv_ms * 1e-3) / 1e12, frac_of_mfma_peak=conv_flops / (conv_ms * 1e-3) / 1e12 / peak,
                ms_per_step=conv_ms, flops_per_step=conv_flops,
                kernels=[dict(name=r["name"], launches=r["launches"], ms=r["ms"],
                              tflops=r["flops"] / (r["ms"] * 1e-3) / 1e12) for r in kp],
                by_shape=shape_rows)
    swap = dict(gib_out=pstats["bytes_out"] / GiB, gib_in=pstats["bytes_in"] / GiB,
                d2h_gbs=(pstats["bytes_out"] / 1e9) / (pstats["d2h_ms"] * 1e-3) if pstats["d2h_ms"] > 0 else None,
                h2d_gbs=(pstats["bytes_in"] / 1e9) / (pstats["h2d_ms"] * 1e-3) if pstats["h2d_ms"] > 0 else None,
                d2h_ms=pstats["d2h_ms"], h2d_ms=pstats["h2d_ms"],
                copy_times="events around every copy" if timed_swaps else "bytes / calibrated link rate",
                calibrated_link_gbs=dict(d2h=cal["link"][0] / 1e9, h2d=cal["link"][1] / 1e9),
                note="the headline plan; the swap engine under load is in swap_points")
    if sec0 is not None and summ["n_swapped"] > 0:
        copy_s = (swap["d2h_ms"] + swap["h2d_ms"]) * 1e-3
        noswap = dict(ms_per_step=sec0 * 1e3, images_per_s=k / sec0, pool_gib=big / GiB,
                      hidden_fraction=(1.0 - (sec - sec0) / copy_s) if copy_s > 0 else None)
        swap["hidden_fraction"] = noswap["hidden_fraction"]

    # ---- CPU baseline: the oracle, as it stands, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle as O
        kc = args.cpu_sample_k
        params = S.init_params(net)
        img, lab = S.make_batch(net, 1, 0)
        O.train_step(net.as_array(), chw, params, img, lab, 0.1)        # warm-up: library and threads
        img, lab = S.make_batch(net, kc, 0)
        t = time.perf_counter()
        O.train_step(net.as_array(), chw, params, img, lab, 0.1)
        dt = time.perf_counter() - t
        cpu = dict(value=kc / dt, unit="images/s", cores=int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())),
                   kind="oracle", sample=f"one {args.net} training step at minibatch {kc} ({dt:.1f} s) after a one-image warm-up step")

    out = dict(
        metric="train images/s (ResNet-152 fp32, 8 GiB HBM budget) + conv MFMA utilisation" if (args.net, args.dtype, args.budget_gib) == ("resnet152", "f32", 8.0)
        else f"train images/s ({args.net} {args.dtype}, {args.budget_gib} GiB HBM budget) + conv MFMA utilisation",
        value=value, unit="images/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
        ms_per_step=sec * 1e3, higher_is_better=True, scaling="weak", vs_baseline=None, dtype=args.dtype,
        data="synthetic",
        config=dict(workload=f"{args.net} {'fp32' if args.dtype == 'f32' else 'bf16 (fp32 master weights and statistics)'} training step, 224x224x3 N(0,1) images, 1000 classes, "
                             f"minibatch {k}, device-memory budget {args.budget_gib} GiB, planner mode {args.mode}",
                    minibatch=k, budget_gib=args.budget_gib, strides="v1", optimizer="plain SGD lr 0.1",
                    wgrad_stream=not args.serial, graph_replay=graph_choice),
        roofline=roofline, cpu_baseline=cpu, pcie_inclusive=pcie_inclusive, conv=conv, swap=swap, swap_points=swap_points,
        noswap_reference=noswap,
        plan=dict(n_maps=summ["n_maps"], n_swapped=summ["n_swapped"], peak_gib=summ["peak_bytes"] / GiB,
                  layer_peak_gib=summ["layer_peak_bytes"] / GiB, noswap_peak_gib=summ["noswap_peak_bytes"] / GiB,
                  predicted_ms=summ["t_iter"] * 1e3, predicted_stall_ms=summ["t_stall"] * 1e3,
                  predicted_compute_ms=summ["t_compute"] * 1e3, plan_ms=summ["plan_ms"],
                  host_issue_ms=stats["host_issue_ms"], host_wait_ms=stats["host_wait_ms"],
                  host_busy_ms=stats["host_issue_ms"] - stats["host_wait_ms"]),
        step_ms_by_kind=by_kind, hbm_bound_steps=hbm, sweep=sweep, noswap_max_k=noswap_max_k, tuner=tuner, loss=loss,
        paper_context="AccUDNN on an NVIDIA M40 (Caffe + cuDNN): ResNet-152, 12 GB budget, k=54, 24 images/s "
                      "(Table 1); 8.3 GB at k=32 with 64% of maps offloaded (Sec. 6.3)")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
