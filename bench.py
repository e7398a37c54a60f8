#!/usr/bin/env python3
"""Benchmark of the hot path: ResNet-152 fp32 training steps under an 8 GiB device-memory
budget on one MI355X (benchmark configs[3]), synthetic ImageNet-shaped data.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--k auto|N] [--budget-gib 8]

Prints ONE JSON line.  `value` = images/s over exactly K timed steps at the headline
minibatch, inputs resident in HBM.  `roofline` prices the dominant convolution kernel
(by total time in a step) against the fp32 MFMA peak; `cpu_baseline` times the CPU oracle
on a bounded sample of the same workload.
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
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--k", default="auto", help="headline minibatch, or 'auto' = best of the sweep")
    ap.add_argument("--sweep", default="32,64,128,256", help="minibatch sizes of the sweep (configs[3])")
    ap.add_argument("--budget-gib", type=float, default=8.0)
    ap.add_argument("--net", default="resnet152", choices=["vgg16", "resnet18", "resnet34", "resnet50", "resnet101", "resnet152"])
    ap.add_argument("--mode", default="dynamic", choices=["dynamic", "naive", "none"])
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"],
                    help="storage of activations / gradients / kernel-side weights (bf16: configs[4])")
    ap.add_argument("--serial", action="store_true",
                    help="weight gradients on the compute stream instead of their own (every kernel runs alone: "
                         "the setting in which single kernels are timed)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-noswap-reference", action="store_true")
    ap.add_argument("--cpu-sample-k", type=int, default=12)
    return ap.parse_args()


# HBM bytes per launch of the dominant kernel (igemm_kernel<direct>), from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs of this script, scaled by what the same counters read for sgd_kernel
# (profiles/resnet152_k41_hbm_traffic_pmc.txt).  Known for the profiled workload only.
MEASURED_TRAFFIC_BYTES = {("resnet152", 41, 8.0): 71.2e6}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards by data parallelism, see DESIGN.md); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
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
    trainable, host_need = [], 256
    for k in sweep_ks:
        try:
            s = probe.plan_swaps(k, budget, B.PLAN_NAIVE_ALL)
            trainable.append(k)
            host_need = max(host_need, s["host_bytes"])
        except B.AccError as e:
            log(f"k={k}: not trainable under {args.budget_gib} GiB ({e})")
    lo, hi = 1, 4096
    while lo < hi:                                   # largest k that fits with nothing swapped
        mid = (lo + hi + 1) // 2
        try:
            probe.plan_swaps(mid, budget, B.PLAN_NONE)
            lo = mid
        except B.AccError:
            hi = mid - 1
    noswap_max_k = lo
    if args.k == "auto" and noswap_max_k not in trainable:
        trainable = sorted(trainable + [noswap_max_k])     # the largest minibatch that needs no swap
    probe.close()
    if not trainable:
        print("bench.py: no minibatch of the sweep is trainable under the budget", file=sys.stderr)
        sys.exit(1)

    torch.cuda.set_device(0)
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

    def batch(k, step):
        if (k, step) not in cache:
            img, lab = S.make_batch(net, k, step)
            cache[(k, step)] = (torch.from_numpy(img).cuda(), lab)
        return cache[(k, step)]

    def run(k, steps, warmup, first_step=0):
        imgs = [batch(k, first_step + i) for i in range(min(2, steps + warmup))]
        for i in range(warmup):
            ctx.train_step(*imgs[i % len(imgs)], 0.1)
        torch.cuda.synchronize()
        t = time.perf_counter()
        loss = 0.0
        for i in range(steps):
            loss = ctx.train_step(*imgs[i % len(imgs)], 0.1)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / steps, loss

    # ---- sweep (configs[3]): short runs, to find the throughput-optimal minibatch
    sweep = []
    for k in trainable:
        summ = ctx.plan_swaps(k, budget, mode)
        sec, loss = run(k, 3, 1)
        sweep.append(dict(k=k, images_per_s=k / sec, ms_per_step=sec * 1e3, n_swapped=summ["n_swapped"],
                          n_maps=summ["n_maps"], gib_swapped_each_way=summ["bytes_swapped"] / GiB,
                          peak_gib=summ["peak_bytes"] / GiB, predicted_ms=summ["t_iter"] * 1e3,
                          predicted_stall_ms=summ["t_stall"] * 1e3, plan_ms=summ["plan_ms"]))
        log("sweep", sweep[-1])
    best = max(sweep, key=lambda r: r["images_per_s"])
    k = best["k"] if args.k == "auto" else int(args.k)
    cache = {key: v for key, v in cache.items() if key[0] == k}

    # ---- headline: W warm-up steps, then exactly K timed steps
    summ = ctx.plan_swaps(k, budget, mode)
    sec, loss = run(k, args.steps, args.warmup)
    value = k / sec
    stats = ctx.stats()

    # ---- roofline of the dominant kernel: events directly around every convolution launch,
    # and per-step / per-copy times.  The library refuses event timing for plans that swap
    # more than 24 GiB per iteration; then the kernels are timed in the uncapped no-swap
    # context below (same kernels, same shapes) and the copies are not timed one by one.
    def profiled(c_):
        c_.set_profiling(3)
        c_.train_step(*batch(k, 0), 0.1)
        c_.train_step(*batch(k, 1), 0.1)
        r = (c_.kernel_profile(), c_.step_times_ms(), c_.stats())
        c_.set_profiling(0)
        return r

    timed_swaps = summ["host_bytes"] <= (24 << 30)
    if timed_swaps:
        kp, step_ms, pstats = profiled(ctx)
    names = [ctx.step_info(j)["name"] for j in range(ctx.step_count())]
    # bytes of the tensors every step reads and writes (the headline plan is the installed one)
    step_bytes = []
    for j in range(ctx.step_count()):
        reads, writes = ctx.step_io(j)
        step_bytes.append(sum(ctx.tensor_info(t)["bytes"] for t in set(reads) | set(writes)))
    ctx.close()
    del ctx
    torch.cuda.empty_cache()

    # ---- same minibatch with nothing swapped in an uncapped pool: what the swaps cost
    noswap = None
    sec0 = None
    if (not args.no_noswap_reference and summ["n_swapped"] > 0) or not timed_swaps:
        big = int(summ["noswap_peak_bytes"] * 1.02) + (64 << 20)
        ctx2 = B.Context(net.as_array(), chw, pool_bytes=big, host_bytes=256, dtype=dtype)
        ctx2.set_weights(S.init_params(net))
        if args.serial:
            ctx2.set_wgrad_overlap(False)
        ctx2.plan_swaps(k, big, B.PLAN_NONE)
        imgs = batch(k, 0)
        ctx2.train_step(*imgs, 0.1)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(5):
            ctx2.train_step(*imgs, 0.1)
        torch.cuda.synchronize()
        sec0 = (time.perf_counter() - t) / 5
        if not timed_swaps:
            kp, step_ms, _ = profiled(ctx2)
            pstats = dict(stats, d2h_ms=stats["bytes_out"] / cal["link"][0] * 1e3,
                          h2d_ms=stats["bytes_in"] / cal["link"][1] * 1e3)
        ctx2.close()
        del ctx2
        torch.cuda.empty_cache()

    dom = max(kp, key=lambda r: r["ms"])
    conv_flops = sum(r["flops"] for r in kp)
    conv_ms = sum(r["ms"] for r in kp)
    ach = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
    # bf16 mode: the forward / data-gradient kernel multiplies bf16 on the matrix cores (dense peak
    # 2.5 PFLOP/s); the weight-gradient kernel widens its operands and uses the fp32 instruction
    peak = 2500.0 if (args.dtype == "bf16" and dom["name"].startswith("igemm")) else PEAK_FP32_MFMA_TFLOPS
    roofline = dict(bound="mfma", kernel=dom["name"], achieved=ach, peak=peak, unit="TFLOP/s",
                    frac=ach / peak,
                    traffic=MEASURED_TRAFFIC_BYTES.get((args.net, k, args.budget_gib)) if args.dtype == "f32" else None, launches_per_step=dom["launches"],
                    avg_launch_us=dom["ms"] * 1e3 / dom["launches"],
                    flop_per_launch=dom["flops"] / dom["launches"],
                    timed_in=("two extra steps of the headline context" if timed_swaps else "the no-swap run of the same minibatch") +
                             ", weight gradients on the compute stream so that every kernel is timed alone")
    # step-level view: BN / pooling / update steps against the HBM roofline
    by_kind, bytes_by_kind = {}, {}
    for n_, ms, nb in zip(names, step_ms, step_bytes):
        by_kind[n_] = by_kind.get(n_, 0.0) + float(ms)
        bytes_by_kind[n_] = bytes_by_kind.get(n_, 0) + nb
    # batch norm (+ReLU, +add) against the HBM roofline: bytes of the tensors the steps touch
    # (each counted once per step, although backward reads x and dy twice) over their time
    hbm = {n_: dict(gb_per_step=bytes_by_kind[n_] / 1e9, ms_per_step=by_kind[n_],
                    gbs=bytes_by_kind[n_] / 1e9 / (by_kind[n_] * 1e-3), frac_of_hbm_peak=bytes_by_kind[n_] / 1e9 /
                    (by_kind[n_] * 1e-3) / 8000.0)
           for n_ in ("bn_fwd", "bn_bwd", "maxpool_fwd", "maxpool_bwd") if by_kind.get(n_, 0) > 0}
    conv = dict(tflops=conv_flops / (conv_ms * 1e-3) / 1e12, frac_of_mfma_peak=conv_flops / (conv_ms * 1e-3) / 1e12 /
                PEAK_FP32_MFMA_TFLOPS, ms_per_step=conv_ms, flops_per_step=conv_flops,
                kernels=[dict(name=r["name"], launches=r["launches"], ms=r["ms"],
                              tflops=r["flops"] / (r["ms"] * 1e-3) / 1e12) for r in kp])
    swap = dict(gib_out=pstats["bytes_out"] / GiB, gib_in=pstats["bytes_in"] / GiB,
                d2h_gbs=(pstats["bytes_out"] / 1e9) / (pstats["d2h_ms"] * 1e-3) if pstats["d2h_ms"] > 0 else None,
                h2d_gbs=(pstats["bytes_in"] / 1e9) / (pstats["h2d_ms"] * 1e-3) if pstats["h2d_ms"] > 0 else None,
                d2h_ms=pstats["d2h_ms"], h2d_ms=pstats["h2d_ms"],
                copy_times="events around every copy" if timed_swaps else "bytes / calibrated link rate")
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
        img, lab = S.make_batch(net, kc, 0)
        params = S.init_params(net)
        t = time.perf_counter()
        O.train_step(net.as_array(), chw, params, img, lab, 0.1)
        dt = time.perf_counter() - t
        cpu = dict(value=kc / dt, unit="images/s", cores=int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())),
                   kind="oracle", sample=f"one {args.net} training step at minibatch {kc} ({dt:.1f} s)")

    out = dict(
        metric="train images/s (ResNet-152 fp32, 8 GiB HBM budget) + conv MFMA utilisation" if (args.net, args.dtype, args.budget_gib) == ("resnet152", "f32", 8.0)
        else f"train images/s ({args.net} {args.dtype}, {args.budget_gib} GiB HBM budget) + conv MFMA utilisation",
        value=value, unit="images/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
        ms_per_step=sec * 1e3, higher_is_better=True, scaling="weak", vs_baseline=None, dtype=args.dtype,
        data="synthetic",
        config=dict(workload=f"{args.net} {'fp32' if args.dtype == 'f32' else 'bf16 (fp32 master weights and statistics)'} training step, 224x224x3 N(0,1) images, 1000 classes, "
                             f"minibatch {k}, device-memory budget {args.budget_gib} GiB, planner mode {args.mode}",
                    minibatch=k, budget_gib=args.budget_gib, strides="v1", optimizer="plain SGD lr 0.1",
                    wgrad_stream=not args.serial),
        roofline=roofline, cpu_baseline=cpu, conv=conv, swap=swap, noswap_reference=noswap,
        plan=dict(n_maps=summ["n_maps"], n_swapped=summ["n_swapped"], peak_gib=summ["peak_bytes"] / GiB,
                  layer_peak_gib=summ["layer_peak_bytes"] / GiB, noswap_peak_gib=summ["noswap_peak_bytes"] / GiB,
                  predicted_ms=summ["t_iter"] * 1e3, predicted_stall_ms=summ["t_stall"] * 1e3,
                  predicted_compute_ms=summ["t_compute"] * 1e3, plan_ms=summ["plan_ms"],
                  host_issue_ms=stats["host_issue_ms"]),
        step_ms_by_kind=by_kind, hbm_bound_steps=hbm, sweep=sweep, noswap_max_k=noswap_max_k, tuner=tuner, loss=loss,
        paper_context="AccUDNN on an NVIDIA M40 (Caffe + cuDNN): ResNet-152, 12 GB budget, k=54, 24 images/s "
                      "(Table 1); 8.3 GB at k=32 with 64% of maps offloaded (Sec. 6.3)")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
