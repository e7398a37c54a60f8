"""Checks of the performance model against the machine, in the manner of the paper's model
validation (Sec. 6.2: throughput against the minibatch per layer type, the predicted against
the observed course of one iteration, memory in use and bytes swapped over the iteration).

Everything here reads what the library already records (the calibration table, the plan, the
simulated and the observed timeline); nothing of the method is computed in Python.

    python -m paper_1901_06773_amd.validate --net resnet152 --k 64 --budget-gib 8
"""
import argparse
import json
import sys
from collections import defaultdict

import numpy as np

OP_LOAD, OP_COMPUTE, OP_OFFLOAD, OP_PREFETCH = 0, 1, 2, 3


# ----------------------------------------------------------------- throughput against k
def step_classes(ctx, net):
    """Class label of every step: convolutions by filter size and direction, the rest by kind."""
    out = []
    for j in range(ctx.step_count()):
        info = ctx.step_info(j)
        name = info["name"]
        if name.startswith("conv") and info["layer"] >= 0:
            l = net.layers[info["layer"]]
            name = f"{name}_{l.r}x{l.s}"
        out.append(name)
    return out


def throughput_curves(ctx, net):
    """From the calibration table: for every class of steps and every measured minibatch the
    summed time, and the rate it implies: TFLOP/s for the steps that have FLOPs (Eq. 1: linear
    in k), GB/s over the bytes of the tensors they read and write for the others."""
    cal = ctx.get_calibration()
    if not cal["ks"]:
        raise RuntimeError("calibrate first")
    k_plan = ctx.k
    classes = step_classes(ctx, net)
    flops_img, bytes_img = defaultdict(float), defaultdict(float)
    steps_of = defaultdict(list)
    for j, cls in enumerate(classes):
        info = ctx.step_info(j)
        steps_of[cls].append(j)
        flops_img[cls] += info["flops"] / k_plan
        reads, writes = ctx.step_io(j)
        bytes_img[cls] += sum(ctx.tensor_info(t)["bytes"] for t in set(reads) | set(writes)) / k_plan
    curves = {}
    for cls, steps in steps_of.items():
        rows = []
        for i, k in enumerate(cal["ks"]):
            sec = float(cal["seconds"][i, steps].sum())
            row = dict(k=k, ms=sec * 1e3)
            if flops_img[cls] > 0:
                row["tflops"] = flops_img[cls] * k / sec / 1e12
            else:
                row["gbs"] = bytes_img[cls] * k / sec / 1e9
            rows.append(row)
        curves[cls] = rows
    return curves


# ------------------------------------------------------------------ predicted vs observed
def _busy_overlap(intervals, busy):
    """Length of the part of `intervals` covered by the (sorted, disjoint) `busy` intervals."""
    total = 0.0
    starts = [b[0] for b in busy]
    for a0, a1 in intervals:
        i = max(0, int(np.searchsorted(starts, a0)) - 1)
        while i < len(busy) and busy[i][0] < a1:
            total += max(0.0, min(a1, busy[i][1]) - max(a0, busy[i][0]))
            i += 1
    return total


def timeline_summary(tl):
    """Iteration time, stall (idle time of the compute stream between its first and last step),
    copy time per direction and the fraction of it that runs while the compute stream is busy."""
    comp = [(e["t_start"], e["t_end"]) for e in tl if e["op"] == OP_COMPUTE]
    out = [(e["t_start"], e["t_end"]) for e in tl if e["op"] == OP_OFFLOAD]
    inn = [(e["t_start"], e["t_end"]) for e in tl if e["op"] == OP_PREFETCH]
    busy = sum(b - a for a, b in comp)
    span = comp[-1][1] - comp[0][0]
    copies = out + inn
    copy_s = sum(b - a for a, b in copies)
    return dict(t_iter=max(b for _, b in comp + copies) if copies else comp[-1][1], t_compute=busy, t_stall=span - busy,
                d2h_s=sum(b - a for a, b in out), h2d_s=sum(b - a for a, b in inn),
                copy_hidden_fraction=(_busy_overlap(copies, comp) / copy_s) if copy_s > 0 else None)


def dependency_violations(ctx, tl, slack=20e-6):
    """Instructions whose observed start precedes the observed end of something the plan makes
    them wait for (the step, offload or prefetch named by wait_step / wait_d2h / wait_h2d), or
    of the previous instruction on their own stream.  Empty when the streams and events of the
    executor order the work as planned.  slack: resolution of the event clock."""
    ins = ctx.instructions()
    end_step, end_d2h, end_h2d = {}, {}, {}
    last_on_stream = {}
    bad = []
    for i, (a, e) in enumerate(zip(ins, tl)):
        if e["t_start"] < 0:        # input loads carry no timing events
            continue
        deps = []
        if a["wait_step"] >= 0 and a["wait_step"] in end_step:
            deps.append(("step", a["wait_step"], end_step[a["wait_step"]]))
        if a["wait_d2h"] >= 0 and a["wait_d2h"] in end_d2h:
            deps.append(("offload", a["wait_d2h"], end_d2h[a["wait_d2h"]]))
        if a["wait_h2d"] >= 0 and a["wait_h2d"] in end_h2d:
            deps.append(("prefetch", a["wait_h2d"], end_h2d[a["wait_h2d"]]))
        stream = {OP_COMPUTE: "c", OP_OFFLOAD: "o", OP_PREFETCH: "i", OP_LOAD: "i"}[a["op"]]
        if stream in last_on_stream:
            deps.append(("stream", stream, last_on_stream[stream]))
        for what, which, t in deps:
            if e["t_start"] + slack < t:
                bad.append(dict(instr=i, op=a["op"], arg=a["arg"], waits_for=what, id=which,
                                early_by_us=(t - e["t_start"]) * 1e6))
        last_on_stream[stream] = e["t_end"]
        if a["op"] == OP_COMPUTE:
            end_step[a["arg"]] = e["t_end"]
        elif a["op"] == OP_OFFLOAD:
            end_d2h[a["seq"]] = e["t_end"]
        elif a["op"] == OP_PREFETCH:
            end_h2d[a["seq"]] = e["t_end"]
    return bad


def compare_timelines(ctx):
    """Predicted (Algorithm 1's simulation) against observed (events) for the installed plan."""
    pred, obs = ctx.timeline(False), ctx.timeline(True)
    ps, os_ = timeline_summary(pred), timeline_summary(obs)
    t0 = next(e["t_start"] for e in obs if e["op"] == OP_COMPUTE) - next(e["t_start"] for e in pred if e["op"] == OP_COMPUTE)
    dev = [abs((o["t_start"] - t0) - p["t_start"]) for p, o in zip(pred, obs) if p["op"] == OP_COMPUTE]
    dur = [((o["t_end"] - o["t_start"]), (p["t_end"] - p["t_start"])) for p, o in zip(pred, obs) if p["op"] == OP_COMPUTE]
    return dict(predicted=ps, observed=os_,
                start_deviation_ms=dict(mean=float(np.mean(dev)) * 1e3, max=float(np.max(dev)) * 1e3),
                step_time_error=dict(sum_abs_ms=float(sum(abs(a - b) for a, b in dur)) * 1e3),
                dependency_violations=dependency_violations(ctx, obs))


# ----------------------------------------------------------------------- memory over time
def memory_curve(ctx, observed=False, points=64):
    """Bytes of the pool in use and bytes moved out / in so far, sampled over the iteration.
    A tensor occupies the pool from the start of the instruction that writes it first (its
    producing step, the input load or its prefetch) to the end of its last use; a swapped
    map leaves when both its offload and its last forward use are done, and returns with its
    prefetch."""
    tl = ctx.timeline(observed)
    ins = ctx.instructions()
    step_t = {}
    off_t, pre_t = {}, {}
    load_t = {}
    for a, e in zip(ins, tl):
        if a["op"] == OP_COMPUTE:
            step_t[a["arg"]] = (e["t_start"], e["t_end"])
        elif a["op"] == OP_OFFLOAD:
            off_t[a["arg"]] = (e["t_start"], e["t_end"], e["bytes"])
        elif a["op"] == OP_PREFETCH:
            pre_t[a["arg"]] = (e["t_start"], e["t_end"], e["bytes"])
        else:
            load_t[a["arg"]] = (max(e["t_start"], 0.0), max(e["t_end"], 0.0))
    events = []            # (time, delta bytes in pool)
    for t in range(ctx.tensor_count()):
        ti = ctx.tensor_info(t)
        if ti["bytes"] == 0 or ti["producer_step"] < 0 and t not in load_t:
            continue
        born = load_t[t][0] if t in load_t else step_t[ti["producer_step"]][0]
        last = step_t[ti["last_step"]][1]
        if ti["swapped"] and t in off_t and t in pre_t:
            gone = max(off_t[t][1], step_t[ti["last_fwd_step"]][1])
            events += [(born, ti["bytes"]), (gone, -ti["bytes"]), (pre_t[t][0], ti["bytes"]), (last, -ti["bytes"])]
        else:
            events += [(born, ti["bytes"]), (last, -ti["bytes"])]
    events.sort()
    t_end = max(e["t_end"] for e in tl)
    grid = np.linspace(0.0, t_end, points)
    times = np.array([e[0] for e in events])
    cum = np.cumsum([e[1] for e in events])
    outs = sorted((v[1], v[2]) for v in off_t.values())
    inns = sorted((v[1], v[2]) for v in pre_t.values())

    def moved(series, t):
        return int(sum(b for te, b in series if te <= t))
    rows = []
    for t in grid:
        i = int(np.searchsorted(times, t, side="right")) - 1
        rows.append(dict(t_ms=float(t) * 1e3, pool_bytes=int(cum[i]) if i >= 0 else 0,
                         bytes_out=moved(outs, t), bytes_in=moved(inns, t)))
    return dict(peak_dynamic_bytes=int(cum.max()) if len(cum) else 0, series=rows)


# --------------------------------------------------------------------------------- report
def format_report(rep):
    lines = [f"{rep['net']} at minibatch {rep['k']}, budget {rep['budget_gib']} GiB: "
             f"{rep['plan']['n_swapped']} of {rep['plan']['n_maps']} maps swapped, "
             f"{rep['plan']['bytes_swapped'] / 2**30:.2f} GiB each way", ""]
    lines.append("Throughput against the minibatch, per class of steps (calibration table):")
    ks = [r["k"] for r in next(iter(rep["throughput"].values()))]
    lines.append(f"  {'class':22s}" + "".join(f"{'k=' + str(k):>10s}" for k in ks) + "   unit")
    for cls, rows in rep["throughput"].items():
        unit = "TFLOP/s" if "tflops" in rows[0] else "GB/s"
        vals = [r.get("tflops", r.get("gbs")) for r in rows]
        if sum(r["ms"] for r in rows) < 0.05 * len(rows) or not any(vals):
            continue                                  # under 50 us per iteration (noise), or no rate defined
        lines.append(f"  {cls:22s}" + "".join(f"{v:10.1f}" for v in vals) + f"   {unit}")
    c = rep["timeline"]
    lines += ["", "One iteration, predicted by the simulation of the plan against observed with events:",
              f"  {'':24s}{'predicted':>12s}{'observed':>12s}"]
    for key, label, scale in (("t_iter", "iteration ms", 1e3), ("t_compute", "compute ms", 1e3), ("t_stall", "stall ms", 1e3),
                              ("d2h_s", "offload copies ms", 1e3), ("h2d_s", "prefetch copies ms", 1e3),
                              ("copy_hidden_fraction", "copies under compute", 1.0)):
        p, o = c["predicted"][key], c["observed"][key]
        fmt = (lambda v: f"{v * scale:12.2f}") if p is not None and o is not None else (lambda v: f"{'-':>12s}")
        lines.append(f"  {label:24s}{fmt(p)}{fmt(o)}")
    lines.append(f"  start of a step, observed against predicted: mean |dev| {c['start_deviation_ms']['mean']:.2f} ms, "
                 f"max {c['start_deviation_ms']['max']:.2f} ms")
    lines.append(f"  instructions that started before something they wait for had ended: {len(c['dependency_violations'])}")
    lines += ["", "Memory over the iteration (observed times): pool bytes in use above the resident weights, bytes moved so far",
              f"  {'t ms':>8s}{'pool GiB':>10s}{'out GiB':>10s}{'in GiB':>10s}"]
    for r in rep["memory_observed"]["series"][::4]:
        lines.append(f"  {r['t_ms']:8.1f}{r['pool_bytes'] / 2**30:10.2f}{r['bytes_out'] / 2**30:10.2f}{r['bytes_in'] / 2**30:10.2f}")
    lines.append(f"  peak: {rep['memory_observed']['peak_dynamic_bytes'] / 2**30:.2f} GiB observed order, "
                 f"{rep['memory_predicted']['peak_dynamic_bytes'] / 2**30:.2f} GiB predicted order, "
                 f"{(rep['plan']['peak_bytes'] - rep['plan']['static_bytes']) / 2**30:.2f} GiB the planner's sum of live bytes "
                 f"(a map being copied out is no longer in that sum)")
    return "\n".join(lines)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--net", default="resnet152")
    ap.add_argument("--k", type=int, default=64)
    ap.add_argument("--budget-gib", type=float, default=8.0)
    ap.add_argument("--curve-ks", default="8,16,32", help="further minibatches for the throughput curves")
    ap.add_argument("--json", default="", help="write the full report here")
    args = ap.parse_args(argv)
    import torch
    import synth as S
    from . import binding as B
    net = getattr(S, args.net)()
    chw = (net.in_c, net.in_h, net.in_w)
    budget = int(args.budget_gib * 2**30)
    probe = B.Context(net.as_array(), chw)
    host = probe.plan_swaps(args.k, budget, B.PLAN_NAIVE_ALL)["host_bytes"]
    probe.close()
    torch.cuda.set_device(0)
    ctx = B.Context(net.as_array(), chw, pool_bytes=budget, host_bytes=host + (64 << 20))
    ctx.set_weights(S.init_params(net))
    ks = sorted(set([int(x) for x in args.curve_ks.split(",") if x] + [args.k]))
    # per-class rates: every step alone on the compute stream (with the weight gradients on their
    # own stream a conv backward step's time on the compute stream covers only its data gradient)
    ctx.set_wgrad_overlap(False)
    ctx.calibrate(ks)
    ctx.plan_swaps(args.k, budget, B.PLAN_DYNAMIC)
    curves = throughput_curves(ctx, net)
    # the plan and its prediction: step times as the run will see them
    ctx.set_wgrad_overlap(True)
    ctx.calibrate(ks)
    plan = ctx.plan_swaps(args.k, budget, B.PLAN_DYNAMIC)
    img, lab = S.make_batch(net, args.k, 0)
    img = torch.from_numpy(img).cuda()
    for _ in range(2):
        ctx.train_step(img, lab, 0.1)
    ctx.set_profiling(1)
    ctx.train_step(img, lab, 0.1)
    ctx.set_profiling(0)
    rep = dict(net=args.net, k=args.k, budget_gib=args.budget_gib, plan=plan, throughput=curves,
               timeline=compare_timelines(ctx), memory_predicted=memory_curve(ctx, False),
               memory_observed=memory_curve(ctx, True))
    print(format_report(rep))
    if args.json:
        with open(args.json, "w") as f:
            json.dump(rep, f, indent=1)
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
