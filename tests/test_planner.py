"""CPU tests of the static analyzer, the performance model, Algorithm 1 / Eq. 4 / Eq. 6 and
the pin-back strategy (body of Algorithm 2), through planning-only contexts of the C ABI.

Pins: figures published for the ResNets (He et al., Table 1: 3.8 / 7.6 / 11.3 x 10^9
multiply-adds), exact linearity in the minibatch (Eq. 1), closed forms of Algorithm 1 on a
chain of identical layers, an independent plain-Python checker of every plan (oracle/
plan_check.py: memory model, data residency, happens-before over streams and events, timing
recurrences) and brute force over all swap sets of toy networks."""
import itertools
import os
import re

import numpy as np
import pytest

import synth as S
from oracle import plan_check as PC

MiB, GiB = 1 << 20, 1 << 30


def B():
    from paper_1901_06773_amd import binding
    return binding


def ctx_of(net):
    return B().Context(net.as_array(), (net.in_c, net.in_h, net.in_w))


def chain(n_units=6, c=32, hw=8, classes=8):
    """conv1x1(c->c) -> BN -> ReLU, n_units times, at constant resolution: every feature
    map that survives into backward has the same size."""
    net = S.NetSpec(f"chain{n_units}", c, hw, hw, classes)
    x = -1
    for _ in range(n_units):
        x = net.add(S.Layer(S.CONV, in0=x, cin=c, cout=c, r=1, s=1, stride=1, pad=0))
        x = net.add(S.Layer(S.BN, in0=x, cin=c, cout=c))
        x = net.add(S.Layer(S.RELU, in0=x, cin=c, cout=c))
    g = net.add(S.Layer(S.GAP, in0=x, cin=c, cout=c))
    f = net.add(S.Layer(S.FC, in0=g, cin=c, cout=classes))
    net.add(S.Layer(S.SOFTMAX_CE, in0=f, cin=classes, cout=1))
    return net


# ------------------------------------------------------------------ ABI surface
def test_library_exports_every_declared_symbol():
    b = B()
    hdr = open(os.path.join(os.path.dirname(__file__), "..", "include", "accudnn.h")).read()
    declared = set(re.findall(r"\b(acc_[a-z0-9_]+)\s*\(", hdr))
    assert len(declared) >= 30
    for name in declared:
        assert hasattr(b.lib(), name), f"{name} is declared in accudnn.h but not exported"
    assert declared == set(b.EXPORTED_SYMBOLS), declared ^ set(b.EXPORTED_SYMBOLS)


def test_single_operations_refuse_bad_arguments_before_any_launch():
    """Every acc_op_* call checks its arguments on the host and returns ACC_EINVAL without launching anything:
    null and misaligned pointers, an unknown storage type, shapes the kernels do not take, sizes beyond
    their 32-bit index ranges.  (No GPU is needed for a call that must not reach one; the pointers are
    made-up addresses that nothing dereferences.)"""
    b = B()
    L = b.lib()
    P, Q, R = 0x10000, 0x20000, 0x30000          # 16-byte aligned, never dereferenced
    E = b.ACC_EINVAL
    conv = lambda x=P, w=Q, y=R, n=2, h=8, wd=8, cin=32, cout=32, r=3, s=3, st=1, pad=1, dt=b.F32: \
        L.acc_op_conv_fwd(x, w, y, n, h, wd, cin, cout, r, s, st, pad, dt, None)
    assert conv(x=None) == E and conv(w=None) == E and conv(y=None) == E
    assert conv(x=P + 8) == E                    # 16 bytes at a time
    assert conv(dt=7) == E
    assert conv(s=1) == E                        # square filters only
    assert conv(pad=3) == E and conv(st=0) == E and conv(n=0) == E and conv(h=1, wd=1, pad=0) == E
    assert conv(n=65536, h=256, wd=256) == E     # 2^32 output positions: beyond the kernels' row index
    assert L.acc_op_conv_dgrad(P, Q, R, 2, 8, 8, 32, 32, 3, 3, 1, 1, 0, None, 0, b.F32, None) == E   # needs its workspace
    assert L.acc_op_conv_wgrad(P, Q, R + 4, 2, 8, 8, 32, 32, 3, 3, 1, 1, None, 0, b.F32, None) == E
    bn = lambda x=P, rows=64, c=32, ws=R, dt=b.F32: L.acc_op_bn_fwd(x, Q, Q, None, P, Q, Q, rows, c, 1, 1e-5, ws, dt, None)
    assert bn(x=None) == E and bn(ws=None) == E and bn(rows=0) == E and bn(c=30) == E and bn(dt=-1) == E
    assert L.acc_op_bn_bwd(P, Q, None, Q, Q, Q, P, Q, Q, None, 64, 6, R, b.F32, None) == E
    assert L.acc_op_bn_fwd_noalloc(P, Q, Q, None, P, Q, Q, 64, 2048 + 4, 1, 1e-5, b.F32, None) == E
    assert b"ACC_NOALLOC_BN_MAX_C" in L.acc_last_error(None)
    pool = lambda x=P, c=8, r=3, st=2, pad=1, dt=b.F32: L.acc_op_maxpool_fwd(x, Q, 2, 8, 8, c, r, st, pad, dt, None)
    assert pool(x=None) == E and pool(c=6) == E and pool(pad=3) == E and pool(st=0) == E and pool(dt=9) == E
    assert L.acc_op_maxpool_bwd(P, None, R, 2, 8, 8, 8, 3, 2, 1, 0, b.F32, None) == E
    assert L.acc_op_gap_fwd(P, None, 2, 49, 64, b.F32, None) == E and L.acc_op_gap_fwd(P, Q, 2, 0, 64, b.F32, None) == E
    assert L.acc_op_gap_bwd(None, Q, 2, 49, 64, 0, b.F32, None) == E
    assert L.acc_op_softmax_ce(P, Q, None, None, None, 4, 10, b.F32, None) == E       # nothing asked for
    assert L.acc_op_softmax_ce(P, Q, R, None, None, 4, 10, b.F32, None) == E          # rows without the mean
    assert L.acc_op_softmax_ce(P, None, R, R, None, 4, 10, b.F32, None) == E
    assert L.acc_op_softmax_ce(P, Q, R, R, None, 0, 10, b.F32, None) == E


def test_execution_without_resources_fails_loudly():
    b = B()
    net = S.bottleneck_unit()
    ctx = ctx_of(net)
    with pytest.raises(b.AccError) as e:
        ctx.set_weights(S.init_params(net))
    assert e.value.status == b.ACC_ESTATE
    with pytest.raises(b.AccError) as e:
        ctx.calibrate([2])
    assert e.value.status == b.ACC_ESTATE


def test_malformed_networks_are_rejected():
    b = B()
    net = S.bottleneck_unit()
    arr = net.as_array().copy()
    arr[0, 3] = 63                                     # conv cin does not match its input
    with pytest.raises(b.AccError) as e:
        b.Context(arr, (64, 16, 16))
    assert e.value.status == b.ACC_EINVAL
    arr = net.as_array().copy()
    arr[-1, 0] = S.GAP                                 # no loss at the end
    with pytest.raises(b.AccError):
        b.Context(arr, (64, 16, 16))
    ctx_of(S.resnet((1, 1), in_hw=32, width=8, variant="v1.5"))      # strided 3x3 with a data gradient: fine
    # a 3x3 convolution with stride 4 and padding 2 would need a negatively padded part
    net = S.NetSpec("odd_stride", 8, 16, 16, 10)
    a = net.add(S.Layer(S.CONV, in0=-1, cin=8, cout=8, r=1, s=1, stride=1, pad=0))
    a = net.add(S.Layer(S.BN, in0=a, cin=8, cout=8))
    a = net.add(S.Layer(S.RELU, in0=a, cin=8, cout=8))
    a = net.add(S.Layer(S.CONV, in0=a, cin=8, cout=8, r=3, s=3, stride=4, pad=2))
    a = net.add(S.Layer(S.BN, in0=a, cin=8, cout=8))
    a = net.add(S.Layer(S.RELU, in0=a, cin=8, cout=8))
    a = net.add(S.Layer(S.GAP, in0=a, cin=8, cout=8))
    a = net.add(S.Layer(S.FC, in0=a, cin=8, cout=10))
    net.add(S.Layer(S.SOFTMAX_CE, in0=a, cin=10, cout=1))
    with pytest.raises(b.AccError) as e:
        ctx_of(net)
    assert "strided" in str(e.value)


# ------------------------------------------------------------ static information
def published():
    out = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "published_figures.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


PUB = published()


def test_memory_stays_under_the_figures_the_paper_prints_for_caffe():
    """Sec. 6.3 A: ResNet-152 at minibatch 32 takes more than 24 GB resident and 2.5 GB with
    every map swapped in the paper's Caffe; the fused step here must need less of both, and
    the same order of reduction (network-wide to layer-wide)."""
    b = B()
    ctx = ctx_of(S.resnet152())
    s = ctx.plan_swaps(32, 1 << 40, b.PLAN_NAIVE_ALL)
    assert s["noswap_peak_bytes"] < PUB["resnet152_k32_resident_gb_upper"] * 1e9
    assert s["layer_peak_bytes"] < PUB["resnet152_k32_layerwise_gb_upper"] * 1e9
    assert s["noswap_peak_bytes"] > 4 * s["layer_peak_bytes"]
    # the retention set, counted here from the layer records alone: inputs of conv / fc / bn /
    # max-pool / loss (needed again in backward) and ReLU outputs (their own mask)
    net = S.resnet152()
    shape, kept = {}, set()
    for i, l in enumerate(net.layers):
        c, h, w = (net.in_c, net.in_h, net.in_w) if l.in0 < 0 else shape[l.in0]
        if l.kind in (S.CONV, S.MAXPOOL):
            h, w = (h + 2 * l.pad - l.r) // l.stride + 1, (w + 2 * l.pad - l.s) // l.stride + 1
            c = l.cout if l.kind == S.CONV else c
        elif l.kind == S.GAP:
            h = w = 1
        elif l.kind == S.FC:
            c, h, w = l.cout, 1, 1
        shape[i] = (c, h, w)
        if l.kind in (S.CONV, S.FC, S.BN, S.MAXPOOL, S.SOFTMAX_CE):
            kept.add(l.in0)
        if l.kind == S.RELU:
            kept.add(i)
    per_image = sum(4 * np.prod((net.in_c, net.in_h, net.in_w) if t < 0 else shape[t]) for t in kept)
    assert s["n_maps"] == len(kept) == 310
    assert s["bytes_maps"] == 32 * per_image == 32 * 171_614_112


@pytest.mark.parametrize("name,gmacs", [("resnet18", PUB["resnet18_gmacs"]), ("resnet34", PUB["resnet34_gmacs"]),
                                        ("resnet50", PUB["resnet50_gmacs"]), ("resnet101", PUB["resnet101_gmacs"]),
                                        ("resnet152", PUB["resnet152_gmacs"])])
def test_flops_match_the_published_multiply_adds(name, gmacs):
    """Forward multiply-adds per 224x224 image (convolutions and the FC layer)."""
    b = B()
    ctx = ctx_of(getattr(S, name)())
    ctx.plan_swaps(1, 1 << 40, b.PLAN_NONE)
    fwd = sum(ctx.step_info(j)["flops"] for j in range(ctx.step_count()) if ctx.step_info(j)["backward"] == 0)
    assert abs(fwd / 2 / 1e9 - gmacs) < 0.1
    # backward does twice the forward work, minus the data gradient of the stem
    bwd = sum(ctx.step_info(j)["flops"] for j in range(ctx.step_count()) if ctx.step_info(j)["backward"] == 1)
    stem = 2 * 112 * 112 * 64 * 3 * 49
    assert bwd == pytest.approx(2 * fwd - stem, rel=1e-12)


def test_vgg16_flops_and_maps():
    """VGG-16 (conv + bias + ReLU fused into one step each, FC over the flattened 7x7x512 map):
    forward multiply-adds within 2 % of the published 15.3 G (convolutions 15.35 G and the three
    FC layers 0.12 G), backward twice that minus the first layer's data gradient; the maps kept
    for backward are the image, the 13 ReLU outputs, the 5 pooled maps, the 2 hidden FC outputs
    and the logits."""
    b = B()
    ctx = ctx_of(S.vgg16())
    k = 64                      # (every map a whole number of 256-byte units)
    s = ctx.plan_swaps(k, 1 << 40, b.PLAN_NONE)
    fwd = sum(ctx.step_info(j)["flops"] for j in range(ctx.step_count()) if ctx.step_info(j)["backward"] == 0) / k
    assert fwd / 2 / 1e9 == pytest.approx(PUB["vgg16_gmacs"], rel=0.02)
    bwd = sum(ctx.step_info(j)["flops"] for j in range(ctx.step_count()) if ctx.step_info(j)["backward"] == 1) / k
    assert bwd == pytest.approx(2 * fwd - 2 * 224 * 224 * 64 * 3 * 9, rel=1e-12)
    assert s["n_maps"] == 1 + 13 + 5 + 2 + 1
    per_image = 4 * (3 * 224 * 224 + 2 * 64 * 224 ** 2 + 2 * 128 * 112 ** 2 + 3 * 256 * 56 ** 2 + 3 * 512 * 28 ** 2 +
                     3 * 512 * 14 ** 2 + 64 * 112 ** 2 + 128 * 56 ** 2 + 256 * 28 ** 2 + 512 * 14 ** 2 + 512 * 7 ** 2 + 2 * 4096 + 1000)
    assert s["bytes_maps"] == k * per_image


def test_sizes_and_flops_are_linear_in_the_minibatch():
    """Eq. 1 and static information 2: feature-map bytes and FLOPs scale with k exactly."""
    b = B()
    ctx = ctx_of(S.resnet50())
    ctx.plan_swaps(4, 1 << 40, b.PLAN_NONE)
    t4 = [ctx.tensor_info(t) for t in range(ctx.tensor_count())]
    f4 = [ctx.step_info(j)["flops"] for j in range(ctx.step_count())]
    s4 = ctx.plan_swaps(4, 1 << 40, b.PLAN_NONE)
    ctx.plan_swaps(12, 1 << 40, b.PLAN_NONE)
    t12 = [ctx.tensor_info(t) for t in range(ctx.tensor_count())]
    f12 = [ctx.step_info(j)["flops"] for j in range(ctx.step_count())]
    s12 = ctx.plan_swaps(12, 1 << 40, b.PLAN_NONE)
    for a, c in zip(t4, t12):
        if a["is_map"]:      # exact up to the 256-byte rounding of each object
            assert abs(c["bytes"] - 3 * a["bytes"]) < 3 * 256
            if a["bytes"] % (256 * 4) == 0:
                assert c["bytes"] == 3 * a["bytes"]
    assert all(c == 3 * a for a, c in zip(f4, f12))
    assert abs(s12["bytes_maps"] - 3 * s4["bytes_maps"]) < 3 * 256 * s4["n_maps"]
    # retention set of ResNet-50: every conv input and every BN input, fp32
    assert s4["bytes_maps"] / 4 / MiB == pytest.approx(76.9, abs=1.0)


def test_gmap_lifetimes_are_consistent():
    b = B()
    net = S.resnet((1, 1), in_hw=32, width=8, classes=10)
    ctx = ctx_of(net)
    ctx.plan_swaps(2, 1 << 40, b.PLAN_NONE)
    ns = ctx.step_count()
    first, last = {}, {}
    for j in range(ns):
        r, w = ctx.step_io(j)
        for t in r + w:
            first.setdefault(t, j)
            last[t] = j
        for t in r:
            assert first[t] < j or t in (0, 1), f"step {j} reads tensor {t} before anything wrote it"
    for t in range(ctx.tensor_count()):
        info = ctx.tensor_info(t)
        assert info["last_step"] == last[t]
        if info["is_map"]:
            assert info["last_fwd_step"] < info["first_bwd_step"]


# ------------------------------------------------- every plan is a valid plan
CASES = [
    ("config1", lambda: S.bottleneck_unit(), 2),
    ("mini_w8", lambda: S.resnet((1, 2), in_hw=32, classes=10, width=8), 3),
    ("mini_w32", lambda: S.resnet((1, 1, 2, 1), in_hw=64, classes=100, width=32), 5),
    ("chain", lambda: chain(), 4),
]


@pytest.mark.parametrize("name,make,k", CASES)
def test_plans_pass_the_independent_checker(name, make, k):
    b = B()
    net = make()
    ctx = ctx_of(net)
    s0 = ctx.plan_swaps(k, 1 << 40, b.PLAN_NAIVE_ALL)
    lo, hi, stat = s0["layer_peak_bytes"], s0["noswap_peak_bytes"], s0["static_bytes"]
    plans = [(b.PLAN_NONE, int(hi * 1.05)), (b.PLAN_NAIVE_ALL, int(lo * 1.15) + 65536), (b.PLAN_NAIVE_ALL, hi)]
    plans += [(b.PLAN_DYNAMIC, int(lo + f * (hi - lo))) for f in (0.2, 0.3, 0.5, 0.7, 0.9, 1.2)]
    for mode, budget in plans:
        s = ctx.plan_swaps(k, budget, mode)
        res = PC.check_plan(PC.gather(ctx), budget, stat)
        assert res["n_swapped"] == s["n_swapped"]
        # the checker counts an object from its first use, the planner from its (possibly
        # earlier) allocation
        assert stat + res["peak_dynamic_bytes"] <= s["peak_bytes"] <= budget
        if mode == b.PLAN_NAIVE_ALL:
            assert s["n_swapped"] == s["n_maps"]
        if mode == b.PLAN_NONE:
            assert s["n_swapped"] == 0
            assert stat + res["peak_dynamic_bytes"] == s["peak_bytes"] == s["noswap_peak_bytes"]
    # random explicit swap sets
    rng = np.random.default_rng(1)
    for _ in range(5):
        mask = rng.integers(0, 2, s0["n_maps"])
        ctx.plan_explicit(k, int(hi * 1.05), list(mask))
        PC.check_plan(PC.gather(ctx), int(hi * 1.05), stat)


def test_resnet50_plans_pass_the_checker():
    b = B()
    net = S.resnet50()
    ctx = ctx_of(net)
    for k, budget in ((32, 2 * GiB), (64, 4 * GiB)):
        s = ctx.plan_swaps(k, budget, b.PLAN_DYNAMIC)
        res = PC.check_plan(PC.gather(ctx), budget, s["static_bytes"])
        assert 0 < res["n_swapped"] == s["n_swapped"] < s["n_maps"]
        assert s["peak_bytes"] <= budget


def test_checker_detects_planted_mistakes():
    """The checker itself is pinned: a dropped wait, a wrong offset and a missing prefetch,
    planted in a copy of a good plan, must each be reported."""
    b = B()
    net = S.resnet((1, 2), in_hw=32, classes=10, width=8)
    ctx = ctx_of(net)
    s0 = ctx.plan_swaps(3, 1 << 40, b.PLAN_NAIVE_ALL)
    budget = int(s0["layer_peak_bytes"] * 1.15) + 65536
    s = ctx.plan_swaps(3, budget, b.PLAN_NAIVE_ALL)
    good = PC.gather(ctx)
    PC.check_plan(good, budget, s["static_bytes"])
    import copy
    # (1) drop every wait of the prefetches: they now race with the previous occupants
    bad = copy.deepcopy(good)
    for ins in bad["instrs"]:
        if ins["op"] == PC.PREFETCH:
            ins["wait_step"] = ins["wait_d2h"] = -1
    with pytest.raises(PC.PlanError):
        PC.check_plan(bad, budget, s["static_bytes"])
    # (2) a compute step that no longer waits for its prefetched input
    bad = copy.deepcopy(good)
    for ins in bad["instrs"]:
        if ins["op"] == PC.COMPUTE:
            ins["wait_h2d"] = -1
    with pytest.raises(PC.PlanError):
        PC.check_plan(bad, budget, s["static_bytes"])
    # (3) two live tensors on the same bytes
    bad = copy.deepcopy(good)
    maps = [t for t, info in enumerate(bad["tensors"]) if info["is_map"]]
    bad["tensors"][maps[3]]["offset"] = bad["tensors"][maps[2]]["offset"]
    with pytest.raises(PC.PlanError):
        PC.check_plan(bad, budget, s["static_bytes"])
    # (4) a prefetch removed
    bad = copy.deepcopy(good)
    bad["instrs"] = [i for n, i in enumerate(bad["instrs"]) if not (i["op"] == PC.PREFETCH and i["seq"] == 5)]
    with pytest.raises(PC.PlanError):
        PC.check_plan(bad, budget, s["static_bytes"])


# ------------------------------------------- Algorithm 1: closed forms and replay
def test_simulated_times_equal_the_independent_replay():
    b = B()
    net = S.resnet((1, 1, 2, 1), in_hw=64, classes=100, width=32)
    ctx = ctx_of(net)
    flops_s, bytes_s, launch, d2h, h2d, lat = 40e12, 2e12, 5e-6, 20e9, 25e9, 8e-6
    ctx.set_cost_model(flops_s, bytes_s, launch, d2h, h2d, lat)
    s0 = ctx.plan_swaps(5, 1 << 40, b.PLAN_NAIVE_ALL)
    for frac in (0.2, 0.6):
        budget = int(s0["layer_peak_bytes"] + frac * (s0["noswap_peak_bytes"] - s0["layer_peak_bytes"]))
        s = ctx.plan_swaps(5, budget, b.PLAN_DYNAMIC)
        plan = PC.gather(ctx)
        cost = [st["t_compute"] for st in plan["steps"]]
        rep = PC.replay_times(plan, cost, d2h, h2d, lat)
        assert rep["t_iter"] == pytest.approx(s["t_iter"], rel=1e-12)
        assert rep["t_stall"] == pytest.approx(s["t_stall"], rel=1e-9, abs=1e-12)
        for j, st in enumerate(plan["steps"]):
            assert rep["t_ready"][j] == pytest.approx(st["t_ready"], abs=1e-12)
            assert rep["t_end"][j] == pytest.approx(st["t_end"], abs=1e-12)
        assert sum(cost) == pytest.approx(s["t_compute"], rel=1e-12)          # Eq. 2


def _chain_setup(c_time, p_time, budget_factor):
    """Chain of identical units, every step costs c_time, every map copy p_time."""
    b = B()
    net = chain(n_units=6, c=32, hw=8)
    ctx = ctx_of(net)
    k = 4
    map_bytes = k * 32 * 8 * 8 * 4
    ctx.set_cost_model(1e30, 1e30, 0.0, map_bytes / p_time, map_bytes / p_time, 0.0)
    ctx.set_step_times([c_time] * ctx.step_count())
    s0 = ctx.plan_swaps(k, 1 << 40, b.PLAN_NAIVE_ALL)
    return b, ctx, k, s0, map_bytes


def test_algorithm1_unlimited_memory_prefetch_chain():
    """With memory to spare the swap-in stream never waits for a release: prefetches run
    back to back, so the q-th map needed in backward is ready p after the (q-1)-th
    (t_ready accumulates the transfer times), and backward runs without stall iff p <= c."""
    for c_time, p_time in ((1e-3, 0.5e-3), (1e-3, 2e-3)):
        b, ctx, k, s0, map_bytes = _chain_setup(c_time, p_time, None)
        s = ctx.plan_explicit(k, 1 << 40, [1] * s0["n_maps"])
        plan = PC.gather(ctx)
        PC.check_plan(plan, 1 << 40, s["static_bytes"])
        pre = [i for i in plan["instrs"] if i["op"] == PC.PREFETCH]
        big = [i for i in pre if plan["tensors"][i["arg"]]["bytes"] == map_bytes]
        rep = PC.replay_times(plan, [c_time] * ctx.step_count(), map_bytes / p_time, map_bytes / p_time, 0.0)
        # consecutive equal-size prefetches complete exactly p apart once the link is the bottleneck
        n_fwd = sum(1 for st in plan["steps"] if st["backward"] == 0)
        bwd_ready = [plan["steps"][j]["t_ready"] for j in range(n_fwd, ctx.step_count())]
        assert all(b2 >= a for a, b2 in zip(bwd_ready, bwd_ready[1:]))          # monotone
        stall_bwd = sum(max(0.0, plan["steps"][j]["t_start"] - plan["steps"][j - 1]["t_end"])
                        for j in range(n_fwd + 1, ctx.step_count()))
        if p_time <= c_time:
            assert stall_bwd == pytest.approx(0.0, abs=1e-12)        # Eq. 6 holds in backward
        else:
            # link-bound: the last backward step that needs a map ends no earlier than all
            # the copies, which run back to back at p each
            assert s["t_iter"] >= len(big) * p_time
            assert stall_bwd > 0
        assert rep["t_iter"] == pytest.approx(s["t_iter"], rel=1e-12)


def test_algorithm1_one_map_of_room_serialises():
    """With room for the active area only, a prefetch can start only after the step that
    releases memory has finished, so compute and transfer alternate: every backward step
    that needs a swapped map pays its full transfer time (Algorithm 1, third branch)."""
    c_time, p_time = 1e-3, 3e-3
    b, ctx, k, s0, map_bytes = _chain_setup(c_time, p_time, None)
    # the layer-wise peak plus the little that first fit needs on top of the sum of the live
    # bytes (5 % here: the peak is 23 maps' worth, most of it weight-gradient workspace)
    s = None
    for extra in (4096, map_bytes // 4, map_bytes // 2, 3 * map_bytes // 4, map_bytes, 5 * map_bytes // 4):
        tight = s0["layer_peak_bytes"] + extra
        try:
            s = ctx.plan_swaps(k, tight, b.PLAN_NAIVE_ALL)
            break
        except b.AccError:
            continue
    assert s is not None, "the active area plus one and a quarter maps must be enough"
    plan = PC.gather(ctx)
    PC.check_plan(plan, tight, s["static_bytes"])
    n_pref = sum(1 for i in plan["instrs"] if i["op"] == PC.PREFETCH and plan["tensors"][i["arg"]]["bytes"] == map_bytes)
    roomy = ctx.plan_swaps(k, 1 << 40, b.PLAN_NAIVE_ALL)
    # the tight plan cannot be faster than the roomy one, and exposes at least the transfer
    # time that exceeds the compute time of the steps in between
    assert s["t_iter"] >= roomy["t_iter"] - 1e-12
    assert s["t_stall"] >= n_pref * (p_time - 2 * c_time) - 1e-9


# ------------------------------------------------------- Algorithm 2 (body)
def test_no_swap_when_everything_fits_and_untrainable_below_the_layer_peak():
    b = B()
    net = S.resnet50()
    ctx = ctx_of(net)
    s = ctx.plan_swaps(32, 64 * GiB, b.PLAN_DYNAMIC)          # BASELINE configs[1]: zero swaps
    assert s["n_swapped"] == 0 and s["bytes_swapped"] == 0 and s["t_stall"] < 1e-3
    lo = ctx.plan_swaps(32, 1 << 40, b.PLAN_NAIVE_ALL)["layer_peak_bytes"]
    with pytest.raises(b.AccError) as e:
        ctx.plan_swaps(32, int(lo * 0.9), b.PLAN_DYNAMIC)
    assert e.value.status == b.ACC_EUNTRAINABLE
    with pytest.raises(b.AccError) as e:
        ctx.plan_swaps(32, 1 * MiB, b.PLAN_DYNAMIC)
    assert e.value.status == b.ACC_EPOOL                      # below parameters + gradients


def test_swapped_bytes_shrink_as_the_budget_grows():
    b = B()
    ctx = ctx_of(S.resnet152())
    prev = None
    for gib in (6, 8, 10, 12, 16, 24):
        s = ctx.plan_swaps(64, gib * GiB, b.PLAN_DYNAMIC)
        assert s["peak_bytes"] <= gib * GiB
        if prev is not None:
            assert s["bytes_swapped"] <= prev
        prev = s["bytes_swapped"]
    assert prev == 0


def test_planner_against_brute_force_on_toy_networks():
    """All 2^m swap sets of a network with m <= 10 maps go through plan_explicit; the
    planner's choice must be feasible and close to the best predicted iteration time."""
    b = B()
    net = chain(n_units=4, c=32, hw=8)          # 11 maps: 2048 swap sets
    ctx = ctx_of(net)
    k = 4
    ctx.set_cost_model(2e12, 1e11, 4e-6, 1e9, 1e9, 5e-6)       # slow link: swapping is costly
    s0 = ctx.plan_swaps(k, 1 << 40, b.PLAN_NAIVE_ALL)
    m = s0["n_maps"]
    assert m <= 12
    lo, hi = s0["layer_peak_bytes"], s0["noswap_peak_bytes"]
    # (the pool of this toy is mostly workspaces; first fit needs 5 % more than the sum of the
    # live bytes, which is 0.4 of the way from the layer-wise to the no-swap peak)
    for frac in (0.45, 0.6, 0.9):
        budget = int(lo + frac * (hi - lo))
        best = None
        for mask in itertools.product((0, 1), repeat=m):
            try:
                s = ctx.plan_explicit(k, budget, list(mask))
            except b.AccError:
                continue
            if best is None or s["t_iter"] < best:
                best = s["t_iter"]
        s = ctx.plan_swaps(k, budget, b.PLAN_DYNAMIC)
        assert s["peak_bytes"] <= budget
        assert s["t_iter"] <= best * 1.10, (frac, s["t_iter"], best)


# ------------------------------------------------- efficiency-optimal minibatch (Alg. 2, Eq. 7, Eq. 9)
def _budget_between(ctx, k_fit, k_swap):
    """A budget under which k_fit still trains without swapping but k_fit + 1 does not."""
    b = B()
    lo = ctx.plan_swaps(k_fit, 1 << 40, b.PLAN_NONE)["peak_bytes"]
    hi = ctx.plan_swaps(k_fit + 1, 1 << 40, b.PLAN_NONE)["peak_bytes"]
    assert lo < hi
    # just below what k_fit + 1 needs at the very least: first fit may need a little more than
    # the sum of the live bytes, so k_fit gets all the room there is
    budget = hi - 256
    ctx.plan_swaps(k_fit, budget, b.PLAN_NONE)
    with pytest.raises(b.AccError):
        ctx.plan_swaps(k_fit + 1, budget, b.PLAN_NONE)
    return budget


def test_tuner_bounds_agree_with_the_planner():
    b = B()
    net = S.resnet((1, 1, 2, 1), in_hw=64, classes=100, width=32)
    ctx = ctx_of(net)
    ctx.set_cost_model(40e12, 3e12, 4e-6, 50e9, 50e9, 1e-5)
    budget = _budget_between(ctx, 12, 13)
    res, summ = ctx.tune_minibatch(budget, 1, 200)
    # the winner's plan is the installed one
    assert ctx.k == res["k_best"] and summ["t_iter"] == pytest.approx(res["t_iter"])
    assert len(ctx.instructions()) == summ["n_instr"]
    assert res["k_noswap_max"] == 12
    ctx.plan_swaps(12, budget, b.PLAN_NONE)
    with pytest.raises(b.AccError):
        ctx.plan_swaps(13, budget, b.PLAN_NONE)
    kmax = res["k_trainable_max"]
    assert 13 <= kmax <= 200
    ctx.plan_swaps(kmax, budget, b.PLAN_NAIVE_ALL)          # k_max trains with everything swapped ...
    if kmax < 200:
        with pytest.raises(b.AccError) as e:                  # ... and k_max + 1 does not (Eq. 4)
            ctx.plan_swaps(kmax + 1, budget, b.PLAN_DYNAMIC)
        assert e.value.status == b.ACC_EUNTRAINABLE
    # no evaluated minibatch is predicted faster
    assert res["images_per_s"] == pytest.approx(res["k_best"] / res["t_iter"])
    for k in list(range(1, 13)) + [13, kmax]:
        s = ctx.plan_swaps(k, budget, b.PLAN_DYNAMIC)
        assert k / s["t_iter"] <= res["images_per_s"] * (1 + 1e-9), k


def test_tuner_follows_measured_step_times():
    """Step times that rise in stairs of 8 images (what tile quantisation does to a GPU):
    the best minibatch is the top of the last full stair that fits, not the largest one."""
    b = B()
    net = chain(n_units=4, c=32, hw=8)
    ctx = ctx_of(net)
    ns = ctx.step_count()
    ks = list(range(1, 41))
    table = np.array([[1e-4 * (-(-k // 8)) for _ in range(ns)] for k in ks])
    ctx.set_calibration(ks, table, (1e7, 1e7, 1e-5))     # a slow link: swapping never pays here
    budget = _budget_between(ctx, 21, 22)
    res, _ = ctx.tune_minibatch(budget, 1, 40)
    assert res["k_noswap_max"] == 21
    assert res["k_best"] == 16                      # 16 images cost two stairs, 17..21 cost three
    # with room for 24 the third stair is full
    res, _ = ctx.tune_minibatch(_budget_between(ctx, 24, 25), 1, 40)
    assert res["k_best"] == 24


def test_tuner_reports_an_untrainable_range():
    b = B()
    net = S.bottleneck_unit()
    ctx = ctx_of(net)
    s = ctx.plan_swaps(4, 1 << 40, b.PLAN_NAIVE_ALL)
    with pytest.raises(b.AccError) as e:
        ctx.tune_minibatch(s["static_bytes"] + 1024, 4, 8)
    assert e.value.status == b.ACC_EUNTRAINABLE
    with pytest.raises(b.AccError):
        ctx.tune_minibatch(1 << 30, 8, 4)            # empty range


def test_adaptive_learning_rate_closed_forms():
    """Eq. 9 against what it must reduce to: q = 1 gives the base rate, q = 2 gives
    a(2 - a c), a -> 0 gives the linear scaling rule q a, q -> infinity gives 1/c."""
    b = B()
    a, c = 0.1, 0.7
    assert b.adaptive_lr(a, c, 1.0) == pytest.approx(a, rel=1e-14)
    assert b.adaptive_lr(a, c, 2.0) == pytest.approx(a * (2 - a * c), rel=1e-14)
    assert b.adaptive_lr(1e-9, c, 8.0) == pytest.approx(8e-9, rel=1e-6)
    assert b.adaptive_lr(a, c, 1e6) == pytest.approx(1 / c, rel=1e-12)
    # the contraction factors of Eq. 8 match: (1 - a c)^(q) == 1 - a* c
    q = 4.2
    assert (1 - a * c) ** q == pytest.approx(1 - b.adaptive_lr(a, c, q) * c, rel=1e-13)
    assert np.isnan(b.adaptive_lr(2.0, 0.7, 2.0)) and np.isnan(b.adaptive_lr(0.1, 0.0, 2.0))


# ------------------------------------------------------------ timeline of the simulation
@pytest.mark.parametrize("budget_gib", [64, 3, 2])
def test_simulated_timeline_is_consistent_with_the_plan(budget_gib):
    """The per-instruction times of Algorithm 1's simulation: every instruction starts after
    what it waits for and after its predecessor on its stream; compute entries are the
    t_start / t_end of the steps; the last end is the predicted iteration; replaying
    allocations and releases along those times never exceeds the planned pool peak, ends
    empty, and has moved every swapped byte out and back."""
    from paper_1901_06773_amd import validate as V
    b = B()
    net = S.resnet50()
    ctx = ctx_of(net)
    s = ctx.plan_swaps(64, budget_gib << 30, b.PLAN_DYNAMIC)
    assert (s["n_swapped"] > 0) == (budget_gib < 64)
    tl = ctx.timeline()
    assert len(tl) == s["n_instr"]
    assert V.dependency_violations(ctx, tl, slack=0.0) == []
    for e in tl:
        if e["op"] == V.OP_COMPUTE:
            info = ctx.step_info(e["arg"])
            assert (e["t_start"], e["t_end"]) == (info["t_start"], info["t_end"])
    assert max(e["t_end"] for e in tl) == pytest.approx(s["t_iter"], rel=1e-12)
    summ = V.timeline_summary(tl)
    assert summ["t_compute"] == pytest.approx(s["t_compute"], rel=1e-9)
    mem = V.memory_curve(ctx, observed=False, points=200)
    # (a map being copied out still occupies its block although the planner's sum of live bytes
    # has let go of it, so the replay may exceed that sum, never the pool)
    cap = min(budget_gib << 30, s["noswap_peak_bytes"]) - s["static_bytes"]
    assert 0.5 * (s["peak_bytes"] - s["static_bytes"]) < mem["peak_dynamic_bytes"] <= cap
    last = mem["series"][-1]
    assert last["pool_bytes"] == 0 and last["bytes_out"] == last["bytes_in"] == s["bytes_swapped"]
    # a planning-only context has nothing observed
    with pytest.raises(b.AccError) as e:
        ctx.timeline(observed=True)
    assert e.value.status == b.ACC_ESTATE
