"""GPU parity of the whole training step (C ABI: acc_create / acc_plan_swaps /
acc_train_step) against the CPU oracle, and the invariant that swapping feature
maps out and back in never changes a single bit of the result."""
import time

import numpy as np
import pytest
import torch

import oracle as O
import synth as S

pytestmark = pytest.mark.gpu

TOL = 1e-4            # fp32: relative, per tensor (l2 and max norm)
MiB = 1 << 20


def B():
    from paper_1901_06773_amd import binding
    return binding


def close(gpu, ref, what, tol=TOL):
    gpu = np.asarray(gpu, np.float64); ref = np.asarray(ref, np.float64)
    assert np.isfinite(gpu).all(), f"{what}: non-finite values"
    nr = np.linalg.norm(ref)
    err = np.linalg.norm(gpu - ref)
    assert err <= tol * max(nr, 1e-30), f"{what}: rel l2 {err / max(nr, 1e-30):.3e}"
    assert np.abs(gpu - ref).max() <= tol * max(np.abs(ref).max(), 1e-30), f"{what}: max norm"


def wide_chain():
    """Three wide convolutions at 12x12: few output tiles and long K, so the convolution
    kernels cut their tail tiles along K, and the weight gradient is reduced over several
    splits (the paths that hand partial sums from one workgroup to another)."""
    net = S.NetSpec("wide_chain", 128, 12, 12, 10)
    x = -1
    for cin, cout, r in ((128, 128, 3), (128, 256, 1), (256, 128, 3)):
        x = net.add(S.Layer(S.CONV, in0=x, cin=cin, cout=cout, r=r, s=r, stride=1, pad=r // 2))
        x = net.add(S.Layer(S.BN, in0=x, cin=cout, cout=cout))
        x = net.add(S.Layer(S.RELU, in0=x, cin=cout, cout=cout))
    g = net.add(S.Layer(S.GAP, in0=x, cin=128, cout=128))
    f = net.add(S.Layer(S.FC, in0=g, cin=128, cout=10))
    net.add(S.Layer(S.SOFTMAX_CE, in0=f, cin=10, cout=1))
    return net


def tall_chain():
    """1x1 convolutions over 8 x 56 x 56 positions (25088 GEMM rows, 392 row tiles) with up to 256
    channels: many output tiles per CU and few K chunks per tile, forward (64 -> 256, with the
    batch-norm sums in its epilogue) and as a data gradient (of 256 -> 64, with the mask and
    the backward sums): the shape of the 1x1 expansions of the large networks."""
    net = S.NetSpec("tall_chain", 64, 56, 56, 10)
    x = -1
    for cin, cout in ((64, 256), (256, 64), (64, 128)):
        x = net.add(S.Layer(S.CONV, in0=x, cin=cin, cout=cout, r=1, s=1, stride=1, pad=0))
        x = net.add(S.Layer(S.BN, in0=x, cin=cout, cout=cout))
        x = net.add(S.Layer(S.RELU, in0=x, cin=cout, cout=cout))
    g = net.add(S.Layer(S.GAP, in0=x, cin=128, cout=128))
    f = net.add(S.Layer(S.FC, in0=g, cin=128, cout=10))
    net.add(S.Layer(S.SOFTMAX_CE, in0=f, cin=10, cout=1))
    return net


NETS = {
    "config1_unit": (lambda: S.bottleneck_unit(), 2),                       # BASELINE configs[0]
    "mini_resnet_w8": (lambda: S.resnet((1, 2), in_hw=32, classes=10, width=8), 3),
    "mini_resnet_w32": (lambda: S.resnet((1, 1, 2, 1), in_hw=64, classes=100, width=32), 5),
    # 30 x 30 input: the stem leaves 15 x 15 for the max-pool (odd: ragged last windows and blocks)
    "mini_resnet_odd": (lambda: S.resnet((1, 1), in_hw=30, classes=10, width=8), 3),
    "wide_chain": (wide_chain, 6),
    "tall_chain": (tall_chain, 8),
    # strided 3x3 convolutions with a data gradient: basic blocks (18/34-layer style) and v1.5 strides
    "mini_resnet_basic": (lambda: S.resnet((2, 1, 1), in_hw=48, classes=10, width=32, block="basic"), 3),
    "mini_resnet_v15": (lambda: S.resnet((1, 2), in_hw=32, classes=10, width=8, variant="v1.5"), 3),
    # VGG style: conv + bias + ReLU, 2x2 max-pools, FC + ReLU over the flattened map (no batch norm)
    "mini_vgg": (lambda: S.vgg(cfg=((32, 32), (64, 64), (64,)), in_c=3, in_hw=32, classes=10, fc=96), 4),
}



def tight_pool(probe, k, s0):
    """The smallest pool, in steps of 5 % of the dynamic part above the layer-wise peak, in which
    the plan that swaps every map can be laid out (first fit needs a little more than the sum
    of the live bytes)."""
    b = B()
    stat = s0["static_bytes"]
    for f in (1.0, 1.05, 1.10, 1.15, 1.20, 1.25):
        tight = stat + int((s0["layer_peak_bytes"] - stat) * f) + 64 * 1024
        try:
            probe.plan_swaps(k, tight, b.PLAN_NAIVE_ALL)
            return tight
        except b.AccError:
            continue
    raise AssertionError("no layout within 25 % of the layer-wise peak")


def run_gpu(net, params, k, mode, budget, steps=1, pool=None, host=256 * MiB, lr=0.1, explicit=None, dtype=0,
            wgrad_stream=True, overlap=True):
    b = B()
    ctx = b.Context(net.as_array(), (net.in_c, net.in_h, net.in_w), pool_bytes=pool or budget, host_bytes=host,
                    dtype=dtype, wgrad_stream=wgrad_stream)
    ctx.set_weights(params)
    if not overlap:
        ctx.set_wgrad_overlap(False)
    summ = ctx.plan_explicit(k, budget, explicit) if explicit is not None else ctx.plan_swaps(k, budget, mode)
    losses = []
    for s in range(steps):
        img, lab = S.make_batch(net, k, s)
        losses.append(ctx.train_step(torch.from_numpy(img).pin_memory(), lab, lr))
    out = dict(losses=losses, grads=ctx.get_grads(), weights=ctx.get_weights(), summary=summ, stats=ctx.stats())
    ctx.close()
    return out


@pytest.mark.parametrize("name", list(NETS))
def test_step_matches_oracle(name):
    make, k = NETS[name]
    net = make()
    params = S.init_params(net)
    img, lab = S.make_batch(net, k, 0)
    o_loss, o_w, o_g = O.train_step(net.as_array(), (net.in_c, net.in_h, net.in_w), params, img, lab, 0.1)
    g = run_gpu(net, params, k, B().PLAN_NONE, 512 * MiB)
    close(g["losses"][0], o_loss, f"{name} loss")
    for i, (a, r) in enumerate(zip(g["grads"], o_g)):
        if r.size:
            close(a, r, f"{name} grad of layer {i} ({S.KIND_NAMES[net.layers[i].kind]})")
    for i, (a, r) in enumerate(zip(g["weights"], o_w)):
        if r.size:
            close(a, r, f"{name} updated weights of layer {i}")


@pytest.mark.parametrize("name", ["config1_unit", "mini_resnet_w8", "mini_vgg"])
def test_minibatch_of_one(name):
    """The degenerate minibatch: batch-norm statistics over H x W alone, one-row GEMMs in the head,
    a single image's worth of tiles everywhere."""
    make, _ = NETS[name]
    net = make()
    params = S.init_params(net)
    img, lab = S.make_batch(net, 1, 0)
    o_loss, o_w, o_g = O.train_step(net.as_array(), (net.in_c, net.in_h, net.in_w), params, img, lab, 0.1)
    g = run_gpu(net, params, 1, B().PLAN_NONE, 512 * MiB)
    close(g["losses"][0], o_loss, f"{name} loss")
    for i, (a, r) in enumerate(zip(g["grads"], o_g)):
        if r.size:
            close(a, r, f"{name} grad of layer {i} ({S.KIND_NAMES[net.layers[i].kind]})")
    for i, (a, r) in enumerate(zip(g["weights"], o_w)):
        if r.size:
            close(a, r, f"{name} updated weights of layer {i}")


def test_resnet152_at_full_input_size_is_as_close_to_the_exact_step_as_fp32_allows():
    """The benchmark's network at 224x224 and a minibatch the oracle finishes in seconds.
    152 layers at random initialisation amplify rounding: the oracle run with fp32 storage
    and the oracle run entirely in double differ by 1-4 % in the gradients (by 1e-6 in the
    loss), so 1e-4 against either is not a meaningful bar here.  What is: the GPU step must
    be as close to the exact (double) step as the fp32-storage oracle is, within a factor 4
    per gradient tensor (the bound of the full-depth tests: ReLU decisions that differ move
    every earlier gradient, and which ones differ depends on the order in which a kernel adds
    its products; observed 2.6 to 3.1 over the kernel versions), plus 1e-3 (ten times the
    one-layer tolerance) for what fp32 MFMA accumulation adds over 155 convolutions where the
    oracle accumulates in double; the loss within 1e-4.  The comparison that does hold 1e-4 at
    this depth, with the discrete decisions taken from the same values on both sides, is in
    test_gpu_full_nets.py."""
    net = S.resnet152()
    k = 4
    params = S.init_params(net)
    img, lab = S.make_batch(net, k, 0)
    chw = (net.in_c, net.in_h, net.in_w)
    l32, _, g32 = O.train_step(net.as_array(), chw, params, img, lab, 0.1)
    l64, _, g64 = O.train_step(net.as_array(), chw, [p.astype(np.float64) for p in params],
                               img.astype(np.float64), lab, 0.1)
    g = run_gpu(net, params, k, B().PLAN_NONE, 2048 * MiB)
    close(g["losses"][0], l64, "loss against the exact step")
    close(g["losses"][0], l32, "loss against the fp32-storage oracle")
    worst = 0.0
    for i, (a, r32, r64) in enumerate(zip(g["grads"], g32, g64)):
        if not r64.size:
            continue
        n64 = np.linalg.norm(r64)
        e_gpu = np.linalg.norm(np.asarray(a, np.float64) - r64) / n64
        e_o32 = np.linalg.norm(r32.astype(np.float64) - r64) / n64
        worst = max(worst, e_gpu / max(e_o32, 1e-6))
        assert np.isfinite(e_gpu) and e_gpu <= 4.0 * e_o32 + 1e-3, \
            f"layer {i} ({S.KIND_NAMES[net.layers[i].kind]}): gpu {e_gpu:.3e}, fp32 oracle {e_o32:.3e}"
    print(f"worst gpu / fp32-oracle error ratio against the exact step: {worst:.2f}")


def test_three_steps_follow_the_oracle():
    make, k = NETS["config1_unit"]
    net = make()
    params = S.init_params(net)
    g = run_gpu(net, params, k, B().PLAN_NONE, 64 * MiB, steps=3)
    p = params
    for s in range(3):
        img, lab = S.make_batch(net, k, s)
        o_loss, p, _ = O.train_step(net.as_array(), (net.in_c, net.in_h, net.in_w), p, img, lab, 0.1)
        close(g["losses"][s], o_loss, f"loss of step {s}", TOL * 10)


def bit_equal(a, b, what):
    for i, (x, y) in enumerate(zip(a, b)):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32)), f"{what}: layer {i} differs"


@pytest.mark.parametrize("name", list(NETS))
def test_swapping_everything_is_bit_exact(name):
    """Naive strategy (Sec. 3.1): every feature map out and back in, in a pool just
    above the layer-wise peak, against the run that keeps everything resident."""
    make, k = NETS[name]
    net = make()
    params = S.init_params(net)
    b = B()
    ref = run_gpu(net, params, k, b.PLAN_NONE, 512 * MiB, steps=2)
    probe = b.Context(net.as_array(), (net.in_c, net.in_h, net.in_w))
    s0 = probe.plan_swaps(k, 1 << 40, b.PLAN_NAIVE_ALL)
    stat = s0["static_bytes"]             # weights, gradients, statistics, kernel scratch: always resident
    tight = tight_pool(probe, k, s0)
    probe.close()
    # (where one layer's working set is most of what the whole network keeps, as in the single
    # block and the small VGG, the two peaks lie too close for the comparison to say anything)
    if s0["noswap_peak_bytes"] - stat > 1.25 * (s0["layer_peak_bytes"] - stat):
        assert tight < s0["noswap_peak_bytes"]
    out = run_gpu(net, params, k, b.PLAN_NAIVE_ALL, tight, steps=2)
    assert out["summary"]["n_swapped"] == out["summary"]["n_maps"] > 0
    assert out["stats"]["bytes_out"] == out["stats"]["bytes_in"] == out["summary"]["bytes_swapped"]
    assert out["stats"]["peak_pool_bytes"] <= tight
    assert np.float32(out["losses"][0]).view(np.uint32) == np.float32(ref["losses"][0]).view(np.uint32)
    assert np.float32(out["losses"][1]).view(np.uint32) == np.float32(ref["losses"][1]).view(np.uint32)
    bit_equal(out["grads"], ref["grads"], "gradients")
    bit_equal(out["weights"], ref["weights"], "weights")


@pytest.mark.parametrize("frac", [0.35, 0.6, 0.85])
def test_dynamic_plans_are_bit_exact(frac):
    """Planner-chosen partial swaps at budgets between the layer-wise peak and the
    no-swap peak."""
    make, k = NETS["mini_resnet_w32"]
    net = make()
    params = S.init_params(net)
    b = B()
    ref = run_gpu(net, params, k, b.PLAN_NONE, 512 * MiB, steps=2)
    probe = b.Context(net.as_array(), (net.in_c, net.in_h, net.in_w))
    s0 = probe.plan_swaps(k, 1 << 40, b.PLAN_NAIVE_ALL)
    probe.close()
    lo, hi = s0["layer_peak_bytes"], s0["noswap_peak_bytes"]
    budget = int(lo + frac * (hi - lo))
    out = run_gpu(net, params, k, b.PLAN_DYNAMIC, budget, steps=2)
    assert 0 < out["summary"]["n_swapped"] < out["summary"]["n_maps"]
    assert out["summary"]["peak_bytes"] <= budget
    assert out["losses"] == ref["losses"]
    bit_equal(out["grads"], ref["grads"], "gradients")
    bit_equal(out["weights"], ref["weights"], "weights")


def test_random_swap_sets_are_bit_exact():
    make, k = NETS["mini_resnet_w8"]
    net = make()
    params = S.init_params(net)
    b = B()
    ref = run_gpu(net, params, k, b.PLAN_NONE, 256 * MiB)
    probe = b.Context(net.as_array(), (net.in_c, net.in_h, net.in_w))
    n_maps = probe.plan_swaps(k, 1 << 40, b.PLAN_NONE)["n_maps"]
    probe.close()
    rng = np.random.default_rng(0)
    for trial in range(4):
        mask = rng.integers(0, 2, n_maps)
        out = run_gpu(net, params, k, None, 256 * MiB, explicit=list(mask))
        assert out["summary"]["n_swapped"] == int(mask.sum())
        assert out["losses"] == ref["losses"], f"trial {trial}"
        bit_equal(out["grads"], ref["grads"], f"gradients, trial {trial}")


def test_device_resident_input_and_error_paths():
    make, k = NETS["config1_unit"]
    net = make()
    params = S.init_params(net)
    b = B()
    ctx = b.Context(net.as_array(), (net.in_c, net.in_h, net.in_w), pool_bytes=64 * MiB, host_bytes=MiB)
    img, lab = S.make_batch(net, k, 0)
    with pytest.raises(b.AccError) as e:
        ctx.train_step(torch.from_numpy(img).cuda(), lab, 0.1)       # no plan yet
    assert e.value.status == b.ACC_ESTATE
    with pytest.raises(b.AccError) as e:
        ctx.plan_swaps(k, 128 * MiB, b.PLAN_NONE)                    # budget above the pool
    assert e.value.status == b.ACC_EPOOL
    with pytest.raises(b.AccError) as e:
        ctx.plan_swaps(k, 300 * 1024, b.PLAN_DYNAMIC)                # below the layer-wise peak
    assert e.value.status in (b.ACC_EUNTRAINABLE, b.ACC_EPOOL)
    with pytest.raises(b.AccError) as e:
        ctx.plan_swaps(4096, 64 * MiB, b.PLAN_NAIVE_ALL)             # not even one layer's working set fits
    assert e.value.status == b.ACC_EUNTRAINABLE
    with pytest.raises(b.AccError) as e:
        bad = lab.copy(); bad[0] = net.classes                       # a label that is no class
        ctx.plan_swaps(k, 64 * MiB, b.PLAN_NONE)
        ctx.train_step(torch.from_numpy(img).cuda(), bad, 0.1)
    assert e.value.status == b.ACC_EINVAL
    ctx.set_weights(params)
    ctx.plan_swaps(k, 64 * MiB, b.PLAN_DYNAMIC)
    l_dev = ctx.train_step(torch.from_numpy(img).cuda(), lab, 0.1)
    ctx.set_weights(params)
    l_host = ctx.train_step(torch.from_numpy(img).pin_memory(), lab, 0.1)
    assert l_dev == l_host
    ctx.close()


def test_host_arena_too_small_for_the_swapped_maps():
    """A plan whose swapped maps need more pinned host memory than the context was given is refused
    with ACC_EHOSTMEM, exactly; the same plan is accepted once the arena is large enough."""
    make, k = NETS["mini_resnet_w32"]
    net = make()
    b = B()
    chw = (net.in_c, net.in_h, net.in_w)
    probe = b.Context(net.as_array(), chw)
    need = probe.plan_swaps(k, 1 << 40, b.PLAN_NAIVE_ALL)
    probe.close()
    assert need["host_bytes"] > 4 * MiB
    ctx = b.Context(net.as_array(), chw, pool_bytes=512 * MiB, host_bytes=need["host_bytes"] - 256)
    with pytest.raises(b.AccError) as e:
        ctx.plan_swaps(k, 512 * MiB, b.PLAN_NAIVE_ALL)
    assert e.value.status == b.ACC_EHOSTMEM
    ctx.close()
    ctx = b.Context(net.as_array(), chw, pool_bytes=512 * MiB, host_bytes=need["host_bytes"])
    assert ctx.plan_swaps(k, 512 * MiB, b.PLAN_NAIVE_ALL)["n_swapped"] == need["n_swapped"]
    ctx.close()


# ------------------------------------------------------------------ verification mode of the swap engine
@pytest.mark.parametrize("name,k", [("mini_resnet_w32", 5), ("mini_resnet_basic", 3), ("mini_vgg", 4), ("resnet50", 16)])
@pytest.mark.parametrize("mode", ["none", "naive_all", "dynamic"])
def test_poisoned_memory_is_never_read_and_the_budget_is_never_exceeded(name, k, mode):
    """ACC_DEBUG_POISON: every byte of the pool that holds no live tensor holds a NaN pattern
    (before the iteration, after a block's release, until a prefetch has landed), and so does
    the host arena until an offload has landed.  A plan that orders every use after the data's
    arrival and before the block's release therefore gives finite results with the very bits
    of the unpoisoned resident run; one with a missing wait would read NaNs.  The pool is made
    32 MiB larger than the budget: the scan after the iteration must find the highest written
    byte inside the budget (acc_train_step itself returns ACC_EPOOL otherwise), at or below
    where the plan's highest block ends, and above the sum of the live bytes' low-water mark."""
    b = B()
    net = NETS[name][0]() if name in NETS else getattr(S, name)()
    params = S.init_params(net)
    chw = (net.in_c, net.in_h, net.in_w)
    probe = b.Context(net.as_array(), chw)
    s_all = probe.plan_swaps(k, 1 << 40, b.PLAN_NAIVE_ALL)
    s_none = probe.plan_swaps(k, 1 << 40, b.PLAN_NONE)
    stat = s_all["static_bytes"]
    if mode == "none":
        pmode, budget = b.PLAN_NONE, int(s_none["peak_bytes"] * 1.05) + 8 * MiB
    elif mode == "naive_all":
        pmode, budget = b.PLAN_NAIVE_ALL, tight_pool(probe, k, s_all)
    else:
        pmode, budget = b.PLAN_DYNAMIC, (s_all["layer_peak_bytes"] + s_none["peak_bytes"]) // 2
        for _ in range(4):      # a budget the planner can lay out (first fit needs some slack above the live bytes)
            try:
                probe.plan_swaps(k, budget, pmode)
                break
            except b.AccError:
                budget = int(budget * 1.08)
    probe.close()
    ref = run_gpu(net, params, k, b.PLAN_NONE, int(s_none["peak_bytes"] * 1.05) + 64 * MiB, steps=2, host=MiB)

    ctx = b.Context(net.as_array(), chw, pool_bytes=budget + 32 * MiB, host_bytes=s_all["host_bytes"] + MiB)
    ctx.set_weights(params)
    summ = ctx.plan_swaps(k, budget, pmode)
    ctx.set_debug(True)
    losses = []
    for s in range(2):
        img, lab = S.make_batch(net, k, s)
        losses.append(ctx.train_step(torch.from_numpy(img).pin_memory(), lab, 0.1))
        st = ctx.stats()
        assert st["peak_is_measured"] == 1
        assert stat < st["peak_pool_bytes"] <= budget, (st["peak_pool_bytes"], budget)
        assert st["touched_pool_bytes"] <= st["peak_pool_bytes"]
        # every live byte was written at some point; alignment padding of the blocks is not
        assert st["touched_pool_bytes"] > stat + 0.5 * (summ["layer_peak_bytes"] - stat)
    grads, weights = ctx.get_grads(), ctx.get_weights()
    ctx.set_debug(False)
    ctx.close()
    if mode == "naive_all":
        assert summ["n_swapped"] == summ["n_maps"] > 0
    for a in grads:
        assert np.isfinite(a).all()
    for a, r in zip(losses, ref["losses"]):
        assert np.isfinite(a) and np.float32(a).view(np.uint32) == np.float32(r).view(np.uint32)
    bit_equal(grads, ref["grads"], "gradients")
    bit_equal(weights, ref["weights"], "weights")


def test_resnet152_at_the_benchmark_size_swapped_and_resident_agree_bit_for_bit():
    """The benchmark's network and minibatch (ResNet-152, 224x224, k = 41): a planner-chosen
    partial swap under 5 GiB against the resident run under 8 GiB, two steps, every bit of
    loss and updated weights; and the loss of the first step is what 1000 classes at random
    initialisation give (ln 1000 plus the spread of the logits)."""
    GiB = 1 << 30
    net = S.resnet152()
    k = 41
    params = S.init_params(net)
    b = B()
    ref = run_gpu(net, params, k, b.PLAN_NONE, 8 * GiB, steps=2, host=64 * MiB)
    probe = b.Context(net.as_array(), (net.in_c, net.in_h, net.in_w))
    need = probe.plan_swaps(k, 5 * GiB, b.PLAN_DYNAMIC)
    probe.close()
    assert need["n_swapped"] > 0
    out = run_gpu(net, params, k, b.PLAN_DYNAMIC, 5 * GiB, steps=2, host=need["host_bytes"] + 64 * MiB)
    assert out["summary"]["n_swapped"] > 0 and out["stats"]["bytes_out"] == out["summary"]["bytes_swapped"]
    assert out["stats"]["peak_pool_bytes"] <= 5 * GiB
    for a, r in zip(out["losses"], ref["losses"]):
        assert np.float32(a).view(np.uint32) == np.float32(r).view(np.uint32)
    bit_equal(out["weights"], ref["weights"], "weights")
    assert np.log(1000.0) < ref["losses"][0] < np.log(1000.0) + 3.0


# ------------------------------------------------------------------ bf16 storage (configs[4]'s arithmetic)
def l2_close(gpu, ref, what, tol):
    gpu = np.asarray(gpu, np.float64); ref = np.asarray(ref, np.float64)
    assert np.isfinite(gpu).all(), f"{what}: non-finite values"
    err = np.linalg.norm(gpu - ref) / max(np.linalg.norm(ref), 1e-30)
    assert err <= tol, f"{what}: rel l2 {err:.3e}"


def _bf(a):
    """round an fp32 array to bf16 (nearest even) and back"""
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(torch.bfloat16).float().numpy()


def bf16_chain_step(net, params, img, lab):
    """The step of a conv-BN-ReLU chain (+ GAP, FC, loss) put together from the oracle's layer
    functions, with every stored tensor rounded to bf16 where the GPU path stores one: conv
    outputs, BN+ReLU outputs, pooled features, logits (before and after the bias), and the
    gradient of each of them; weights rounded for the kernels; statistics, weight gradients
    and the loss in fp32.  -> (loss, grads per layer)"""
    L = net.layers
    grads = [np.zeros(0, np.float32)] * len(L)
    acts = {-1: _bf(img)}
    saved = {}
    i = 0
    while L[i].kind == S.CONV:
        cv, bn = L[i], L[i + 1]
        assert bn.kind == S.BN and L[i + 2].kind == S.RELU
        w16 = _bf(params[i].reshape(cv.cout, cv.cin, cv.r, cv.s))
        x = acts[cv.in0]
        z = _bf(O.conv_fwd(x, w16, cv.stride, cv.pad))
        gamma, beta = params[i + 1][:bn.cin], params[i + 1][bn.cin:]
        y, mean, istd = O.bn_fwd(z, gamma, beta, O.BN_EPS)
        a = _bf(O.relu_fwd(y))
        saved[i] = (x, w16, z, gamma, mean, istd, a)
        acts[i + 2] = a
        i += 3
    gap_l, fc_l = L[i], L[i + 1]
    assert gap_l.kind == S.GAP and fc_l.kind == S.FC and L[i + 2].kind == S.SOFTMAX_CE
    feat_in = acts[gap_l.in0]
    feat = _bf(O.gap_fwd(feat_in))
    W, bias = params[i + 1][:fc_l.cout * fc_l.cin], params[i + 1][fc_l.cout * fc_l.cin:]
    p16 = np.concatenate([_bf(W), np.zeros_like(bias)])
    logits = _bf(_bf(O.fc_fwd(feat, p16, fc_l.cout)) + bias)
    loss, dz = O.softmax_ce(logits, lab)
    dz = _bf(dz)
    dfeat, dparam = O.fc_bwd(feat, p16, dz)
    grads[i + 1] = dparam
    g = _bf(O.gap_bwd(_bf(dfeat), feat_in.shape))
    i -= 3
    while i >= 0:
        cv = L[i]
        x, w16, z, gamma, mean, istd, a = saved[i]
        gm = O.relu_bwd(a, g)
        dz_, dgamma, dbeta = O.bn_bwd(z, gm, gamma, mean, istd)
        grads[i + 1] = np.concatenate([dgamma, dbeta])
        dz_ = _bf(dz_)
        grads[i] = O.conv_wgrad(x, dz_, w16.shape, cv.stride, cv.pad).ravel()
        if i > 0:
            g = _bf(O.conv_dgrad(dz_, w16, x.shape, cv.stride, cv.pad))
        i -= 3
    return loss, grads


def test_bf16_step_equals_its_layers_put_together():
    """At random initialisation batch-norm backward cancels most of the incoming gradient,
    which amplifies bf16 rounding of the stored tensors to 10-50 % in the weight gradients:
    against the fp32 oracle only the loss can be held to 2e-2 (next test).  What pins the
    bf16 path is this: the GPU step against the same layers taken from the oracle one by
    one with bf16 rounding at exactly the tensors the GPU stores.  Then only the accumulation
    order and rare rounding ties differ: 2e-2 per gradient tensor holds with a wide margin."""
    net = wide_chain()
    k = 6
    params = S.init_params(net)
    img, lab = S.make_batch(net, k, 0)
    e_loss, e_g = bf16_chain_step(net, params, img, lab)
    b = B()
    g = run_gpu(net, params, k, b.PLAN_NONE, 512 * MiB, dtype=b.BF16, lr=0.0)
    l2_close(g["losses"][0], e_loss, "loss", 1e-4)
    worst = 0.0
    for i, (a, r) in enumerate(zip(g["grads"], e_g)):
        if r.size:
            worst = max(worst, np.linalg.norm(np.asarray(a, np.float64) - r) / np.linalg.norm(r))
            l2_close(a, r, f"grad of layer {i} ({S.KIND_NAMES[net.layers[i].kind]})", 2e-2)
    print(f"worst relative l2 distance of a gradient tensor: {worst:.2e}")


def _output_shapes(net):
    """(c, h, w) of every layer's output."""
    out = []
    for l in net.layers:
        c, h, w = (net.in_c, net.in_h, net.in_w) if l.in0 < 0 else out[l.in0]
        if l.kind in (S.CONV, S.MAXPOOL):
            co = l.cout if l.kind == S.CONV else c
            out.append((co, O.out_dim(h, l.r, l.stride, l.pad), O.out_dim(w, l.s, l.stride, l.pad)))
        elif l.kind == S.GAP:
            out.append((c, 1, 1))
        elif l.kind == S.FC:
            out.append((l.cout, 1, 1))
        elif l.kind == S.SOFTMAX_CE:
            out.append((1, 1, 1))
        else:
            out.append((c, h, w))
    return out


@pytest.mark.parametrize("name", ["config1_unit", "mini_resnet_w8", "mini_resnet_w32", "wide_chain", "tall_chain", "resnet50"])
def test_bf16_step_against_the_fp32_oracle(name):
    """Activations, their gradients and the weights the kernels read stored as bf16, fp32
    accumulation, fp32 master weights and statistics, against the fp32 oracle (configs[4]'s
    arithmetic; ResNet-50 at its full input size and minibatch 8 is the deep case).
    End to end: the loss within 2e-2, every gradient finite.  Gradient tensors: compared in a
    second iteration that runs on the oracle's forward activations (rounded to bf16 on their
    way in, acc_inject_output), so that ReLU masks and max-pool winners are taken from the
    same values on both sides: per tensor the relative l2 distance is printed; 2e-2 must hold
    for nine tensors in ten and 1e-1 for all (the exceptions sit where a batch norm over few
    positions cancels most of the incoming gradient: bf16 rounding of the stored gradient,
    2^-9 per element, is amplified there).  Without the injection the gradients of the two
    sides are 8-130 % apart at random initialisation, the fp32 paths' 1-5 % for the same reason
    times the coarser rounding."""
    if name in NETS:
        make, k = NETS[name]
        net = make()
    else:
        net, k = getattr(S, name)(), 8
    chw = (net.in_c, net.in_h, net.in_w)
    params = S.init_params(net)
    img, lab = S.make_batch(net, k, 0)
    shp = _output_shapes(net)
    stored = [i for i, l in enumerate(net.layers) if l.kind in (S.CONV, S.RELU, S.MAXPOOL)]
    sizes = {i: k * int(np.prod(shp[i])) for i in stored}
    o_loss, o_w, o_g, o_acts = O.train_step(net.as_array(), chw, params, img, lab, 0.1, want_acts=stored, act_sizes=sizes)
    b = B()
    probe = b.Context(net.as_array(), chw, dtype=b.BF16)
    pool = int(probe.plan_swaps(k, 1 << 40, b.PLAN_NONE)["peak_bytes"] * 1.05) + 64 * MiB
    probe.close()
    ctx = b.Context(net.as_array(), chw, pool_bytes=pool, host_bytes=MiB, dtype=b.BF16)
    ctx.set_weights(params)
    ctx.plan_swaps(k, pool, b.PLAN_NONE)
    pinned = torch.from_numpy(img).pin_memory()
    loss = ctx.train_step(pinned, lab, 0.0)
    l2_close(loss, o_loss, f"{name} loss", 2e-2)
    for a in ctx.get_grads():
        assert np.isfinite(a).all()
    ctx.inject_outputs({i: o_acts[i].reshape(k, *shp[i]).transpose(0, 2, 3, 1) for i in stored})
    loss2 = ctx.train_step(pinned, lab, 0.0)
    grads = ctx.get_grads()
    ctx.stop_captures()
    ctx.close()
    l2_close(loss2, o_loss, f"{name} loss on the oracle's activations", 2e-2)
    errs = {}
    for i, (a, r) in enumerate(zip(grads, o_g)):
        if r.size:
            errs[i] = float(np.linalg.norm(np.asarray(a, np.float64) - r) / np.linalg.norm(r))
    over = {i: e for i, e in errs.items() if e > 2e-2}
    print(f"\n{name} k={k} bf16 against the fp32 oracle: loss {abs(loss - o_loss) / o_loss:.1e}; {len(errs)} gradient tensors, "
          f"median {np.median(list(errs.values())):.1e}, max {max(errs.values()):.1e}; beyond 2e-2: "
          + (", ".join(f"layer {i} ({S.KIND_NAMES[net.layers[i].kind]}) {e:.1e}" for i, e in over.items()) or "none"))
    assert len(over) <= 0.1 * len(errs), over
    assert max(errs.values()) <= 1e-1, over


def test_bf16_maps_take_half_the_memory_and_swap_bit_exactly():
    b = B()
    make, k = NETS["mini_resnet_w32"]
    net = make()
    params = S.init_params(net)
    chw = (net.in_c, net.in_h, net.in_w)
    p32 = b.Context(net.as_array(), chw)
    p16 = b.Context(net.as_array(), chw, dtype=b.BF16)
    s32 = p32.plan_swaps(k, 1 << 40, b.PLAN_NAIVE_ALL)
    s16 = p16.plan_swaps(k, 1 << 40, b.PLAN_NAIVE_ALL)
    tight = tight_pool(p16, k, s16)
    p32.close(); p16.close()
    assert s16["n_maps"] == s32["n_maps"]
    assert abs(s16["bytes_maps"] * 2 - s32["bytes_maps"]) <= 512 * s32["n_maps"]      # halves, up to 256-byte rounding
    ref = run_gpu(net, params, k, b.PLAN_NONE, 512 * MiB, steps=2, dtype=b.BF16)
    out = run_gpu(net, params, k, b.PLAN_NAIVE_ALL, tight, steps=2, dtype=b.BF16)
    assert out["summary"]["n_swapped"] == out["summary"]["n_maps"] > 0
    assert out["stats"]["bytes_out"] == out["stats"]["bytes_in"] == s16["bytes_swapped"]
    for a, r in zip(out["losses"], ref["losses"]):
        assert np.float32(a).view(np.uint32) == np.float32(r).view(np.uint32)
    bit_equal(out["grads"], ref["grads"], "gradients")
    bit_equal(out["weights"], ref["weights"], "weights")


# ------------------------------------------------------------------ the baseline's configurations
GiB = 1 << 30


def _budgeted_vs_resident(net, k, budget, expect_swaps, dtype=0, steps=2):
    b = B()
    params = S.init_params(net)
    chw = (net.in_c, net.in_h, net.in_w)
    probe = b.Context(net.as_array(), chw, dtype=dtype)
    plan = probe.plan_swaps(k, budget, b.PLAN_DYNAMIC)
    resident = probe.plan_swaps(k, 1 << 40, b.PLAN_NONE)
    probe.close()
    assert plan["peak_bytes"] <= budget
    assert (plan["n_swapped"] > 0) == expect_swaps, plan["n_swapped"]
    out = run_gpu(net, params, k, b.PLAN_DYNAMIC, budget, steps=steps, host=plan["host_bytes"] + 64 * MiB, dtype=dtype)
    assert out["stats"]["peak_pool_bytes"] <= budget
    assert all(np.isfinite(l) for l in out["losses"])
    if expect_swaps:
        ref = run_gpu(net, params, k, b.PLAN_NONE, resident["peak_bytes"] + 64 * MiB, steps=steps, dtype=dtype)
        for a, r in zip(out["losses"], ref["losses"]):
            assert np.float32(a).view(np.uint32) == np.float32(r).view(np.uint32)
        bit_equal(out["weights"], ref["weights"], "weights")
    return plan, out


def test_config_resnet50_uncapped_needs_no_swap():
    """configs[1]: ResNet-50, minibatch 32, no memory cap: the planner must choose zero swaps."""
    plan, out = _budgeted_vs_resident(S.resnet50(), 32, 64 * GiB, expect_swaps=False)
    assert plan["n_swapped"] == 0 and out["stats"]["bytes_out"] == 0


def test_config_resnet101_under_12_gib():
    """configs[2]: ResNet-101, minibatch 64, 12 GiB: planner-chosen swaps, same bits as the
    resident run."""
    net = S.resnet101()
    plan, out = _budgeted_vs_resident(net, 64, 12 * GiB, expect_swaps=_needs_swap(net, 64, 12 * GiB))
    assert out["stats"]["bytes_out"] == plan["bytes_swapped"]


def _needs_swap(net, k, budget, dtype=0):
    b = B()
    probe = b.Context(net.as_array(), (net.in_c, net.in_h, net.in_w), dtype=dtype)
    need = probe.plan_swaps(k, 1 << 40, b.PLAN_NONE)["peak_bytes"] > budget
    probe.close()
    return need


def test_config_resnet152_under_8_gib_at_twice_the_resident_minibatch():
    """configs[3]: ResNet-152 under 8 GiB at minibatch 64 (the resident maximum is 46)."""
    plan, out = _budgeted_vs_resident(S.resnet152(), 64, 8 * GiB, expect_swaps=True)
    assert out["stats"]["bytes_out"] == plan["bytes_swapped"] > 2 * GiB


def test_resnet34_under_4_gib_swaps_and_keeps_the_bits():
    """The basic-block network of the paper's Table 1 (strided 3x3 data gradients) at its full
    input size: minibatch 192 needs 5.7 GiB resident; under 4 GiB the planner swaps, and the
    weights after two steps are those of the resident run, bit for bit."""
    plan, out = _budgeted_vs_resident(S.resnet34(), 192, 4 * GiB, expect_swaps=True)
    assert out["stats"]["bytes_out"] == plan["bytes_swapped"] > 0


def test_vgg16_at_full_size_swapping_everything_keeps_the_bits():
    """VGG-16 of the paper's Table 1 at 224 x 224 (conv + bias + ReLU in one launch, 2 x 2 max-pools, the
    25088 -> 4096 fully connected layer): every map offloaded and brought back, under 2.5 GiB at minibatch
    16, against the resident run.  (The planner itself swaps nothing here: the backward step of the second
    convolution alone needs nearly the whole resident peak, so swapping buys this network next to nothing.)"""
    b = B()
    net = S.vgg16()
    k = 16
    params = S.init_params(net)
    chw = (net.in_c, net.in_h, net.in_w)
    probe = b.Context(net.as_array(), chw)
    plan = probe.plan_swaps(k, int(2.5 * GiB), b.PLAN_NAIVE_ALL)
    resident = probe.plan_swaps(k, 1 << 40, b.PLAN_NONE)
    probe.close()
    assert plan["n_swapped"] == plan["n_maps"] > 0
    out = run_gpu(net, params, k, b.PLAN_NAIVE_ALL, int(2.5 * GiB), steps=2, host=plan["host_bytes"] + 64 * MiB)
    assert out["stats"]["bytes_out"] == plan["bytes_swapped"] > 0
    assert out["stats"]["peak_pool_bytes"] <= int(2.5 * GiB)
    ref = run_gpu(net, params, k, b.PLAN_NONE, int(resident["peak_bytes"] * 1.05) + 64 * MiB, steps=2)
    for a, r in zip(out["losses"], ref["losses"]):
        assert np.isfinite(a) and np.float32(a).view(np.uint32) == np.float32(r).view(np.uint32)
    bit_equal(out["weights"], ref["weights"], "weights")


def test_config_resnet152_bf16_under_24_gib():
    """configs[4]: ResNet-152 with bf16 storage, 24 GiB; at minibatch 320 (the resident maximum
    is 291) so that the resident reference run stays small."""
    b = B()
    plan, out = _budgeted_vs_resident(S.resnet152(), 320, 24 * GiB, expect_swaps=True, dtype=b.BF16, steps=1)
    assert out["stats"]["bytes_out"] == plan["bytes_swapped"] > 0


@pytest.mark.parametrize("name", ["mini_resnet_w32", "mini_resnet_basic", "wide_chain"])
def test_weight_gradient_stream_changes_no_bit(name):
    """Weight gradients on their own stream beside the data gradients (the default), on the
    compute stream although the context has the extra stream, and in a context created with
    three streams only: the same losses, gradients and weights, bit for bit, with everything
    resident and with every map swapped."""
    make, k = NETS[name]
    net = make()
    params = S.init_params(net)
    b = B()
    probe = b.Context(net.as_array(), (net.in_c, net.in_h, net.in_w))
    s0 = probe.plan_swaps(k, 1 << 40, b.PLAN_NAIVE_ALL)
    tight = tight_pool(probe, k, s0)
    probe.close()
    for mode, budget in ((b.PLAN_NONE, 512 * MiB), (b.PLAN_NAIVE_ALL, tight)):
        ref = run_gpu(net, params, k, mode, budget, steps=2)
        for kw in (dict(overlap=False), dict(wgrad_stream=False)):
            out = run_gpu(net, params, k, mode, budget, steps=2, **kw)
            for a, r in zip(out["losses"], ref["losses"]):
                assert np.float32(a).view(np.uint32) == np.float32(r).view(np.uint32)
            bit_equal(out["grads"], ref["grads"], f"gradients {kw}")
            bit_equal(out["weights"], ref["weights"], f"weights {kw}")


# ------------------------------------------------------------------ Algorithm 2's outer search on the machine
@pytest.mark.timeout(600)
def test_tuned_minibatch_is_the_fastest_measured_one():
    """acc_tune_minibatch on the benchmark's workload (ResNet-152, 8 GiB), with the cost model
    calibrated on this machine, against a measured sweep: the minibatch it picks must be within
    3 % of the best images/s measured at itself, its two neighbours, the largest minibatch that
    needs no swap, a smaller one and one that swaps; and the iteration time it predicted for its
    choice within 10 % of the measured one."""
    b = B()
    net = S.resnet152()
    chw = (net.in_c, net.in_h, net.in_w)
    budget = 8 * GiB
    probe = b.Context(net.as_array(), chw)
    lo, hi = 1, 512
    while lo < hi:
        mid = (lo + hi + 1) // 2
        try:
            probe.plan_swaps(mid, budget, b.PLAN_NONE); lo = mid
        except b.AccError:
            hi = mid - 1
    k_fit = lo
    k_swap = k_fit + 6
    host = probe.plan_swaps(k_swap, budget, b.PLAN_NAIVE_ALL)["host_bytes"]
    probe.close()
    ctx = b.Context(net.as_array(), chw, pool_bytes=budget, host_bytes=host + 64 * MiB)
    ctx.set_weights(S.init_params(net))
    ctx.calibrate(list(range(k_fit - 15, k_fit + 1)))
    tuned, plan = ctx.tune_minibatch(budget, 1, k_swap + 10)
    k_best = tuned["k_best"]
    assert tuned["k_noswap_max"] == k_fit and 1 <= k_best <= tuned["k_trainable_max"]

    def measure(k):
        ctx.plan_swaps(k, budget, b.PLAN_DYNAMIC)
        img, lab = S.make_batch(net, k, 0)
        img = torch.from_numpy(img).cuda()
        ctx.train_step(img, lab, 0.0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(4):
            ctx.train_step(img, lab, 0.0)
        torch.cuda.synchronize()
        return k / ((time.perf_counter() - t0) / 4)

    rates = {}
    for k in sorted({k_best, max(1, k_best - 1), min(k_best + 1, tuned["k_trainable_max"]), k_fit, 32, k_swap}):
        rates[k] = measure(k)
    ctx.close()
    print("\nmeasured images/s:", {k: round(v, 1) for k, v in rates.items()}, "tuner:", tuned)
    assert rates[k_best] >= 0.97 * max(rates.values()), (k_best, rates)
    assert k_best / tuned["t_iter"] == pytest.approx(rates[k_best], rel=0.10)
    assert rates[k_swap] < rates[k_best]          # on this link a swap costs more than the larger minibatch gains


def test_capture_injection_and_launch_profile_hooks():
    """The parity hooks of the ABI on the single bottleneck block: a captured output is what the oracle
    computes; a fused-away layer, a bad layer and a buffer that is too small are refused; an injected
    output replaces the library's own for the rest of the iteration (injecting zeros for the block's last
    ReLU output makes every image's logits equal to the FC bias, so the loss is ln 10 exactly); the
    per-launch profile names every convolution of the step with its role and flops."""
    net = S.bottleneck_unit()
    k = 2
    b = B()
    chw = (net.in_c, net.in_h, net.in_w)
    params = S.init_params(net)
    img, lab = S.make_batch(net, k, 0)
    relus = [i for i, l in enumerate(net.layers) if l.kind == S.RELU]
    convs = [i for i, l in enumerate(net.layers) if l.kind == S.CONV]
    bns = [i for i, l in enumerate(net.layers) if l.kind == S.BN]
    want = convs + relus
    shp = _output_shapes(net)
    sizes = {i: k * int(np.prod(shp[i])) for i in want}
    o_loss, _, _, o_acts = O.train_step(net.as_array(), chw, params, img, lab, 0.0, want_acts=want, act_sizes=sizes)
    ctx = b.Context(net.as_array(), chw, pool_bytes=64 * MiB, host_bytes=MiB)
    ctx.set_weights(params)
    ctx.plan_swaps(k, 64 * MiB, b.PLAN_NONE)
    lib = b.lib()
    buf = torch.empty(1 << 20, dtype=torch.uint8).pin_memory()
    assert lib.acc_capture_output(ctx._h, bns[0], buf.data_ptr(), buf.numel()) == b.ACC_EINVAL      # fused into its ReLU's step
    assert lib.acc_capture_output(ctx._h, len(net.layers), buf.data_ptr(), buf.numel()) == b.ACC_EINVAL
    assert lib.acc_capture_output(ctx._h, convs[0], buf.data_ptr(), 16) == b.ACC_OK                  # too small: refused at the step
    with pytest.raises(b.AccError) as e:
        ctx.train_step(torch.from_numpy(img).pin_memory(), lab, 0.0)
    assert e.value.status == b.ACC_EINVAL
    ctx.stop_captures()
    caps = ctx.capture_outputs(want, shp, k)
    loss = ctx.train_step(torch.from_numpy(img).pin_memory(), lab, 0.0)
    close(loss, o_loss, "loss")
    for i in want:
        c, h, w = shp[i]
        close(caps[i].numpy().transpose(0, 3, 1, 2), o_acts[i].reshape(k, c, h, w), f"captured output of layer {i}")
    ctx.stop_captures()
    last = relus[-1]
    ctx.inject_outputs({last: np.zeros((k, shp[last][1], shp[last][2], shp[last][0]), np.float32)})
    loss0 = ctx.train_step(torch.from_numpy(img).pin_memory(), lab, 0.0)
    assert abs(loss0 - np.log(net.classes)) < 1e-6          # FC bias is zero at initialisation: uniform softmax
    ctx.stop_captures()
    ctx.set_profiling(2)
    ctx.train_step(torch.from_numpy(img).pin_memory(), lab, 0.0)
    prof = ctx.launch_profile()
    ctx.set_profiling(0)
    ctx.close()
    by_role = {r: [p for p in prof if p["role"] == r and net.layers[p["layer"]].kind == S.CONV] for r in ("fwd", "dgrad", "wgrad")}
    assert sorted(p["layer"] for p in by_role["fwd"]) == convs and sorted(p["layer"] for p in by_role["wgrad"]) == convs
    assert sorted(p["layer"] for p in by_role["dgrad"]) == convs[1:]          # the first layer needs no data gradient
    for p in prof:
        l = net.layers[p["layer"]]
        if l.kind == S.CONV:
            assert p["flops"] == 2.0 * k * shp[p["layer"]][1] * shp[p["layer"]][2] * l.cout * l.cin * l.r * l.s and p["ms"] >= 0


# ------------------------------------------------------------------ graph replay
@pytest.mark.parametrize("name", ["mini_resnet_w32", "mini_resnet_basic", "mini_vgg", "wide_chain", "config1_unit"])
@pytest.mark.parametrize("wgrad_stream", [True, False])
def test_graph_replay_changes_no_bit(name, wgrad_stream):
    """acc_set_graph: the compute part of an iteration that swaps nothing is recorded into a HIP graph
    in its first run and replayed afterwards.  Five iterations on changing batches and learning rates
    (the first records, four replay), with the program's own eager work and synchronisations between
    the replays (gradients and weights are read back after every step), against the ordinary run:
    every loss, every gradient and every weight of every step, bit for bit.  Then a new plan at another
    minibatch (the recording is discarded and made again), one profiled step in between (runs the
    ordinary way), and a plan that swaps (never uses the graph)."""
    make, k = NETS[name]
    net = make()
    params = S.init_params(net)
    b = B()
    chw = (net.in_c, net.in_h, net.in_w)

    def run(graph, kk, mode, budget, steps, profiled_at=None):
        ctx = b.Context(net.as_array(), chw, pool_bytes=512 * MiB, host_bytes=256 * MiB, wgrad_stream=wgrad_stream)
        ctx.set_weights(params)
        ctx.set_graph(graph)
        ctx.plan_swaps(kk, budget, mode)
        out = []
        for s in range(steps):
            img, lab = S.make_batch(net, kk, s)
            if profiled_at == s:
                ctx.set_profiling(1)
            loss = ctx.train_step(torch.from_numpy(img).pin_memory(), lab, 0.1 / (s + 1))
            ctx.set_profiling(0)
            out.append((loss, ctx.get_grads(), ctx.get_weights()))
        # a second plan in the same context
        ctx.plan_swaps(kk + 1, budget, mode)
        for s in range(2):
            img, lab = S.make_batch(net, kk + 1, 10 + s)
            loss = ctx.train_step(torch.from_numpy(img).cuda(), lab, 0.05)
            out.append((loss, ctx.get_grads(), ctx.get_weights()))
        ctx.close()
        return out

    for mode, budget in ((b.PLAN_NONE, 512 * MiB),):
        ref = run(False, k, mode, budget, 5)
        got = run(True, k, mode, budget, 5, profiled_at=3)
        for s, ((l0, g0, w0), (l1, g1, w1)) in enumerate(zip(ref, got)):
            assert np.float32(l0).view(np.uint32) == np.float32(l1).view(np.uint32), f"loss of step {s}"
            bit_equal(g1, g0, f"gradients of step {s}")
            bit_equal(w1, w0, f"weights of step {s}")
    # with graph mode on, a plan that swaps runs the ordinary way and keeps its bits
    probe = b.Context(net.as_array(), chw)
    s0 = probe.plan_swaps(k, 1 << 40, b.PLAN_NAIVE_ALL)
    tight = tight_pool(probe, k, s0)
    probe.close()
    ctx = b.Context(net.as_array(), chw, pool_bytes=tight, host_bytes=256 * MiB, wgrad_stream=wgrad_stream)
    ctx.set_weights(params)
    ctx.set_graph(True)
    ctx.plan_swaps(k, tight, b.PLAN_NAIVE_ALL)
    img, lab = S.make_batch(net, k, 0)
    loss = ctx.train_step(torch.from_numpy(img).pin_memory(), lab, 0.1)
    assert np.float32(loss).view(np.uint32) == np.float32(ref[0][0]).view(np.uint32)
    bit_equal(ctx.get_weights(), ref[0][2], "weights of the swapped step")
    ctx.close()


# ------------------------------------------------------------------ model validation (Sec. 6.2)
@pytest.mark.parametrize("case", ["mini_naive", "resnet50_dynamic"])
def test_observed_timeline_obeys_the_plan_and_tracks_the_prediction(case):
    """A step run with events around every step and copy: on the device no instruction starts
    before the step, offload or prefetch that the plan makes it wait for has ended (the three
    streams and their events order the work as Algorithm 1 assumes); memory replayed along
    the observed times stays inside the pool; and, with the cost model calibrated on this
    machine, the observed iteration is within 15 % of the predicted one."""
    from paper_1901_06773_amd import validate as V
    b = B()
    if case == "mini_naive":
        make, k = NETS["mini_resnet_w32"]
        net, mode = make(), b.PLAN_NAIVE_ALL
        probe = b.Context(net.as_array(), (net.in_c, net.in_h, net.in_w))
        s0 = probe.plan_swaps(k, 1 << 40, mode)
        probe.close()
        budget = s0["static_bytes"] + int((s0["layer_peak_bytes"] - s0["static_bytes"]) * 1.5)
        host = s0["host_bytes"] + 64 * MiB
    else:
        net, k, mode, budget = S.resnet50(), 64, b.PLAN_DYNAMIC, 3 * GiB
        host = 6 * GiB
    ctx = b.Context(net.as_array(), (net.in_c, net.in_h, net.in_w), pool_bytes=budget, host_bytes=host)
    ctx.set_weights(S.init_params(net))
    ctx.calibrate([k])
    plan = ctx.plan_swaps(k, budget, mode)
    assert plan["n_swapped"] > 0
    img, lab = S.make_batch(net, k, 0)
    img = torch.from_numpy(img).cuda()
    ctx.train_step(img, lab, 0.1)
    ctx.set_profiling(1)
    ctx.train_step(img, lab, 0.1)
    ctx.set_profiling(0)
    obs = ctx.timeline(observed=True)
    assert len(obs) == plan["n_instr"]
    assert V.dependency_violations(ctx, obs) == []
    rep = V.compare_timelines(ctx)
    mem = V.memory_curve(ctx, observed=True, points=400)
    assert mem["peak_dynamic_bytes"] <= budget - plan["static_bytes"]
    assert mem["series"][-1]["bytes_out"] == mem["series"][-1]["bytes_in"] == plan["bytes_swapped"]
    if case == "resnet50_dynamic":
        assert rep["observed"]["t_iter"] == pytest.approx(rep["predicted"]["t_iter"], rel=0.15)
        curves = V.throughput_curves(ctx, net)
        assert curves["conv_fwd_3x3"][0]["tflops"] > 20 and curves["bn_fwd"][0]["gbs"] > 500
    ctx.close()
