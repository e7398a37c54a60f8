"""GPU parity of whole training steps of the full-depth networks of the baseline's
configurations (ResNet-50 at minibatch 32, ResNet-101 at 32, ResNet-152 at 16; 224 x 224 inputs)
against the CPU oracle, through the C ABI.

What can be held to 1e-4 at this depth and what cannot.

 * The loss can (end to end).
 * Every layer's forward output can, given the same input: in the second iteration below
   each stored output is captured before it is overwritten with the oracle's, so it is the
   library's result on the oracle's input.
 * Every gradient tensor and every updated weight tensor can, given the same discrete
   decisions.  A ReLU passes the gradient where its stored output is positive; of the ~3e8
   stored outputs a few per million lie within rounding of zero and the two sides decide
   those differently; at random initialisation each such decision moves the gradients of all
   earlier layers visibly.  A floating-point value that decides a discrete outcome has to be
   the same value on both sides before outcomes can be compared, so the gradients are taken
   from an iteration in which the library's stored activations are overwritten with the
   oracle's right after each is produced (acc_inject_output): masks and max-pool winners
   then come from the same numbers.
 * End-to-end activations and the gradients of an independent pass cannot, for ANY fp32
   implementation: these networks at random initialisation amplify a perturbation of 3e-8
   per stored tensor (rounding to fp32, the only difference between the oracle with fp32
   storage and the oracle in double) to 3e-4 at the last ReLU of ResNet-152 and to 0.4-1 %
   in the gradient tensors.  Against that yardstick the library is held to a fixed multiple
   of the fp32-storage oracle's own distance from the exact (double) step: 16 x (+1e-4) for
   activations - fp32 accumulation over up to 4608 products leaves up to 2e-6 per layer,
   measured per layer below, against 3.5e-8 of storage rounding; accumulated, 6-9 x is
   observed - and 4 x (+1e-3) for gradient tensors (decisions that differ grow with the
   square root of that)."""
import time

import numpy as np
import pytest
import torch

import oracle as O
import synth as S

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]

TOL = 1e-4
MiB = 1 << 20


def B():
    from paper_1901_06773_amd import binding
    return binding


def shapes_of(net):
    """(c, h, w) of every layer's output."""
    out = []
    for l in net.layers:
        c, h, w = (net.in_c, net.in_h, net.in_w) if l.in0 < 0 else out[l.in0]
        if l.kind == S.CONV:
            out.append((l.cout, O.out_dim(h, l.r, l.stride, l.pad), O.out_dim(w, l.s, l.stride, l.pad)))
        elif l.kind == S.MAXPOOL:
            out.append((c, O.out_dim(h, l.r, l.stride, l.pad), O.out_dim(w, l.s, l.stride, l.pad)))
        elif l.kind == S.GAP:
            out.append((c, 1, 1))
        elif l.kind == S.FC:
            out.append((l.cout, 1, 1))
        elif l.kind == S.SOFTMAX_CE:
            out.append((1, 1, 1))
        else:
            out.append((c, h, w))
    return out


def rel(a, r):
    a = np.asarray(a, np.float64).ravel(); r = np.asarray(r, np.float64).ravel()
    return (np.linalg.norm(a - r) / max(np.linalg.norm(r), 1e-300),
            np.abs(a - r).max() / max(np.abs(r).max(), 1e-300))


def full_net_case(name, k):
    b = B()
    net = getattr(S, name)()
    chw = (net.in_c, net.in_h, net.in_w)
    params = S.init_params(net)
    img, lab = S.make_batch(net, k, 0)
    shp = shapes_of(net)
    # stored outputs: convolutions (inputs of the batch norms), ReLU outputs of bn(+add)+relu, pooling, FC
    stored = [i for i, l in enumerate(net.layers) if l.kind in (S.CONV, S.RELU, S.MAXPOOL, S.GAP, S.FC)]
    sizes = {i: k * int(np.prod(shp[i])) for i in stored}
    t0 = time.time()
    o_loss, o_w, o_g, o_acts = O.train_step(net.as_array(), chw, params, img, lab, 0.1, want_acts=stored, act_sizes=sizes)
    t1 = time.time()
    x_loss, _, x_g, x_acts = O.train_step(net.as_array(), chw, [p.astype(np.float64) for p in params],
                                          img.astype(np.float64), lab, 0.1, want_acts=stored, act_sizes=sizes)
    print(f"\n{name} k={k}: oracle step {t1 - t0:.1f} s, in double {time.time() - t1:.1f} s, loss {o_loss:.6f} / {x_loss:.6f}")

    probe = b.Context(net.as_array(), chw)
    pool = int(probe.plan_swaps(k, 1 << 40, b.PLAN_NONE)["peak_bytes"] * 1.05) + 64 * MiB
    probe.close()
    ctx = b.Context(net.as_array(), chw, pool_bytes=pool, host_bytes=MiB)
    ctx.set_weights(params)
    ctx.plan_swaps(k, pool, b.PLAN_NONE)
    caps = ctx.capture_outputs(stored, shp, k)
    pinned = torch.from_numpy(img).pin_memory()

    # ---- independent step: loss and every stored activation
    loss = ctx.train_step(pinned, lab, 0.1)
    g_free = ctx.get_grads()
    assert abs(loss - o_loss) <= TOL * abs(o_loss), (loss, o_loss)
    worst_l2 = worst_ratio = 0.0
    first_over = None
    flips = total = 0
    for i in stored:
        c, h, w = shp[i]
        got = caps[i].numpy().transpose(0, 3, 1, 2)
        ref = o_acts[i].reshape(k, c, h, w)
        exact = x_acts[i].reshape(k, c, h, w)
        assert np.isfinite(got).all(), f"activation of layer {i}"
        e_gpu, m_gpu = rel(got, exact)
        e_o32, m_o32 = rel(ref, exact)
        worst_l2 = max(worst_l2, e_gpu)
        worst_ratio = max(worst_ratio, e_gpu / max(e_o32, 1e-5))
        if first_over is None and e_gpu > TOL:
            first_over = (i, e_gpu, e_o32)
        what = f"activation of layer {i} ({S.KIND_NAMES[net.layers[i].kind]})"
        assert e_gpu <= TOL + 16 * e_o32, f"{what}: rel l2 {e_gpu:.3e}, fp32-storage oracle {e_o32:.3e}"
        assert m_gpu <= TOL + 16 * m_o32, f"{what}: max norm {m_gpu:.3e}, fp32-storage oracle {m_o32:.3e}"
        if net.layers[i].kind == S.RELU:
            flips += int(((got > 0) != (ref > 0)).sum()); total += got.size
    last = stored[-3]
    print(f"  loss rel. error {abs(loss - o_loss) / abs(o_loss):.2e}; {len(stored)} stored activations end to end against the "
          f"exact step: worst rel l2 {worst_l2:.2e} (fp32-storage oracle at the last ReLU: "
          f"{rel(o_acts[last], x_acts[last])[0]:.2e}), worst ratio to the oracle's own distance {worst_ratio:.1f}; first beyond "
          f"1e-4: {'none' if first_over is None else 'layer %d (gpu %.2e, oracle %.2e)' % first_over}")
    print(f"  ReLU outputs whose sign differs between the two sides: {flips} of {total} ({flips / total:.1e})")

    # ---- second iteration on the oracle's activations: every gradient and updated weight tensor
    ctx.set_weights(params)
    inject = [i for i in stored if net.layers[i].kind in (S.CONV, S.RELU, S.MAXPOOL)]
    ctx.inject_outputs({i: o_acts[i].reshape(k, *shp[i]).transpose(0, 2, 3, 1) for i in inject})
    loss2 = ctx.train_step(pinned, lab, 0.1)
    assert abs(loss2 - o_loss) <= TOL * abs(o_loss)
    grads, weights = ctx.get_grads(), ctx.get_weights()
    ctx.stop_captures()
    ctx.close()
    # each layer on the oracle's input (captured before the injection overwrote it)
    worst = 0.0
    for i in stored:
        c, h, w = shp[i]
        e2, em = rel(caps[i].numpy().transpose(0, 3, 1, 2), o_acts[i].reshape(k, c, h, w))
        worst = max(worst, e2, em)
        assert e2 <= TOL and em <= TOL, f"layer {i} ({S.KIND_NAMES[net.layers[i].kind]}) on the oracle's input: {e2:.3e} / {em:.3e}"
    print(f"  every layer's forward output on the oracle's input: worst {worst:.2e} (l2 or max norm)")
    worst = 0.0
    for i, (a, r) in enumerate(zip(grads, o_g)):
        if r.size:
            e2, em = rel(a, r)
            worst = max(worst, e2, em)
            assert np.isfinite(a).all() and e2 <= TOL and em <= TOL, \
                f"gradient of layer {i} ({S.KIND_NAMES[net.layers[i].kind]}): rel l2 {e2:.3e}, max norm {em:.3e}"
    for i, (a, r) in enumerate(zip(weights, o_w)):
        if r.size:
            e2, em = rel(a, r)
            assert e2 <= TOL and em <= TOL, f"updated weights of layer {i}: rel l2 {e2:.3e}, max norm {em:.3e}"
    print(f"  same decisions on both sides: worst gradient tensor {worst:.2e} (l2 or max norm) of {sum(1 for r in o_g if r.size)}")

    # ---- the independent step's gradients: how far, against the exact step
    ratios, e_gs, e_os = [], [], []
    for i, (a, r32, r64) in enumerate(zip(g_free, o_g, x_g)):
        if not r64.size:
            continue
        n64 = np.linalg.norm(r64)
        e_gpu = np.linalg.norm(np.asarray(a, np.float64) - r64) / n64
        e_o32 = np.linalg.norm(r32.astype(np.float64) - r64) / n64
        e_gs.append(e_gpu); e_os.append(e_o32); ratios.append(e_gpu / max(e_o32, 1e-4))
        assert np.isfinite(e_gpu) and e_gpu <= 4.0 * e_o32 + 1e-3, \
            f"layer {i} ({S.KIND_NAMES[net.layers[i].kind]}): gpu {e_gpu:.3e}, fp32-storage oracle {e_o32:.3e}"
    print(f"  independent step against the exact one, per gradient tensor: gpu median {np.median(e_gs):.2e} "
          f"max {max(e_gs):.2e}; fp32-storage oracle median {np.median(e_os):.2e} max {max(e_os):.2e}; "
          f"worst ratio {max(ratios):.2f}")


def test_resnet50_minibatch_32_against_the_oracle():
    """configs[1]."""
    full_net_case("resnet50", 32)


def test_resnet101_minibatch_32_against_the_oracle():
    """The network of configs[2] at the largest minibatch the oracle finishes within a minute."""
    full_net_case("resnet101", 32)


def test_resnet152_minibatch_16_against_the_oracle():
    """The benchmark's network (configs[3])."""
    full_net_case("resnet152", 16)
