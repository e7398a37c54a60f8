"""Pins for the whole training step of the CPU oracle: central finite
differences of the double build, a cross-check against torch's CPU autograd
(library routine, never the oracle itself), float-vs-double agreement, the SGD
update rule, and the seeded input recipe."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle as O
import synth as S

NETS = {
    "config1_unit": lambda: S.bottleneck_unit(),                      # BASELINE configs[0]
    "mini_resnet_v1": lambda: S.resnet((1, 2), in_hw=20, classes=7, width=4),
    "mini_resnet_v15": lambda: S.resnet((2, 1), in_hw=18, classes=5, width=4, variant="v1.5"),
    "mini_resnet_basic": lambda: S.resnet((2, 1), in_hw=20, classes=6, width=4, block="basic"),
    # conv + bias + ReLU stages, 2x2 max-pools, three FC layers over the flattened map
    "mini_vgg": lambda: S.vgg(cfg=((4, 4), (6,)), in_c=3, in_hw=12, classes=5, fc=10),
}


def as64(params):
    return [p.astype(np.float64) for p in params]


def perturbed_params(net, seed=42):
    """He-normal weights, plus random gamma/beta/bias so that no gradient path is
    hidden behind an exact one or zero."""
    params = S.init_params(net, seed)
    rng = np.random.default_rng(seed)
    for i, l in enumerate(net.layers):
        if l.kind == S.BN:
            params[i] = (params[i] + 0.2 * rng.standard_normal(params[i].size)).astype(np.float32)
        if l.kind == S.FC:
            params[i][-l.cout:] = 0.1 * rng.standard_normal(l.cout)
        if l.kind == S.BIAS:
            params[i] = (0.1 * rng.standard_normal(l.cin)).astype(np.float32)
    return params


def loss_only(net, params, img, lab):
    return O.train_step(net.as_array(), (net.in_c, net.in_h, net.in_w), params, img, lab, 0.0)[0]


def torch_step(net, params, img, lab, eps=O.BN_EPS):
    """Forward/backward of the layer list with torch CPU ops in float64."""
    tp = []
    for l, p in zip(net.layers, params):
        t = torch.from_numpy(np.asarray(p, np.float64).copy())
        tp.append(t.requires_grad_(True) if t.numel() else t)
    x_in = torch.from_numpy(img.astype(np.float64))
    outs = []
    get = lambda i: x_in if i < 0 else outs[i]
    loss = None
    for l, p in zip(net.layers, tp):
        x = get(l.in0)
        if l.kind == S.CONV:
            y = F.conv2d(x, p.view(l.cout, l.cin, l.r, l.s), stride=l.stride, padding=l.pad)
        elif l.kind == S.BN:
            y = F.batch_norm(x, None, None, p[:l.cin], p[l.cin:], training=True, eps=eps)
        elif l.kind == S.RELU:
            y = F.relu(x)
        elif l.kind == S.ADD:
            y = x + get(l.in1)
        elif l.kind == S.BIAS:
            y = x + p.view(1, -1, 1, 1)
        elif l.kind == S.MAXPOOL:
            y = F.max_pool2d(x, l.r, l.stride, l.pad)
        elif l.kind == S.GAP:
            y = x.mean(dim=(2, 3))
        elif l.kind == S.FC:
            n = l.cout * l.cin
            y = x.reshape(x.shape[0], -1) @ p[:n].view(l.cout, l.cin).T + p[n:]
        elif l.kind == S.SOFTMAX_CE:
            y = F.cross_entropy(x, torch.from_numpy(lab).long())
            loss = y
        outs.append(y)
    loss.backward()
    grads = [p.grad.numpy() if p.numel() else np.zeros(0) for p in tp]
    return loss.item(), grads


@pytest.mark.parametrize("name", list(NETS))
def test_step_vs_torch_autograd(name):
    net = NETS[name]()
    params = as64(perturbed_params(net))
    img, lab = S.make_batch(net, 3)
    img = img.astype(np.float64)
    loss, newp, grads = O.train_step(net.as_array(), (net.in_c, net.in_h, net.in_w), params, img, lab, 0.1)
    tloss, tgrads = torch_step(net, params, img, lab)
    assert math.isclose(loss, tloss, rel_tol=1e-12)
    for i, (g, tg) in enumerate(zip(grads, tgrads)):
        if g.size:
            scale = max(np.abs(tg).max(), 1e-30)
            assert np.abs(g - tg).max() <= 1e-9 * scale, f"layer {i} ({S.KIND_NAMES[net.layers[i].kind]})"
    # SGD: theta <- theta - lr * grad, with the loss taken at the pre-update weights
    for p, g, q in zip(params, grads, newp):
        np.testing.assert_allclose(q, p - 0.1 * g, rtol=0, atol=1e-15)


@pytest.mark.parametrize("name", list(NETS))
def test_step_central_finite_differences(name):
    """h = 1e-5, >= 64 sampled coordinates per parameter tensor (all, if fewer)."""
    net = NETS[name]()
    params = as64(perturbed_params(net))
    img, lab = S.make_batch(net, 2)
    img = img.astype(np.float64)
    _, _, grads = O.train_step(net.as_array(), (net.in_c, net.in_h, net.in_w), params, img, lab, 0.0)
    rng = np.random.default_rng(3)
    h = 1e-5
    for i, g in enumerate(grads):
        if not g.size:
            continue
        idx = rng.choice(g.size, size=min(64, g.size), replace=False)
        fd = np.zeros(idx.size)
        for j, e in enumerate(idx):
            keep = params[i][e]
            params[i][e] = keep + h
            lp = loss_only(net, params, img, lab)
            params[i][e] = keep - h
            lm = loss_only(net, params, img, lab)
            params[i][e] = keep
            fd[j] = (lp - lm) / (2 * h)
        err = np.linalg.norm(fd - g[idx]) / max(np.linalg.norm(g[idx]), 1e-30)
        assert err <= 1e-6, f"layer {i} ({S.KIND_NAMES[net.layers[i].kind]}): rel err {err:.2e}"


@pytest.mark.parametrize("name", list(NETS))
def test_float_build_agrees_with_double_build(name):
    net = NETS[name]()
    params = perturbed_params(net)
    img, lab = S.make_batch(net, 4)
    l32, p32, g32 = O.train_step(net.as_array(), (net.in_c, net.in_h, net.in_w), params, img, lab, 0.1)
    l64, p64, g64 = O.train_step(net.as_array(), (net.in_c, net.in_h, net.in_w), as64(params),
                                 img.astype(np.float64), lab, 0.1)
    assert abs(l32 - l64) <= 1e-5 * abs(l64)
    for i, (a, b) in enumerate(zip(g32, g64)):
        if a.size:
            assert np.linalg.norm(a - b) <= 1e-5 * np.linalg.norm(b), f"layer {i}"
    for a, b in zip(p32, p64):
        if a.size:
            assert np.linalg.norm(a - b) <= 1e-5 * np.linalg.norm(b)


def test_maxpool_tie_break_does_not_change_weight_gradients():
    """Ties in the stem's max-pool occur only among zeros of the preceding ReLU,
    whose own gradient mask is zero, so any tie-break gives the same weight
    gradients: shifting the images so that many ReLU outputs are zero must still
    agree with torch (which breaks ties its own way)."""
    net = NETS["mini_resnet_v1"]()
    params = as64(perturbed_params(net))
    # a strongly negative beta in the stem BN makes most stem ReLU outputs exactly zero
    params[1][net.layers[1].cin:] = -1.5
    img, lab = S.make_batch(net, 2)
    img = img.astype(np.float64)
    loss, _, grads = O.train_step(net.as_array(), (net.in_c, net.in_h, net.in_w), params, img, lab, 0.0)
    tloss, tgrads = torch_step(net, params, img, lab)
    assert math.isclose(loss, tloss, rel_tol=1e-12)
    for g, tg in zip(grads, tgrads):
        if g.size:
            assert np.abs(g - tg).max() <= 1e-9 * max(np.abs(tg).max(), 1e-30)


def test_malformed_spec_is_rejected():
    net = S.bottleneck_unit()
    arr = net.as_array().copy()
    arr[0, 3] = 63      # cin of the first conv no longer matches the input
    with pytest.raises(ValueError):
        O.train_step(arr, (64, 16, 16), S.init_params(net), *S.make_batch(net, 2), 0.1)


# ------------------------------------------------------------- input recipe
def test_splitmix64_known_values():
    """First outputs of splitmix64 for seed 0 (values published with the reference
    implementation of the generator by its author)."""
    v = S.splitmix64(0, 0, 3)
    assert [int(x) for x in v] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_rng_is_counter_based_and_normal():
    a = S.normal(5, 1001)
    b = S.normal(5, 400)
    np.testing.assert_array_equal(a[:400], b)
    z = S.normal(11, 200000)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01
    assert abs(np.mean(z ** 3)) < 0.03 and abs(np.mean(z ** 4) - 3) < 0.06
    lab = S.labels_uniform(3, 10000, 10)
    assert lab.min() == 0 and lab.max() == 9 and np.bincount(lab).min() > 800


def test_resnet_specs_match_published_parameter_counts():
    """Bottleneck ResNet-50/101/152 parameter counts (conv + BN affine + FC), the
    figures quoted for these networks everywhere: 25.56 M / 44.55 M / 60.19 M."""
    assert S.param_count(S.resnet50()) == 25_557_032
    assert S.param_count(S.resnet101()) == 44_549_160
    assert S.param_count(S.resnet152()) == 60_192_808
    # the basic-block networks (two 3x3 convolutions per block): 11.69 M / 21.80 M
    assert S.param_count(S.resnet18()) == 11_689_512
    assert S.param_count(S.resnet34()) == 21_797_672
    # configuration D of the VGG paper ("138M" in its table of parameter counts)
    assert S.param_count(S.vgg16()) == 138_357_544
    net = S.bottleneck_unit()
    assert [l.kind for l in net.layers][:11] == [S.CONV, S.BN, S.RELU, S.CONV, S.BN, S.RELU,
                                                  S.CONV, S.BN, S.ADD, S.RELU, S.GAP]
