"""Pins for the layer functions of the CPU oracle: each is checked against
something other than itself (brute force, a library special case, a closed form,
an adjoint identity), chosen so that a dropped term, a wrong sign or index, or a
transposed operand fails at least one of them."""
import itertools
import math

import numpy as np
import pytest
import scipy.signal
import torch
import torch.nn.functional as F

import oracle as O

RNG = np.random.default_rng(7)


def rnd(*shape, dtype=np.float64):
    return RNG.standard_normal(shape).astype(dtype)


CONV_CASES = [  # n, cin, h, w, cout, r, stride, pad
    (2, 3, 7, 7, 4, 3, 1, 1),
    (2, 3, 8, 9, 4, 3, 2, 1),
    (1, 2, 9, 9, 3, 1, 2, 0),      # odd size, strided 1x1
    (2, 3, 11, 10, 2, 7, 2, 3),    # stem-like
    (1, 4, 5, 5, 4, 1, 1, 0),
    (2, 2, 6, 6, 3, 3, 2, 0),
    (1, 1, 7, 8, 1, 5, 3, 2),
]


def brute_conv(x, w, stride, pad):
    """Definition of cross-correlation, one output element at a time, Python loops."""
    n, cin, h, wd = x.shape
    cout, _, r, s = w.shape
    ho, wo = (h + 2 * pad - r) // stride + 1, (wd + 2 * pad - s) // stride + 1
    y = np.zeros((n, cout, ho, wo))
    for i, co, oy, ox in itertools.product(range(n), range(cout), range(ho), range(wo)):
        acc = 0.0
        for ci, kr, kt in itertools.product(range(cin), range(r), range(s)):
            iy, ix = oy * stride + kr - pad, ox * stride + kt - pad
            if 0 <= iy < h and 0 <= ix < wd:
                acc += x[i, ci, iy, ix] * w[co, ci, kr, kt]
        y[i, co, oy, ox] = acc
    return y


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_fwd_brute_force(case):
    n, cin, h, wd, cout, r, stride, pad = case
    x, w = rnd(n, cin, h, wd), rnd(cout, cin, r, r)
    np.testing.assert_allclose(O.conv_fwd(x, w, stride, pad), brute_conv(x, w, stride, pad),
                               rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_fwd_vs_torch_library(case):
    n, cin, h, wd, cout, r, stride, pad = case
    x, w = rnd(n, cin, h, wd), rnd(cout, cin, r, r)
    ref = F.conv2d(torch.from_numpy(x), torch.from_numpy(w), stride=stride, padding=pad).numpy()
    np.testing.assert_allclose(O.conv_fwd(x, w, stride, pad), ref, rtol=1e-11, atol=1e-11)


def test_conv_1x1_is_matmul():
    x, w = rnd(3, 5, 4, 6), rnd(7, 5, 1, 1)
    ref = np.einsum("oc,nchw->nohw", w[:, :, 0, 0], x)
    np.testing.assert_allclose(O.conv_fwd(x, w), ref, rtol=1e-12, atol=1e-12)


def test_conv_full_window_is_fc():
    x, w = rnd(3, 4, 5, 5), rnd(6, 4, 5, 5)
    ref = x.reshape(3, -1) @ w.reshape(6, -1).T
    np.testing.assert_allclose(O.conv_fwd(x, w).reshape(3, 6), ref, rtol=1e-12, atol=1e-12)


def test_conv_delta_kernel_shifts():
    x = rnd(1, 1, 6, 7)
    for kr, kt in itertools.product(range(3), range(3)):
        w = np.zeros((1, 1, 3, 3)); w[0, 0, kr, kt] = 1.0
        y = O.conv_fwd(x, w, 1, 1)
        ref = np.zeros_like(x)
        for oy, ox in itertools.product(range(6), range(7)):
            iy, ix = oy + kr - 1, ox + kt - 1
            if 0 <= iy < 6 and 0 <= ix < 7:
                ref[0, 0, oy, ox] = x[0, 0, iy, ix]
        np.testing.assert_array_equal(y, ref)


def test_conv_single_channel_is_correlate2d():
    x, w = rnd(1, 1, 9, 8), rnd(1, 1, 3, 3)
    ref = scipy.signal.correlate2d(x[0, 0], w[0, 0], mode="valid")
    np.testing.assert_allclose(O.conv_fwd(x, w)[0, 0], ref, rtol=1e-12, atol=1e-12)
    ref_same = scipy.signal.correlate2d(x[0, 0], w[0, 0], mode="same")
    np.testing.assert_allclose(O.conv_fwd(x, w, 1, 1)[0, 0], ref_same, rtol=1e-12, atol=1e-12)


def test_conv_linearity():
    x1, x2, w1, w2 = rnd(2, 3, 6, 6), rnd(2, 3, 6, 6), rnd(4, 3, 3, 3), rnd(4, 3, 3, 3)
    a, b = 0.7, -1.3
    np.testing.assert_allclose(O.conv_fwd(a * x1 + b * x2, w1, 2, 1),
                               a * O.conv_fwd(x1, w1, 2, 1) + b * O.conv_fwd(x2, w1, 2, 1), atol=1e-12)
    np.testing.assert_allclose(O.conv_fwd(x1, a * w1 + b * w2, 2, 1),
                               a * O.conv_fwd(x1, w1, 2, 1) + b * O.conv_fwd(x1, w2, 2, 1), atol=1e-12)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_adjoint_identities(case):
    """<conv(x,w),dy> = <x,dgrad(dy,w)> = <w,wgrad(x,dy)>: exact up to rounding."""
    n, cin, h, wd, cout, r, stride, pad = case
    x, w = rnd(n, cin, h, wd), rnd(cout, cin, r, r)
    y = O.conv_fwd(x, w, stride, pad)
    dy = rnd(*y.shape)
    lhs = float(np.sum(y * dy))
    dx = O.conv_dgrad(dy, w, x.shape, stride, pad)
    dw = O.conv_wgrad(x, dy, w.shape, stride, pad)
    assert math.isclose(lhs, float(np.sum(x * dx)), rel_tol=1e-11, abs_tol=1e-11)
    assert math.isclose(lhs, float(np.sum(w * dw)), rel_tol=1e-11, abs_tol=1e-11)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_grads_vs_torch_autograd(case):
    n, cin, h, wd, cout, r, stride, pad = case
    x, w = rnd(n, cin, h, wd), rnd(cout, cin, r, r)
    tx = torch.from_numpy(x).requires_grad_(True)
    tw = torch.from_numpy(w).requires_grad_(True)
    ty = F.conv2d(tx, tw, stride=stride, padding=pad)
    dy = rnd(*ty.shape)
    ty.backward(torch.from_numpy(dy))
    np.testing.assert_allclose(O.conv_dgrad(dy, w, x.shape, stride, pad), tx.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(O.conv_wgrad(x, dy, w.shape, stride, pad), tw.grad.numpy(), rtol=1e-11, atol=1e-11)


def test_conv_f32_rounds_once():
    """float storage with double accumulation: within half an ulp of the f64 result."""
    x, w = rnd(2, 16, 8, 8, dtype=np.float32), rnd(8, 16, 3, 3, dtype=np.float32)
    y32 = O.conv_fwd(x, w, 1, 1)
    y64 = O.conv_fwd(x.astype(np.float64), w.astype(np.float64), 1, 1)
    np.testing.assert_array_equal(y32, y64.astype(np.float32))


# ----------------------------------------------------------------- batch norm
def test_bn_fwd_closed_form_moments():
    x = rnd(4, 5, 3, 3) * 2.5 + 1.0
    gamma, beta = rnd(5), rnd(5)
    eps = 1e-5
    y, mean, istd = O.bn_fwd(x, gamma, beta, eps)
    var = x.var(axis=(0, 2, 3))          # numpy's default is the biased variance
    np.testing.assert_allclose(mean, x.mean(axis=(0, 2, 3)), rtol=1e-13)
    np.testing.assert_allclose(istd, 1 / np.sqrt(var + eps), rtol=1e-13)
    np.testing.assert_allclose(y.mean(axis=(0, 2, 3)), beta, atol=1e-13)
    np.testing.assert_allclose(y.var(axis=(0, 2, 3)), gamma ** 2 * var / (var + eps), rtol=1e-12)


def test_bn_single_element_gives_beta():
    x = rnd(1, 3, 1, 1)
    gamma, beta = rnd(3), rnd(3)
    y, mean, istd = O.bn_fwd(x, gamma, beta, 1e-5)
    np.testing.assert_allclose(y[0, :, 0, 0], beta, atol=1e-15)
    np.testing.assert_allclose(istd, 1 / math.sqrt(1e-5), rtol=1e-14)


def test_bn_vs_torch_library_and_autograd():
    x, gamma, beta = rnd(3, 4, 5, 2) + 0.5, rnd(4), rnd(4)
    tx = torch.from_numpy(x).requires_grad_(True)
    tg = torch.from_numpy(gamma).requires_grad_(True)
    tb = torch.from_numpy(beta).requires_grad_(True)
    ty = F.batch_norm(tx, None, None, tg, tb, training=True, eps=1e-5)
    y, mean, istd = O.bn_fwd(x, gamma, beta, 1e-5)
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-11, atol=1e-11)
    dy = rnd(*x.shape)
    ty.backward(torch.from_numpy(dy))
    dx, dg, db = O.bn_bwd(x, dy, gamma, mean, istd)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(dg, tg.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-11, atol=1e-11)


def test_bn_bwd_orthogonality():
    """dx sums to zero in every channel; its product with xhat sums to the closed form
    gamma*istd*dgamma*eps*istd^2 (zero only for eps = 0, since sum xhat^2 = m*var/(var+eps))."""
    x, gamma, dy = rnd(4, 3, 4, 4), rnd(3), rnd(4, 3, 4, 4)
    _, mean, istd = O.bn_fwd(x, gamma, np.zeros(3), 1e-5)
    dx, dg, db = O.bn_bwd(x, dy, gamma, mean, istd)
    xhat = (x - mean[None, :, None, None]) * istd[None, :, None, None]
    np.testing.assert_allclose(dx.sum(axis=(0, 2, 3)), 0, atol=1e-12)
    np.testing.assert_allclose((dx * xhat).sum(axis=(0, 2, 3)), gamma * istd * dg * 1e-5 * istd ** 2,
                               rtol=1e-9, atol=1e-13)
    np.testing.assert_allclose(db, dy.sum(axis=(0, 2, 3)), rtol=1e-13)
    np.testing.assert_allclose(dg, (dy * xhat).sum(axis=(0, 2, 3)), rtol=1e-12)


# ---------------------------------------------------------- ReLU, pooling, FC
def test_relu():
    x = np.array([-1.0, 0.0, 2.0, -0.0, 3.5])
    y = O.relu_fwd(x)
    np.testing.assert_array_equal(y, [0, 0, 2, 0, 3.5])
    np.testing.assert_array_equal(O.relu_bwd(y, np.ones(5)), [0, 0, 1, 0, 1])   # ReLU'(0) = 0


def test_maxpool_brute_force_and_first_max_tie_break():
    x = rnd(2, 3, 7, 8)
    x[0, 0, 0:3, 0:3] = 5.0          # a window full of ties: first in scan order wins
    y, arg = O.maxpool_fwd(x, 3, 2, 1)
    n, c, h, wd = x.shape
    for i, ch, oy, ox in itertools.product(range(n), range(c), range(y.shape[2]), range(y.shape[3])):
        best, where = None, None
        for kr, kt in itertools.product(range(3), range(3)):
            iy, ix = oy * 2 + kr - 1, ox * 2 + kt - 1
            if 0 <= iy < h and 0 <= ix < wd and (best is None or x[i, ch, iy, ix] > best):
                best, where = x[i, ch, iy, ix], iy * wd + ix
        assert y[i, ch, oy, ox] == best and arg[i, ch, oy, ox] == where
    ty = F.max_pool2d(torch.from_numpy(x), 3, 2, 1).numpy()
    np.testing.assert_array_equal(y, ty)


def test_maxpool_bwd_vs_torch_autograd():
    x = rnd(2, 2, 9, 9)             # continuous values: no ties
    tx = torch.from_numpy(x).requires_grad_(True)
    ty = F.max_pool2d(tx, 3, 2, 1)
    dy = rnd(*ty.shape)
    ty.backward(torch.from_numpy(dy))
    _, arg = O.maxpool_fwd(x, 3, 2, 1)
    dx = O.maxpool_bwd(dy, arg, x.shape)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-13, atol=1e-13)
    assert math.isclose(dx.sum(), dy.sum(), rel_tol=1e-12)


def test_gap_and_fc():
    x = rnd(3, 4, 5, 5)
    np.testing.assert_allclose(O.gap_fwd(x), x.mean(axis=(2, 3)), rtol=1e-13)
    dy = rnd(3, 4)
    np.testing.assert_allclose(O.gap_bwd(dy, x.shape), np.broadcast_to(dy[:, :, None, None] / 25, x.shape), rtol=1e-13)
    xin, W, b = rnd(3, 6), rnd(5, 6), rnd(5)
    param = np.concatenate([W.ravel(), b])
    np.testing.assert_allclose(O.fc_fwd(xin, param, 5), xin @ W.T + b, rtol=1e-12, atol=1e-12)
    dz = rnd(3, 5)
    dx, dparam = O.fc_bwd(xin, param, dz)
    np.testing.assert_allclose(dx, dz @ W, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dparam[:30].reshape(5, 6), dz.T @ xin, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dparam[30:], dz.sum(axis=0), rtol=1e-12, atol=1e-12)


# ----------------------------------------------------------------- softmax-CE
@pytest.mark.parametrize("classes", [10, 1000])
def test_softmax_ce_zero_logits_is_log_classes(classes):
    z = np.zeros((4, classes))
    loss, dz = O.softmax_ce(z, np.arange(4) % classes)
    assert math.isclose(loss, math.log(classes), rel_tol=1e-14)
    np.testing.assert_allclose(dz.sum(axis=1), 0, atol=1e-15)


def test_softmax_ce_shift_invariance_rowsums_and_library():
    z = rnd(5, 7) * 3
    lab = np.array([0, 6, 3, 3, 1], np.int32)
    loss, dz = O.softmax_ce(z, lab)
    loss2, dz2 = O.softmax_ce(z + 100.0, lab)
    assert math.isclose(loss, loss2, rel_tol=1e-12)
    np.testing.assert_allclose(dz, dz2, atol=1e-14)
    np.testing.assert_allclose(dz.sum(axis=1), 0, atol=1e-15)
    tz = torch.from_numpy(z).requires_grad_(True)
    tl = F.cross_entropy(tz, torch.from_numpy(lab).long())
    tl.backward()
    assert math.isclose(loss, tl.item(), rel_tol=1e-12)
    np.testing.assert_allclose(dz, tz.grad.numpy(), atol=1e-14)
    # huge logits must not overflow (max-subtracted)
    loss3, _ = O.softmax_ce(np.array([[1000.0, 0.0]]), np.array([0], np.int32))
    assert math.isclose(loss3, 0.0, abs_tol=1e-12)
