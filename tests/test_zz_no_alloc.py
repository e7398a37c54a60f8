"""acc_op_bn_fwd_noalloc (the entry point for callers that cannot allocate: its reduction
workspace is a device array built into the library) against acc_op_bn_fwd with a
caller-supplied workspace: same kernels, so every output bit must agree; two calls in a row,
the second on a smaller input, so that what the first call left in the shared array is there
when the second runs.  The existing entry point is itself held to the oracle in
test_gpu_ops.py; the first call here is checked against the oracle as well."""
import numpy as np
import pytest
import torch

import oracle as O
import synth as S

pytestmark = pytest.mark.gpu


def B():
    from paper_1901_06773_amd import binding
    return binding


def rnd(seed, *shape):
    return S.normal(seed, int(np.prod(shape))).astype(np.float32).reshape(shape)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def both_ways(n, c, h, w, variant, seed):
    b = B()
    x = rnd(seed, n, h, w, c) * np.float32(1.3) + np.float32(0.2)          # NHWC
    gamma = (1.0 + 0.2 * rnd(seed + 1, c)).astype(np.float32)
    beta = (0.1 * rnd(seed + 2, c)).astype(np.float32)
    res = rnd(seed + 3, n, h, w, c) if variant == "add_relu" else None
    relu = variant != "plain"
    xd, gd, bd = dev(x), dev(gamma), dev(beta)
    rd = dev(res) if res is not None else None
    out = {}
    for which in ("workspace", "noalloc"):
        y = torch.full_like(xd, float("nan"))
        mean = torch.full((c,), float("nan"), device="cuda")
        istd = torch.full((c,), float("nan"), device="cuda")
        if which == "workspace":
            ws = torch.empty(b.op_bn_workspace(c), dtype=torch.uint8, device="cuda")
            b.op_bn_fwd(xd, gd, bd, rd, y, mean, istd, relu, O.BN_EPS, ws)
        else:
            b.op_bn_fwd_noalloc(xd, gd, bd, rd, y, mean, istd, relu, O.BN_EPS)
        torch.cuda.synchronize()
        out[which] = (y.cpu().numpy(), mean.cpu().numpy(), istd.cpu().numpy())
    for a, r, what in zip(out["noalloc"], out["workspace"], ("y", "mean", "istd")):
        assert np.isfinite(a).all(), what
        assert np.array_equal(a.view(np.uint32), r.view(np.uint32)), f"{what} differs ({n},{c},{h},{w}) {variant}"
    return x, gamma, beta, res, relu, out["noalloc"]


def test_two_calls_in_a_row_match_the_entry_point_with_a_workspace():
    # first call: every column slice, hundreds of row slabs
    x, gamma, beta, res, relu, (y, mean, istd) = both_ways(9, 2048, 14, 14, "add_relu", 11)
    xn = np.ascontiguousarray(x.transpose(0, 3, 1, 2))
    bn, o_mean, o_istd = O.bn_fwd(xn, gamma, beta, O.BN_EPS)
    ref = O.relu_fwd(bn + np.ascontiguousarray(res.transpose(0, 3, 1, 2)))
    got = y.transpose(0, 3, 1, 2).astype(np.float64)
    assert np.linalg.norm(got - ref) <= 1e-4 * np.linalg.norm(ref)
    assert np.abs(mean - o_mean).max() <= 1e-5 * np.abs(o_mean).max()
    assert np.abs(istd - o_istd).max() <= 1e-5 * np.abs(o_istd).max()
    # second call: fewer channels, fewer rows (ragged), another variant; the array still holds
    # the first call's partial sums beyond what this one writes
    both_ways(3, 64, 7, 9, "relu", 21)
    # third: bf16-free single-slab case
    both_ways(1, 12, 1, 1, "plain", 31)


def test_sizes_beyond_the_built_in_workspace_are_refused():
    b = B()
    c = 2048 + 4
    x = torch.zeros(2, 1, 1, c, device="cuda")
    v = torch.zeros(c, device="cuda")
    with pytest.raises(b.AccError) as e:
        b.op_bn_fwd_noalloc(x, v, v, None, torch.zeros_like(x), v.clone(), v.clone(), False, 1e-5)
    assert e.value.status == b.ACC_EINVAL and "ACC_NOALLOC_BN_MAX_C" in str(e.value)
