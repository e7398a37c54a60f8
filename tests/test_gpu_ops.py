"""GPU parity of the single operations (C ABI acc_op_*) against the CPU oracle,
element by element, on seeded inputs that span several tiles and a ragged tail.

Tolerance (fp32 MFMA / fp32 vector arithmetic against the oracle's double
accumulation): ||gpu - oracle||_2 <= 1e-4 ||oracle||_2 and
max|gpu - oracle| <= 1e-4 max|oracle| per tensor."""
import numpy as np
import pytest
import torch

import oracle as O
import synth as S

pytestmark = pytest.mark.gpu

TOL = 1e-4


def B():
    from paper_1901_06773_amd import binding
    return binding


def close(gpu: np.ndarray, ref: np.ndarray, what: str, tol: float = TOL):
    gpu = gpu.astype(np.float64); ref = ref.astype(np.float64)
    assert gpu.shape == ref.shape, what
    assert np.isfinite(gpu).all(), f"{what}: non-finite values"
    nr = np.linalg.norm(ref)
    assert np.linalg.norm(gpu - ref) <= tol * max(nr, 1e-30), \
        f"{what}: rel l2 {np.linalg.norm(gpu - ref) / max(nr, 1e-30):.3e}"
    assert np.abs(gpu - ref).max() <= tol * max(np.abs(ref).max(), 1e-30), \
        f"{what}: max abs {np.abs(gpu - ref).max():.3e} vs scale {np.abs(ref).max():.3e}"


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def nhwc(a):   # NCHW numpy -> NHWC numpy
    return np.ascontiguousarray(a.transpose(0, 2, 3, 1))


def nchw(a):
    return np.ascontiguousarray(a.transpose(0, 3, 1, 2))


def ohwi(w):   # OIHW -> OHWI
    return np.ascontiguousarray(w.transpose(0, 2, 3, 1))


def oihw(w):
    return np.ascontiguousarray(w.transpose(0, 3, 1, 2))


def rnd(seed, *shape):
    return S.normal(seed, int(np.prod(shape))).astype(np.float32).reshape(shape)


CONV_CASES = [  # n, h, w, cin, cout, r, stride, pad
    (2, 14, 14, 64, 96, 3, 1, 1),      # fast path, N tail, M = 392 (ragged over 128 and 64)
    (3, 9, 9, 128, 256, 1, 1, 0),      # 1x1, M = 243
    (2, 16, 16, 64, 128, 1, 2, 0),     # strided 1x1 (projection shortcut)
    (2, 9, 9, 32, 64, 1, 2, 0),        # strided 1x1, odd size
    (5, 28, 28, 32, 64, 3, 1, 1),      # several tiles (M = 3920)
    (2, 16, 16, 16, 16, 3, 1, 1),      # config-1 sized: per-element path
    (2, 16, 16, 64, 16, 1, 1, 0),      # fast loader with cout < 64
    (2, 12, 10, 20, 24, 3, 1, 1),      # channels not a multiple of 32, non-square image
    (1, 7, 7, 96, 40, 3, 1, 1),        # single image, ragged everything
    (2, 23, 23, 8, 16, 7, 2, 3),       # stem-like filter
    (8, 57, 55, 64, 256, 1, 1, 0),     # 1x1 expansion: 392 row tiles (ragged M) x 4, two chunks each
    (8, 57, 55, 256, 64, 1, 1, 0),     # 1x1 reduction: eight chunks; its data gradient is the expansion
    (16, 32, 32, 256, 64, 1, 1, 0),    # exactly 256 tiles of eight chunks: the last launch shape of the two-group kernel
    (1, 128, 129, 256, 64, 1, 1, 0),   # 258 tiles: the first one beyond it
    (2, 8, 8, 224, 64, 1, 1, 0),       # seven chunks: too short for two groups
    (2, 9, 7, 288, 40, 1, 1, 0),       # nine chunks in two groups (5 + 4), ragged rows and columns
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_fwd(case):
    n, h, w, cin, cout, r, stride, pad = case
    x = rnd(1, n, cin, h, w); wt = rnd(2, cout, cin, r, r) * np.float32(np.sqrt(2.0 / (cin * r * r)))
    ref = O.conv_fwd(x, wt, stride, pad)
    dx, dw = dev(nhwc(x)), dev(ohwi(wt))
    y = torch.full((n, ref.shape[2], ref.shape[3], cout), float("nan"), device="cuda")
    B().op_conv_fwd(dx, dw, y, stride, pad)
    torch.cuda.synchronize()
    close(nchw(y.cpu().numpy()), ref, f"conv_fwd {case}")


STRIDED_DGRAD_CASES = [  # data gradient cut by the residue of the dx position
    (2, 16, 16, 64, 64, 3, 2, 1),      # the down-sampling 3x3 of the basic-block / v1.5 networks
    (3, 15, 13, 32, 64, 3, 2, 1),      # odd sizes: the residue classes differ in size
    (2, 14, 14, 64, 32, 3, 2, 0),      # no padding: row and column paddings of the parts differ
    (2, 12, 12, 32, 32, 2, 2, 0),      # 2x2 stride 2: every part is a 1x1
    (2, 17, 17, 32, 32, 5, 3, 2),      # stride 3, nine parts
    (2, 16, 16, 20, 24, 3, 2, 1),      # per-element loader
    (2, 13, 13, 32, 32, 1, 3, 0),      # 1x1 stride 3 through the same split (most classes empty)
]


@pytest.mark.parametrize("case", CONV_CASES + STRIDED_DGRAD_CASES)
@pytest.mark.parametrize("accumulate", [False, True])
def test_conv_dgrad(case, accumulate):
    n, h, w, cin, cout, r, stride, pad = case
    wt = rnd(2, cout, cin, r, r) * np.float32(np.sqrt(2.0 / (cin * r * r)))
    ho, wo = O.out_dim(h, r, stride, pad), O.out_dim(w, r, stride, pad)
    dy = rnd(3, n, cout, ho, wo)
    ref = O.conv_dgrad(dy, wt, (n, cin, h, w), stride, pad)
    base = rnd(4, n, cin, h, w) if accumulate else None
    if accumulate:
        ref = (ref.astype(np.float64) + base).astype(np.float32)
    b = B()
    ws = torch.empty(max(b.op_conv_workspace(n, h, w, cin, cout, r, stride, pad), 256), dtype=torch.uint8, device="cuda")
    dxt = dev(nhwc(base)) if accumulate else torch.full((n, h, w, cin), float("nan"), device="cuda")
    b.op_conv_dgrad(dev(nhwc(dy)), dev(ohwi(wt)), dxt, stride, pad, ws, accumulate)
    torch.cuda.synchronize()
    close(nchw(dxt.cpu().numpy()), ref, f"conv_dgrad {case} acc={accumulate}")


WGRAD_CASES = CONV_CASES + [
    (16, 28, 28, 64, 64, 3, 1, 1),     # M = 12544: split over the minibatch positions
    (4, 14, 14, 256, 128, 1, 1, 0),    # 128-wide column tiles
    (8, 1, 1, 64, 10, 1, 1, 0),        # fc-shaped, cout not a multiple of 4
]


@pytest.mark.parametrize("case", WGRAD_CASES)
def test_conv_wgrad(case):
    n, h, w, cin, cout, r, stride, pad = case
    x = rnd(1, n, cin, h, w)
    ho, wo = O.out_dim(h, r, stride, pad), O.out_dim(w, r, stride, pad)
    dy = rnd(3, n, cout, ho, wo)
    ref = O.conv_wgrad(x, dy, (cout, cin, r, r), stride, pad)
    b = B()
    ws = torch.empty(max(b.op_conv_workspace(n, h, w, cin, cout, r, stride, pad), 256), dtype=torch.uint8, device="cuda")
    dw = torch.full((cout, r, r, cin), float("nan"), device="cuda")
    b.op_conv_wgrad(dev(nhwc(x)), dev(nhwc(dy)), dw, stride, pad, ws)
    torch.cuda.synchronize()
    close(oihw(dw.cpu().numpy()), ref, f"conv_wgrad {case}")


POOL_CASES = [  # n, c, h, w, r, stride, pad
    (2, 64, 16, 16, 3, 2, 1),
    (3, 12, 15, 13, 3, 2, 1),       # odd sizes: ragged last windows, channels not a multiple of 32
    (2, 8, 8, 8, 2, 2, 0),          # VGG's pool: windows do not overlap
    (2, 16, 9, 9, 3, 1, 1),         # stride 1: every position in up to nine windows
    (41, 64, 112, 112, 3, 2, 1),    # the stem's pool at the benchmark minibatch
]


@pytest.mark.parametrize("case", POOL_CASES)
def test_maxpool_fwd_bwd(case):
    """Forward: the same maxima, bit for bit.  Backward: the gradient goes to the first maximum of every
    window in row-major order (the oracle's rule); a position that wins several windows adds their
    gradients, in an order of its own, hence a tolerance.  The input is rounded to multiples of 1/4 so
    that windows do hold equal values and the tie rule is exercised."""
    n, c, h, w, r, stride, pad = case
    x = np.round(rnd(11, n, c, h, w) * 4) / np.float32(4)
    y_ref, arg = O.maxpool_fwd(x, r, stride, pad)
    dy = rnd(12, *y_ref.shape)
    dx_ref = O.maxpool_bwd(dy, arg, x.shape)
    b = B()
    xd = dev(nhwc(x))
    y = torch.full((n, y_ref.shape[2], y_ref.shape[3], c), float("nan"), device="cuda")
    b.op_maxpool_fwd(xd, y, r, stride, pad)
    dx = torch.full((n, h, w, c), float("nan"), device="cuda")
    b.op_maxpool_bwd(xd, dev(nhwc(dy)), dx, r, stride, pad)
    base = rnd(13, n, c, h, w)
    dxa = dev(nhwc(base))
    b.op_maxpool_bwd(xd, dev(nhwc(dy)), dxa, r, stride, pad, accumulate=True)
    torch.cuda.synchronize()
    assert np.array_equal(nchw(y.cpu().numpy()), y_ref), f"maxpool_fwd {case}"
    close(nchw(dx.cpu().numpy()), dx_ref, f"maxpool_bwd {case}", 1e-6)
    close(nchw(dxa.cpu().numpy()), dx_ref.astype(np.float64) + base, f"maxpool_bwd accumulate {case}", 1e-6)


@pytest.mark.parametrize("case", [(41, 2048, 7, 7), (3, 20, 5, 3), (2, 64, 1, 1)])
def test_gap_fwd_bwd(case):
    n, c, h, w = case
    x = rnd(14, n, c, h, w)
    y_ref = O.gap_fwd(x)
    dy = rnd(15, n, c)
    dx_ref = O.gap_bwd(dy, x.shape)
    b = B()
    y = torch.full((n, c), float("nan"), device="cuda")
    b.op_gap_fwd(dev(nhwc(x)), y)
    dx = torch.full((n, h, w, c), float("nan"), device="cuda")
    b.op_gap_bwd(dev(dy), dx)
    torch.cuda.synchronize()
    close(y.cpu().numpy(), y_ref, f"gap_fwd {case}")
    close(nchw(dx.cpu().numpy()), dx_ref, f"gap_bwd {case}")


@pytest.mark.parametrize("case", [(41, 1000), (3, 10), (1, 7), (300, 1000)])
def test_softmax_ce(case):
    """Loss and gradient against the oracle; logits scaled so that exp() of the unshifted values would
    overflow in fp32 (the maximum is subtracted first); zero logits give ln(classes)."""
    # (the gradient is held to 1e-4 per tensor like every other operation)
    n, classes = case
    z = rnd(16, n, classes) * np.float32(40.0)
    lab = S.labels_uniform(17, n, classes)
    loss_ref, dz_ref = O.softmax_ce(z, lab)
    b = B()
    zd, ld = dev(z), dev(lab)
    rows = torch.full((n,), float("nan"), device="cuda")
    loss = torch.full((1,), float("nan"), device="cuda")
    dz = torch.full((n, classes), float("nan"), device="cuda")
    b.op_softmax_ce(zd, ld, rows, loss, dz)
    zeros = torch.zeros((n, classes), device="cuda")
    loss0 = torch.full((1,), float("nan"), device="cuda")
    b.op_softmax_ce(zeros, ld, rows.clone(), loss0, None)
    torch.cuda.synchronize()
    # (the kernel works relative to the row maximum, so the loss keeps its digits even where it is the small
    # difference of two large logits: the (1, 7) case, loss 1.7e-3 beside logits of 70)
    close(loss.cpu().numpy(), np.array([loss_ref], np.float32), f"softmax_ce loss {case}", 1e-5)
    close(dz.cpu().numpy(), dz_ref, f"softmax_ce dz {case}")
    assert abs(float(loss0.item()) - np.log(classes)) <= 1e-6 * np.log(classes)
    assert abs(float(dz.sum().item())) < 1e-5          # every row of the gradient sums to zero


BN_CASES = [  # n, c, h, w
    (2, 16, 16, 16),
    (3, 64, 7, 9),
    (2, 256, 14, 14),
    (5, 2048, 3, 3),       # two column slices
    (1, 12, 1, 1),         # single element per channel: variance 0
    (4, 1024, 1, 1),
    (37, 64, 11, 13),      # many slabs, ragged rows
]


@pytest.mark.parametrize("case", BN_CASES)
@pytest.mark.parametrize("variant", ["plain", "relu", "add_relu"])
def test_bn_fwd_bwd(case, variant):
    bn_case(case, variant)


@pytest.mark.parametrize("case,variant", [((41, 256, 56, 56), "add_relu"), ((41, 1024, 14, 14), "add_relu"),
                                          ((41, 64, 112, 112), "relu"), ((41, 256, 14, 14), "relu"),
                                          ((41, 2048, 7, 7), "add_relu")])
def test_bn_full_size(case, variant):
    """The batch-norm shapes of ResNet-152 that move the most bytes, at the benchmark's
    minibatch (thousands of row slabs, every column slice), element by element; and two of the
    small ones, whose finishing pass runs inside the apply launch (256 slabs: two batches of
    partial loads per workgroup; 2048 channels: 64 column slices)."""
    bn_case(case, variant)


def _bn_sweep():
    """Seeded shapes around the boundaries of the batch-norm launch shapes: rows (n*h*w) below and above one
    trip of 128 rows per workgroup, around 32-row and 512-row multiples (the number of partial sums, where the
    finishing pass moves into the apply launch and where it does not), channel counts that fill a 32-channel
    slice partly, exactly, and several times."""
    rows = [1, 2, 31, 33, 127, 129, 500, 2047, 2049, 8191, 8193, 16383, 16385, 20001]
    chans = [4, 8, 28, 32, 36, 60, 64, 100, 256, 260]
    u = S.splitmix64(31, 0, 2 * len(rows))
    out = []
    for i, r in enumerate(rows):
        c = chans[int(u[2 * i] % len(chans))]
        h = [1, 3, 7][int(u[2 * i + 1] % 3)]
        if r % h:
            h = 1
        out.append((r // h, c, h, 1, ["plain", "relu", "add_relu"][i % 3]))
    return out


@pytest.mark.parametrize("n,c,h,w,variant", _bn_sweep())
def test_bn_shape_sweep(n, c, h, w, variant):
    bn_case((n, c, h, w), variant)


def bn_case(case, variant):
    n, c, h, w = case
    x = rnd(5, n, c, h, w) * np.float32(1.7) + np.float32(0.3)
    gamma = (1.0 + 0.2 * rnd(6, c)).astype(np.float32)
    beta = (0.1 * rnd(7, c)).astype(np.float32)
    res = rnd(8, n, c, h, w) if variant == "add_relu" else None
    relu = variant != "plain"
    bn, mean, istd = O.bn_fwd(x, gamma, beta, O.BN_EPS)
    pre = bn if res is None else bn + res
    ref_y = O.relu_fwd(pre) if relu else pre
    b = B()
    ws = torch.empty(b.op_bn_workspace(c), dtype=torch.uint8, device="cuda")
    xd = dev(nhwc(x))
    y = torch.full_like(xd, float("nan"))
    m_d = torch.empty(c, device="cuda"); i_d = torch.empty(c, device="cuda")
    b.op_bn_fwd(xd, dev(gamma), dev(beta), dev(nhwc(res)) if res is not None else None, y, m_d, i_d, relu, O.BN_EPS, ws)
    torch.cuda.synchronize()
    close(nchw(y.cpu().numpy()), ref_y, f"bn_fwd y {case} {variant}")
    close(m_d.cpu().numpy(), mean, "bn mean", 1e-5)
    close(i_d.cpu().numpy(), istd, "bn istd", 1e-5)

    # backward: dy masked by the ReLU output, dx / dgamma / dbeta; masked gradient in place
    dy = rnd(9, n, c, h, w)
    g = O.relu_bwd(ref_y, dy) if relu else dy
    ref_dx, ref_dg, ref_db = O.bn_bwd(x, g, gamma, mean, istd)
    dyd = dev(nhwc(dy))
    dxd = torch.full_like(xd, float("nan"))
    dg_d = torch.empty(c, device="cuda"); db_d = torch.empty(c, device="cuda")
    y_ref_d = dev(nhwc(ref_y))     # mask taken from the oracle's output: same decision on both sides
    b.op_bn_bwd(xd, dyd, y_ref_d if relu else None, dev(gamma), dev(mean.astype(np.float32)),
                dev(istd.astype(np.float32)), dxd, dg_d, db_d, dyd if variant == "add_relu" else None, ws)
    torch.cuda.synchronize()
    scale = 1e-4 if n * h * w > 1 else 1e-3
    close(nchw(dxd.cpu().numpy()), ref_dx, f"bn_bwd dx {case} {variant}", scale)
    close(dg_d.cpu().numpy(), ref_dg, "bn dgamma", scale)
    close(db_d.cpu().numpy(), ref_db, "bn dbeta")
    if variant == "add_relu":
        np.testing.assert_array_equal(nchw(dyd.cpu().numpy()), g)   # masking is exact


def test_bad_arguments_are_rejected():
    b = B()
    x = torch.zeros(1, 4, 4, 8, device="cuda")
    w = torch.zeros(8, 3, 3, 8, device="cuda")
    y = torch.zeros(1, 4, 4, 8, device="cuda")
    with pytest.raises(b.AccError):
        b.op_conv_fwd(x, w, y, 0, 1)        # stride 0
    with pytest.raises(b.AccError):
        b.op_conv_fwd(x, w, y, 1, 3)        # pad >= r
    ws = torch.empty(1 << 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(b.AccError):
        b.op_conv_dgrad(y, w, torch.zeros(1, 14, 14, 8, device="cuda"), 4, 2, ws)  # 3x3 stride 4 pad 2: not supported
    # a view that starts one element into its buffer: contiguous, but not 16-byte aligned
    buf = torch.zeros(x.numel() + 4, device="cuda")
    x_off = buf[1:1 + x.numel()].view(x.shape)
    assert x_off.data_ptr() % 16 == 4 and x_off.is_contiguous()
    with pytest.raises(b.AccError):
        b.op_conv_fwd(x_off, w, y, 1, 1)
    dw = torch.zeros_like(w)
    with pytest.raises(b.AccError):
        b.op_conv_wgrad(x_off, y, dw, 1, 1, ws)


# ------------------------------------------------------------------ full-size layers, sampled
FULL_CASES = [  # the layer shapes of ResNet-152 that carry most of the work, at the benchmark's minibatch
    (41, 14, 14, 256, 256, 3, 1, 1),
    (41, 14, 14, 1024, 256, 1, 1, 0),
    (41, 14, 14, 256, 1024, 1, 1, 0),
    (41, 28, 28, 128, 128, 3, 1, 1),
    (41, 56, 56, 64, 256, 1, 1, 0),
    (41, 56, 56, 256, 512, 1, 2, 0),     # strided projection
    (41, 7, 7, 512, 512, 3, 1, 1),
    (41, 224, 224, 3, 64, 7, 2, 3),      # stem (per-element loader)
]


def _sample(rng, shape, count):
    return [tuple(int(rng.integers(0, d)) for d in shape) for _ in range(count)]


@pytest.mark.parametrize("case", FULL_CASES)
def test_conv_full_size_sampled(case):
    """Full benchmark shapes (too large for the oracle's whole tensor in seconds): 150 sampled
    outputs of each of the three GEMMs against the definition written out in float64."""
    n, h, w, cin, cout, r, stride, pad = case
    b = B()
    g = torch.Generator(device="cuda").manual_seed(1234)
    x = torch.randn(n, h, w, cin, device="cuda", generator=g)
    wt = torch.randn(cout, r, r, cin, device="cuda", generator=g) * float(np.sqrt(2.0 / (cin * r * r)))
    ho, wo = (h + 2 * pad - r) // stride + 1, (w + 2 * pad - r) // stride + 1
    dy = torch.randn(n, ho, wo, cout, device="cuda", generator=g)
    y = torch.full((n, ho, wo, cout), float("nan"), device="cuda")
    b.op_conv_fwd(x, wt, y, stride, pad)
    ws = torch.empty(max(b.op_conv_workspace(n, h, w, cin, cout, r, stride, pad), 256), dtype=torch.uint8, device="cuda")
    dw = torch.full((cout, r, r, cin), float("nan"), device="cuda")
    b.op_conv_wgrad(x, dy, dw, stride, pad, ws)
    do_dgrad = stride == 1 or r == 1
    if do_dgrad:
        dx = torch.full((n, h, w, cin), float("nan"), device="cuda")
        b.op_conv_dgrad(dy, wt, dx, stride, pad, ws, False)
    torch.cuda.synchronize()
    X, W_, DY = x.cpu().numpy().astype(np.float64), wt.cpu().numpy().astype(np.float64), dy.cpu().numpy().astype(np.float64)
    Y, DW = y.cpu().numpy(), dw.cpu().numpy()
    assert np.isfinite(Y).all() and np.isfinite(DW).all()
    rng = np.random.default_rng(7)
    Xp = np.pad(X, ((0, 0), (pad, pad), (pad, pad), (0, 0)))
    scale_y, scale_dw = np.abs(Y).max(), np.abs(DW).max()
    for (i, p, q, co) in _sample(rng, (n, ho, wo, cout), 150):
        ref = np.sum(Xp[i, p * stride:p * stride + r, q * stride:q * stride + r, :] * W_[co])
        assert abs(Y[i, p, q, co] - ref) <= TOL * scale_y, ("fwd", case, (i, p, q, co))
    for (co, kr, kt, ci) in _sample(rng, (cout, r, r, cin), 150):
        # dw[co,kr,kt,ci] = sum over images and output positions of dy * the input under tap (kr, kt)
        patch = Xp[:, kr:kr + (ho - 1) * stride + 1:stride, kt:kt + (wo - 1) * stride + 1:stride, ci]
        ref = np.sum(patch * DY[:, :, :, co])
        assert abs(DW[co, kr, kt, ci] - ref) <= TOL * scale_dw, ("wgrad", case, (co, kr, kt, ci))
    if do_dgrad:
        DX = dx.cpu().numpy()
        assert np.isfinite(DX).all()
        scale_dx = np.abs(DX).max()
        for (i, iy, ix, ci) in _sample(rng, (n, h, w, cin), 150):
            ref = 0.0
            for kr in range(r):
                for kt in range(r):
                    py, px = iy + pad - kr, ix + pad - kt
                    if py % stride or px % stride:
                        continue
                    py //= stride; px //= stride
                    if 0 <= py < ho and 0 <= px < wo:
                        ref += np.dot(DY[i, py, px, :], W_[:, kr, kt, ci])
            assert abs(DX[i, iy, ix, ci] - ref) <= TOL * scale_dx, ("dgrad", case, (i, iy, ix, ci))


# ------------------------------------------------------------------ bf16 storage
BF16_CASES = [
    (2, 14, 14, 64, 96, 3, 1, 1),      # fast path (channels a multiple of 64), N tail
    (3, 9, 9, 128, 256, 1, 1, 0),
    (2, 16, 16, 64, 128, 1, 2, 0),     # strided 1x1
    (5, 28, 28, 64, 64, 3, 1, 1),      # several tiles
    (2, 16, 16, 32, 16, 3, 1, 1),      # 32 channels: per-element path in bf16
    (2, 12, 10, 20, 24, 3, 1, 1),      # ragged channels
    (2, 23, 23, 8, 16, 7, 2, 3),       # stem-like
    # input channels a multiple of 128: the weight gradient runs on the bf16 matrix cores (128 x 128 tiles)
    (4, 14, 14, 256, 128, 3, 1, 1),    # filter taps and padding; 784 rows = 12 chunks of 64 and a ragged one
    (6, 14, 14, 128, 200, 3, 1, 1),    # output channels end inside the second row of tiles
    (8, 28, 28, 128, 128, 3, 2, 1),    # strided 3x3
    (9, 7, 7, 512, 512, 1, 2, 0),      # strided 1x1
    (41, 14, 14, 256, 256, 3, 1, 1),   # benchmark-sized layer: the minibatch range is cut into parts
    # at least 256 tiles of 128 x 128: forward and data gradient run in the 128 x 128 bf16 kernel
    (16, 56, 56, 64, 128, 1, 1, 0),    # one chunk of K, 392 row tiles
    (44, 28, 28, 128, 128, 3, 1, 1),   # taps and padding; 34496 rows: the last row tile is half full
    (44, 56, 56, 128, 128, 1, 2, 0),   # strided gather forward, scattering data gradient
    (44, 28, 28, 128, 200, 1, 1, 0),   # output channels end inside the second column of tiles
]


def bf(a: np.ndarray) -> torch.Tensor:
    """numpy fp32 -> device bf16 (round to nearest even)"""
    return torch.from_numpy(np.ascontiguousarray(a)).cuda().to(torch.bfloat16)


def f32(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy()


@pytest.mark.parametrize("case", BF16_CASES)
def test_conv_bf16(case):
    """bf16 operands, fp32 accumulation: against the oracle run on the same bf16-rounded
    operands the only differences are the accumulation order and the final rounding of a
    bf16 output (relative 2^-9 per element); the weight gradient is fp32 and held to 1e-4."""
    n, h, w, cin, cout, r, stride, pad = case
    b = B()
    xb = bf(nhwc(rnd(1, n, cin, h, w)))
    wb = bf(ohwi(rnd(2, cout, cin, r, r) * np.float32(np.sqrt(2.0 / (cin * r * r)))))
    x, wt = nchw(f32(xb)), oihw(f32(wb))                         # what the kernels really see
    ho, wo = O.out_dim(h, r, stride, pad), O.out_dim(w, r, stride, pad)
    dyb = bf(nhwc(rnd(3, n, cout, ho, wo)))
    dy = nchw(f32(dyb))
    y = torch.full((n, ho, wo, cout), float("nan"), device="cuda", dtype=torch.bfloat16)
    b.op_conv_fwd(xb, wb, y, stride, pad)
    ws = torch.empty(max(b.op_conv_workspace(n, h, w, cin, cout, r, stride, pad), 256), dtype=torch.uint8, device="cuda")
    dw = torch.full((cout, r, r, cin), float("nan"), device="cuda")
    b.op_conv_wgrad(xb, dyb, dw, stride, pad, ws)
    torch.cuda.synchronize()
    close(nchw(f32(y)), O.conv_fwd(x, wt, stride, pad), f"bf16 conv_fwd {case}", 8e-3)
    close(oihw(dw.cpu().numpy()), O.conv_wgrad(x, dy, (cout, cin, r, r), stride, pad), f"bf16 conv_wgrad {case}")
    if stride == 1 or r == 1:
        for accumulate in (False, True):
            base = bf(nhwc(rnd(4, n, cin, h, w)))
            dx = base.clone() if accumulate else torch.full((n, h, w, cin), float("nan"), device="cuda", dtype=torch.bfloat16)
            b.op_conv_dgrad(dyb, wb, dx, stride, pad, ws, accumulate)
            torch.cuda.synchronize()
            ref = O.conv_dgrad(dy, wt, (n, cin, h, w), stride, pad)
            if accumulate:
                ref = ref + nchw(f32(base))
            close(nchw(f32(dx)), ref, f"bf16 conv_dgrad {case} acc={accumulate}", 8e-3)


@pytest.mark.parametrize("case", [(3, 64, 7, 9), (2, 256, 14, 14), (37, 64, 11, 13)])
@pytest.mark.parametrize("variant", ["plain", "add_relu"])
def test_bn_bf16(case, variant):
    n, c, h, w = case
    b = B()
    xb = bf(nhwc(rnd(5, n, c, h, w) * np.float32(1.7) + np.float32(0.3)))
    x = nchw(f32(xb))
    gamma = (1.0 + 0.2 * rnd(6, c)).astype(np.float32)
    beta = (0.1 * rnd(7, c)).astype(np.float32)
    relu = variant != "plain"
    resb = bf(nhwc(rnd(8, n, c, h, w))) if relu else None
    bn, mean, istd = O.bn_fwd(x, gamma, beta, O.BN_EPS)
    pre = bn if resb is None else bn + nchw(f32(resb))
    ref_y = O.relu_fwd(pre) if relu else pre
    ws = torch.empty(b.op_bn_workspace(c), dtype=torch.uint8, device="cuda")
    y = torch.full_like(xb, float("nan"))
    m_d = torch.empty(c, device="cuda"); i_d = torch.empty(c, device="cuda")
    b.op_bn_fwd(xb, dev(gamma), dev(beta), resb, y, m_d, i_d, relu, O.BN_EPS, ws)
    torch.cuda.synchronize()
    close(nchw(f32(y)), ref_y, f"bf16 bn_fwd {case} {variant}", 8e-3)
    close(m_d.cpu().numpy(), mean, "bn mean", 1e-5)       # statistics are fp32 sums of the bf16 values
    close(i_d.cpu().numpy(), istd, "bn istd", 1e-5)
    # backward on the stored (bf16) output, so that both sides take the same ReLU decisions
    y_used = nchw(f32(y))
    dyb = bf(nhwc(rnd(9, n, c, h, w)))
    dy = nchw(f32(dyb))
    g = O.relu_bwd(y_used, dy) if relu else dy
    ref_dx, ref_dg, ref_db = O.bn_bwd(x, g, gamma, mean, istd)
    dxd = torch.full_like(xb, float("nan"))
    dg_d = torch.empty(c, device="cuda"); db_d = torch.empty(c, device="cuda")
    b.op_bn_bwd(xb, dyb, y if relu else None, dev(gamma), m_d, i_d, dxd, dg_d, db_d, dyb if relu else None, ws)
    torch.cuda.synchronize()
    close(nchw(f32(dxd)), ref_dx, f"bf16 bn_bwd dx {case} {variant}", 8e-3)
    close(dg_d.cpu().numpy(), ref_dg, "bn dgamma", 1e-4)
    close(db_d.cpu().numpy(), ref_db, "bn dbeta", 1e-4)
    if relu:
        np.testing.assert_array_equal(nchw(f32(dyb)), g)      # masking is exact
