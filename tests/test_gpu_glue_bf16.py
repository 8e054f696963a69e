"""GPU parity of the layers between the convolutions of a bf16 step (the `_t` entry points with LC_BF16): batch
normalisation (plain, fused with residual / ReLU, backward through the ReLU), overlapping max pooling, the gradient
at a residual block's output, global average pooling.  Inputs are drawn in fp32, rounded once to bf16 on the host,
and those exact values feed both sides; the oracle works in float64 on them.

Tolerances.  A bf16 output is the fp32 result rounded once, so it can differ from the rounded oracle value by one
bf16 step (2^-8 relative) where the fp32 result sits next to a rounding boundary, plus the fp32 error of the
layer itself (1e-4 tensor-scaled, as for the fp32 kernels): |gpu - oracle| <= 2^-8 |oracle| + 2e-4 max|oracle|
element by element.  fp32 outputs (statistics, dgamma, dbeta, pooled means) keep the fp32 tolerances.  Max pooling
forwards values unchanged: values and indices are compared bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from oracle import batchnorm as obn
from oracle import resnet as ores
from oracle import tiny_cnn as otc
from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
EPS = 1e-5
BF = lc.LC_BF16
NHWC = lc.LC_NHWC


def _bf(a):
    """fp32 array -> (bf16 bit patterns, the values they denote)"""
    bits = synth.to_bf16_bits(a)
    return bits, synth.bf16_bits_to_f32(bits)


def _dev(bits_nchw):
    return torch.from_numpy(np.ascontiguousarray(gu.to_layout(bits_nchw, NHWC)).view(np.int16)).to(gu.DEV)


def _back(t):
    """device bf16 tensor in NHWC -> fp32 values in NCHW order"""
    return gu.from_layout(synth.bf16_bits_to_f32(t.cpu().numpy().view(np.uint16)), NHWC)


def _close_bf16(got, ref, extra=2e-4):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape and np.all(np.isfinite(got))
    bound = np.abs(ref) * 2.0 ** -8 + extra * float(np.max(np.abs(ref)))
    bad = np.abs(got - ref) > bound
    assert not bad.any(), f"{int(bad.sum())} of {bad.size} beyond one bf16 step; worst {float(np.max(np.abs(got - ref) - bound))}"


BN_SHAPES = {
    "resnet_56x56_c64": (8, 64, 56, 56),
    "resnet_7x7_c2048": (16, 2048, 7, 7),
    "c8_one_group": (3, 8, 5, 7),
    "c24_ragged_rows": (5, 24, 9, 11),
    "one_pixel_per_image": (64, 16, 1, 1),
    "many_slabs": (32, 16, 64, 64),
}


def _bn_case(shape, seed):
    n, c, h, w = shape
    xb, x = _bf(synth.normal(shape, seed) * 1.5 + 0.4)
    dyb, dy = _bf(synth.normal(shape, seed + 1))
    rb, res = _bf(synth.normal(shape, seed + 4))
    gamma = (1.0 + 0.5 * synth.normal((c,), seed + 2)).astype(np.float32)
    beta = (0.5 * synth.normal((c,), seed + 3)).astype(np.float32)
    return (xb, x), (dyb, dy), (rb, res), gamma, beta


@pytest.mark.parametrize("name", list(BN_SHAPES))
def test_batchnorm_bf16_forward_and_backward_match_oracle(name):
    shape = BN_SHAPES[name]
    n, c, h, w = shape
    (xb, x), (dyb, dy), _, gamma, beta = _bn_case(shape, 9100 + 10 * list(BN_SHAPES).index(name))
    xd, dyd, gd, bd = _dev(xb), _dev(dyb), gu.dev(gamma), gu.dev(beta)
    y, dx = torch.full_like(xd, -1), torch.full_like(xd, -1)
    mean, invstd, dg, db = (torch.empty(c, device=gu.DEV) for _ in range(4))
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, NHWC))
    lc.batchnorm_fwd_t(BF, xd, gd, bd, None, y, mean, invstd, n, c, h, w, EPS, False, NHWC, ws)
    lc.batchnorm_bwd_t(BF, xd, dyd, gd, None, mean, invstd, dx, dg, db, n, c, h, w, False, NHWC, ws)
    torch.cuda.synchronize()
    oy, omean, oinv = obn.forward(x, gamma, beta, EPS)
    odx, odg, odb = obn.backward(x, dy, gamma, EPS)
    _close_bf16(_back(y), oy)
    _close_bf16(_back(dx), odx)
    assert gu.scaled_err(mean.cpu().numpy(), omean) <= 1e-5
    assert np.max(np.abs(invstd.cpu().numpy() - oinv) / oinv) <= 1e-4
    assert gu.scaled_err(dg.cpu().numpy(), odg) <= 1e-4
    assert gu.scaled_err(db.cpu().numpy(), odb) <= 1e-4


@pytest.mark.parametrize("relu,residual", [(True, False), (False, True), (True, True)], ids=["relu", "residual", "residual_relu"])
def test_batchnorm_bf16_fused_forward(relu, residual):
    shape = (6, 32, 14, 14)
    n, c, h, w = shape
    (xb, x), _, (rb, res), gamma, beta = _bn_case(shape, 9300)
    xd, gd, bd = _dev(xb), gu.dev(gamma), gu.dev(beta)
    rd = _dev(rb) if residual else None
    y = torch.full_like(xd, -1)
    mean, invstd = torch.empty(c, device=gu.DEV), torch.empty(c, device=gu.DEV)
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, NHWC))
    lc.batchnorm_fwd_t(BF, xd, gd, bd, rd, y, mean, invstd, n, c, h, w, EPS, relu, NHWC, ws)
    torch.cuda.synchronize()
    want, _, _ = obn.forward(x, gamma, beta, EPS)
    if residual:
        want = want + res.astype(np.float64)
    if relu:
        want = np.maximum(want, 0.0)
    _close_bf16(_back(y), want)


def test_batchnorm_bf16_backward_through_relu():
    """Elements whose output the oracle puts within 1e-4 of zero get dy = 0 on both sides: there fp32 and float64 may
    disagree on the sign."""
    shape = (6, 32, 14, 14)
    n, c, h, w = shape
    (xb, x), (_, dy), _, gamma, beta = _bn_case(shape, 9400)
    oy, _, _ = obn.forward(x, gamma, beta, EPS)
    dyb, dy = _bf(np.where(np.abs(oy) < 1e-4, 0.0, dy).astype(np.float32))
    xd, dyd, gd, bd = _dev(xb), _dev(dyb), gu.dev(gamma), gu.dev(beta)
    y, dx = torch.full_like(xd, -1), torch.full_like(xd, -1)
    mean, invstd, dg, db = (torch.empty(c, device=gu.DEV) for _ in range(4))
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, NHWC))
    lc.batchnorm_fwd_t(BF, xd, gd, bd, None, y, mean, invstd, n, c, h, w, EPS, True, NHWC, ws)
    lc.batchnorm_bwd_t(BF, xd, dyd, gd, bd, mean, invstd, dx, dg, db, n, c, h, w, True, NHWC, ws)
    torch.cuda.synchronize()
    odx, odg, odb = obn.backward(x, np.where(oy > 0.0, dy, 0.0), gamma, EPS)
    _close_bf16(_back(dx), odx)
    assert gu.scaled_err(dg.cpu().numpy(), odg) <= 1e-4
    assert gu.scaled_err(db.cpu().numpy(), odb) <= 1e-4
    # the mask the backward pass rebuilds is the mask of the stored (rounded) output
    masked = torch.full_like(xd, -1)
    dx2, dg2, db2 = torch.full_like(xd, -1), torch.empty(c, device=gu.DEV), torch.empty(c, device=gu.DEV)
    lc.relu_add_bwd_t(BF, y, dyd, None, masked, xd.numel())
    lc.batchnorm_bwd_t(BF, xd, masked, gd, None, mean, invstd, dx2, dg2, db2, n, c, h, w, False, NHWC, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(dx.cpu().numpy(), dx2.cpu().numpy())
    np.testing.assert_array_equal(dg.cpu().numpy(), dg2.cpu().numpy())
    np.testing.assert_array_equal(db.cpu().numpy(), db2.cpu().numpy())


def test_batchnorm_bf16_reruns_are_bit_identical_and_f32_dtype_is_the_fp32_call():
    n, c, h, w = 16, 128, 28, 28
    xb, _ = _bf(synth.normal((n, c, h, w), 9500))
    xd = _dev(xb)
    g, b = gu.dev(np.ones(c, np.float32)), gu.dev(np.zeros(c, np.float32))
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, NHWC))
    outs = []
    for _ in range(2):
        y, m, s = torch.full_like(xd, -1), torch.empty(c, device=gu.DEV), torch.empty(c, device=gu.DEV)
        lc.batchnorm_fwd_t(BF, xd, g, b, None, y, m, s, n, c, h, w, EPS, False, NHWC, ws)
        torch.cuda.synchronize()
        outs.append((y.cpu().numpy(), m.cpu().numpy(), s.cpu().numpy()))
    for a, bb in zip(*outs):
        np.testing.assert_array_equal(a, bb)
    xf = gu.dev(synth.normal((n, h, w, c), 9501))
    res = []
    for typed in (True, False):
        y, m, s = torch.empty_like(xf), torch.empty(c, device=gu.DEV), torch.empty(c, device=gu.DEV)
        if typed:
            lc.batchnorm_fwd_t(lc.LC_F32, xf, g, b, None, y, m, s, n, c, h, w, EPS, True, NHWC, ws)
        else:
            lc.batchnorm_fwd_ex(xf, g, b, None, y, m, s, n, c, h, w, EPS, True, NHWC, ws)
        torch.cuda.synchronize()
        res.append((y.cpu().numpy(), m.cpu().numpy(), s.cpu().numpy()))
    for a, bb in zip(*res):
        np.testing.assert_array_equal(a, bb)


def test_bf16_layers_refuse_what_they_do_not_take():
    n, c, h, w = 2, 12, 4, 4                                   # 12 channels: not whole 16-byte groups
    x = torch.zeros(n * h * w * c, dtype=torch.int16, device=gu.DEV)
    f = torch.zeros(c, device=gu.DEV)
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, NHWC))
    with pytest.raises(lc.LarsConvError, match="unsupported"):
        lc.batchnorm_fwd_t(BF, x, f, f, None, x.clone(), f.clone(), f.clone(), n, c, h, w, EPS, False, NHWC, ws)
    with pytest.raises(lc.LarsConvError, match="unsupported"):
        lc.maxpool_fwd_t(BF, x, x.clone(), torch.zeros(x.numel(), dtype=torch.uint8, device=gu.DEV), n, c, h, w, 2, 2, 0, NHWC)
    with pytest.raises(lc.LarsConvError, match="unsupported"):
        lc.relu_add_bwd_t(BF, x, x, None, x.clone(), 12)
    x16 = torch.zeros(n * h * w * 16, dtype=torch.int16, device=gu.DEV)
    f16 = torch.zeros(16, device=gu.DEV)
    with pytest.raises(lc.LarsConvError, match="unsupported"):
        lc.batchnorm_fwd_t(BF, x16, f16, f16, None, x16.clone(), f16.clone(), f16.clone(), n, 16, h, w, EPS, False, lc.LC_NCHW, ws)
    with pytest.raises(lc.LarsConvError, match="misaligned"):
        lc.batchnorm_fwd_t(BF, x16[1:], f16, f16, None, x16.clone(), f16.clone(), f16.clone(), n, 16, h, w - 1, EPS, False, NHWC, ws)
    with pytest.raises(lc.LarsConvError, match="unsupported"):
        lc.global_avgpool_fwd_t(7, x16, torch.zeros(n * 16, device=gu.DEV), n, 16, h, w, NHWC)


POOLS = {
    "resnet_stem_3x3_s2_p1": ((4, 64, 28, 28), 3, 2, 1),
    "alexnet_3x3_s2": ((3, 96, 13, 13), 3, 2, 0),
    "odd_image_3x3_s2_p1": ((3, 16, 11, 9), 3, 2, 1),
    "one_pixel_3x3_s2_p1": ((2, 8, 1, 1), 3, 2, 1),
    "one_column_3x3_s2_p1": ((1, 8, 5, 1), 3, 2, 1),
    "2x2_s2": ((2, 8, 6, 8), 2, 2, 0),
    "odd_image_5x5_s3_p2": ((2, 16, 11, 9), 5, 3, 2),
}


@pytest.mark.parametrize("name", list(POOLS))
def test_maxpool_bf16(name):
    shape, window, stride, pad = POOLS[name]
    n, c, h, w = shape
    xb, x = _bf(synth.normal(shape, 9600 + list(POOLS).index(name)))
    oy, oidx = ores.maxpool(x, window, stride, pad)
    ph, pw = oy.shape[2:]
    dyb, dy = _bf(synth.normal(oy.shape, 9650))
    xd, dyd = _dev(xb), _dev(dyb)
    y = torch.full((n, ph, pw, c), -1, dtype=torch.int16, device=gu.DEV)
    idx = torch.full((n, ph, pw, c), 255, dtype=torch.uint8, device=gu.DEV)
    dx = torch.full_like(xd, -1)
    lc.maxpool_fwd_t(BF, xd, y, idx, n, c, h, w, window, stride, pad, NHWC)
    lc.maxpool_bwd_t(BF, dyd, idx, dx, n, c, h, w, window, stride, pad, NHWC)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(_back(y), oy.astype(np.float32))
    np.testing.assert_array_equal(idx.cpu().numpy().transpose(0, 3, 1, 2), oidx)
    odx = ores.maxpool_bwd(oidx, dy, (h, w), window, stride, pad)
    got = _back(dx)
    _close_bf16(got, odx, extra=0.0)
    assert np.mean(got == oracle.round_to_bf16(odx)) >= 0.999         # sums of up to four bf16 values: fp32 nearly always holds them exactly


@pytest.mark.parametrize("mode", ["both_masked", "one_masked", "sum_only"])
def test_relu_add_bwd_bf16(mode):
    count = 8 * 12345                                                   # several blocks and a ragged last one
    yb, y = _bf(synth.normal((count,), 9700))
    ab, a = _bf(synth.normal((count,), 9701))
    bb, b = _bf(synth.normal((count,), 9702))
    dv = lambda bits: torch.from_numpy(bits.view(np.int16)).to(gu.DEV)   # noqa: E731
    yd, ad, bd = dv(yb), dv(ab), dv(bb)
    dx = torch.full_like(ad, -1)
    if mode == "both_masked":
        lc.relu_add_bwd_t(BF, yd, ad, bd, dx, count)
        want = np.where(y > 0, a.astype(np.float64) + b, 0.0)
    elif mode == "one_masked":
        lc.relu_add_bwd_t(BF, yd, ad, None, dx, count)
        want = np.where(y > 0, a.astype(np.float64), 0.0)
    else:
        lc.relu_add_bwd_t(BF, None, ad, bd, dx, count)
        want = a.astype(np.float64) + b
    torch.cuda.synchronize()
    got = synth.bf16_bits_to_f32(dx.cpu().numpy().view(np.uint16))
    _close_bf16(got, want, extra=0.0)
    assert np.mean(got == oracle.round_to_bf16(want)) >= 0.9999          # the fp32 sum of two bf16 values is exact unless they lie 2^16 apart


def test_device_rounding_to_bf16_takes_ties_to_even():
    """The kernels round with the device's fp32 -> bf16 conversion; here its ties: sums a + b (exact in fp32) that
    lie exactly between two bf16 values, just above and just below, for both signs and many exponents, against the
    oracle's integer rounding."""
    mant = np.arange(128, 256, dtype=np.float64)                              # 1.0000000b .. 1.1111111b: even and odd last bits
    a, b = [], []
    for e in range(-20, 21, 3):
        av = mant / 128.0 * 2.0 ** e
        half = 2.0 ** (e - 8)                                                 # half a bf16 step of av
        for bv in (half, -half, half * (1 + 2.0 ** -7), half * (1 - 2.0 ** -7), -half * (1 + 2.0 ** -7), 3 * half, 0.0):
            for sign in (1.0, -1.0):
                a.append(sign * av)
                b.append(np.full_like(av, sign * bv))
    a, b = np.concatenate(a).astype(np.float32), np.concatenate(b).astype(np.float32)
    ab, av_ = _bf(a)
    bb, bv_ = _bf(b)
    assert np.array_equal(av_, a) and np.array_equal(bv_, b) and a.size % 8 == 0    # all inputs are bf16 values
    want = a.astype(np.float64) + b.astype(np.float64)
    assert np.array_equal(want, (a + b).astype(np.float64))                   # the fp32 sum is exact
    ties = np.mean((want.astype(np.float32).view(np.uint32) & 0xFFFF) == 0x8000)
    assert ties > 0.2                                                         # and many of them are ties
    dv = lambda bits: torch.from_numpy(bits.view(np.int16)).to(gu.DEV)        # noqa: E731
    dx = torch.full((a.size,), -1, dtype=torch.int16, device=gu.DEV)
    lc.relu_add_bwd_t(BF, None, dv(ab), dv(bb), dx, a.size)
    torch.cuda.synchronize()
    got = synth.bf16_bits_to_f32(dx.cpu().numpy().view(np.uint16))
    np.testing.assert_array_equal(got, oracle.round_to_bf16(want))
    # infinities stay, NaN stays NaN
    spec = np.array([np.inf, -np.inf, np.nan, 0.0, -0.0, 3.0e38, -3.0e38, 1e-40], np.float32)
    sb, _ = _bf(np.zeros(8, np.float32))
    hi = (spec.view(np.uint32) >> 16).astype(np.uint16)                       # truncated patterns: exact bf16 inputs
    out = torch.full((8,), -1, dtype=torch.int16, device=gu.DEV)
    lc.relu_add_bwd_t(BF, None, dv(hi), dv(sb), out, 8)
    torch.cuda.synchronize()
    res = synth.bf16_bits_to_f32(out.cpu().numpy().view(np.uint16))
    assert np.isposinf(res[0]) and np.isneginf(res[1]) and np.isnan(res[2])
    np.testing.assert_array_equal(res[3:], synth.bf16_bits_to_f32(hi)[3:])


def test_global_avgpool_bf16():
    for shape in ((6, 2048, 7, 7), (3, 8, 5, 3), (2, 24, 1, 1)):
        n, c, h, w = shape
        xb, x = _bf(synth.normal(shape, 9800) + 0.3)
        dy = synth.normal((n, c), 9801)
        y = torch.full((n, c), float("nan"), device=gu.DEV)
        dx = torch.full((n, h, w, c), -1, dtype=torch.int16, device=gu.DEV)
        lc.global_avgpool_fwd_t(BF, _dev(xb), y, n, c, h, w, NHWC)
        lc.global_avgpool_bwd_t(BF, gu.dev(dy), dx, n, c, h, w, NHWC)
        torch.cuda.synchronize()
        assert gu.scaled_err(y.cpu().numpy(), otc.global_avgpool(x.astype(np.float64))) <= 1e-5
        _close_bf16(_back(dx), otc.global_avgpool_bwd(dy.astype(np.float64), h, w), extra=1e-6)


def test_maxpool_bf16_ties_and_padding():
    """Equal values: the first tap in row-major window order that lies inside the image wins (at the border that is not
    tap 0); all-negative values: padding never wins."""
    n, c, h, w = 2, 8, 6, 6
    for value in (1.5, -2.0):
        xb, x = _bf(np.full((n, c, h, w), value, np.float32))
        oy, oidx = ores.maxpool(x, 3, 2, 1)
        y = torch.full((n, 3, 3, c), -1, dtype=torch.int16, device=gu.DEV)
        idx = torch.full((n, 3, 3, c), 255, dtype=torch.uint8, device=gu.DEV)
        lc.maxpool_fwd_t(BF, _dev(xb), y, idx, n, c, h, w, 3, 2, 1, NHWC)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(_back(y), np.full((n, c, 3, 3), value, np.float32))
        got = idx.cpu().numpy().transpose(0, 3, 1, 2)
        np.testing.assert_array_equal(got, oidx)
        assert got[0, 0, 0, 0] == 4 and got[0, 0, 0, 1] == 3 and got[0, 0, 1, 0] == 1 and got[0, 0, 1, 1] == 0


def test_typed_calls_with_fp32_are_the_fp32_calls():
    n, c, h, w = 3, 16, 9, 9
    x = gu.dev(synth.normal((n, h, w, c), 9870))
    dy = gu.dev(synth.normal((n, 5, 5, c), 9871))
    outs = []
    for typed in (True, False):
        y = torch.full((n, 5, 5, c), float("nan"), device=gu.DEV)
        idx = torch.full((n, 5, 5, c), 255, dtype=torch.uint8, device=gu.DEV)
        dx, s, g = torch.full_like(x, float("nan")), torch.full_like(x, float("nan")), torch.full((n, c), float("nan"), device=gu.DEV)
        gx = torch.full_like(x, float("nan"))
        if typed:
            lc.maxpool_fwd_t(lc.LC_F32, x, y, idx, n, c, h, w, 3, 2, 1, NHWC)
            lc.maxpool_bwd_t(lc.LC_F32, dy, idx, dx, n, c, h, w, 3, 2, 1, NHWC)
            lc.relu_add_bwd_t(lc.LC_F32, x, x, dx, s, x.numel())
            lc.global_avgpool_fwd_t(lc.LC_F32, x, g, n, c, h, w, NHWC)
            lc.global_avgpool_bwd_t(lc.LC_F32, g, gx, n, c, h, w, NHWC)
        else:
            lc.maxpool_fwd(x, y, idx, n, c, h, w, 3, 2, 1, NHWC)
            lc.maxpool_bwd(dy, idx, dx, n, c, h, w, 3, 2, 1, NHWC)
            lc.relu_add_bwd(x, x, dx, s, x.numel())
            lc.global_avgpool_fwd(x, g, n, c, h, w, NHWC)
            lc.global_avgpool_bwd(g, gx, n, c, h, w, NHWC)
        torch.cuda.synchronize()
        outs.append([t.cpu().numpy() for t in (y, idx, dx, s, g, gx)])
    for a, b in zip(*outs):
        np.testing.assert_array_equal(a, b)


def test_batchnorm_bf16_constant_tensor():
    """A constant input: the batch variance is exactly zero on both sides (the pivot is the value itself), y = beta rounded
    to bf16, and the backward pass stays finite with dx = gamma / sqrt(eps) * (dy - mean(dy)) rounded."""
    n, c, h, w = 4, 16, 3, 3
    xb, x = _bf(np.full((n, c, h, w), 2.5, np.float32))
    dyb, dy = _bf(synth.normal((n, c, h, w), 9880))
    gamma = (1.0 + 0.5 * synth.normal((c,), 9881)).astype(np.float32)
    beta = synth.normal((c,), 9882)
    xd, dyd, gd, bd = _dev(xb), _dev(dyb), gu.dev(gamma), gu.dev(beta)
    y, dx = torch.full_like(xd, -1), torch.full_like(xd, -1)
    mean, invstd, dg, db = (torch.empty(c, device=gu.DEV) for _ in range(4))
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, NHWC))
    lc.batchnorm_fwd_t(BF, xd, gd, bd, None, y, mean, invstd, n, c, h, w, EPS, False, NHWC, ws)
    lc.batchnorm_bwd_t(BF, xd, dyd, gd, None, mean, invstd, dx, dg, db, n, c, h, w, False, NHWC, ws)
    torch.cuda.synchronize()
    assert np.allclose(invstd.cpu().numpy(), 1.0 / np.sqrt(EPS), rtol=1e-5)
    np.testing.assert_array_equal(mean.cpu().numpy(), np.full(c, 2.5, np.float32))
    oy, _, _ = obn.forward(x, gamma, beta, EPS)
    _close_bf16(_back(y), oy, extra=1e-3)                 # |x - mean| is 0 or one fp32 step, times 1/sqrt(eps) = 316
    odx, odg, odb = obn.backward(x, dy, gamma, EPS)
    assert gu.scaled_err(db.cpu().numpy(), odb) <= 1e-4
    assert np.max(np.abs(dg.cpu().numpy() - odg)) <= 1e-6
    _close_bf16(_back(dx), odx, extra=1e-4)


@pytest.mark.parametrize("bf16", [False, True], ids=["fp32", "bf16"])
@pytest.mark.parametrize("two", [True, False], ids=["two_gradients", "one_gradient"])
@pytest.mark.parametrize("shape", [(6, 32, 14, 14), (3, 8, 5, 7), (16, 256, 7, 7), (2, 64, 56, 56)], ids=["14x14", "ragged", "wide", "many_rows"])
def test_block_gradient_joined_with_batchnorm_sums_equals_the_two_plain_calls(shape, two, bf16):
    """relu_add_bwd_bnsums_t + batchnorm_bwd_presummed_t against relu_add_bwd_t + batchnorm_bwd_t: bit for bit, and the
    plain pair is itself checked against the oracle elsewhere in this file and in test_gpu_batchnorm.py."""
    n, c, h, w = shape
    dtype = BF if bf16 else lc.LC_F32

    def put(a):
        if bf16:
            return _dev(_bf(a)[0])
        return gu.dev(gu.to_layout(a, NHWC))
    z = put((synth.normal(shape, 9900) * 1.5 + 0.4).astype(np.float32))
    y = put(synth.normal(shape, 9901))                    # the block's output: its sign is the mask
    g1, g2 = put(synth.normal(shape, 9902)), put(synth.normal(shape, 9903))
    gamma = gu.dev((1.0 + 0.5 * synth.normal((c,), 9904)).astype(np.float32))
    beta = gu.dev(synth.normal((c,), 9905))
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, NHWC))
    mean, invstd = torch.empty(c, device=gu.DEV), torch.empty(c, device=gu.DEV)
    a = torch.empty_like(z)
    lc.batchnorm_fwd_t(dtype, z, gamma, beta, None, a, mean, invstd, n, c, h, w, EPS, False, NHWC, ws)
    outs = []
    for joined in (False, True):
        fill = -1 if bf16 else float("nan")
        d_pre, dz = torch.full_like(z, fill), torch.full_like(z, fill)
        dg, db = torch.empty(c, device=gu.DEV), torch.empty(c, device=gu.DEV)
        if joined:
            lc.relu_add_bwd_bnsums_t(dtype, y, g1, g2 if two else None, d_pre, z, mean, invstd, n, c, h, w, NHWC, ws)
            lc.batchnorm_bwd_presummed_t(dtype, z, d_pre, gamma, mean, invstd, dz, dg, db, n, c, h, w, NHWC, ws)
        else:
            lc.relu_add_bwd_t(dtype, y, g1, g2 if two else None, d_pre, z.numel())
            lc.batchnorm_bwd_t(dtype, z, d_pre, gamma, None, mean, invstd, dz, dg, db, n, c, h, w, False, NHWC, ws)
        torch.cuda.synchronize()
        outs.append([t.cpu().numpy() for t in (d_pre, dz, dg, db)])
    for u, v in zip(*outs):
        np.testing.assert_array_equal(u, v)
    assert np.all(np.isfinite(outs[1][2])) and np.any(outs[1][1] != 0)


@pytest.mark.parametrize("bf16", [False, True], ids=["fp32", "bf16"])
@pytest.mark.parametrize("two", [True, False], ids=["two_gradients", "one_gradient"])
@pytest.mark.parametrize("case", [(6, 32, 14, 14, 2), (3, 8, 5, 7, 2), (2, 64, 56, 56, 2), (5, 16, 9, 9, 3), (4, 8, 1, 6, 2)],
                         ids=["14x14", "odd_sizes", "many_rows", "stride_3", "one_row"])
def test_block_gradient_from_gradients_on_the_stride_grid(case, two, bf16):
    """relu_add_bwd_bnsums_grid_t takes the arriving gradients as [n, ceil(h/s), ceil(w/s), c] tensors that hold the pixels
    (i s, j s) only (what backward-data of a strided 1x1 convolution produces on its output grid).  Bit for bit the result of
    relu_add_bwd_bnsums_t on the same gradients scattered into zero tensors, sums included (checked through
    batchnorm_bwd_presummed_t); stride 1 is the plain call."""
    n, c, h, w, s = case
    hq, wq = (h + s - 1) // s, (w + s - 1) // s
    dtype = BF if bf16 else lc.LC_F32
    shape, qshape = (n, c, h, w), (n, c, hq, wq)

    def put(a):
        if bf16:
            return _dev(_bf(a)[0])
        return gu.dev(gu.to_layout(a, NHWC))
    z = put((synth.normal(shape, 9950) * 1.5 + 0.4).astype(np.float32))
    y = put(synth.normal(shape, 9951))
    small = [synth.normal(qshape, 9952), synth.normal(qshape, 9953)]
    full = []
    for a in small:
        f = np.zeros(shape, dtype=np.float32)
        f[:, :, ::s, ::s] = a
        full.append(f)
    g_small, g_full = [put(a) for a in small], [put(a) for a in full]
    gamma = gu.dev((1.0 + 0.5 * synth.normal((c,), 9954)).astype(np.float32))
    beta = gu.dev(synth.normal((c,), 9955))
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, NHWC))
    mean, invstd = torch.empty(c, device=gu.DEV), torch.empty(c, device=gu.DEV)
    a = torch.empty_like(z)
    lc.batchnorm_fwd_t(dtype, z, gamma, beta, None, a, mean, invstd, n, c, h, w, EPS, False, NHWC, ws)
    outs = []
    for grid in (False, True):
        fill = -1 if bf16 else float("nan")
        d_pre, dz = torch.full_like(z, fill), torch.full_like(z, fill)
        dg, db = torch.empty(c, device=gu.DEV), torch.empty(c, device=gu.DEV)
        if grid:
            lc.relu_add_bwd_bnsums_grid_t(dtype, y, g_small[0], g_small[1] if two else None, d_pre, z, mean, invstd, n, c, h, w, s, NHWC, ws)
        else:
            lc.relu_add_bwd_bnsums_t(dtype, y, g_full[0], g_full[1] if two else None, d_pre, z, mean, invstd, n, c, h, w, NHWC, ws)
        lc.batchnorm_bwd_presummed_t(dtype, z, d_pre, gamma, mean, invstd, dz, dg, db, n, c, h, w, NHWC, ws)
        torch.cuda.synchronize()
        outs.append([t.cpu().numpy() for t in (d_pre, dz, dg, db)])
    for u, v in zip(*outs):
        np.testing.assert_array_equal(u, v)
    assert np.all(np.isfinite(outs[1][2])) and np.any(outs[1][0] != 0)
    # stride 1: the plain call
    d1, d2 = torch.empty_like(z), torch.empty_like(z)
    lc.relu_add_bwd_bnsums_grid_t(dtype, y, g_full[0], None, d1, z, mean, invstd, n, c, h, w, 1, NHWC, ws)
    lc.relu_add_bwd_bnsums_t(dtype, y, g_full[0], None, d2, z, mean, invstd, n, c, h, w, NHWC, ws)
    torch.cuda.synchronize()
    assert torch.equal(d1.view(torch.int16) if bf16 else d1, d2.view(torch.int16) if bf16 else d2)
