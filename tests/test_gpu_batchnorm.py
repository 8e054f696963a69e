"""GPU parity: batchnorm_fwd / batchnorm_bwd through the C ABI against the numpy float64 oracle, both layouts,
vector and scalar paths, shapes from ResNet-50 and AlexNet-BN down to single pixels.  Tolerance 1e-4 tensor-scaled
(fp32 per-thread partial sums of x - pivot and its square, fp64 combination)."""
import numpy as np
import pytest
import torch

from oracle import batchnorm as obn
from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 1e-4
EPS = 1e-5

SHAPES = {
    "resnet_56x56_c64": (8, 64, 56, 56),
    "resnet_7x7_c2048": (16, 2048, 7, 7),
    "alexnet_13x13_c384": (8, 384, 13, 13),
    "alexnet_c96": (3, 96, 27, 27),
    "odd_channels_scalar_path": (5, 7, 9, 11),
    "one_pixel_per_image": (64, 10, 1, 1),
    "single_image": (1, 12, 6, 5),
    "many_slabs": (32, 16, 64, 64),
}


def _lay(a, layout):
    return np.ascontiguousarray(a.transpose(0, 2, 3, 1)) if layout == lc.LC_NHWC else np.ascontiguousarray(a)


def _unlay(a, layout):
    return a.transpose(0, 3, 1, 2) if layout == lc.LC_NHWC else a


def _run(shape, layout, seed, offset=0):
    n, c, h, w = shape
    x = (synth.normal(shape, seed) * 2.0 + 0.7).astype(np.float32)          # non-zero mean
    dy = synth.normal(shape, seed + 1)
    gamma = (1.0 + 0.5 * synth.normal((c,), seed + 2)).astype(np.float32)
    beta = synth.normal((c,), seed + 3)

    def put(a):                                                               # optional misalignment by `offset` floats
        buf = torch.empty(a.size + offset, dtype=torch.float32, device=gu.DEV)
        v = buf[offset:]
        v.copy_(torch.from_numpy(np.ascontiguousarray(a).reshape(-1)))
        return v
    xd, dyd = put(_lay(x, layout)), put(_lay(dy, layout))
    gd, bd = gu.dev(gamma), gu.dev(beta)
    y, dx = torch.empty_like(xd), torch.empty_like(xd)
    mean, invstd, dg, db = (torch.empty(c, device=gu.DEV) for _ in range(4))
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, layout))
    lc.batchnorm_fwd(xd, gd, bd, y, mean, invstd, n, c, h, w, EPS, layout, ws)
    lc.batchnorm_bwd(xd, dyd, gd, mean, invstd, dx, dg, db, n, c, h, w, layout, ws)
    torch.cuda.synchronize()
    shp = (n, h, w, c) if layout == lc.LC_NHWC else shape
    oy, omean, oinv = obn.forward(x, gamma, beta, EPS)
    odx, odg, odb = obn.backward(x, dy, gamma, EPS)
    assert gu.scaled_err(_unlay(y.cpu().numpy().reshape(shp), layout), oy) <= TOL
    assert gu.scaled_err(mean.cpu().numpy(), omean) <= 1e-5
    assert np.max(np.abs(invstd.cpu().numpy() - oinv) / oinv) <= 1e-4
    assert gu.scaled_err(_unlay(dx.cpu().numpy().reshape(shp), layout), odx) <= TOL
    assert gu.scaled_err(dg.cpu().numpy(), odg) <= TOL
    assert gu.scaled_err(db.cpu().numpy(), odb) <= TOL


@pytest.mark.parametrize("layout", [lc.LC_NHWC, lc.LC_NCHW], ids=["nhwc", "nchw"])
@pytest.mark.parametrize("name", list(SHAPES))
def test_forward_and_backward_match_oracle(name, layout):
    _run(SHAPES[name], layout, 8300 + 10 * list(SHAPES).index(name))


def test_misaligned_tensors_take_the_scalar_path():
    _run((4, 16, 9, 9), lc.LC_NHWC, 8500, offset=1)


def test_reruns_are_bit_identical():
    n, c, h, w = 16, 128, 28, 28
    x = gu.dev(synth.normal((n, h, w, c), 8600))
    g, b = gu.dev(np.ones(c, np.float32)), gu.dev(np.zeros(c, np.float32))
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, lc.LC_NHWC))
    outs = []
    for _ in range(2):
        y, m, s = torch.empty_like(x), torch.empty(c, device=gu.DEV), torch.empty(c, device=gu.DEV)
        lc.batchnorm_fwd(x, g, b, y, m, s, n, c, h, w, EPS, lc.LC_NHWC, ws)
        torch.cuda.synchronize()
        outs.append((y.cpu().numpy(), m.cpu().numpy(), s.cpu().numpy()))
    for a, bb in zip(outs[0], outs[1]):
        np.testing.assert_array_equal(a, bb)


# ---------------------------------------------------------------- fused forms
def _fused_case(shape, seed):
    n, c, h, w = shape
    x = (synth.normal(shape, seed) * 1.5 - 0.3).astype(np.float32)
    dy = synth.normal(shape, seed + 1)
    res = synth.normal(shape, seed + 4)
    gamma = (1.0 + 0.5 * synth.normal((c,), seed + 2)).astype(np.float32)
    beta = (0.5 * synth.normal((c,), seed + 3)).astype(np.float32)
    return x, dy, res, gamma, beta


@pytest.mark.parametrize("layout", [lc.LC_NHWC, lc.LC_NCHW], ids=["nhwc", "nchw"])
@pytest.mark.parametrize("shape", [(6, 32, 14, 14), (3, 7, 5, 9)], ids=["vector", "scalar"])
@pytest.mark.parametrize("relu,residual", [(True, False), (False, True), (True, True)], ids=["relu", "residual", "residual_relu"])
def test_fused_forward_matches_oracle(shape, layout, relu, residual):
    n, c, h, w = shape
    x, _, res, gamma, beta = _fused_case(shape, 8700)
    xd, gd, bd = gu.dev(_lay(x, layout)), gu.dev(gamma), gu.dev(beta)
    rd = gu.dev(_lay(res, layout)) if residual else None
    y = torch.empty_like(xd)
    mean, invstd = torch.empty(c, device=gu.DEV), torch.empty(c, device=gu.DEV)
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, layout))
    lc.batchnorm_fwd_ex(xd, gd, bd, rd, y, mean, invstd, n, c, h, w, EPS, relu, layout, ws)
    torch.cuda.synchronize()
    want, _, _ = obn.forward(x, gamma, beta, EPS)
    if residual:
        want = want + res.astype(np.float64)
    if relu:
        want = np.maximum(want, 0.0)
    assert gu.scaled_err(_unlay(y.cpu().numpy(), layout), want) <= TOL


@pytest.mark.parametrize("layout", [lc.LC_NHWC, lc.LC_NCHW], ids=["nhwc", "nchw"])
@pytest.mark.parametrize("shape", [(6, 32, 14, 14), (3, 7, 5, 9)], ids=["vector", "scalar"])
def test_backward_through_relu_matches_oracle(shape, layout):
    """The gradient is taken as zero where the batch-norm output is not positive.  Elements whose output the
    oracle puts within 1e-4 of zero get dy = 0 on both sides: there fp32 and float64 may disagree on the sign."""
    n, c, h, w = shape
    x, dy, _, gamma, beta = _fused_case(shape, 8800)
    oy, _, _ = obn.forward(x, gamma, beta, EPS)
    dy = np.where(np.abs(oy) < 1e-4, 0.0, dy).astype(np.float32)
    xd, dyd, gd, bd = gu.dev(_lay(x, layout)), gu.dev(_lay(dy, layout)), gu.dev(gamma), gu.dev(beta)
    y, dx = torch.empty_like(xd), torch.empty_like(xd)
    mean, invstd, dg, db = (torch.empty(c, device=gu.DEV) for _ in range(4))
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, layout))
    lc.batchnorm_fwd_ex(xd, gd, bd, None, y, mean, invstd, n, c, h, w, EPS, True, layout, ws)
    lc.batchnorm_bwd_ex(xd, dyd, gd, bd, mean, invstd, dx, dg, db, n, c, h, w, True, layout, ws)
    torch.cuda.synchronize()
    odx, odg, odb = obn.backward(x, np.where(oy > 0.0, dy, 0.0), gamma, EPS)
    assert gu.scaled_err(_unlay(dx.cpu().numpy(), layout), odx) <= TOL
    assert gu.scaled_err(dg.cpu().numpy(), odg) <= TOL
    assert gu.scaled_err(db.cpu().numpy(), odb) <= TOL


@pytest.mark.parametrize("layout", [lc.LC_NHWC, lc.LC_NCHW], ids=["nhwc", "nchw"])
def test_rebuilt_mask_is_the_mask_of_the_stored_output(layout):
    """batchnorm_bwd_ex(relu) on dy must equal batchnorm_bwd on dy masked with the stored forward output > 0,
    bit for bit: the backward pass rebuilds the forward's value exactly."""
    n, c, h, w = 8, 64, 28, 28
    x, dy, _, gamma, beta = _fused_case((n, c, h, w), 8900)
    xd, dyd, gd, bd = gu.dev(_lay(x, layout)), gu.dev(_lay(dy, layout)), gu.dev(gamma), gu.dev(beta)
    y = torch.empty_like(xd)
    mean, invstd = torch.empty(c, device=gu.DEV), torch.empty(c, device=gu.DEV)
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, layout))
    lc.batchnorm_fwd_ex(xd, gd, bd, None, y, mean, invstd, n, c, h, w, EPS, True, layout, ws)
    outs = []
    for fused in (True, False):
        dx, dg, db = torch.empty_like(xd), torch.empty(c, device=gu.DEV), torch.empty(c, device=gu.DEV)
        if fused:
            lc.batchnorm_bwd_ex(xd, dyd, gd, bd, mean, invstd, dx, dg, db, n, c, h, w, True, layout, ws)
        else:
            masked = torch.empty_like(xd)
            lc.relu_add_bwd(y, dyd, None, masked, xd.numel())
            lc.batchnorm_bwd(xd, masked, gd, mean, invstd, dx, dg, db, n, c, h, w, layout, ws)
        torch.cuda.synchronize()
        outs.append((dx.cpu().numpy(), dg.cpu().numpy(), db.cpu().numpy()))
    assert float((y > 0).float().mean()) > 0.2             # the mask is not trivial
    for a, b in zip(*outs):
        np.testing.assert_array_equal(a, b)


@pytest.mark.parametrize("layout", [lc.LC_NHWC, lc.LC_NCHW], ids=["nhwc", "nchw"])
def test_degenerate_batches(layout):
    """One value per channel (the batch variance is 0, y = beta, dx = 0 up to rounding) and a constant tensor."""
    for shape, const in (((1, 8, 1, 1), None), ((4, 8, 3, 3), 2.5)):
        n, c, h, w = shape
        x = synth.normal(shape, 8950) if const is None else np.full(shape, const, np.float32)
        dy = synth.normal(shape, 8951)
        gamma = (1.0 + 0.5 * synth.normal((c,), 8952)).astype(np.float32)
        beta = synth.normal((c,), 8953)
        xd, dyd, gd, bd = gu.dev(_lay(x, layout)), gu.dev(_lay(dy, layout)), gu.dev(gamma), gu.dev(beta)
        y, dx = torch.empty_like(xd), torch.empty_like(xd)
        mean, invstd, dg, db = (torch.empty(c, device=gu.DEV) for _ in range(4))
        ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, layout))
        lc.batchnorm_fwd(xd, gd, bd, y, mean, invstd, n, c, h, w, EPS, layout, ws)
        lc.batchnorm_bwd(xd, dyd, gd, mean, invstd, dx, dg, db, n, c, h, w, layout, ws)
        torch.cuda.synchronize()
        oy, omean, oinv = obn.forward(x, gamma, beta, EPS)
        odx, odg, odb = obn.backward(x, dy, gamma, EPS)
        assert np.allclose(invstd.cpu().numpy(), 1.0 / np.sqrt(EPS), rtol=1e-5)          # variance exactly 0 on both sides
        assert np.allclose(oinv, 1.0 / np.sqrt(EPS), rtol=1e-12)
        assert np.max(np.abs(_unlay(y.cpu().numpy(), layout) - oy)) <= 1e-3               # |x - mean| <= 1 ulp, times 1/sqrt(eps) = 316
        assert gu.scaled_err(db.cpu().numpy(), odb) <= TOL
        # xhat is exactly 0 on both sides (the mean of equal values is exact), so dgamma = 0 and
        # dx = gamma / sqrt(eps) * (dy - mean(dy)): values of order 1e3, compared at fp32 rounding of that scale
        assert np.max(np.abs(dg.cpu().numpy() - odg)) <= 1e-6
        bound = 1e-5 * float(np.max(np.abs(gamma))) / np.sqrt(EPS) * float(np.max(np.abs(dy)))
        assert np.max(np.abs(_unlay(dx.cpu().numpy(), layout) - odx)) <= bound


@pytest.mark.parametrize("layout", [lc.LC_NHWC, lc.LC_NCHW], ids=["nhwc", "nchw"])
def test_mean_far_from_zero_against_the_spread(layout):
    """Mean 10, spread 0.05: sums of x and x^2 in fp32 would lose the variance to cancellation."""
    n, c, h, w = 8, 16, 12, 12
    x = (10.0 + 0.05 * synth.normal((n, c, h, w), 8960)).astype(np.float32)
    gamma = np.ones(c, np.float32)
    beta = np.zeros(c, np.float32)
    xd, gd, bd = gu.dev(_lay(x, layout)), gu.dev(gamma), gu.dev(beta)
    y = torch.empty_like(xd)
    mean, invstd = torch.empty(c, device=gu.DEV), torch.empty(c, device=gu.DEV)
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, layout))
    lc.batchnorm_fwd(xd, gd, bd, y, mean, invstd, n, c, h, w, EPS, layout, ws)
    torch.cuda.synchronize()
    oy, omean, oinv = obn.forward(x, gamma, beta, EPS)
    assert np.max(np.abs(invstd.cpu().numpy() - oinv) / oinv) <= 1e-5
    assert gu.scaled_err(_unlay(y.cpu().numpy(), layout), oy) <= TOL


def test_full_size_stem_output_sampled():
    """The largest tensor of the ResNet-50 step at its real size (batch 256, 112x112, 64 channels: 205 M values, the
    launch geometry bench.py times): statistics and channel gradients against float64 sums over the whole tensor,
    y and dx on sampled elements."""
    n, c, h, w = 256, 64, 112, 112
    gen = torch.Generator(device=gu.DEV)
    gen.manual_seed(8970)
    x = torch.randn((n, h, w, c), generator=gen, device=gu.DEV) * 1.7 + 0.4
    dy = torch.randn((n, h, w, c), generator=gen, device=gu.DEV)
    gamma = (1.0 + 0.3 * synth.normal((c,), 8971)).astype(np.float32)
    beta = (0.2 * synth.normal((c,), 8972)).astype(np.float32)
    gd, bd = gu.dev(gamma), gu.dev(beta)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    mean, invstd, dg, db = (torch.empty(c, device=gu.DEV) for _ in range(4))
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, lc.LC_NHWC))
    lc.batchnorm_fwd(x, gd, bd, y, mean, invstd, n, c, h, w, EPS, lc.LC_NHWC, ws)
    lc.batchnorm_bwd(x, dy, gd, mean, invstd, dx, dg, db, n, c, h, w, lc.LC_NHWC, ws)
    torch.cuda.synchronize()
    # the oracle's definitions on the whole tensor, in float64, one channel block at a time to bound host memory
    xh = x.cpu().numpy().reshape(-1, c)
    dyh = dy.cpu().numpy().reshape(-1, c)
    m = xh.shape[0]
    omean = xh.mean(axis=0, dtype=np.float64)
    ovar = np.zeros(c)
    odb = dyh.sum(axis=0, dtype=np.float64)
    odg = np.zeros(c)
    for c0 in range(0, c, 8):
        blk = xh[:, c0:c0 + 8].astype(np.float64) - omean[c0:c0 + 8]
        ovar[c0:c0 + 8] = (blk * blk).mean(axis=0)
        odg[c0:c0 + 8] = (dyh[:, c0:c0 + 8] * blk).sum(axis=0) / np.sqrt(ovar[c0:c0 + 8] + EPS)
    oinv = 1.0 / np.sqrt(ovar + EPS)
    assert gu.scaled_err(mean.cpu().numpy(), omean) <= 1e-5
    assert np.max(np.abs(invstd.cpu().numpy() - oinv) / oinv) <= 1e-5
    assert gu.scaled_err(db.cpu().numpy(), odb) <= TOL
    assert gu.scaled_err(dg.cpu().numpy(), odg) <= TOL
    rows = synth.uniform_int(4096, 8973, m)
    xs, dys = xh[rows].astype(np.float64), dyh[rows].astype(np.float64)
    xhat = (xs - omean) * oinv
    want_y = gamma * xhat + beta
    want_dx = gamma * oinv * (dys - odb / m - xhat * odg / m)
    got_y = y.reshape(-1, c)[torch.from_numpy(rows).to(gu.DEV)].cpu().numpy()
    got_dx = dx.reshape(-1, c)[torch.from_numpy(rows).to(gu.DEV)].cpu().numpy()
    assert np.max(np.abs(got_y - want_y)) <= TOL * np.max(np.abs(want_y))
    assert np.max(np.abs(got_dx - want_dx)) <= TOL * np.max(np.abs(want_dx))
