"""GPU parity of batchnorm_fwd_pair_t, y = relu?(bn(x) + bn2(x2)) in one stream pass (the output of a residual block whose
shortcut has a projection): against the float64 oracle (two batch norms, a sum, a clamp), and against the two plain calls
it replaces.  fp32 in both layouts (statistics by a pass over each tensor) and in NHWC with the statistics handed over by
the convolutions that made x and x2 (conv2d_fwd_stats); bf16 in NHWC, where the fused form rounds once (the shortcut's
value is not rounded to bf16 before the sum), so it lies within one bf16 step of the float64 value.
Tolerances: 1e-4 tensor-scaled in fp32 (as for batch norm); one bf16 step element by element in bf16."""
import numpy as np
import pytest
import torch

import oracle
from oracle import batchnorm as obn
from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 1e-4
EPS = 1e-5
NHWC = lc.LC_NHWC

SHAPES = {
    "block_output_56x56": (4, 256, 56, 56),
    "block_output_7x7": (16, 2048, 7, 7),
    "odd_channels_scalar_path": (5, 7, 9, 11),
    "one_pixel_per_image": (64, 12, 1, 1),
}


def _params(c, seed):
    return ((1.0 + 0.5 * synth.normal((c,), seed)).astype(np.float32), synth.normal((c,), seed + 1),
            (1.0 + 0.5 * synth.normal((c,), seed + 2)).astype(np.float32), synth.normal((c,), seed + 3))


def _want(x, x2, g1, b1, g2, b2, relu):
    y1, m1, i1 = obn.forward(x, g1, b1, EPS)
    y2, m2, i2 = obn.forward(x2, g2, b2, EPS)
    y = y1 + y2
    return (np.maximum(y, 0.0) if relu else y), m1, i1, m2, i2


@pytest.mark.parametrize("relu", [True, False], ids=["relu", "no_relu"])
@pytest.mark.parametrize("layout", [lc.LC_NCHW, lc.LC_NHWC], ids=["nchw", "nhwc"])
@pytest.mark.parametrize("name", list(SHAPES))
def test_pair_fp32_matches_oracle_and_the_two_plain_calls(name, layout, relu):
    n, c, h, w = SHAPES[name]
    seed = 8800 + 10 * list(SHAPES).index(name)
    x = (synth.normal((n, c, h, w), seed) * 1.5 + 0.4).astype(np.float32)
    x2 = (synth.normal((n, c, h, w), seed + 1) * 0.7 - 0.2).astype(np.float32)
    g1, b1, g2, b2 = _params(c, seed + 2)
    xd, x2d = gu.dev(gu.to_layout(x, layout)), gu.dev(gu.to_layout(x2, layout))
    gd = [gu.dev(a) for a in (g1, b1, g2, b2)]
    y = torch.full_like(xd, float("nan"))
    m1, i1, m2, i2 = (torch.full((c,), float("nan"), device=gu.DEV) for _ in range(4))
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, layout))
    lc.batchnorm_fwd_pair_t(lc.LC_F32, xd, gd[0], gd[1], None, 0, x2d, gd[2], gd[3], None, 0, y, m1, i1, m2, i2, n, c, h, w, EPS, relu,
                            layout, ws)
    torch.cuda.synchronize()
    want, om1, oi1, om2, oi2 = _want(x, x2, g1, b1, g2, b2, relu)
    got = gu.from_layout(y.cpu().numpy(), layout)
    assert np.all(np.isfinite(got))
    assert gu.scaled_err(got, want) <= TOL
    for a, b in ((m1, om1), (m2, om2)):
        assert gu.scaled_err(a.cpu().numpy(), b) <= 1e-5
    for a, b in ((i1, oi1), (i2, oi2)):
        assert np.max(np.abs(a.cpu().numpy() - b) / b) <= 1e-4
    # the two calls it replaces
    mid, y2 = torch.empty_like(xd), torch.empty_like(xd)
    ma, ia, mb, ib = (torch.empty(c, device=gu.DEV) for _ in range(4))
    lc.batchnorm_fwd_t(lc.LC_F32, x2d, gd[2], gd[3], None, mid, mb, ib, n, c, h, w, EPS, False, layout, ws)
    lc.batchnorm_fwd_t(lc.LC_F32, xd, gd[0], gd[1], mid, y2, ma, ia, n, c, h, w, EPS, relu, layout, ws)
    torch.cuda.synchronize()
    assert gu.scaled_err(got, gu.from_layout(y2.cpu().numpy(), layout)) <= 2e-6
    np.testing.assert_array_equal(m1.cpu().numpy(), ma.cpu().numpy())
    np.testing.assert_array_equal(i2.cpu().numpy(), ib.cpu().numpy())


@pytest.mark.parametrize("bf16", [False, True], ids=["fp32", "bf16"])
def test_pair_with_the_statistics_of_both_convolutions(bf16):
    """A projection block in small: x -> 1x1 convolution (the block's last) and x0 -> strided 1x1 projection, both with
    conv2d_fwd_stats; the pair takes both sets of pieces.  Against the oracle on the device's own convolution outputs."""
    n, c_in, hw, k = 8, 64, 14, 256
    seed = 8900
    dtype = lc.LC_BF16 if bf16 else lc.LC_F32

    def put(a_nchw):
        a = gu.to_layout(a_nchw, NHWC)
        return torch.from_numpy(synth.to_bf16_bits(a).view(np.int16)).to(gu.DEV) if bf16 else gu.dev(a)

    def get(t):
        a = t.cpu().numpy()
        return gu.from_layout(synth.bf16_bits_to_f32(a.view(np.uint16)) if bf16 else a, NHWC)

    xa = synth.normal((n, c_in, hw, hw), seed)
    xb = synth.normal((n, 2 * c_in, 2 * hw, 2 * hw), seed + 1)
    wa = synth.normal((k, c_in, 1, 1), seed + 2, std=0.2)
    wb = synth.normal((k, 2 * c_in, 1, 1), seed + 3, std=0.15)
    da = gu.desc_for(xa.shape, wa.shape, 1, 0, NHWC, dtype)
    db = gu.desc_for(xb.shape, wb.shape, 2, 0, NHWC, dtype)
    ta, tb = lc.conv2d_fwd_stats_count(da), lc.conv2d_fwd_stats_count(db)
    assert ta > 0 and tb > 0
    tdt = torch.int16 if bf16 else torch.float32
    za = torch.empty((n, hw, hw, k), dtype=tdt, device=gu.DEV)
    zb = torch.empty((n, hw, hw, k), dtype=tdt, device=gu.DEV)
    sa = torch.full((ta, k, 2), float("nan"), dtype=torch.float32, device=gu.DEV)
    sb = torch.full((tb, k, 2), float("nan"), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_fwd_stats(da, put(xa), put(wa), za, sa, gu.workspace(lc.conv2d_workspace_bytes(da, lc.LC_PASS_FWD)))
    lc.conv2d_fwd_stats(db, put(xb), put(wb), zb, sb, gu.workspace(lc.conv2d_workspace_bytes(db, lc.LC_PASS_FWD)))
    g1, b1, g2, b2 = _params(k, seed + 4)
    gd = [gu.dev(a) for a in (g1, b1, g2, b2)]
    y = torch.full_like(za, -1 if bf16 else float("nan"))
    m1, i1, m2, i2 = (torch.full((k,), float("nan"), device=gu.DEV) for _ in range(4))
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, k, hw, hw, NHWC))
    lc.batchnorm_fwd_pair_t(dtype, za, gd[0], gd[1], sa, ta, zb, gd[2], gd[3], sb, tb, y, m1, i1, m2, i2, n, k, hw, hw, EPS, True, NHWC, ws)
    torch.cuda.synchronize()
    want, om1, oi1, om2, oi2 = _want(get(za), get(zb), g1, b1, g2, b2, True)
    got = get(y)
    assert np.all(np.isfinite(got))
    assert gu.scaled_err(m1.cpu().numpy(), om1) <= 1e-5 and gu.scaled_err(m2.cpu().numpy(), om2) <= 1e-5
    assert np.max(np.abs(i1.cpu().numpy() - oi1) / oi1) <= 1e-4 and np.max(np.abs(i2.cpu().numpy() - oi2) / oi2) <= 1e-4
    if bf16:
        assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -8 + 2e-4 * float(np.max(np.abs(want))))
        assert gu.scaled_err(got, oracle.round_to_bf16(want)) <= 2e-2
    else:
        assert gu.scaled_err(got, want) <= TOL


def test_pair_bf16_against_the_two_plain_calls():
    """bf16: the two plain calls round the shortcut's batch-norm output to bf16 before the sum, the pair does not; both lie
    within a bf16 step of the float64 value, so they differ by at most two steps, and in few elements."""
    n, c, h, w = 6, 128, 14, 14
    bits = lambda a: torch.from_numpy(synth.to_bf16_bits(np.ascontiguousarray(a.transpose(0, 2, 3, 1))).view(np.int16)).to(gu.DEV)   # noqa: E731
    back = lambda t: synth.bf16_bits_to_f32(t.cpu().numpy().view(np.uint16)).transpose(0, 3, 1, 2)                                    # noqa: E731
    x = (synth.normal((n, c, h, w), 8950) + 0.3).astype(np.float32)
    x2 = (synth.normal((n, c, h, w), 8951) * 0.5).astype(np.float32)
    g1, b1, g2, b2 = _params(c, 8952)
    gd = [gu.dev(a) for a in (g1, b1, g2, b2)]
    xd, x2d = bits(x), bits(x2)
    y, mid, y2 = (torch.full_like(xd, -1) for _ in range(3))
    st = [torch.empty(c, device=gu.DEV) for _ in range(8)]
    ws = gu.workspace(lc.batchnorm_workspace_bytes(n, c, h, w, NHWC))
    lc.batchnorm_fwd_pair_t(lc.LC_BF16, xd, gd[0], gd[1], None, 0, x2d, gd[2], gd[3], None, 0, y, st[0], st[1], st[2], st[3], n, c, h, w, EPS,
                            True, NHWC, ws)
    lc.batchnorm_fwd_t(lc.LC_BF16, x2d, gd[2], gd[3], None, mid, st[6], st[7], n, c, h, w, EPS, False, NHWC, ws)
    lc.batchnorm_fwd_t(lc.LC_BF16, xd, gd[0], gd[1], mid, y2, st[4], st[5], n, c, h, w, EPS, True, NHWC, ws)
    torch.cuda.synchronize()
    got, plain = back(y), back(y2)
    want, *_ = _want(back(xd), back(x2d), g1, b1, g2, b2, True)
    assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -8 + 2e-4 * float(np.max(np.abs(want))))
    assert np.all(np.abs(got - plain) <= np.abs(plain) * 2.0 ** -6 + 1e-3 * float(np.max(np.abs(want))))
    assert np.mean(got == plain) >= 0.7
    np.testing.assert_array_equal(st[0].cpu().numpy(), st[4].cpu().numpy())
    np.testing.assert_array_equal(st[3].cpu().numpy(), st[7].cpu().numpy())
