"""GPU parity for grouped convolutions (the original AlexNet's layers, the paper's Table "Scaling Ratio for AlexNet and
ResNet50") through the C ABI against the grouped CPU oracle, fp32 and bf16, both layouts.  Tolerances as for the
one-group layers: fp32 <= 1e-4 tensor-scaled; bf16 y, dx <= 2e-2 and within one bf16 step of the exact value, dw <= 1e-4."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu

# n, c, h, w, k, r, s, stride, pad, groups
SHAPES = {
    "alexnet_conv2_small": (2, 96, 13, 13, 256, 5, 5, 1, 2, 2),
    "alexnet_conv4_small": (3, 384, 7, 7, 384, 3, 3, 1, 1, 2),
    "three_groups_ragged": (2, 24, 11, 9, 36, 3, 2, (2, 1), (1, 0), 3),
    "depthwise": (2, 16, 9, 9, 16, 3, 3, 1, 1, 16),
    "odd_slice_sizes": (2, 10, 8, 8, 6, 3, 3, 1, 1, 2),          # 5 channels and 3 filters per group
    "strided_1x1": (2, 64, 15, 15, 128, 1, 1, 2, 0, 4),
}


def _inputs(shape, seed):
    n, c, h, w, k, r, s, stride, pad, g = shape
    x = synth.normal((n, c, h, w), seed)
    wt = synth.normal((k, c // g, r, s), seed + 1, std=float(np.sqrt(2.0 * g / (c * r * s))))
    p, q = oracle.out_shape(h, w, r, s, stride, pad)
    dy = synth.normal((n, k, p, q), seed + 2)
    return x, wt, dy


def _desc(shape, layout, dtype):
    n, c, h, w, k, r, s, stride, pad, g = shape
    d = gu.desc_for((n, c, h, w), (k, c // g, r, s), stride, pad, layout, dtype)
    return dataclasses.replace(d, groups=g)


@pytest.mark.parametrize("layout", [lc.LC_NHWC, lc.LC_NCHW], ids=["nhwc", "nchw"])
@pytest.mark.parametrize("name", list(SHAPES))
def test_grouped_three_passes_match_oracle_fp32(name, layout):
    shape = SHAPES[name]
    n, c, h, w, k, r, s, stride, pad, g = shape
    x, wt, dy = _inputs(shape, 8000 + 10 * list(SHAPES).index(name))
    d = _desc(shape, layout, lc.LC_F32)
    print(f"grouped case {name} layout {layout} desc {d}", flush=True)
    xl, wl, dyl = gu.to_layout(x, layout), gu.to_layout(wt, layout), gu.to_layout(dy, layout)
    y = gu.from_layout(gu.gpu_fwd(d, xl, wl), layout)
    assert gu.scaled_err(y, oracle.conv2d_fwd_grouped(x, wt, g, stride, pad)) <= 1e-4
    dx = gu.from_layout(gu.gpu_bwd_data(d, dyl, wl), layout)
    assert gu.scaled_err(dx, oracle.conv2d_bwd_data_grouped(dy, wt, g, (h, w), stride, pad)) <= 1e-4
    # gpu_bwd_weight sizes dw from the descriptor's c: take the grouped filter shape instead
    dshape = (k, c // g, r, s) if layout == lc.LC_NCHW else (k, r, s, c // g)
    dw = torch.full(dshape, float("nan"), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_bwd_weight(d, gu.dev(xl), gu.dev(dyl), dw, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT)))
    torch.cuda.synchronize()
    assert gu.scaled_err(gu.from_layout(dw.cpu().numpy(), layout), oracle.conv2d_bwd_weight_grouped(x, dy, g, (r, s), stride, pad)) <= 1e-4


def _bits(a):
    return synth.to_bf16_bits(a)


def _dev_bf16(bits_l):
    return torch.from_numpy(np.ascontiguousarray(bits_l).view(np.int16)).to(gu.DEV)


def _back(t):
    return synth.bf16_bits_to_f32(t.cpu().numpy().view(np.uint16))


@pytest.mark.parametrize("layout", [lc.LC_NHWC, lc.LC_NCHW], ids=["nhwc", "nchw"])
@pytest.mark.parametrize("name", ["alexnet_conv2_small", "alexnet_conv4_small", "three_groups_ragged", "odd_slice_sizes"])
def test_grouped_three_passes_match_oracle_bf16(name, layout):
    shape = SHAPES[name]
    n, c, h, w, k, r, s, stride, pad, g = shape
    raw = _inputs(shape, 8500 + 10 * list(SHAPES).index(name))
    xb, wb, dyb = (_bits(a) for a in raw)
    x, wt, dy = (synth.bf16_bits_to_f32(b) for b in (xb, wb, dyb))
    d = _desc(shape, layout, lc.LC_BF16)
    print(f"grouped bf16 case {name} layout {layout} desc {d}", flush=True)
    p, q = lc.conv2d_out_shape(d)
    xd, wd, dyd = (_dev_bf16(gu.to_layout(a, layout)) for a in (xb, wb, dyb))
    y = torch.full((n, k, p, q) if layout == lc.LC_NCHW else (n, p, q, k), -1, dtype=torch.int16, device=gu.DEV)
    lc.conv2d_fwd(d, xd, wd, y, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)))
    dx = torch.full((n, c, h, w) if layout == lc.LC_NCHW else (n, h, w, c), -1, dtype=torch.int16, device=gu.DEV)
    lc.conv2d_bwd_data(d, dyd, wd, dx, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_DATA)))
    dw = torch.full((k, c // g, r, s) if layout == lc.LC_NCHW else (k, r, s, c // g), float("nan"), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_bwd_weight(d, xd, dyd, dw, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT)))
    torch.cuda.synchronize()
    ref_y = oracle.conv2d_fwd_grouped(x, wt, g, stride, pad)
    ref_dx = oracle.conv2d_bwd_data_grouped(dy, wt, g, (h, w), stride, pad)
    ref_dw = oracle.conv2d_bwd_weight_grouped(x, dy, g, (r, s), stride, pad)
    got_y, got_dx = gu.from_layout(_back(y), layout), gu.from_layout(_back(dx), layout)
    assert gu.scaled_err(got_y, oracle.round_to_bf16(ref_y)) <= 2e-2
    assert gu.scaled_err(got_dx, oracle.round_to_bf16(ref_dx)) <= 2e-2
    assert np.all(np.abs(got_y - ref_y) <= np.abs(ref_y) * 2.0 ** -7 + 1e-6 * np.max(np.abs(ref_y)))
    assert np.all(np.abs(got_dx - ref_dx) <= np.abs(ref_dx) * 2.0 ** -7 + 1e-6 * np.max(np.abs(ref_dx)))
    assert gu.scaled_err(gu.from_layout(dw.cpu().numpy(), layout), ref_dw) <= 1e-4


def test_full_size_grouped_alexnet_layer_sampled():
    # conv2 of the original AlexNet at the benchmark's batch: 256 x 27 x 27 x 96 -> 256 filters of 5x5 over 48 channels
    cs = synth.alexnet_grouped_convs(256)[1]
    g, cg, kg = cs.groups, cs.c // cs.groups, cs.k // cs.groups
    x = synth.normal((cs.n, cs.h, cs.w, cs.c), 8800)
    wt = synth.normal((cs.k, cs.r, cs.s, cg), 8801, std=float(np.sqrt(2.0 / (cg * cs.r * cs.s))))
    d = lc.ConvDesc(cs.n, cs.c, cs.h, cs.w, cs.k, cs.r, cs.s, cs.stride, cs.stride, cs.pad, cs.pad, lc.LC_F32, lc.LC_NHWC, g)
    print(f"full-size grouped layer {d}", flush=True)
    y = gu.gpu_fwd(d, x, wt)
    coords = synth.sample_coords(2048, (cs.n, cs.k, cs.p, cs.q), 8802)
    # every sampled output is a one-group output of its group's slices: the pinned single-element evaluator applies
    worst = 0.0
    for grp in range(g):
        sel = coords[(coords[:, 1] // kg) == grp].copy()
        got = y[sel[:, 0], sel[:, 2], sel[:, 3], sel[:, 1]]
        sel[:, 1] -= grp * kg
        ref, mag = oracle.conv2d_fwd_at(np.ascontiguousarray(x[..., grp * cg:(grp + 1) * cg]), wt[grp * kg:(grp + 1) * kg], sel,
                                        cs.stride, cs.pad, oracle.NHWC)
        worst = max(worst, float(np.max(np.abs(got - ref) / mag)))
    print(f"worst |err| / sum|terms| = {worst:.2e}", flush=True)
    assert worst <= 1e-5
