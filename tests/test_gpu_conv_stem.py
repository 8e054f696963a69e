"""GPU parity of the fp32 kernels for ResNet's first layer (7x7 window, stride 2, padding 3, 3 -> 64 channels, NHWC, output
height and width multiples of 16), forward and backward-weight, which run a tile of 16 x 16 output pixels from an input slab
in LDS: one tile and several
per block, images of odd height and width (the last window rows and columns hang over the edge on both sides or on one),
more than one tile per image in both directions, more blocks than tiles.  Each result is compared with the float64 oracle
element by element (1e-4 tensor-scaled: both sides use the same fp32 operands, the GPU sums 147 products in fp32) and with
the general kernel's result (LARSCONV_NO_STEM_DIRECT, read whenever a call is planned).  The statistics the kernel hands
to batch norm (one piece per 4 x 16 block of output pixels) are checked piece by piece in test_gpu_conv_stats.py; the layer
at its full size (256 x 224 x 224 x 3) is a case of test_gpu_conv.py's sampled full-size test."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 1e-4
NHWC = lc.LC_NHWC

SHAPES = {
    # n, h, w
    "one_tile": (1, 32, 32),
    "tall_images": (3, 64, 32),
    "odd_height_and_width": (2, 31, 63),
    "several_tiles_each_way": (2, 96, 64),
    "many_small_images": (70, 32, 32),
}


@pytest.fixture
def restore_env():
    old = os.environ.get("LARSCONV_NO_STEM_DIRECT")
    os.environ.pop("LARSCONV_NO_STEM_DIRECT", None)
    yield
    if old is None:
        os.environ.pop("LARSCONV_NO_STEM_DIRECT", None)
    else:
        os.environ["LARSCONV_NO_STEM_DIRECT"] = old


@pytest.mark.parametrize("name", list(SHAPES))
def test_first_layer_kernel_matches_oracle_and_general_kernel(name, restore_env):
    n, h, w = SHAPES[name]
    seed = 5300 + 10 * list(SHAPES).index(name)
    x = synth.normal((n, 3, h, w), seed)
    wt = synth.normal((64, 3, 7, 7), seed + 1, std=float(np.sqrt(2.0 / 147)))
    d = gu.desc_for(x.shape, wt.shape, 2, 3, NHWC)
    p, q = lc.conv2d_out_shape(d)
    assert p % 16 == 0 and q % 16 == 0
    print(f"first-layer case {name} desc {d} -> {p} x {q}", flush=True)
    xl, wl = gu.to_layout(x, NHWC), gu.to_layout(wt, NHWC)
    y = gu.from_layout(gu.gpu_fwd(d, xl, wl), NHWC)
    ref = oracle.conv2d_fwd(x, wt, 2, 3)
    assert np.all(np.isfinite(y))                                  # every element written (the output starts as NaN)
    assert gu.scaled_err(y, ref) <= TOL
    assert lc.conv2d_fwd_stats_count(d) == n * (p // 16) * (q // 16) * 4
    os.environ["LARSCONV_NO_STEM_DIRECT"] = "1"
    other = gu.from_layout(gu.gpu_fwd(d, xl, wl), NHWC)
    assert gu.scaled_err(other, ref) <= TOL
    assert gu.scaled_err(y, other) <= 1e-5


@pytest.mark.parametrize("name", list(SHAPES))
def test_first_layer_filter_gradient_matches_oracle_and_general_kernel(name, restore_env):
    n, h, w = SHAPES[name]
    seed = 5500 + 10 * list(SHAPES).index(name)
    x = synth.normal((n, 3, h, w), seed)
    d = gu.desc_for(x.shape, (64, 3, 7, 7), 2, 3, NHWC)
    p, q = lc.conv2d_out_shape(d)
    dy = synth.normal((n, 64, p, q), seed + 2)
    print(f"first-layer filter gradient case {name} desc {d}", flush=True)
    xl, dyl = gu.to_layout(x, NHWC), gu.to_layout(dy, NHWC)
    dw = gu.from_layout(gu.gpu_bwd_weight(d, xl, dyl), NHWC)
    ref = oracle.conv2d_bwd_weight(x, dy, (7, 7), 2, 3)
    assert np.all(np.isfinite(dw))
    assert gu.scaled_err(dw, ref) <= TOL
    np.testing.assert_array_equal(dw, gu.from_layout(gu.gpu_bwd_weight(d, xl, dyl), NHWC))   # fixed order: reruns are bit-identical
    # the squared norm for LARS comes out of the sum over the blocks' partials
    count = lc.conv2d_bwd_weight_sq_count(d)
    pieces = torch.full((count,), float("nan"), dtype=torch.float64, device=gu.DEV)
    dw2 = torch.full((64, 7, 7, 3), float("nan"), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_bwd_weight_sq(d, gu.dev(xl), gu.dev(dyl), dw2, pieces, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT)))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(gu.from_layout(dw2.cpu().numpy(), NHWC), dw)
    want = float(np.sum(dw.astype(np.float64) ** 2))
    assert abs(float(pieces.sum().item()) - want) <= 1e-6 * want
    os.environ["LARSCONV_NO_STEM_DIRECT"] = "1"
    other = gu.from_layout(gu.gpu_bwd_weight(d, xl, dyl), NHWC)
    assert gu.scaled_err(other, ref) <= TOL
    assert gu.scaled_err(dw, other) <= 2e-5


@pytest.mark.parametrize("name", list(SHAPES))
def test_first_layer_bf16_forward_matches_oracle_and_general_path(name, restore_env):
    """bf16 operands and result, fp32 sums, one rounding: within one bf16 step of the float64 value element by element, and
    equal to the result of the path over 2x2 pixel blocks in all but a few elements (same products, another order)."""
    n, h, w = SHAPES[name]
    seed = 5600 + 10 * list(SHAPES).index(name)
    xb = synth.to_bf16_bits(synth.normal((n, 3, h, w), seed))
    wb = synth.to_bf16_bits(synth.normal((64, 3, 7, 7), seed + 1, std=float(np.sqrt(2.0 / 147))))
    x, wt = synth.bf16_bits_to_f32(xb), synth.bf16_bits_to_f32(wb)
    d = gu.desc_for(x.shape, wt.shape, 2, 3, NHWC, lc.LC_BF16)
    p, q = lc.conv2d_out_shape(d)
    put = lambda bits: torch.from_numpy(np.ascontiguousarray(gu.to_layout(bits, NHWC)).view(np.int16)).to(gu.DEV)   # noqa: E731
    xd, wd = put(xb), put(wb)

    def run():
        y = torch.full((n, p, q, 64), -1, dtype=torch.int16, device=gu.DEV)
        lc.conv2d_fwd(d, xd, wd, y, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)))
        torch.cuda.synchronize()
        return gu.from_layout(synth.bf16_bits_to_f32(y.cpu().numpy().view(np.uint16)), NHWC)

    y = run()
    ref = oracle.conv2d_fwd(x, wt, 2, 3)
    assert np.all(np.isfinite(y))                                  # the fill pattern is a NaN
    assert gu.scaled_err(y, oracle.round_to_bf16(ref)) <= 2e-2
    assert np.all(np.abs(y - ref) <= np.abs(ref) * 2.0 ** -7 + 1e-6 * float(np.max(np.abs(ref))))
    assert lc.conv2d_fwd_stats_count(d) == n * (p // 16) * (q // 16) * 4
    os.environ["LARSCONV_NO_STEM_DIRECT"] = "1"
    other = run()
    assert np.mean(y == other) >= 0.99
    assert np.all(np.abs(y - other) <= np.abs(other) * 2.0 ** -7 + 1e-6 * float(np.max(np.abs(other))))


@pytest.mark.parametrize("name", list(SHAPES))
def test_first_layer_bf16_filter_gradient_matches_oracle_and_general_path(name, restore_env):
    """bf16 x and dy, fp32 sums and dw: exact products of bf16 values, so the result agrees with the float64 oracle on the
    same operands to fp32 summation error, and with the path over 2x2 pixel blocks likewise."""
    n, h, w = SHAPES[name]
    seed = 5700 + 10 * list(SHAPES).index(name)
    xb = synth.to_bf16_bits(synth.normal((n, 3, h, w), seed))
    x = synth.bf16_bits_to_f32(xb)
    d = gu.desc_for(x.shape, (64, 3, 7, 7), 2, 3, NHWC, lc.LC_BF16)
    p, q = lc.conv2d_out_shape(d)
    dyb = synth.to_bf16_bits(synth.normal((n, 64, p, q), seed + 2))
    dy = synth.bf16_bits_to_f32(dyb)
    put = lambda bits: torch.from_numpy(np.ascontiguousarray(gu.to_layout(bits, NHWC)).view(np.int16)).to(gu.DEV)   # noqa: E731
    xd, dyd = put(xb), put(dyb)

    def run(sq=False):
        dw = torch.full((64, 7, 7, 3), float("nan"), dtype=torch.float32, device=gu.DEV)
        ws = gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT))
        pieces = None
        if sq:
            pieces = torch.full((lc.conv2d_bwd_weight_sq_count(d),), float("nan"), dtype=torch.float64, device=gu.DEV)
            lc.conv2d_bwd_weight_sq(d, xd, dyd, dw, pieces, ws)
        else:
            lc.conv2d_bwd_weight(d, xd, dyd, dw, ws)
        torch.cuda.synchronize()
        return gu.from_layout(dw.cpu().numpy(), NHWC), pieces

    dw, _ = run()
    ref = oracle.conv2d_bwd_weight(x, dy, (7, 7), 2, 3)
    assert np.all(np.isfinite(dw))
    assert gu.scaled_err(dw, ref) <= TOL
    np.testing.assert_array_equal(dw, run()[0])
    dw2, pieces = run(sq=True)
    np.testing.assert_array_equal(dw2, dw)
    want = float(np.sum(dw.astype(np.float64) ** 2))
    assert abs(float(pieces.sum().item()) - want) <= 1e-6 * want
    os.environ["LARSCONV_NO_STEM_DIRECT"] = "1"
    other, _ = run()
    assert gu.scaled_err(other, ref) <= TOL
    assert gu.scaled_err(dw, other) <= 2e-5


def test_other_first_layers_keep_the_general_kernel(restore_env):
    """Shapes next to the one the kernel takes: an output that is not a multiple of 16, another filter count, stride or
    padding, NCHW.  All must still be right (the general kernel runs them)."""
    cases = [((2, 3, 40, 40), (64, 3, 7, 7), 2, 3, NHWC), ((2, 3, 32, 32), (32, 3, 7, 7), 2, 3, NHWC),
             ((2, 3, 35, 35), (64, 3, 7, 7), 1, 3, NHWC), ((2, 3, 34, 34), (64, 3, 7, 7), 2, 2, NHWC),
             ((2, 3, 32, 32), (64, 3, 7, 7), 2, 3, lc.LC_NCHW)]
    for i, (xs, ws, stride, pad, layout) in enumerate(cases):
        x = synth.normal(xs, 5400 + i)
        wt = synth.normal(ws, 5450 + i, std=0.1)
        d = gu.desc_for(xs, ws, stride, pad, layout)
        y = gu.from_layout(gu.gpu_fwd(d, gu.to_layout(x, layout), gu.to_layout(wt, layout)), layout)
        assert gu.scaled_err(y, oracle.conv2d_fwd(x, wt, stride, pad)) <= TOL
        p, q = lc.conv2d_out_shape(d)
        dy = synth.normal((xs[0], ws[0], p, q), 5480 + i)
        dw = gu.from_layout(gu.gpu_bwd_weight(d, gu.to_layout(x, layout), gu.to_layout(dy, layout)), layout)
        assert gu.scaled_err(dw, oracle.conv2d_bwd_weight(x, dy, (7, 7), stride, pad)) <= TOL
