"""GPU parity of the bf16 backward-weight kernel that stages a 3x3 stride-1 pad-1 layer's activations once for all nine taps
(a ring of padded-image positions in LDS; channel and filter counts multiples of 64).  The library sends a layer there only
when its images are at least 24 pixels wide; these tests lower that threshold (LARSCONV_WGRAD_SLAB_MIN_W, read whenever a
call is planned) so that shapes the oracle finishes in seconds reach the kernel: several images per split and several
splits per image, images narrower and wider than the 32 positions of a step, the widest image the kernel takes (a longer
ring), rectangular images, one-row images, more than one tile of filters and of channels, and a single split (the kernel
writes dw itself).  Every result is also compared with the gathering kernel's
(LARSCONV_NO_WGRAD_SLAB): both add exact products of bf16 values in fp32, in a different order.
Tolerance as for every bf16 filter gradient: 1e-4 tensor-scaled against the float64 oracle on the same bf16 operands."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL_DW = 1e-4
NHWC = lc.LC_NHWC

SHAPES = {
    # n, c, h, w, k
    "two_images_14x14": (2, 64, 14, 14, 64),
    "narrow_6x6_many_images": (37, 64, 6, 6, 64),
    "rect_9x11_two_filter_tiles": (5, 64, 9, 11, 128),
    "rect_12x7_two_channel_tiles": (3, 128, 12, 7, 64),
    "one_image_28x28": (1, 64, 28, 28, 64),
    "wide_rows_56x56": (2, 64, 56, 56, 64),
    "widest_image_8x93": (2, 64, 8, 93, 64),
    "four_tiles_7x7": (6, 128, 7, 7, 128),
    "one_row_images_1x40": (9, 64, 1, 40, 64),
    "single_split_writes_dw": (1, 64, 6, 6, 64),
}


@pytest.fixture
def slab_for_small_shapes():
    saved = {k: os.environ.get(k) for k in ("LARSCONV_WGRAD_SLAB_MIN_W", "LARSCONV_NO_WGRAD_SLAB")}
    os.environ["LARSCONV_WGRAD_SLAB_MIN_W"] = "6"
    os.environ.pop("LARSCONV_NO_WGRAD_SLAB", None)
    yield
    for k, v in saved.items():
        if v is None:
            os.environ.pop(k, None)
        else:
            os.environ[k] = v


def _dev(bits_nchw):
    return torch.from_numpy(np.ascontiguousarray(gu.to_layout(bits_nchw, NHWC)).view(np.int16)).to(gu.DEV)


def _run(d, xd, dyd, k, c, sq=False):
    dw = torch.full((k, 3, 3, c), float("nan"), dtype=torch.float32, device=gu.DEV)
    ws = gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT))      # planned under the current environment
    pieces = None
    if sq:
        pieces = torch.full((lc.conv2d_bwd_weight_sq_count(d),), float("nan"), dtype=torch.float64, device=gu.DEV)
        lc.conv2d_bwd_weight_sq(d, xd, dyd, dw, pieces, ws)
    else:
        lc.conv2d_bwd_weight(d, xd, dyd, dw, ws)
    torch.cuda.synchronize()
    return gu.from_layout(dw.cpu().numpy(), NHWC), (pieces.cpu().numpy() if sq else None)


@pytest.mark.parametrize("name", list(SHAPES))
def test_wgrad_slab_matches_oracle_and_gathering_kernel(name, slab_for_small_shapes):
    n, c, h, w, k = SHAPES[name]
    seed = 6700 + 10 * list(SHAPES).index(name)
    xb = synth.to_bf16_bits(synth.normal((n, c, h, w), seed))
    dyb = synth.to_bf16_bits(synth.normal((n, k, h, w), seed + 2))
    x, dy = synth.bf16_bits_to_f32(xb), synth.bf16_bits_to_f32(dyb)
    d = gu.desc_for(x.shape, (k, c, 3, 3), 1, 1, NHWC, lc.LC_BF16)
    print(f"wgrad slab case {name} desc {d}", flush=True)
    xd, dyd = _dev(xb), _dev(dyb)
    dw, _ = _run(d, xd, dyd, k, c)
    ref = oracle.conv2d_bwd_weight(x, dy, (3, 3), 1, 1)
    assert np.all(np.isfinite(dw))
    assert gu.scaled_err(dw, ref) <= TOL_DW
    again, _ = _run(d, xd, dyd, k, c)
    np.testing.assert_array_equal(dw, again)                     # fixed order of the splits: reruns are bit-identical
    os.environ["LARSCONV_NO_WGRAD_SLAB"] = "1"
    other, _ = _run(d, xd, dyd, k, c)
    assert gu.scaled_err(other, ref) <= TOL_DW
    assert gu.scaled_err(dw, other) <= 1e-5                      # same products, fp32 sums in another order


def test_wgrad_slab_squared_norm_pieces(slab_for_small_shapes):
    """conv2d_bwd_weight_sq on a layer the kernel takes: the pieces of the squared norm come out of the split reduction
    behind it and add up to the squared norm of the dw it wrote."""
    n, c, h, w, k = 4, 64, 14, 14, 128
    xb = synth.to_bf16_bits(synth.normal((n, c, h, w), 6900))
    dyb = synth.to_bf16_bits(synth.normal((n, k, h, w), 6901))
    d = gu.desc_for((n, c, h, w), (k, c, 3, 3), 1, 1, NHWC, lc.LC_BF16)
    dw, pieces = _run(d, _dev(xb), _dev(dyb), k, c, sq=True)
    want = float(np.sum(dw.astype(np.float64) ** 2))
    assert abs(float(pieces.sum()) - want) <= 1e-6 * want
    plain, _ = _run(d, _dev(xb), _dev(dyb), k, c)
    np.testing.assert_array_equal(dw, plain)


def test_wgrad_slab_full_size_sampled():
    """res2a_3x3 of the bf16 workload at its full size (512 x 56 x 56 x 64 -> 64): the launch configuration bench.py times,
    without the threshold override.  Sampled filter-gradient elements (sums over 1.6 million pixels), all nine taps of the
    first and the last (filter, channel) pair among them."""
    n, c, hw, k = 512, 64, 56, 64
    seed = 6950
    xb = synth.to_bf16_bits(synth.normal((n, hw, hw, c), seed))
    dyb = synth.to_bf16_bits(synth.normal((n, hw, hw, k), seed + 2))
    x, dy = synth.bf16_bits_to_f32(xb), synth.bf16_bits_to_f32(dyb)
    d = lc.ConvDesc(n, c, hw, hw, k, 3, 3, 1, 1, 1, 1, lc.LC_BF16, NHWC)
    dv = lambda bits: torch.from_numpy(bits.view(np.int16)).to(gu.DEV)       # noqa: E731
    dw = torch.full((k, 3, 3, c), float("nan"), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_bwd_weight(d, dv(xb), dv(dyb), dw, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT)))
    torch.cuda.synchronize()
    dw = dw.cpu().numpy()
    assert np.all(np.isfinite(dw))
    corners = np.array([[k_, c_, r_, s_] for (k_, c_) in ((0, 0), (k - 1, c - 1)) for r_ in range(3) for s_ in range(3)], dtype=np.int32)
    cw = np.concatenate([synth.sample_coords(96, (k, c, 3, 3), seed + 5), corners])
    ref, _ = oracle.conv2d_bwd_weight_at(x, dy, (3, 3), cw, 1, 1, oracle.NHWC)
    assert np.max(np.abs(dw[cw[:, 0], cw[:, 2], cw[:, 3], cw[:, 1]] - ref)) <= TOL_DW * np.max(np.abs(ref))
