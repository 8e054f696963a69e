"""GPU parity of the bf16 kernel that stages a tile's activation slab once for all nine taps of a 3x3 stride-1 pad-1
window (forward, and backward-data, which is the same convolution of dy with the re-ordered filter).  The library sends a
layer there only when its tiles fill the chip; these tests lower that threshold (LARSCONV_SLAB_MIN_TILES, read on every
call) so that small shapes the oracle finishes in seconds reach the kernel: several images per tile (the empty virtual row
between images), images narrower than a tile and wider than one, ragged last tiles in both directions, odd filter counts
(single 2-byte stores instead of column pairs), 2x2 images, and the widest slab the kernel takes.  Every result is also
compared bit for bit with the main kernel's (threshold back up): both add the same products in a different order, so they
agree to fp32 rounding and after the bf16 rounding differ in a few elements by one step at most.
Tolerances as for every bf16 convolution: 2e-2 tensor-scaled against the rounded oracle value."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL_BF16 = 2e-2
NHWC = lc.LC_NHWC

SHAPES = {
    # n, c, h, w, k
    "two_images_14x14": (2, 64, 14, 14, 128),
    "three_images_7x7_ragged_columns": (3, 32, 7, 7, 96),
    "rect_9x11_k40": (5, 64, 9, 11, 40),
    "one_image_28x28_c96": (1, 96, 28, 28, 64),
    "wide_rows_56x56": (2, 32, 56, 56, 64),
    "many_tiny_images_3x5_k160": (40, 32, 3, 5, 160),
    "images_2x2": (64, 32, 2, 2, 64),
    "odd_filter_count": (2, 32, 8, 8, 33),
    "resnet_14_stage_256": (4, 256, 14, 14, 256),
}


@pytest.fixture
def slab_for_small_shapes():
    old = os.environ.get("LARSCONV_SLAB_MIN_TILES")
    os.environ["LARSCONV_SLAB_MIN_TILES"] = "1"
    yield
    if old is None:
        del os.environ["LARSCONV_SLAB_MIN_TILES"]
    else:
        os.environ["LARSCONV_SLAB_MIN_TILES"] = old


def _dev(bits_nchw):
    return torch.from_numpy(np.ascontiguousarray(gu.to_layout(bits_nchw, NHWC)).view(np.int16)).to(gu.DEV)


def _back(t):
    return gu.from_layout(synth.bf16_bits_to_f32(t.cpu().numpy().view(np.uint16)), NHWC)


def _run(d, xd, wd, dyd, n, c, h, w, k):
    y = torch.full((n, h, w, k), -1, dtype=torch.int16, device=gu.DEV)
    dx = torch.full((n, h, w, c), -1, dtype=torch.int16, device=gu.DEV)
    lc.conv2d_fwd(d, xd, wd, y, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)))
    lc.conv2d_bwd_data(d, dyd, wd, dx, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_DATA)))
    torch.cuda.synchronize()
    return _back(y), _back(dx)


@pytest.mark.parametrize("name", list(SHAPES))
def test_slab_kernel_matches_oracle_and_main_kernel(name, slab_for_small_shapes):
    n, c, h, w, k = SHAPES[name]
    seed = 6100 + 10 * list(SHAPES).index(name)
    xb = synth.to_bf16_bits(synth.normal((n, c, h, w), seed))
    wb = synth.to_bf16_bits(synth.normal((k, c, 3, 3), seed + 1, std=float(np.sqrt(2.0 / (9 * c)))))
    dyb = synth.to_bf16_bits(synth.normal((n, k, h, w), seed + 2))
    x, wt, dy = (synth.bf16_bits_to_f32(b) for b in (xb, wb, dyb))
    d = gu.desc_for(x.shape, wt.shape, 1, 1, NHWC, lc.LC_BF16)
    print(f"slab case {name} desc {d}", flush=True)
    xd, wd, dyd = _dev(xb), _dev(wb), _dev(dyb)
    y, dx = _run(d, xd, wd, dyd, n, c, h, w, k)
    ref_y = oracle.conv2d_fwd(x, wt, 1, 1)
    ref_dx = oracle.conv2d_bwd_data(dy, wt, (h, w), 1, 1)
    assert gu.scaled_err(y, oracle.round_to_bf16(ref_y)) <= TOL_BF16
    assert gu.scaled_err(dx, oracle.round_to_bf16(ref_dx)) <= TOL_BF16
    for got, ref in ((y, ref_y), (dx, ref_dx)):            # element by element: within one bf16 step of the float64 value
        assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -7 + 1e-5 * float(np.max(np.abs(ref))))
    # the main kernel on the same operands
    os.environ["LARSCONV_SLAB_MIN_TILES"] = "1000000000"
    y2, dx2 = _run(d, xd, wd, dyd, n, c, h, w, k)
    for a, b in ((y, y2), (dx, dx2)):
        assert np.mean(a == b) >= 0.99
        assert np.all(np.abs(a - b) <= np.abs(b) * 2.0 ** -7 + 1e-6 * float(np.max(np.abs(b))))


def test_slab_kernel_full_size_sampled():
    """res3a_3x3 of the bf16 workload at its full size (512 x 28 x 28 x 128 -> 128, 3136 tiles): the launch configuration
    bench.py times, without the threshold override.  Sampled outputs of forward and backward-data, corners included."""
    n, c, hw, k = 512, 128, 28, 128
    seed = 6500
    xb = synth.to_bf16_bits(synth.normal((n, hw, hw, c), seed))
    wb = synth.to_bf16_bits(synth.normal((k, 3, 3, c), seed + 1, std=float(np.sqrt(2.0 / (9 * c)))))
    dyb = synth.to_bf16_bits(synth.normal((n, hw, hw, k), seed + 2))
    x, wt, dy = (synth.bf16_bits_to_f32(b) for b in (xb, wb, dyb))
    d = lc.ConvDesc(n, c, hw, hw, k, 3, 3, 1, 1, 1, 1, lc.LC_BF16, NHWC)
    dv = lambda bits: torch.from_numpy(bits.view(np.int16)).to(gu.DEV)       # noqa: E731
    xd, wd, dyd = dv(xb), dv(wb), dv(dyb)
    y = torch.full((n, hw, hw, k), -1, dtype=torch.int16, device=gu.DEV)
    dx = torch.full((n, hw, hw, c), -1, dtype=torch.int16, device=gu.DEV)
    lc.conv2d_fwd(d, xd, wd, y, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)))
    lc.conv2d_bwd_data(d, dyd, wd, dx, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_DATA)))
    torch.cuda.synchronize()
    y = synth.bf16_bits_to_f32(y.cpu().numpy().view(np.uint16))
    dx = synth.bf16_bits_to_f32(dx.cpu().numpy().view(np.uint16))
    corners = np.array([[n_, k_, p_, q_] for n_ in (0, n - 1) for k_ in (0, k - 1) for p_ in (0, hw - 1) for q_ in (0, hw - 1)], dtype=np.int32)
    cy = np.concatenate([synth.sample_coords(2048, (n, k, hw, hw), seed + 3), corners])
    ref, _ = oracle.conv2d_fwd_at(x, wt, cy, 1, 1, oracle.NHWC)
    got = y[cy[:, 0], cy[:, 2], cy[:, 3], cy[:, 1]]
    assert np.max(np.abs(got - oracle.round_to_bf16(ref))) <= TOL_BF16 * np.max(np.abs(ref))
    assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -7 + 1e-5 * np.max(np.abs(ref)))
    cx = np.concatenate([synth.sample_coords(2048, (n, c, hw, hw), seed + 4), corners])
    ref, _ = oracle.conv2d_bwd_data_at(dy, wt, (hw, hw), cx, 1, 1, oracle.NHWC)
    got = dx[cx[:, 0], cx[:, 2], cx[:, 3], cx[:, 1]]
    assert np.max(np.abs(got - oracle.round_to_bf16(ref))) <= TOL_BF16 * np.max(np.abs(ref))
    assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -7 + 1e-5 * np.max(np.abs(ref)))
    assert np.all(np.isfinite(y)) and np.all(np.isfinite(dx))            # every element was written (the fill pattern is a NaN)
