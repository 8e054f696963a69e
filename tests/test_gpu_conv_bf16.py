"""GPU parity for bf16 operands (fp32 accumulation): inputs are drawn in fp32, rounded once to bf16 on the
host, and those exact values feed both sides.  The oracle sums in double; its result is rounded to bf16 for
the comparison with y / dx (bf16 outputs) and left unrounded for dw (fp32 output).
Tolerances: y, dx  max |gpu - oracle| / max |oracle| <= 2e-2 (one bf16 ulp is 2^-8 = 3.9e-3 relative);
dw <= 1e-4 as for fp32 operands (the products of bf16 values are exact in fp32, only the sums round)."""
import numpy as np
import pytest
import torch

import oracle
from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL_BF16, TOL_DW = 2e-2, 1e-4

SHAPES = {
    "3x3_multi_tile": (2, 64, 14, 14, 96, 3, 3, 1, 1),
    "3x3_wide": (3, 32, 10, 12, 160, 3, 3, 1, 1),
    "1x1_plain": (3, 256, 7, 7, 512, 1, 1, 1, 0),
    "1x1_stride2_odd": (2, 64, 15, 15, 128, 1, 1, 2, 0),
    "stem_7x7_s2": (2, 3, 30, 30, 64, 7, 7, 2, 3),            # NHWC: 2x2 pixel blocks; NCHW: c padded to 8; backward-data through fp32
    "5x5_p2": (2, 16, 13, 13, 32, 5, 5, 1, 2),
    "3x3_stride2": (2, 32, 17, 17, 48, 3, 3, 2, 1),           # strided window: backward-data phase by phase
    "3x3_stride2_k24": (2, 32, 17, 17, 24, 3, 3, 2, 1),       # fewer filters than a k-step: backward-data through fp32
    "phases_3x3_s2_p1_v15": (2, 128, 14, 14, 128, 3, 3, 2, 1),
    "phases_3x3_s2_odd_channels_out": (3, 33, 15, 13, 64, 3, 3, 2, 1),     # dx rows of 33 channels: 2-byte stores
    "phases_5x5_s2_p2": (2, 16, 13, 12, 32, 5, 5, 2, 2),
    "phases_some_rows_without_taps": (2, 16, 9, 9, 32, 1, 3, 2, (0, 1)),
    "odd_channels": (2, 6, 9, 9, 10, 3, 3, 1, 1),             # k = 10: backward-data through fp32, scalar filter gradient
    "k8_c24": (2, 24, 9, 9, 8, 3, 3, 1, 1),
    "full_window_fc": (4, 16, 6, 6, 40, 6, 6, 1, 0),
    "single_everything": (1, 1, 5, 5, 1, 1, 1, 1, 0),
    "fc_1x1_on_1x1": (16, 512, 1, 1, 104, 1, 1, 1, 0),
    "resnet_28_stage": (8, 128, 28, 28, 128, 3, 3, 1, 1),
    # few channels, stride 2: NHWC runs them over 2x2 pixel blocks where that saves multiplications
    "blocks_5x5_s2_p2_c3_ragged": (2, 3, 18, 15, 24, 5, 5, 2, 2),
    "blocks_3x3_s2_p1_c4": (3, 4, 13, 16, 40, 3, 3, 2, 1),
    "blocks_7x7_s2_p0_c1": (2, 1, 21, 20, 16, 7, 7, 2, 0),
    "blocks_rect_7x3_s2_c2": (2, 2, 17, 14, 12, 7, 3, 2, (3, 1)),
    "blocks_7x7_s2_p3_odd_image": (1, 3, 29, 31, 72, 7, 7, 2, 3),
}


def _bf16_inputs(shape, seed):
    n, c, h, w, k, r, s, stride, pad = shape
    p, q = oracle.out_shape(h, w, r, s, stride, pad)
    raw = (synth.normal((n, c, h, w), seed), synth.normal((k, c, r, s), seed + 1, std=float(np.sqrt(2.0 / (c * r * s)))),
           synth.normal((n, k, p, q), seed + 2))
    bits = [synth.to_bf16_bits(a) for a in raw]
    vals = [synth.bf16_bits_to_f32(b) for b in bits]         # what both sides compute with
    return bits, vals


def _dev_bf16(bits_l):
    return torch.from_numpy(np.ascontiguousarray(bits_l).view(np.int16)).to(gu.DEV)


def _back(t):
    return synth.bf16_bits_to_f32(t.cpu().numpy().view(np.uint16))


@pytest.mark.parametrize("layout", [lc.LC_NHWC, lc.LC_NCHW], ids=["nhwc", "nchw"])
@pytest.mark.parametrize("name", list(SHAPES))
def test_three_passes_match_oracle_bf16(name, layout):
    shape = SHAPES[name]
    n, c, h, w, k, r, s, stride, pad = shape
    (xb, wb, dyb), (x, wt, dy) = _bf16_inputs(shape, 5000 + 10 * list(SHAPES).index(name))
    d = gu.desc_for(x.shape, wt.shape, stride, pad, layout, lc.LC_BF16)
    print(f"bf16 case {name} layout {layout} desc {d}", flush=True)
    p, q = lc.conv2d_out_shape(d)
    xd, wd, dyd = (_dev_bf16(gu.to_layout(a, layout)) for a in (xb, wb, dyb))

    yshape = (n, k, p, q) if layout == lc.LC_NCHW else (n, p, q, k)
    y = torch.full(yshape, -1, dtype=torch.int16, device=gu.DEV)
    lc.conv2d_fwd(d, xd, wd, y, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)))
    xshape = (n, c, h, w) if layout == lc.LC_NCHW else (n, h, w, c)
    dx = torch.full(xshape, -1, dtype=torch.int16, device=gu.DEV)
    lc.conv2d_bwd_data(d, dyd, wd, dx, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_DATA)))
    wshape = (k, c, r, s) if layout == lc.LC_NCHW else (k, r, s, c)
    dw = torch.full(wshape, float("nan"), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_bwd_weight(d, xd, dyd, dw, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT)))
    torch.cuda.synchronize()

    ref_y = oracle.conv2d_fwd(x, wt, stride, pad)
    ref_dx = oracle.conv2d_bwd_data(dy, wt, (h, w), stride, pad)
    ref_dw = oracle.conv2d_bwd_weight(x, dy, (r, s), stride, pad)
    got_y = gu.from_layout(_back(y), layout)
    got_dx = gu.from_layout(_back(dx), layout)
    assert gu.scaled_err(got_y, oracle.round_to_bf16(ref_y)) <= TOL_BF16
    assert gu.scaled_err(got_dx, oracle.round_to_bf16(ref_dx)) <= TOL_BF16
    # tighter: at most one bf16 step away from the exact result, element by element
    assert np.all(np.abs(got_y - ref_y) <= np.abs(ref_y) * 2.0 ** -7 + 1e-6 * np.max(np.abs(ref_y)))
    assert np.all(np.abs(got_dx - ref_dx) <= np.abs(ref_dx) * 2.0 ** -7 + 1e-6 * max(np.max(np.abs(ref_dx)), 1e-30))
    assert gu.scaled_err(gu.from_layout(dw.cpu().numpy(), layout), ref_dw) <= TOL_DW


def test_bf16_tensors_need_16_byte_alignment():
    d = lc.ConvDesc(2, 16, 9, 9, 24, 3, 3, 1, 1, 1, 1, lc.LC_BF16, lc.LC_NHWC)
    buf = torch.zeros(1 << 16, dtype=torch.int16, device=gu.DEV)
    y = torch.zeros(2 * 9 * 9 * 24, dtype=torch.int16, device=gu.DEV)
    ws = gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD))
    with pytest.raises(lc.LarsConvError) as e:
        lc.conv2d_fwd(d, buf[1:], buf[8192:], y, ws)
    assert e.value.status == lc.LC_ERR_ALIGN


@pytest.mark.parametrize("name", ["res2a_3x3", "res3a_1x1a", "res4b_1x1a", "res5b_3x3"])
def test_bf16_full_size_batch512_sampled(name):
    """bf16 workload at its full size (batch 512, one worker's share of a 32K batch): sampled outputs."""
    cs = {c.name: c for c in synth.resnet50_convs(512)}[name]
    seed = 7000 + len(name)
    print(f"bf16 full-size {name}: {cs}", flush=True)
    xb = synth.to_bf16_bits(synth.normal((cs.n, cs.h, cs.w, cs.c), seed))
    wb = synth.to_bf16_bits(synth.normal((cs.k, cs.r, cs.s, cs.c), seed + 1, std=synth.he_std(cs)))
    dyb = synth.to_bf16_bits(synth.normal((cs.n, cs.p, cs.q, cs.k), seed + 2))
    x, wt, dy = (synth.bf16_bits_to_f32(b) for b in (xb, wb, dyb))
    d = lc.ConvDesc(cs.n, cs.c, cs.h, cs.w, cs.k, cs.r, cs.s, cs.stride, cs.stride, cs.pad, cs.pad, lc.LC_BF16, lc.LC_NHWC)
    xd, wd, dyd = _dev_bf16(xb), _dev_bf16(wb), _dev_bf16(dyb)
    y = torch.empty((cs.n, cs.p, cs.q, cs.k), dtype=torch.int16, device=gu.DEV)
    dx = torch.empty((cs.n, cs.h, cs.w, cs.c), dtype=torch.int16, device=gu.DEV)
    dw = torch.empty((cs.k, cs.r, cs.s, cs.c), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_fwd(d, xd, wd, y, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)))
    lc.conv2d_bwd_data(d, dyd, wd, dx, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_DATA)))
    lc.conv2d_bwd_weight(d, xd, dyd, dw, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT)))
    torch.cuda.synchronize()
    y, dx, dw = _back(y), _back(dx), dw.cpu().numpy()
    cy = synth.sample_coords(1024, (cs.n, cs.k, cs.p, cs.q), seed + 3)
    ref, _ = oracle.conv2d_fwd_at(x, wt, cy, cs.stride, cs.pad, oracle.NHWC)
    assert np.max(np.abs(y[cy[:, 0], cy[:, 2], cy[:, 3], cy[:, 1]] - oracle.round_to_bf16(ref))) <= TOL_BF16 * np.max(np.abs(ref))
    cx = synth.sample_coords(1024, (cs.n, cs.c, cs.h, cs.w), seed + 4)
    ref, _ = oracle.conv2d_bwd_data_at(dy, wt, (cs.h, cs.w), cx, cs.stride, cs.pad, oracle.NHWC)
    assert np.max(np.abs(dx[cx[:, 0], cx[:, 2], cx[:, 3], cx[:, 1]] - oracle.round_to_bf16(ref))) <= TOL_BF16 * max(np.max(np.abs(ref)), 1e-30)
    cw = synth.sample_coords(128, (cs.k, cs.c, cs.r, cs.s), seed + 5)
    ref, _ = oracle.conv2d_bwd_weight_at(x, dy, (cs.r, cs.s), cw, cs.stride, cs.pad, oracle.NHWC)
    assert np.max(np.abs(dw[cw[:, 0], cw[:, 2], cw[:, 3], cw[:, 1]] - ref)) <= TOL_DW * np.max(np.abs(ref))


def test_bf16_first_layer_full_size_batch512_sampled():
    """The 7x7 stride-2 first layer at the bf16 workload's full size (512 x 224 x 224 x 3): forward and backward-weight run
    in the kernels that keep a tile's input slab in LDS (no workspace for the forward pass, one partial filter gradient
    per resident block for backward-weight).  Sampled outputs; backward-data is not part of a training step for a first
    layer."""
    cs = synth.resnet50_convs(512)[0]
    seed = 7800
    print(f"bf16 full-size first layer: {cs}", flush=True)
    xb = synth.to_bf16_bits(synth.normal((cs.n, cs.h, cs.w, cs.c), seed))
    wb = synth.to_bf16_bits(synth.normal((cs.k, cs.r, cs.s, cs.c), seed + 1, std=synth.he_std(cs)))
    dyb = synth.to_bf16_bits(synth.normal((cs.n, cs.p, cs.q, cs.k), seed + 2))
    x, wt, dy = (synth.bf16_bits_to_f32(b) for b in (xb, wb, dyb))
    d = lc.ConvDesc(cs.n, cs.c, cs.h, cs.w, cs.k, cs.r, cs.s, cs.stride, cs.stride, cs.pad, cs.pad, lc.LC_BF16, lc.LC_NHWC)
    assert lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD) == 0
    assert 0 < lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT) < 100_000_000   # the blocks' partials, no unfolded input
    xd, wd, dyd = _dev_bf16(xb), _dev_bf16(wb), _dev_bf16(dyb)
    y = torch.empty((cs.n, cs.p, cs.q, cs.k), dtype=torch.int16, device=gu.DEV)
    dw = torch.empty((cs.k, cs.r, cs.s, cs.c), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_fwd(d, xd, wd, y, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)))
    lc.conv2d_bwd_weight(d, xd, dyd, dw, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT)))
    torch.cuda.synchronize()
    y, dw = _back(y), dw.cpu().numpy()
    # samples spread over the image, plus the four corners of the first and the last image (padding on two sides each)
    cy = synth.sample_coords(1024, (cs.n, cs.k, cs.p, cs.q), seed + 3)
    corners = np.array([[n_, k_, p_, q_] for n_ in (0, cs.n - 1) for k_ in (0, cs.k - 1) for p_ in (0, cs.p - 1) for q_ in (0, cs.q - 1)],
                       dtype=np.int32)
    cy = np.concatenate([cy, corners])
    ref, _ = oracle.conv2d_fwd_at(x, wt, cy, cs.stride, cs.pad, oracle.NHWC)
    got = y[cy[:, 0], cy[:, 2], cy[:, 3], cy[:, 1]]
    assert np.max(np.abs(got - oracle.round_to_bf16(ref))) <= TOL_BF16 * np.max(np.abs(ref))
    assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -7 + 1e-6 * np.max(np.abs(ref)))
    cw = synth.sample_coords(96, (cs.k, cs.c, cs.r, cs.s), seed + 5)
    ref, _ = oracle.conv2d_bwd_weight_at(x, dy, (cs.r, cs.s), cw, cs.stride, cs.pad, oracle.NHWC)
    assert np.max(np.abs(dw[cw[:, 0], cw[:, 2], cw[:, 3], cw[:, 1]] - ref)) <= TOL_DW * np.max(np.abs(ref))


def test_bf16_wide_tile_ragged_edges_sampled():
    """A result wide and tall enough for the 128x256 tile of the main kernel (at least three rounds of tiles), with a
    ragged last tile in both directions: 103,488 rows (808.5 tiles), 300 columns (256 + 44).  Sampled outputs plus the
    last rows and columns; forward and backward-data (whose result is 320 wide: 256 + 64)."""
    n, c, hw, k = 33, 320, 56, 300
    seed = 7900
    xb = synth.to_bf16_bits(synth.normal((n, hw, hw, c), seed))
    wb = synth.to_bf16_bits(synth.normal((k, 1, 1, c), seed + 1, std=(2.0 / c) ** 0.5))
    dyb = synth.to_bf16_bits(synth.normal((n, hw, hw, k), seed + 2))
    x, wt, dy = (synth.bf16_bits_to_f32(b) for b in (xb, wb, dyb))
    d = lc.ConvDesc(n, c, hw, hw, k, 1, 1, 1, 1, 0, 0, lc.LC_BF16, lc.LC_NHWC)
    xd, wd, dyd = _dev_bf16(xb), _dev_bf16(wb), _dev_bf16(dyb)
    y = torch.empty((n, hw, hw, k), dtype=torch.int16, device=gu.DEV)
    dx = torch.empty((n, hw, hw, c), dtype=torch.int16, device=gu.DEV)
    lc.conv2d_fwd(d, xd, wd, y, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)))
    lc.conv2d_bwd_data(d, dyd, wd, dx, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_DATA)))
    torch.cuda.synchronize()
    y, dx = _back(y), _back(dx)
    assert np.all(np.isfinite(y)) and np.all(np.isfinite(dx))

    def coords(channels, sd):
        rnd = synth.sample_coords(768, (n, channels, hw, hw), sd)
        edge = np.array([[n - 1, ch, hw - 1, q] for ch in (0, 255, 256, channels - 1) for q in (0, hw - 2, hw - 1)] +
                        [[0, ch, 0, 0] for ch in (0, 127, 128, 255, 256, channels - 1)], dtype=rnd.dtype)
        return np.concatenate([rnd, edge])
    cy = coords(k, seed + 3)
    ref, _ = oracle.conv2d_fwd_at(x, wt, cy, 1, 0, oracle.NHWC)
    assert np.max(np.abs(y[cy[:, 0], cy[:, 2], cy[:, 3], cy[:, 1]] - oracle.round_to_bf16(ref))) <= TOL_BF16 * np.max(np.abs(ref))
    cx = coords(c, seed + 4)
    ref, _ = oracle.conv2d_bwd_data_at(dy, wt, (hw, hw), cx, 1, 0, oracle.NHWC)
    assert np.max(np.abs(dx[cx[:, 0], cx[:, 2], cx[:, 3], cx[:, 1]] - oracle.round_to_bf16(ref))) <= TOL_BF16 * np.max(np.abs(ref))
