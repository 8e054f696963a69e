"""GPU parity: conv2d_fwd / conv2d_bwd_data / conv2d_bwd_weight through the C ABI against the CPU
oracle on the same seeded inputs.  Tolerance: max |gpu - oracle| / max |oracle| <= 1e-4 per tensor
(fp32 operands, fp32 MFMA accumulation against the oracle's double sums)."""
import numpy as np
import pytest
import torch

import oracle
from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 1e-4

# n, c, h, w, k, r, s, stride, pad   -- small enough for the full-tensor oracle, large enough to span
# several 128-row tiles with ragged tails in every GEMM dimension
SHAPES = {
    "3x3_multi_tile": (2, 64, 14, 14, 96, 3, 3, 1, 1),
    "3x3_wide": (3, 32, 10, 12, 160, 3, 3, 1, 1),
    "1x1_plain": (3, 256, 7, 7, 512, 1, 1, 1, 0),
    "1x1_stride2_odd": (2, 64, 15, 15, 128, 1, 1, 2, 0),
    "1x1_stride2_even_k64": (2, 128, 16, 16, 64, 1, 1, 2, 0),
    "1x1_stride2_few_filters": (2, 32, 9, 9, 8, 1, 1, 2, 0),
    "stem_7x7_s2": (2, 3, 30, 30, 64, 7, 7, 2, 3),
    "alexnet_11x11_s4": (1, 3, 35, 35, 32, 11, 11, 4, 0),
    "5x5_p2": (2, 16, 13, 13, 32, 5, 5, 1, 2),
    "3x3_stride2": (2, 32, 17, 17, 48, 3, 3, 2, 1),
    "odd_channels": (2, 6, 9, 9, 10, 3, 3, 1, 1),
    "asymmetric": (2, 8, 11, 9, 12, 3, 2, (2, 1), (1, 0)),
    "full_window_fc": (4, 16, 6, 6, 40, 6, 6, 1, 0),
    "full_window_rect_stride3_odd": (3, 5, 3, 5, 7, 3, 5, 3, 0),
    "single_everything": (1, 1, 5, 5, 1, 1, 1, 1, 0),
    "fc_1x1_on_1x1": (16, 512, 1, 1, 100, 1, 1, 1, 0),
    "tiny_cnn_conv1": (16, 3, 32, 32, 16, 3, 3, 1, 1),
    "pad_wider_than_window": (1, 4, 5, 5, 4, 2, 2, 1, 2),
    # few channels, stride 2 (bf16 runs these over 2x2 pixel blocks; here they take the few-channels path)
    "blocks_5x5_s2_p2_c3_ragged": (2, 3, 18, 15, 24, 5, 5, 2, 2),
    "blocks_3x3_s2_p1_c4": (3, 4, 13, 16, 40, 3, 3, 2, 1),
    "blocks_7x7_s2_p0_c1": (2, 1, 21, 20, 16, 7, 7, 2, 0),
    "blocks_rect_7x3_s2_c2": (2, 2, 17, 14, 12, 7, 3, 2, (3, 1)),
    "blocks_7x7_s2_p3_odd_image": (1, 3, 29, 31, 72, 7, 7, 2, 3),
    # strided windows other than 1x1: backward-data runs one GEMM per stride phase (16 or more filters, a multiple of 4)
    "phases_3x3_s2_p1_v15": (2, 128, 14, 14, 128, 3, 3, 2, 1),
    "phases_3x3_s2_p1_odd_image": (3, 32, 15, 13, 64, 3, 3, 2, 1),
    "phases_5x5_s2_p2": (2, 16, 13, 12, 32, 5, 5, 2, 2),
    "phases_3x3_s3_p0": (2, 8, 14, 11, 16, 3, 3, 3, 0),
    "phases_2x2_s2_p0": (2, 24, 12, 10, 40, 2, 2, 2, 0),
    "phases_4x4_s2_p1": (2, 16, 12, 12, 32, 4, 4, 2, 1),
    "phases_stride_1x2": (2, 16, 9, 12, 32, 3, 3, (1, 2), (1, 1)),
    "phases_some_rows_without_taps": (2, 16, 9, 9, 32, 1, 3, 2, (0, 1)),      # window height 1 at stride 2: odd rows of dx stay zero
    "phases_pad_beyond_window": (2, 8, 7, 7, 16, 2, 2, 2, 2),
    "phases_4x4_s4_p0": (1, 8, 16, 16, 32, 4, 4, 4, 0),
    "phases_7x7_s2_many_channels": (2, 20, 19, 18, 24, 7, 7, 2, 3),
}


def _inputs(shape, seed):
    n, c, h, w, k, r, s, stride, pad = shape
    x = synth.normal((n, c, h, w), seed)
    wt = synth.normal((k, c, r, s), seed + 1, std=float(np.sqrt(2.0 / (c * r * s))))
    p, q = oracle.out_shape(h, w, r, s, stride, pad)
    dy = synth.normal((n, k, p, q), seed + 2)
    return x, wt, dy


@pytest.mark.parametrize("layout", [lc.LC_NHWC, lc.LC_NCHW], ids=["nhwc", "nchw"])
@pytest.mark.parametrize("name", list(SHAPES))
def test_three_passes_match_oracle(name, layout):
    shape = SHAPES[name]
    n, c, h, w, k, r, s, stride, pad = shape
    x, wt, dy = _inputs(shape, 1000 + 10 * list(SHAPES).index(name))
    d = gu.desc_for(x.shape, wt.shape, stride, pad, layout)
    xl, wl, dyl = gu.to_layout(x, layout), gu.to_layout(wt, layout), gu.to_layout(dy, layout)
    print(f"case {name} layout {layout} desc {d}", flush=True)

    y = gu.from_layout(gu.gpu_fwd(d, xl, wl), layout)
    assert gu.scaled_err(y, oracle.conv2d_fwd(x, wt, stride, pad)) <= TOL
    dx = gu.from_layout(gu.gpu_bwd_data(d, dyl, wl), layout)
    assert gu.scaled_err(dx, oracle.conv2d_bwd_data(dy, wt, (h, w), stride, pad)) <= TOL
    dw = gu.from_layout(gu.gpu_bwd_weight(d, xl, dyl), layout)
    assert gu.scaled_err(dw, oracle.conv2d_bwd_weight(x, dy, (r, s), stride, pad)) <= TOL


def test_larger_layer_full_tensor():
    # 28x28 stage of ResNet-50 at batch 8: 49 row tiles, reduction 1152, 6272 rows for the filter gradient
    shape = (8, 128, 28, 28, 128, 3, 3, 1, 1)
    x, wt, dy = _inputs(shape, 2000)
    d = gu.desc_for(x.shape, wt.shape, 1, 1, lc.LC_NHWC)
    xl, wl, dyl = (gu.to_layout(a, lc.LC_NHWC) for a in (x, wt, dy))
    assert gu.scaled_err(gu.from_layout(gu.gpu_fwd(d, xl, wl), lc.LC_NHWC), oracle.conv2d_fwd(x, wt, 1, 1)) <= TOL
    assert gu.scaled_err(gu.from_layout(gu.gpu_bwd_data(d, dyl, wl), lc.LC_NHWC),
                         oracle.conv2d_bwd_data(dy, wt, (28, 28), 1, 1)) <= TOL
    assert gu.scaled_err(gu.from_layout(gu.gpu_bwd_weight(d, xl, dyl), lc.LC_NHWC),
                         oracle.conv2d_bwd_weight(x, dy, (3, 3), 1, 1)) <= TOL


def test_misaligned_operands_take_the_scalar_path():
    shape = (2, 16, 9, 9, 24, 3, 3, 1, 1)
    n, c, h, w, k, r, s, stride, pad = shape
    x, wt, dy = _inputs(shape, 2100)
    d = gu.desc_for(x.shape, wt.shape, stride, pad, lc.LC_NHWC)
    xl, wl = gu.to_layout(x, lc.LC_NHWC), gu.to_layout(wt, lc.LC_NHWC)
    xb = torch.empty(xl.size + 1, dtype=torch.float32, device=gu.DEV)
    wb = torch.empty(wl.size + 1, dtype=torch.float32, device=gu.DEV)
    xb[1:].copy_(torch.from_numpy(xl.ravel()))
    wb[1:].copy_(torch.from_numpy(wl.ravel()))
    y = torch.full((n, h, w, k), float("nan"), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_fwd(d, xb[1:], wb[1:], y, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)))
    torch.cuda.synchronize()
    assert gu.scaled_err(gu.from_layout(y.cpu().numpy(), lc.LC_NHWC), oracle.conv2d_fwd(x, wt, stride, pad)) <= TOL


def test_filter_gradient_is_bit_reproducible():
    shape = (4, 64, 28, 28, 64, 3, 3, 1, 1)          # heavy split of the reduction
    x, wt, dy = _inputs(shape, 2200)
    d = gu.desc_for(x.shape, wt.shape, 1, 1, lc.LC_NHWC)
    xl, dyl = gu.to_layout(x, lc.LC_NHWC), gu.to_layout(dy, lc.LC_NHWC)
    a = gu.gpu_bwd_weight(d, xl, dyl)
    b = gu.gpu_bwd_weight(d, xl, dyl)
    assert np.array_equal(a, b)
    assert gu.scaled_err(gu.from_layout(a, lc.LC_NHWC), oracle.conv2d_bwd_weight(x, dy, (3, 3), 1, 1)) <= TOL


# ---- full benchmark sizes (batch 256, the launch configuration bench.py times): sampled outputs ----
FULL = {c.name: c for c in synth.resnet50_convs(256) + synth.resnet50_v15_extra_shapes(256)}
FULL_CASES = ["conv1", "res2a_3x3", "res3a_1x1a", "res4a_proj", "res5b_3x3", "res5c_1x1a", "v15_res3a_3x3s2", "v15_res5a_3x3s2"]


@pytest.mark.parametrize("name", FULL_CASES)
def test_full_size_sampled_outputs_and_adjoint(name):
    cs = FULL[name]
    seed = 3000 + 10 * FULL_CASES.index(name)
    print(f"full-size case {name}: {cs}", flush=True)
    x = synth.normal((cs.n, cs.h, cs.w, cs.c), seed)                       # NHWC directly
    wt = synth.normal((cs.k, cs.r, cs.s, cs.c), seed + 1, std=synth.he_std(cs))
    dy = synth.normal((cs.n, cs.p, cs.q, cs.k), seed + 2)
    d = lc.ConvDesc(cs.n, cs.c, cs.h, cs.w, cs.k, cs.r, cs.s, cs.stride, cs.stride, cs.pad, cs.pad, lc.LC_F32, lc.LC_NHWC)
    xd, wd, dyd = gu.dev(x), gu.dev(wt), gu.dev(dy)
    y = torch.empty((cs.n, cs.p, cs.q, cs.k), dtype=torch.float32, device=gu.DEV)
    dx = torch.empty((cs.n, cs.h, cs.w, cs.c), dtype=torch.float32, device=gu.DEV)
    dw = torch.empty((cs.k, cs.r, cs.s, cs.c), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_fwd(d, xd, wd, y, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)))
    lc.conv2d_bwd_data(d, dyd, wd, dx, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_DATA)))
    lc.conv2d_bwd_weight(d, xd, dyd, dw, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT)))
    torch.cuda.synchronize()
    y, dx, dw = y.cpu().numpy(), dx.cpu().numpy(), dw.cpu().numpy()
    assert np.all(np.isfinite(y)) and np.all(np.isfinite(dx)) and np.all(np.isfinite(dw))

    def nhwc_coords(count, dims_nchw, sd):          # (n, ch, row, col) coordinates for the oracle
        return synth.sample_coords(count, dims_nchw, sd)

    cy = nhwc_coords(2048, (cs.n, cs.k, cs.p, cs.q), seed + 3)
    ref, mag = oracle.conv2d_fwd_at(x, wt, cy, cs.stride, cs.pad, oracle.NHWC)
    got = y[cy[:, 0], cy[:, 2], cy[:, 3], cy[:, 1]]
    assert np.max(np.abs(got - ref)) <= TOL * np.max(np.abs(ref))
    assert np.max(np.abs(got - ref) / mag) <= 1e-5          # against the sum of |terms|: order-independent bound

    cx = nhwc_coords(2048, (cs.n, cs.c, cs.h, cs.w), seed + 4)
    ref, _ = oracle.conv2d_bwd_data_at(dy, wt, (cs.h, cs.w), cx, cs.stride, cs.pad, oracle.NHWC)
    got = dx[cx[:, 0], cx[:, 2], cx[:, 3], cx[:, 1]]
    assert np.max(np.abs(got - ref)) <= TOL * max(np.max(np.abs(ref)), 1e-30)
    if cs.r == 1 and cs.stride == 2:
        assert np.all(dx[:, 1::2, :, :] == 0) and np.all(dx[:, :, 1::2, :] == 0)

    cw = nhwc_coords(256, (cs.k, cs.c, cs.r, cs.s), seed + 5)
    ref, mag = oracle.conv2d_bwd_weight_at(x, dy, (cs.r, cs.s), cw, cs.stride, cs.pad, oracle.NHWC)
    got = dw[cw[:, 0], cw[:, 2], cw[:, 3], cw[:, 1]]
    assert np.max(np.abs(got - ref)) <= TOL * np.max(np.abs(ref))

    # adjoint identity on the GPU's own outputs, sums in float64 on the host
    lhs = float(np.sum(y.astype(np.float64) * dy))
    a = float(np.sum(x.astype(np.float64) * dx))
    b = float(np.sum(wt.astype(np.float64) * dw))
    scale = float(np.sqrt(np.sum(y.astype(np.float64) ** 2) * np.sum(dy.astype(np.float64) ** 2)))
    assert abs(lhs - a) <= 1e-5 * scale and abs(lhs - b) <= 1e-5 * scale


# ---- AlexNet-BN layer shapes at batch 256 (five convolutions, three FC layers as convolutions) ----
ALEX = {c.name: c for c in synth.alexnet_bn_convs(256)}


@pytest.mark.parametrize("name", list(ALEX))
def test_alexnet_bn_layers_full_size_sampled(name):
    cs = ALEX[name]
    seed = 4000 + 10 * list(ALEX).index(name)
    print(f"alexnet layer {name}: {cs}", flush=True)
    x = synth.normal((cs.n, cs.h, cs.w, cs.c), seed)
    wt = synth.normal((cs.k, cs.r, cs.s, cs.c), seed + 1, std=synth.he_std(cs))
    dy = synth.normal((cs.n, cs.p, cs.q, cs.k), seed + 2)
    d = lc.ConvDesc(cs.n, cs.c, cs.h, cs.w, cs.k, cs.r, cs.s, cs.stride, cs.stride, cs.pad, cs.pad, lc.LC_F32, lc.LC_NHWC)
    xd, wd, dyd = gu.dev(x), gu.dev(wt), gu.dev(dy)
    y = torch.empty((cs.n, cs.p, cs.q, cs.k), dtype=torch.float32, device=gu.DEV)
    dx = torch.empty((cs.n, cs.h, cs.w, cs.c), dtype=torch.float32, device=gu.DEV)
    dw = torch.empty((cs.k, cs.r, cs.s, cs.c), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_fwd(d, xd, wd, y, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)))
    lc.conv2d_bwd_data(d, dyd, wd, dx, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_DATA)))
    lc.conv2d_bwd_weight(d, xd, dyd, dw, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT)))
    torch.cuda.synchronize()
    y, dx, dw = y.cpu().numpy(), dx.cpu().numpy(), dw.cpu().numpy()
    cy = synth.sample_coords(1024, (cs.n, cs.k, cs.p, cs.q), seed + 3)
    ref, _ = oracle.conv2d_fwd_at(x, wt, cy, cs.stride, cs.pad, oracle.NHWC)
    assert np.max(np.abs(y[cy[:, 0], cy[:, 2], cy[:, 3], cy[:, 1]] - ref)) <= TOL * np.max(np.abs(ref))
    cx = synth.sample_coords(1024, (cs.n, cs.c, cs.h, cs.w), seed + 4)
    ref, _ = oracle.conv2d_bwd_data_at(dy, wt, (cs.h, cs.w), cx, cs.stride, cs.pad, oracle.NHWC)
    assert np.max(np.abs(dx[cx[:, 0], cx[:, 2], cx[:, 3], cx[:, 1]] - ref)) <= TOL * max(np.max(np.abs(ref)), 1e-30)
    cw = synth.sample_coords(256, (cs.k, cs.c, cs.r, cs.s), seed + 5)
    ref, _ = oracle.conv2d_bwd_weight_at(x, dy, (cs.r, cs.s), cw, cs.stride, cs.pad, oracle.NHWC)
    assert np.max(np.abs(dw[cw[:, 0], cw[:, 2], cw[:, 3], cw[:, 1]] - ref)) <= TOL * np.max(np.abs(ref))
    assert np.all(np.isfinite(y)) and np.all(np.isfinite(dx)) and np.all(np.isfinite(dw))


def test_resnet50_conv_sweep_batch128_sampled():
    """Every distinct ResNet-50 convolution shape at batch 128, each pass checked on sampled outputs."""
    for idx, (cs, count) in enumerate(synth.resnet50_distinct_shapes(128), start=1):
        seed = 6000 + 10 * idx
        print(f"sweep shape {idx}: {cs} (x{count})", flush=True)
        x = synth.normal((cs.n, cs.h, cs.w, cs.c), seed)
        wt = synth.normal((cs.k, cs.r, cs.s, cs.c), seed + 1, std=synth.he_std(cs))
        dy = synth.normal((cs.n, cs.p, cs.q, cs.k), seed + 2)
        d = lc.ConvDesc(cs.n, cs.c, cs.h, cs.w, cs.k, cs.r, cs.s, cs.stride, cs.stride, cs.pad, cs.pad, lc.LC_F32, lc.LC_NHWC)
        xd, wd, dyd = gu.dev(x), gu.dev(wt), gu.dev(dy)
        y = torch.empty((cs.n, cs.p, cs.q, cs.k), dtype=torch.float32, device=gu.DEV)
        dx = torch.empty((cs.n, cs.h, cs.w, cs.c), dtype=torch.float32, device=gu.DEV)
        dw = torch.empty((cs.k, cs.r, cs.s, cs.c), dtype=torch.float32, device=gu.DEV)
        lc.conv2d_fwd(d, xd, wd, y, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)))
        lc.conv2d_bwd_data(d, dyd, wd, dx, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_DATA)))
        lc.conv2d_bwd_weight(d, xd, dyd, dw, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT)))
        torch.cuda.synchronize()
        y, dx, dw = y.cpu().numpy(), dx.cpu().numpy(), dw.cpu().numpy()
        cy = synth.sample_coords(512, (cs.n, cs.k, cs.p, cs.q), seed + 3)
        ref, _ = oracle.conv2d_fwd_at(x, wt, cy, cs.stride, cs.pad, oracle.NHWC)
        assert np.max(np.abs(y[cy[:, 0], cy[:, 2], cy[:, 3], cy[:, 1]] - ref)) <= TOL * np.max(np.abs(ref)), idx
        cx = synth.sample_coords(512, (cs.n, cs.c, cs.h, cs.w), seed + 4)
        ref, _ = oracle.conv2d_bwd_data_at(dy, wt, (cs.h, cs.w), cx, cs.stride, cs.pad, oracle.NHWC)
        assert np.max(np.abs(dx[cx[:, 0], cx[:, 2], cx[:, 3], cx[:, 1]] - ref)) <= TOL * max(np.max(np.abs(ref)), 1e-30), idx
        cw = synth.sample_coords(128, (cs.k, cs.c, cs.r, cs.s), seed + 5)
        ref, _ = oracle.conv2d_bwd_weight_at(x, dy, (cs.r, cs.s), cw, cs.stride, cs.pad, oracle.NHWC)
        assert np.max(np.abs(dw[cw[:, 0], cw[:, 2], cw[:, 3], cw[:, 1]] - ref)) <= TOL * np.max(np.abs(ref)), idx
        del xd, wd, dyd
        torch.cuda.empty_cache()


def test_output_beyond_two_gibibytes_sampled():
    """A 1x1 layer whose output (and output gradient) is larger than 2^31 bytes: the kernels address tiles with
    32-bit offsets relative to per-tile bases, which must hold however large the tensor is."""
    n, c, hw, k = 2200, 64, 14, 1280
    p = q = hw
    assert n * p * q * k * 4 > 2 ** 31
    x = synth.normal((n, hw, hw, c), 9100)
    wt = synth.normal((k, 1, 1, c), 9101, std=float(np.sqrt(2.0 / c)))
    block = synth.normal((30_000_017,), 9102)                       # dY: a long non-periodic-looking block, repeated
    total = n * p * q * k
    dy = np.resize(block, total).reshape(n, p, q, k)
    d = lc.ConvDesc(n, c, hw, hw, k, 1, 1, 1, 1, 0, 0, lc.LC_F32, lc.LC_NHWC)
    xd, wd, dyd = gu.dev(x), gu.dev(wt), gu.dev(dy)
    y = torch.empty((n, p, q, k), dtype=torch.float32, device=gu.DEV)
    dx = torch.empty((n, hw, hw, c), dtype=torch.float32, device=gu.DEV)
    dw = torch.empty((k, 1, 1, c), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_fwd(d, xd, wd, y, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)))
    lc.conv2d_bwd_data(d, dyd, wd, dx, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_DATA)))
    lc.conv2d_bwd_weight(d, xd, dyd, dw, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT)))
    torch.cuda.synchronize()
    # the last rows of the output (beyond the 2 GiB mark) and a sample over everything
    tail = y[-3:].cpu().numpy()
    ref_tail = (x[-3:].reshape(-1, c).astype(np.float64) @ wt.reshape(k, c).astype(np.float64).T).reshape(3, p, q, k)
    assert gu.scaled_err(tail, ref_tail) <= TOL
    y = y.cpu().numpy()
    cy = synth.sample_coords(2048, (n, k, p, q), 9103)
    ref, mag = oracle.conv2d_fwd_at(x, wt, cy, 1, 0, oracle.NHWC)
    got = y[cy[:, 0], cy[:, 2], cy[:, 3], cy[:, 1]]
    assert np.max(np.abs(got - ref)) <= TOL * np.max(np.abs(ref))
    del y
    dx = dx.cpu().numpy()
    cx = synth.sample_coords(1024, (n, c, hw, hw), 9104)
    ref, _ = oracle.conv2d_bwd_data_at(dy, wt, (hw, hw), cx, 1, 0, oracle.NHWC)
    got = dx[cx[:, 0], cx[:, 2], cx[:, 3], cx[:, 1]]
    assert np.max(np.abs(got - ref)) <= TOL * np.max(np.abs(ref))
    # last image of dX: its dY rows lie beyond the 2 GiB mark
    ref_last = (dy[-1].reshape(-1, k).astype(np.float64) @ wt.reshape(k, c).astype(np.float64)).reshape(hw, hw, c)
    assert gu.scaled_err(dx[-1], ref_last) <= TOL
    dw = dw.cpu().numpy()
    cw = synth.sample_coords(128, (k, c, 1, 1), 9105)
    ref, mag = oracle.conv2d_bwd_weight_at(x, dy, (1, 1), cw, 1, 0, oracle.NHWC)
    got = dw[cw[:, 0], cw[:, 2], cw[:, 3], cw[:, 1]]
    assert np.max(np.abs(got - ref)) <= TOL * np.max(np.abs(ref))
