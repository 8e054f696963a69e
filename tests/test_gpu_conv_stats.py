"""GPU parity of the batch-norm statistics that come out of the forward convolution (conv2d_fwd_stats) and of the batch
norm that takes them (batchnorm_fwd_pre), fp32 and bf16, NHWC.

What is checked, per shape:
  * y of conv2d_fwd_stats is bit-identical to y of conv2d_fwd;
  * every piece of the statistics equals the sums of the rows of y it covers (y as the device stored it, summed in
    float64 on the host) to 1e-5 of sum |y| resp. sum y^2 (fp32 sums of at most 128 values);
  * the totals agree with the float64 oracle convolution to the convolution's own tolerance;
  * batchnorm_fwd_pre on (y, statistics) gives the mean and 1/std of the float64 oracle to 1e-5 / 1e-4 and the
    output within the batch-norm tolerances (1e-4 tensor-scaled in fp32; one bf16 step in bf16).
Shapes cover tiles the stream-K blocks share (their sums come from a read-back kernel), ragged last tiles in both
directions, the few-channel first layer over 2x2 pixel blocks, the 256x256 tile of the bf16 kernel, and -- with the
tile threshold lowered -- the slab kernel of the bf16 3x3 layers."""
import numpy as np
import pytest
import torch

import oracle
from oracle import batchnorm as obn
from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
NHWC = lc.LC_NHWC
EPS = 1e-5

SHAPES = {
    # n, c, h, w, k, r, s, stride, pad
    "3x3_multi_tile": (4, 64, 14, 14, 96, 3, 3, 1, 1),                 # 784 rows: 6 whole tiles and a ragged one; 96 columns
    "1x1_many_rows": (8, 64, 28, 28, 256, 1, 1, 1, 0),
    "1x1_stride2": (4, 128, 15, 15, 64, 1, 1, 2, 0),
    "deep_k_few_tiles_stream_k": (2, 512, 7, 7, 512, 3, 3, 1, 1),      # 98 rows x 512 columns, 288 k-steps: tiles are shared
    "ragged_rows_and_columns": (3, 32, 9, 11, 40, 3, 3, 1, 1),
    "stem_7x7_s2_c3": (4, 3, 32, 32, 64, 7, 7, 2, 3),
    "resnet_14_stage": (8, 256, 14, 14, 256, 3, 3, 1, 1),
}
SHAPES_BF16_ONLY = {
    "big_tile_256x256": (64, 128, 28, 28, 512, 1, 1, 1, 0),
}


def _inputs(shape, seed, bf16):
    n, c, h, w, k, r, s, stride, pad = shape
    x = (synth.normal((n, c, h, w), seed) + 0.25).astype(np.float32)
    wt = synth.normal((k, c, r, s), seed + 1, std=float(np.sqrt(2.0 / (c * r * s))))
    if bf16:
        x = synth.bf16_bits_to_f32(synth.to_bf16_bits(x))
        wt = synth.bf16_bits_to_f32(synth.to_bf16_bits(wt))
    return x, wt


def _put(a_nchw, bf16):
    a = gu.to_layout(a_nchw, NHWC)
    if bf16:
        return torch.from_numpy(synth.to_bf16_bits(a).view(np.int16)).to(gu.DEV)
    return gu.dev(a)


def _get(t, bf16):
    a = t.cpu().numpy()
    return synth.bf16_bits_to_f32(a.view(np.uint16)) if bf16 else a


def _case(name, shape, bf16):
    n, c, h, w, k, r, s, stride, pad = shape
    x, wt = _inputs(shape, 9900 + 7 * len(name), bf16)
    dtype = lc.LC_BF16 if bf16 else lc.LC_F32
    d = gu.desc_for(x.shape, wt.shape, stride, pad, NHWC, dtype)
    p, q = lc.conv2d_out_shape(d)
    count = lc.conv2d_fwd_stats_count(d)
    print(f"stats case {name} bf16={bf16} desc {d} pieces {count}", flush=True)
    assert count > 0
    xd, wd = _put(x, bf16), _put(wt, bf16)
    ws = gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD))
    tdt = torch.int16 if bf16 else torch.float32
    y_plain = torch.full((n, p, q, k), -1 if bf16 else float("nan"), dtype=tdt, device=gu.DEV)
    y = torch.full((n, p, q, k), -1 if bf16 else float("nan"), dtype=tdt, device=gu.DEV)
    stats = torch.full((count, k, 2), float("nan"), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_fwd(d, xd, wd, y_plain, ws)
    lc.conv2d_fwd_stats(d, xd, wd, y, stats, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(y.cpu().numpy(), y_plain.cpu().numpy())

    got = stats.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got)), "a piece was not written"
    rows = _get(y, bf16).reshape(n * p * q, k).astype(np.float64)
    m = rows.shape[0]
    if (c, k, r, s, stride, pad) == (3, 64, 7, 7, 2, 3) and p % 16 == 0 and q % 16 == 0:
        # the first-layer kernel: a piece is a 4 x 16 block of one image's output pixels, four to a 16 x 16 tile
        assert count == n * (p // 16) * (q // 16) * 4
        idx = np.arange(m).reshape(n, p, q)
        pieces = [idx[i, 16 * ty + 4 * wv:16 * ty + 4 * wv + 4, 16 * tx:16 * tx + 16].ravel()
                  for i in range(n) for ty in range(p // 16) for tx in range(q // 16) for wv in range(4)]
    else:
        half = next(hf for hf in (64, 128) if 2 * ((m + 2 * hf - 1) // (2 * hf)) == count)
        pieces = [np.arange(t * half, min((t + 1) * half, m)) for t in range(count)]
    for t in range(count):
        part = rows[pieces[t]]
        s1, s2 = part.sum(axis=0), (part * part).sum(axis=0)
        assert np.all(np.abs(got[t, :, 0] - s1) <= 1e-5 * np.abs(part).sum(axis=0) + 1e-30), (t, "sum")
        assert np.all(np.abs(got[t, :, 1] - s2) <= 1e-5 * s2 + 1e-30), (t, "sum of squares")

    ref = oracle.conv2d_fwd(x, wt, stride, pad)                           # NCHW float64
    ref_rows = ref.transpose(0, 2, 3, 1).reshape(m, k)
    tol = 2e-2 if bf16 else 1e-4
    assert gu.scaled_err(got[:, :, 0].sum(axis=0), ref_rows.sum(axis=0)) <= tol * 4      # sums of rounded values: errors partly add
    assert gu.scaled_err(got[:, :, 1].sum(axis=0), (ref_rows ** 2).sum(axis=0)) <= tol * 4

    # batch norm from the handed-over sums, against the oracle on the device's y
    gamma = (1.0 + 0.3 * synth.normal((k,), 9950)).astype(np.float32)
    beta = (0.3 * synth.normal((k,), 9951)).astype(np.float32)
    gd, bd = gu.dev(gamma), gu.dev(beta)
    out = torch.full_like(y, -1 if bf16 else float("nan"))
    mean, invstd = torch.empty(k, device=gu.DEV), torch.empty(k, device=gu.DEV)
    bws = gu.workspace(lc.batchnorm_workspace_bytes(n, k, p, q, NHWC))
    lc.batchnorm_fwd_pre(dtype, y, gd, bd, None, out, mean, invstd, n, k, p, q, EPS, True, NHWC, stats, count, bws)
    torch.cuda.synchronize()
    y_nchw = _get(y, bf16).transpose(0, 3, 1, 2)
    oy, omean, oinv = obn.forward(y_nchw, gamma, beta, EPS)
    oy = np.maximum(oy, 0.0)
    assert gu.scaled_err(mean.cpu().numpy(), omean) <= 1e-5
    assert np.max(np.abs(invstd.cpu().numpy() - oinv) / oinv) <= 1e-4
    got_out = _get(out, bf16).transpose(0, 3, 1, 2)
    if bf16:
        bound = np.abs(oy) * 2.0 ** -8 + 2e-4 * float(np.max(np.abs(oy)))
        assert np.all(np.abs(got_out - oy) <= bound)
    else:
        assert gu.scaled_err(got_out, oy) <= 1e-4


@pytest.mark.parametrize("bf16", [False, True], ids=["fp32", "bf16"])
@pytest.mark.parametrize("name", list(SHAPES))
def test_statistics_out_of_the_convolution(name, bf16):
    _case(name, SHAPES[name], bf16)


@pytest.mark.parametrize("name", list(SHAPES_BF16_ONLY))
def test_statistics_out_of_the_big_tile(name):
    _case(name, SHAPES_BF16_ONLY[name], True)


@pytest.mark.parametrize("name", ["3x3_multi_tile", "ragged_rows_and_columns", "resnet_14_stage"])
def test_statistics_out_of_the_slab_kernel(name):
    import os
    old = os.environ.get("LARSCONV_SLAB_MIN_TILES")
    os.environ["LARSCONV_SLAB_MIN_TILES"] = "1"
    try:
        _case(name, SHAPES[name], True)
    finally:
        if old is None:
            del os.environ["LARSCONV_SLAB_MIN_TILES"]
        else:
            os.environ["LARSCONV_SLAB_MIN_TILES"] = old


def test_layers_without_the_epilogue_say_so():
    d = lc.ConvDesc(2, 16, 8, 8, 32, 3, 3, 1, 1, 1, 1, lc.LC_F32, lc.LC_NCHW)
    assert lc.conv2d_fwd_stats_count(d) == 0
    g = lc.ConvDesc(2, 16, 8, 8, 32, 3, 3, 1, 1, 1, 1, lc.LC_F32, NHWC, groups=2)
    assert lc.conv2d_fwd_stats_count(g) == 0
    odd = lc.ConvDesc(2, 6, 8, 8, 32, 3, 3, 1, 1, 1, 1, lc.LC_F32, NHWC)         # 6 channels: the scalar kernel takes it
    x = torch.zeros(2 * 8 * 8 * 16, device=gu.DEV)
    w = torch.zeros(32 * 9 * 16, device=gu.DEV)
    y = torch.zeros(2 * 8 * 8 * 32, device=gu.DEV)
    st = torch.zeros(2048, dtype=torch.float32, device=gu.DEV)
    for desc in (d, g) + ((odd,) if lc.conv2d_fwd_stats_count(odd) == 0 else ()):
        with pytest.raises(lc.LarsConvError, match="unsupported"):
            lc.conv2d_fwd_stats(desc, x, w, y, st, gu.workspace(max(lc.conv2d_workspace_bytes(desc, lc.LC_PASS_FWD), 256)))


def test_reruns_are_bit_identical():
    shape = SHAPES["deep_k_few_tiles_stream_k"]
    n, c, h, w, k, r, s, stride, pad = shape
    x, wt = _inputs(shape, 9990, False)
    d = gu.desc_for(x.shape, wt.shape, stride, pad, NHWC)
    count = lc.conv2d_fwd_stats_count(d)
    xd, wd = _put(x, False), _put(wt, False)
    ws = gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD))
    runs = []
    for _ in range(2):
        y = torch.empty((n, h, w, k), device=gu.DEV)
        st = torch.full((count, k, 2), float("nan"), dtype=torch.float32, device=gu.DEV)
        lc.conv2d_fwd_stats(d, xd, wd, y, st, ws)
        torch.cuda.synchronize()
        runs.append(st.cpu().numpy())
    np.testing.assert_array_equal(runs[0], runs[1])


def test_statistics_at_full_size_bf16():
    """res2a's 1x1 convolution of the bf16 workload at its full size (512 x 56 x 56 x 64 -> 256: 1.6 M rows, 411 M outputs), the
    launch configuration bench.py times.  What holds at any size: y equals conv2d_fwd's bit for bit; the pieces, added up
    on the host, are the column sums of y as the device stored it (summed in float64 here, channel by channel); the batch
    norm that takes them returns that mean and 1/std and normalises sampled outputs accordingly."""
    n, c, hw, k = 512, 64, 56, 256
    gen = torch.Generator(device=gu.DEV)
    gen.manual_seed(4242)
    x = (torch.randn((n, hw, hw, c), generator=gen, device=gu.DEV) + 0.2).to(torch.bfloat16)
    w = (torch.randn((k, 1, 1, c), generator=gen, device=gu.DEV) * (2.0 / c) ** 0.5).to(torch.bfloat16)
    d = lc.ConvDesc(n, c, hw, hw, k, 1, 1, 1, 1, 0, 0, lc.LC_BF16, NHWC)
    count = lc.conv2d_fwd_stats_count(d)
    assert count > 0
    ws = gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD))
    y0 = torch.empty((n, hw, hw, k), dtype=torch.bfloat16, device=gu.DEV)
    y = torch.empty_like(y0)
    stats = torch.full((count, k, 2), float("nan"), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_fwd(d, x, w, y0, ws)
    lc.conv2d_fwd_stats(d, x, w, y, stats, ws)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y0.view(torch.int16))
    del y0
    got = stats.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    m = n * hw * hw
    s1, s2 = np.zeros(k), np.zeros(k)
    rows = y.view(m, k)
    for lo in range(0, m, 1 << 18):                        # float64 sums on the host, a slice at a time
        part = rows[lo:lo + (1 << 18)].to(torch.float32).cpu().numpy().astype(np.float64)
        s1 += part.sum(axis=0)
        s2 += (part * part).sum(axis=0)
    assert np.all(np.abs(got[:, :, 0].sum(axis=0) - s1) <= 1e-6 * np.sqrt(m) * np.sqrt(s2 / m) + 1e-9 * np.abs(s1))
    assert np.all(np.abs(got[:, :, 1].sum(axis=0) - s2) <= 1e-6 * s2)
    mean_ref, var_ref = s1 / m, s2 / m - (s1 / m) ** 2
    gamma = gu.dev((1.0 + 0.3 * synth.normal((k,), 4243)).astype(np.float32))
    beta = gu.dev((0.3 * synth.normal((k,), 4244)).astype(np.float32))
    out = torch.empty_like(y)
    mean, invstd = torch.empty(k, device=gu.DEV), torch.empty(k, device=gu.DEV)
    bws = gu.workspace(lc.batchnorm_workspace_bytes(n, k, hw, hw, NHWC))
    lc.batchnorm_fwd_pre(lc.LC_BF16, y, gamma, beta, None, out, mean, invstd, n, k, hw, hw, EPS, True, NHWC, stats, count, bws)
    torch.cuda.synchronize()
    assert np.max(np.abs(mean.cpu().numpy() - mean_ref)) <= 1e-5 * float(np.max(np.abs(mean_ref)) + np.sqrt(np.max(var_ref)))
    assert np.max(np.abs(invstd.cpu().numpy() * np.sqrt(var_ref + EPS) - 1.0)) <= 1e-4
    idx = torch.from_numpy(synth.uniform_int(4096, 4245, m)).to(gu.DEV).long()
    ys = rows[idx].to(torch.float32).cpu().numpy().astype(np.float64)
    want = np.maximum((ys - mean_ref) / np.sqrt(var_ref + EPS) * gamma.cpu().numpy().astype(np.float64) + beta.cpu().numpy(), 0.0)
    gots = out.view(m, k)[idx].to(torch.float32).cpu().numpy()
    assert np.all(np.abs(gots - want) <= np.abs(want) * 2.0 ** -8 + 2e-4 * float(np.max(np.abs(want))))
