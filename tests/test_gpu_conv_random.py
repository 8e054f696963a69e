"""GPU parity on seeded random convolution shapes: small tensors with every dimension drawn independently (odd
channel counts, windows up to 5x5 and rectangular, strides up to 3, padding up to 3, one-pixel images), all three
passes in both layouts against the full-tensor oracle.  The table is fixed by the seed, so every run checks the
same 36 cases; it complements the hand-picked shapes of test_gpu_conv.py with combinations nobody thought of."""
import numpy as np
import pytest
import torch

import oracle
from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL, TOL_BF16, TOL_DW = 1e-4, 2e-2, 1e-4


def _draw(count, seed):
    u = synth.uniform01(count * 12, seed).reshape(count, 12)
    cases = []
    for row in u:
        pick = lambda x, lo, hi: lo + int(x * (hi - lo + 1) - 1e-9)
        n, c, k = pick(row[0], 1, 4), pick(row[1], 1, 40), pick(row[2], 1, 70)
        h, w = pick(row[3], 1, 20), pick(row[4], 1, 20)
        sh, sw = pick(row[5], 1, 3), pick(row[6], 1, 3)
        ph, pw = pick(row[7], 0, 3), pick(row[8], 0, 3)
        r = min(pick(row[9], 1, 5), h + 2 * ph)
        s = min(pick(row[10], 1, 5), w + 2 * pw)
        cases.append((n, c, h, w, k, r, s, (sh, sw), (ph, pw)))
    return cases


CASES_F32 = _draw(24, 31000)
CASES_BF16 = _draw(12, 32000)


@pytest.mark.parametrize("layout", [lc.LC_NHWC, lc.LC_NCHW], ids=["nhwc", "nchw"])
@pytest.mark.parametrize("idx", range(len(CASES_F32)))
def test_random_shape_fp32(idx, layout):
    n, c, h, w, k, r, s, stride, pad = CASES_F32[idx]
    x = synth.normal((n, c, h, w), 31100 + idx)
    wt = synth.normal((k, c, r, s), 31200 + idx, std=float(np.sqrt(2.0 / (c * r * s))))
    p, q = oracle.out_shape(h, w, r, s, stride, pad)
    dy = synth.normal((n, k, p, q), 31300 + idx)
    d = gu.desc_for(x.shape, wt.shape, stride, pad, layout)
    print(f"random fp32 case {idx}: {CASES_F32[idx]} layout {layout}", flush=True)
    xl, wl, dyl = gu.to_layout(x, layout), gu.to_layout(wt, layout), gu.to_layout(dy, layout)
    assert gu.scaled_err(gu.from_layout(gu.gpu_fwd(d, xl, wl), layout), oracle.conv2d_fwd(x, wt, stride, pad)) <= TOL
    assert gu.scaled_err(gu.from_layout(gu.gpu_bwd_data(d, dyl, wl), layout), oracle.conv2d_bwd_data(dy, wt, (h, w), stride, pad)) <= TOL
    assert gu.scaled_err(gu.from_layout(gu.gpu_bwd_weight(d, xl, dyl), layout), oracle.conv2d_bwd_weight(x, dy, (r, s), stride, pad)) <= TOL


def _bits(a):
    return synth.to_bf16_bits(a)


def _dev_bf16(bits_l):
    return torch.from_numpy(np.ascontiguousarray(bits_l).view(np.int16)).to(gu.DEV)


def _back(t):
    return synth.bf16_bits_to_f32(t.cpu().numpy().view(np.uint16))


@pytest.mark.parametrize("layout", [lc.LC_NHWC, lc.LC_NCHW], ids=["nhwc", "nchw"])
@pytest.mark.parametrize("idx", range(len(CASES_BF16)))
def test_random_shape_bf16(idx, layout):
    n, c, h, w, k, r, s, stride, pad = CASES_BF16[idx]
    p, q = oracle.out_shape(h, w, r, s, stride, pad)
    xb = _bits(synth.normal((n, c, h, w), 32100 + idx))
    wb = _bits(synth.normal((k, c, r, s), 32200 + idx, std=float(np.sqrt(2.0 / (c * r * s)))))
    dyb = _bits(synth.normal((n, k, p, q), 32300 + idx))
    x, wt, dy = (synth.bf16_bits_to_f32(b) for b in (xb, wb, dyb))
    d = gu.desc_for(x.shape, wt.shape, stride, pad, layout, lc.LC_BF16)
    print(f"random bf16 case {idx}: {CASES_BF16[idx]} layout {layout}", flush=True)
    xd, wd, dyd = (_dev_bf16(gu.to_layout(a, layout)) for a in (xb, wb, dyb))
    nhwc = layout == lc.LC_NHWC
    y = torch.full((n, p, q, k) if nhwc else (n, k, p, q), -1, dtype=torch.int16, device=gu.DEV)
    dx = torch.full((n, h, w, c) if nhwc else (n, c, h, w), -1, dtype=torch.int16, device=gu.DEV)
    dw = torch.full((k, r, s, c) if nhwc else (k, c, r, s), float("nan"), dtype=torch.float32, device=gu.DEV)
    lc.conv2d_fwd(d, xd, wd, y, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)))
    lc.conv2d_bwd_data(d, dyd, wd, dx, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_DATA)))
    lc.conv2d_bwd_weight(d, xd, dyd, dw, gu.workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT)))
    torch.cuda.synchronize()
    assert gu.scaled_err(gu.from_layout(_back(y), layout), oracle.round_to_bf16(oracle.conv2d_fwd(x, wt, stride, pad))) <= TOL_BF16
    assert gu.scaled_err(gu.from_layout(_back(dx), layout), oracle.round_to_bf16(oracle.conv2d_bwd_data(dy, wt, (h, w), stride, pad))) <= TOL_BF16
    assert gu.scaled_err(gu.from_layout(dw.cpu().numpy(), layout), oracle.conv2d_bwd_weight(x, dy, (r, s), stride, pad)) <= TOL_DW
