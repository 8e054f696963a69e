"""Pins for the grouped-convolution oracle: it must be G independent convolutions on channel slices (checked against
the pinned one-group oracle), reduce to the plain oracle for one group, agree with a float64 library convolution, and
make the original AlexNet come out at the parameter and operation counts the paper prints."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_1709_05011_amd import synth

CASES = [  # n, c, h, w, k, r, s, stride, pad, groups
    (2, 6, 7, 6, 4, 3, 2, (1, 1), (1, 0), 2),
    (2, 6, 9, 8, 9, 3, 3, (2, 1), (1, 2), 3),
    (1, 8, 5, 5, 8, 1, 1, (1, 1), (0, 0), 8),          # depthwise: every filter sees one channel
    (3, 4, 6, 7, 6, 2, 3, (2, 2), (0, 1), 2),
]


def _data(case, seed):
    n, c, h, w, k, r, s, stride, pad, g = case
    x = synth.normal((n, c, h, w), seed)
    wt = synth.normal((k, c // g, r, s), seed + 1)
    p, q = oracle.out_shape(h, w, r, s, stride, pad)
    dy = synth.normal((n, k, p, q), seed + 2)
    return x, wt, dy


def _nhwc(a):
    return np.ascontiguousarray(np.transpose(a, (0, 2, 3, 1)))


@pytest.mark.parametrize("case", CASES)
def test_grouped_is_independent_convolutions_on_channel_slices(case):
    n, c, h, w, k, r, s, stride, pad, g = case
    x, wt, dy = _data(case, 700)
    cg, kg = c // g, k // g
    y = oracle.conv2d_fwd_grouped(x, wt, g, stride, pad)
    dx = oracle.conv2d_bwd_data_grouped(dy, wt, g, (h, w), stride, pad)
    dw = oracle.conv2d_bwd_weight_grouped(x, dy, g, (r, s), stride, pad)
    for i in range(g):
        xs, ws, dys = x[:, i * cg:(i + 1) * cg], wt[i * kg:(i + 1) * kg], dy[:, i * kg:(i + 1) * kg]
        np.testing.assert_array_equal(y[:, i * kg:(i + 1) * kg], oracle.conv2d_fwd(xs, ws, stride, pad))
        np.testing.assert_array_equal(dx[:, i * cg:(i + 1) * cg], oracle.conv2d_bwd_data(dys, ws, (h, w), stride, pad))
        np.testing.assert_array_equal(dw[i * kg:(i + 1) * kg], oracle.conv2d_bwd_weight(xs, dys, (r, s), stride, pad))


@pytest.mark.parametrize("case", CASES)
def test_nhwc_is_the_same_numbers_in_another_order(case):
    n, c, h, w, k, r, s, stride, pad, g = case
    x, wt, dy = _data(case, 710)
    y = oracle.conv2d_fwd_grouped(_nhwc(x), _nhwc(wt), g, stride, pad, oracle.NHWC)
    np.testing.assert_array_equal(y, _nhwc(oracle.conv2d_fwd_grouped(x, wt, g, stride, pad)))
    dx = oracle.conv2d_bwd_data_grouped(_nhwc(dy), _nhwc(wt), g, (h, w), stride, pad, oracle.NHWC)
    np.testing.assert_array_equal(dx, _nhwc(oracle.conv2d_bwd_data_grouped(dy, wt, g, (h, w), stride, pad)))
    dw = oracle.conv2d_bwd_weight_grouped(_nhwc(x), _nhwc(dy), g, (r, s), stride, pad, oracle.NHWC)
    np.testing.assert_array_equal(dw, _nhwc(oracle.conv2d_bwd_weight_grouped(x, dy, g, (r, s), stride, pad)))


def test_one_group_is_the_plain_convolution():
    case = (2, 5, 7, 6, 4, 3, 2, (2, 1), (1, 1), 1)
    n, c, h, w, k, r, s, stride, pad, g = case
    x, wt, dy = _data(case, 720)
    np.testing.assert_array_equal(oracle.conv2d_fwd_grouped(x, wt, 1, stride, pad), oracle.conv2d_fwd(x, wt, stride, pad))
    np.testing.assert_array_equal(oracle.conv2d_bwd_data_grouped(dy, wt, 1, (h, w), stride, pad),
                                  oracle.conv2d_bwd_data(dy, wt, (h, w), stride, pad))
    np.testing.assert_array_equal(oracle.conv2d_bwd_weight_grouped(x, dy, 1, (r, s), stride, pad),
                                  oracle.conv2d_bwd_weight(x, dy, (r, s), stride, pad))


@pytest.mark.parametrize("case", CASES)
def test_against_float64_library_convolution_and_its_gradients(case):
    n, c, h, w, k, r, s, stride, pad, g = case
    x, wt, dy = _data(case, 730)
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    tw = torch.tensor(wt, dtype=torch.float64, requires_grad=True)
    ty = torch.nn.functional.conv2d(tx, tw, stride=stride, padding=pad, groups=g)
    ty.backward(torch.tensor(dy, dtype=torch.float64))
    np.testing.assert_allclose(oracle.conv2d_fwd_grouped(x, wt, g, stride, pad), ty.detach().numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.conv2d_bwd_data_grouped(dy, wt, g, (h, w), stride, pad), tx.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.conv2d_bwd_weight_grouped(x, dy, g, (r, s), stride, pad), tw.grad.numpy(), rtol=1e-12, atol=1e-12)


def test_adjoint_identity():
    case = CASES[1]
    n, c, h, w, k, r, s, stride, pad, g = case
    x, wt, dy = _data(case, 740)
    lhs = float(np.sum(oracle.conv2d_fwd_grouped(x, wt, g, stride, pad) * dy))
    assert abs(lhs - float(np.sum(x.astype(np.float64) * oracle.conv2d_bwd_data_grouped(dy, wt, g, (h, w), stride, pad)))) <= 1e-10 * abs(lhs)
    assert abs(lhs - float(np.sum(wt.astype(np.float64) * oracle.conv2d_bwd_weight_grouped(x, dy, g, (r, s), stride, pad)))) <= 1e-10 * abs(lhs)


def test_original_alexnet_matches_the_papers_counts(golden_dir):
    gold = {}
    with open(os.path.join(golden_dir, "paper_model_counts.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if len(line) == 2:
                gold[line[0]] = float(line[1])
    convs = synth.alexnet_grouped_convs(1)
    assert [cs.groups for cs in convs] == [1, 2, 1, 2, 2, 1, 1, 1]
    numels = synth.alexnet_grouped_param_numels()
    assert sum(numels) == 60_965_224 and round(sum(numels) / 1e6) == gold["alexnet_params_M"]         # "61 million"
    flops = sum(cs.flops for cs in convs)
    assert flops == 2 * 724_406_816
    assert abs(flops / 1e9 - gold["alexnet_flops_per_image_G"]) <= 0.06                                 # "1.5 billion" (1.449 G)
    # the paper's ratio is operations per image over parameters, from its own rounded entries
    assert round(gold["alexnet_flops_per_image_G"] * 1e3 / gold["alexnet_params_M"], 1) == gold["alexnet_scaling_ratio"]
    # the ungrouped filters of the batch-norm variant used elsewhere carry more of both
    assert sum(cs.flops for cs in synth.alexnet_bn_convs(1)) > flops


def test_v15_extra_shapes():
    sh = synth.resnet50_v15_extra_shapes(2)
    assert [(cs.c, cs.k, cs.r, cs.stride, cs.h, cs.p) for cs in sh] == [
        (256, 128, 1, 1, 56, 56), (128, 128, 3, 2, 56, 28), (512, 256, 1, 1, 28, 28), (256, 256, 3, 2, 28, 14),
        (1024, 512, 1, 1, 14, 14), (512, 512, 3, 2, 14, 7)]
