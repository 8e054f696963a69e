"""Pins for the AlexNet-BN oracle (oracle/alexnet.py): the paper's layer and parameter counts at full size,
finite differences of the float64 loss, and torch's float64 autograd of the same graph as a third opinion."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import alexnet
from paper_1709_05011_amd import synth

FULL = alexnet.Config(convs=((96, 11, 4, 0, True), (256, 5, 1, 2, True), (384, 3, 1, 1, False), (384, 3, 1, 1, False),
                             (256, 3, 1, 1, True)), fcs=(4096, 4096), classes=1000)
MINI = alexnet.Config(convs=((6, 5, 2, 0, True), (8, 3, 1, 1, True), (10, 3, 1, 1, False), (8, 3, 1, 1, True)), fcs=(24, 16), classes=10)
MINI_HW = (49, 49)


def test_full_size_structure():
    # five convolutions and three fully connected layers; 62,379,720 parameters in 21 tensors with ungrouped filters
    # (the paper quotes 61 M for the grouped original, "ImageNet training with AlexNet")
    shapes = alexnet.param_shapes(FULL, (227, 227))
    assert alexnet.feature_shape(FULL, (227, 227)) == (256, 6, 6)
    assert len(shapes) == 21
    assert [int(np.prod(s)) for s in shapes.values()] == synth.alexnet_bn_param_numels()
    assert sum(int(np.prod(s)) for s in shapes.values()) == 62_379_720
    ours = [(s[1], s[0], s[2]) for n, s in shapes.items() if n.startswith("conv") and n.endswith(".w")]
    assert ours == [(cs.c, cs.k, cs.r) for cs in synth.alexnet_bn_convs(1)[:5]]


def _problem(seed, batch=4):
    params = {}
    for i, (name, shp) in enumerate(alexnet.param_shapes(MINI, MINI_HW).items()):
        if name.endswith(".gamma"):
            params[name] = (1.0 + 0.2 * synth.normal(shp, seed + i)).astype(np.float32)
        elif name.endswith(".beta") or name.endswith(".b"):
            params[name] = (0.2 * synth.normal(shp, seed + i)).astype(np.float32)
        else:
            params[name] = synth.normal(shp, seed + i, std=(2.0 / int(np.prod(shp[1:]))) ** 0.5).astype(np.float32)
    x = synth.normal((batch, 3) + MINI_HW, seed + 1000).astype(np.float32)
    labels = synth.uniform_int(batch, seed + 2000, MINI.classes)
    return x, labels, params


def test_mini_feature_shape_and_trace():
    assert alexnet.feature_shape(MINI, MINI_HW) == (8, 2, 2)          # the first fully connected layer sees a 2x2 map
    x, labels, params = _problem(3)
    trace, grads = alexnet.forward_backward(x, labels, params, MINI)
    assert set(grads) == set(params)
    assert abs(trace["loss"] - alexnet.loss_only(x, labels, params, MINI)) < 1e-5


def test_gradients_match_directional_finite_differences():
    x, labels, params = _problem(7)
    _, grads = alexnet.forward_backward(x, labels, params, MINI)
    for trial in range(3):
        direction = {k: synth.normal(v.shape, 700 + 31 * trial + i).astype(np.float64) for i, (k, v) in enumerate(params.items())}
        h = 1e-7                 # small against the distance of any ReLU input or pool margin from its kink
        plus = {k: params[k].astype(np.float64) + h * direction[k] for k in params}
        minus = {k: params[k].astype(np.float64) - h * direction[k] for k in params}
        fd = (alexnet.loss_only(x, labels, plus, MINI) - alexnet.loss_only(x, labels, minus, MINI)) / (2 * h)
        an = sum(float((grads[k] * direction[k]).sum()) for k in params)
        assert abs(fd - an) <= 2e-4 * max(abs(fd), abs(an), 1e-3), (trial, fd, an)


def test_gradients_match_torch_autograd_float64():
    x, labels, params = _problem(13)
    _, grads = alexnet.forward_backward(x, labels, params, MINI)
    tp = {k: torch.from_numpy(v.astype(np.float64)).requires_grad_(True) for k, v in params.items()}
    a = torch.from_numpy(x.astype(np.float64))
    for i, (k, r, stride, pad, pool) in enumerate(MINI.convs):
        name = f"conv{i + 1}"
        z = F.conv2d(a, tp[name + ".w"], None, stride, pad)
        a = F.relu(F.batch_norm(z, None, None, tp[name + ".gamma"], tp[name + ".beta"], True, 0.0, MINI.eps))
        if pool:
            a = F.max_pool2d(a, 3, 2, 0)
    a = a.flatten(1)
    n_conv, n_fc = len(MINI.convs), len(MINI.fcs) + 1
    for j in range(n_fc):
        name = f"fc{n_conv + 1 + j}"
        a = a @ tp[name + ".w"].flatten(1).T + tp[name + ".b"]
        if j < n_fc - 1:
            a = F.relu(a)
    F.cross_entropy(a, torch.from_numpy(labels.astype(np.int64))).backward()
    for k in params:
        ref = tp[k].grad.numpy()
        err = np.abs(grads[k] - ref).max() / max(np.abs(ref).max(), 1e-12)
        assert err < 2e-5, (k, err)
