"""GPU parity of a WHOLE mixed-precision training step: the bottleneck network at a few channels with bf16
activations, activation gradients and convolution filters (fp32 parameters, parameter gradients, statistics,
classifier and loss), forward, backward and the LARS update on the device through the C ABI, against the float64
oracle that rounds to bf16 at the same places (oracle/resnet.py, forward_backward_bf16).

What can differ: the device computes each layer in fp32, the oracle in float64, and both then round to bf16; where
a value sits next to a rounding boundary the two land one bf16 step (2^-8 relative) apart, and that difference then
travels on through the layers behind it -- more so than in fp32, because a batch norm over few values amplifies it.
The bars: every stored activation within TOL_ACT = 1e-2 tensor-scaled and at least 98 % of its elements bit-equal;
every parameter gradient within TOL_GRAD = 2e-2 tensor-scaled (bf16's step is 3.9e-3); loss within 1e-3.  The LARS
update is then checked at fp32 accuracy on the device's own gradients, and the bf16 filter copies it writes bit
for bit against the rounded fp32 weights."""
import numpy as np
import pytest
import torch

import oracle
from oracle import resnet as ores
from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth
from paper_1709_05011_amd.resnet_step import ResNetStep

import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL_ACT, TOL_GRAD = 1e-2, 2e-2
CFG = ores.Config(stem=(8, 3, 1, 1), widths=(8, 16), blocks=(2, 1), classes=10, in_channels=8)
BATCH, HW = 8, 16


def _problem(seed):
    params = {}
    for i, (name, shp) in enumerate(ores.param_shapes(CFG).items()):
        if name.endswith(".gamma"):
            params[name] = (1.0 + 0.2 * synth.normal(shp, seed + i)).astype(np.float32)
        elif name.endswith(".beta") or name == "fc.b":
            params[name] = (0.2 * synth.normal(shp, seed + i)).astype(np.float32)
        else:
            params[name] = synth.normal(shp, seed + i, std=(2.0 / int(np.prod(shp[1:]))) ** 0.5).astype(np.float32)
    x = synth.bf16_bits_to_f32(synth.to_bf16_bits(synth.normal((BATCH, CFG.in_channels, HW, HW), seed + 1000)))
    labels = synth.uniform_int(BATCH, seed + 2000, CFG.classes)
    return x, labels, params


def _to_device_layout(name, a):
    if name.endswith(".w") and a.ndim == 4:
        return np.ascontiguousarray(a.transpose(0, 2, 3, 1))          # [k, c, r, s] -> [k, r, s, c]
    if name == "fc.w":
        return np.ascontiguousarray(a.reshape(a.shape[0], 1, 1, a.shape[1]))
    return a


def _from_device_layout(name, a, ref_shape):
    if name.endswith(".w") and len(ref_shape) == 4:
        return a.transpose(0, 3, 1, 2)
    return a.reshape(ref_shape)


def _bf16_host(t):
    """device bf16 tensor [n, h, w, c] -> fp32 values [n, c, h, w]"""
    return synth.bf16_bits_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16)).transpose(0, 3, 1, 2)


@pytest.mark.parametrize("pair", [True, False], ids=["paired_batch_norms", "plain_batch_norms"])
def test_whole_bf16_training_step_matches_oracle(pair):
    """``pair``: relu(bn(c3) + bn(projection)) in one pass; the projection's batch-norm output is then never stored and so
    never rounded to bf16, on the device and in the oracle."""
    x, labels, params = _problem(4300)
    trace, grads = ores.forward_backward_bf16(x, labels, params, CFG, pair=pair)

    net = ResNetStep(CFG.stem, CFG.widths, CFG.blocks, CFG.classes, BATCH, (HW, HW), in_channels=CFG.in_channels, dtype=lc.LC_BF16,
                     pair_bn=pair)
    assert list(net.params) == list(params)
    net.load({k: _to_device_layout(k, v) for k, v in params.items()})
    xbits = synth.to_bf16_bits(np.ascontiguousarray(x.transpose(0, 2, 3, 1)))
    xd = torch.from_numpy(xbits.view(np.int16)).to(gu.DEV).view(torch.bfloat16)
    ld = gu.dev(labels.astype(np.int32))
    loss = net.forward(xd, ld)
    net.backward()
    torch.cuda.synchronize()

    assert abs(float(loss.item()) - float(trace["loss"])) <= 1e-3 * max(1.0, abs(float(trace["loss"])))
    assert gu.scaled_err(net.logits.cpu().numpy(), trace["logits"]) <= TOL_ACT
    equal = []
    for name in net.order:
        L = net.layers[name]
        for key, t in ((".z", L.z), (".a", L.a)):
            if t is None:                                                # (a projection's output is not stored when paired)
                continue
            got = _bf16_host(t)
            assert gu.scaled_err(got, trace[name + key]) <= TOL_ACT, name + key
            equal.append(float(np.mean(got == trace[name + key])))
    assert min(equal) >= 0.98, min(equal)
    worst = 0.0
    for k in params:
        got = _from_device_layout(k, net.grads[k].cpu().numpy(), grads[k].shape)
        err = gu.scaled_err(got, grads[k])
        worst = max(worst, err)
        assert err <= TOL_GRAD, (k, err)
    print(f"bit-equal stored activations: min {min(equal):.4f}; worst gradient error {worst:.2e}")

    # the update at fp32 accuracy, on the very w, g, v the device holds
    eta, momentum, wd, lr = 0.001, 0.9, 5e-4, 0.3
    names = list(params)
    f = np.float32
    dev_w = [net.params[k].cpu().numpy().ravel().copy() for k in names]
    dev_g = [net.grads[k].cpu().numpy().ravel().copy() for k in names]
    dev_v = [net.velocity[k].cpu().numpy().ravel().copy() for k in names]
    trust_dev, _ = oracle.lars_step(dev_w, dev_g, dev_v, float(f(eta)), float(f(momentum)), float(f(wd)), float(f(lr)))
    net.lars(eta, momentum, wd, lr)
    torch.cuda.synchronize()
    got_trust = net.trust.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got_trust - trust_dev) / np.abs(trust_dev)) <= 1e-5
    for i, k in enumerate(names):
        got_w = net.params[k].cpu().numpy().ravel()
        assert gu.scaled_err(got_w, dev_w[i]) <= 1e-5, k
        if k in net.lowp:             # the copy the next step's convolutions read: the new weights rounded to nearest even
            bits = net.lowp[k].view(torch.int16).cpu().numpy().view(np.uint16).ravel()
            np.testing.assert_array_equal(bits, synth.to_bf16_bits(got_w))
            np.testing.assert_array_equal(synth.bf16_bits_to_f32(bits), oracle.round_to_bf16(got_w))

    # a second step runs on the updated weights and stays finite
    loss2 = net.step(xd, ld, eta, momentum, wd, lr)
    torch.cuda.synchronize()
    assert np.isfinite(float(loss2.item()))
    for k in names:
        assert torch.isfinite(net.params[k]).all(), k
