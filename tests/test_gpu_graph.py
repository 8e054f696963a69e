"""The library under HIP graph capture: it allocates nothing, never synchronizes and clears memory with fill kernels
only, so a whole training step (every layer call and lars_step) can be captured once and replayed.  The test
captures the step of the few-channel residual network, replays it several times with eager work and synchronizations
in between, and checks every replay against the eager step bit for bit (all reductions run in a fixed order) -- in
fp32 and in mixed precision (bf16 activations and filters, the bf16 filter copies written by the update)."""
import numpy as np
import pytest
import torch

from oracle import resnet as ores
from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth
from paper_1709_05011_amd.resnet_step import ResNetStep

import gpu_util as gu

pytestmark = pytest.mark.gpu
CFG = ores.Config(stem=(8, 3, 1, 1), widths=(4, 8), blocks=(2, 1), classes=10)
CFG_BF16 = ores.Config(stem=(8, 3, 1, 1), widths=(8, 16), blocks=(2, 1), classes=10, in_channels=8)      # channel counts in eights
BATCH, HW = 8, 16
HYPER = (0.02, 0.9, 1e-4, 0.5)


def _init(net, seed):
    gen = torch.Generator(device=gu.DEV)
    gen.manual_seed(seed)
    for name, t in net.params.items():
        if name.endswith(".w"):
            t.copy_(torch.randn(t.shape, generator=gen, device=gu.DEV) * (2.0 / t[0].numel()) ** 0.5)
        elif name.endswith(".gamma"):
            t.fill_(1.0)
        else:
            t.zero_()
    for v in net.velocity.values():
        v.zero_()
    for name, t in net.lowp.items():                       # the bf16 filter copies start as the rounded weights
        t.copy_(net.params[name])


def _state(net):
    return ({k: v.clone() for k, v in net.params.items()}, {k: v.clone() for k, v in net.velocity.items()},
            {k: v.clone() for k, v in net.lowp.items()})


@pytest.mark.parametrize("bf16", [False, True], ids=["fp32", "bf16"])
def test_captured_step_replays_bit_identically(bf16):
    cfg = CFG_BF16 if bf16 else CFG
    make = lambda: ResNetStep(cfg.stem, cfg.widths, cfg.blocks, cfg.classes, BATCH, (HW, HW), in_channels=cfg.in_channels,     # noqa: E731
                              dtype=lc.LC_BF16 if bf16 else lc.LC_F32)
    x = gu.dev(synth.normal((BATCH, HW, HW, cfg.in_channels), 6100))
    if bf16:
        x = x.to(torch.bfloat16)
    labels = gu.dev(synth.uniform_int(BATCH, 6101, cfg.classes).astype(np.int32))

    # eager reference: three steps from the same start
    ref = make()
    _init(ref, 6102)
    ref_losses, ref_states = [], []
    for _ in range(3):
        ref_losses.append(float(ref.step(x, labels, *HYPER).item()))
        ref_states.append(_state(ref))

    net = make()
    _init(net, 6102)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                          # a warm-up step off the capture, then restore the start
        net.step(x, labels, *HYPER)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    _init(net, 6102)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        net.step(x, labels, *HYPER)
    torch.cuda.synchronize()
    _init(net, 6102)                                       # capture does not run the kernels; start over
    scratch = torch.empty(1 << 20, device=gu.DEV)
    for it in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert float(net.loss.item()) == ref_losses[it], (it, float(net.loss.item()), ref_losses[it])
        params, velocity, lowp = ref_states[it]
        for k in params:
            assert torch.equal(net.params[k], params[k]), (it, k)
            assert torch.equal(net.velocity[k], velocity[k]), (it, k)
        for k in lowp:
            assert torch.equal(net.lowp[k].view(torch.int16), lowp[k].view(torch.int16)), (it, k)
        assert bool(lowp) == bf16
        scratch.normal_()                                  # eager work between the replays
        (scratch * 2).sum().item()
