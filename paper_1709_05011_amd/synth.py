"""Seeded synthetic inputs and workload shape lists.

This module is the only code the CPU oracle's tests and the HIP path's tests
have in common.  It holds no arithmetic of the method (no convolution, no
norm, no update rule): only

* a counter-based random generator (splitmix64 finaliser over a 64-bit
  counter, Box-Muller for normals) whose output depends on nothing but
  ``(seed, index)``, so the same bytes are produced here, on the GPU machine and in
  any process;
* rounding of fp32 draws to bf16-representable values (input preparation for
  the bf16 workload);
* the layer shapes of the two networks the paper trains (AlexNet with batch
  norm after every convolution, and the original ResNet-50: Sections "Model
  Selection" and "Scaling up Batch Size"; Table "Scaling Ratio for AlexNet and
  ResNet50" gives the sizes they are checked against) and of the tiny CNN used
  as the whole-path parity case.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Tuple

import numpy as np

_U64 = np.uint64
_MASK = (1 << 64) - 1


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function applied element-wise to uint64 counters."""
    z = (z + _U64(0x9E3779B97F4A7C15)).astype(np.uint64)
    z = (z ^ (z >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> _U64(27))) * _U64(0x94D049BB133111EB)
    return z ^ (z >> _U64(31))


def _counters(seed: int, start: int, count: int, stream: int) -> np.ndarray:
    base = ((seed & _MASK) * 0xD1342543DE82EF95 + stream * 0x632BE59BD9B4E019) & _MASK
    with np.errstate(over="ignore"):
        return _U64(base) + np.arange(start, start + count, dtype=np.uint64) * _U64(0x9E3779B97F4A7C15)


def uniform01(count: int, seed: int, stream: int = 0, start: int = 0) -> np.ndarray:
    """``count`` doubles in (0, 1), element i a function of (seed, stream, start+i) only."""
    with np.errstate(over="ignore"):
        bits = _mix(_counters(seed, start, count, stream))
    return ((bits >> _U64(11)).astype(np.float64) + 0.5) * (1.0 / (1 << 53))


def normal(shape, seed: int, std: float = 1.0, mean: float = 0.0) -> np.ndarray:
    """fp32 array of N(mean, std^2) draws (Box-Muller on two counter streams)."""
    count = int(np.prod(shape, dtype=np.int64))
    out = np.empty(count, dtype=np.float32)
    step = 1 << 22  # bounded temporaries for the large activation tensors
    for lo in range(0, count, step):
        n = min(step, count - lo)
        u1 = uniform01(n, seed, 0, lo)
        u2 = uniform01(n, seed, 1, lo)
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        out[lo:lo + n] = (mean + std * z).astype(np.float32)
    return out.reshape(shape)


def uniform_int(count: int, seed: int, hi: int) -> np.ndarray:
    """int64 labels uniform in [0, hi)."""
    return np.minimum((uniform01(count, seed, 2) * hi).astype(np.int64), hi - 1)


def sample_coords(count: int, dims: Tuple[int, ...], seed: int) -> np.ndarray:
    """``count`` seeded coordinates, int32 [count, len(dims)], each column uniform in its dim."""
    cols = []
    for j, d in enumerate(dims):
        u = uniform01(count, seed, 16 + j)
        cols.append(np.minimum((u * d).astype(np.int64), d - 1))
    return np.stack(cols, axis=1).astype(np.int32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); returns the uint16 patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to the fp32 values they denote (exact)."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------------------
# workload shapes
# --------------------------------------------------------------------------------------

@dataclass(frozen=True)
class ConvShape:
    """One convolution: input N x C x H x W, filter K x C x R x S, stride and zero padding."""
    name: str
    n: int
    c: int
    h: int
    w: int
    k: int
    r: int
    s: int
    stride: int = 1
    pad: int = 0
    groups: int = 1          # filters see c / groups input channels each (c and k are the totals)

    @property
    def p(self) -> int:
        return (self.h + 2 * self.pad - self.r) // self.stride + 1

    @property
    def q(self) -> int:
        return (self.w + 2 * self.pad - self.s) // self.stride + 1

    @property
    def macs(self) -> int:
        return self.n * self.k * self.p * self.q * (self.c // self.groups) * self.r * self.s

    @property
    def flops(self) -> int:
        """Nominal dense count of one pass, 2 per multiply-add, padding taps included."""
        return 2 * self.macs

    @property
    def weight_numel(self) -> int:
        return self.k * (self.c // self.groups) * self.r * self.s

    def with_batch(self, n: int) -> "ConvShape":
        return replace(self, n=n)

    def key(self) -> Tuple[int, ...]:
        return (self.c, self.k, self.r, self.s, self.stride, self.pad, self.h, self.w) + ((self.groups,) if self.groups > 1 else ())


def resnet50_convs(batch: int) -> List[ConvShape]:
    """The 53 convolutions of the original ResNet-50 in network order.

    Original form: in the first block of stages 3, 4 and 5 the stride 2 sits on
    the first 1x1 convolution and on the projection shortcut.  This is the
    variant whose per-image work reproduces the 7.72 G operations the paper
    states in "Benefits of Large-Batch Training".
    """
    out = [ConvShape("conv1", batch, 3, 224, 224, 64, 7, 7, 2, 3)]
    spatial, cin = 56, 64
    for stage, (mid, blocks) in enumerate([(64, 3), (128, 4), (256, 6), (512, 3)], start=2):
        cout = 4 * mid
        for b in range(blocks):
            stride = 2 if (b == 0 and stage > 2) else 1
            pre = f"res{stage}{chr(ord('a') + b)}"
            if b == 0:
                out.append(ConvShape(pre + "_proj", batch, cin, spatial, spatial, cout, 1, 1, stride, 0))
            out.append(ConvShape(pre + "_1x1a", batch, cin, spatial, spatial, mid, 1, 1, stride, 0))
            spatial //= stride
            out.append(ConvShape(pre + "_3x3", batch, mid, spatial, spatial, mid, 3, 3, 1, 1))
            out.append(ConvShape(pre + "_1x1b", batch, mid, spatial, spatial, cout, 1, 1, 1, 0))
            cin = cout
    return out


def resnet50_fc(batch: int) -> ConvShape:
    """The classifier as a 1x1 convolution on a 1x1 map (2048 -> 1000)."""
    return ConvShape("fc1000", batch, 2048, 1, 1, 1000, 1, 1, 1, 0)


def resnet50_distinct_shapes(batch: int) -> List[Tuple[ConvShape, int]]:
    """Distinct convolution shapes of ResNet-50 with the number of times each occurs."""
    seen, order = {}, []
    for cs in resnet50_convs(batch):
        if cs.key() not in seen:
            seen[cs.key()] = [cs, 0]
            order.append(cs.key())
        seen[cs.key()][1] += 1
    return [(seen[k][0], seen[k][1]) for k in order]


def resnet50_param_numels() -> List[int]:
    """Sizes of ResNet-50's 161 parameter tensors: per conv its filter then the batch-norm
    scale and shift of its output channels; last the classifier weight and bias."""
    sizes: List[int] = []
    for cs in resnet50_convs(1):
        sizes += [cs.weight_numel, cs.k, cs.k]
    sizes += [2048 * 1000, 1000]
    return sizes


def alexnet_bn_convs(batch: int) -> List[ConvShape]:
    """AlexNet with batch norm (ungrouped filters): five convolutions, then the three
    fully connected layers expressed as convolutions (6x6 window on the 6x6 map, then 1x1)."""
    return [
        ConvShape("conv1", batch, 3, 227, 227, 96, 11, 11, 4, 0),
        ConvShape("conv2", batch, 96, 27, 27, 256, 5, 5, 1, 2),
        ConvShape("conv3", batch, 256, 13, 13, 384, 3, 3, 1, 1),
        ConvShape("conv4", batch, 384, 13, 13, 384, 3, 3, 1, 1),
        ConvShape("conv5", batch, 384, 13, 13, 256, 3, 3, 1, 1),
        ConvShape("fc6", batch, 256, 6, 6, 4096, 6, 6, 1, 0),
        ConvShape("fc7", batch, 4096, 1, 1, 4096, 1, 1, 1, 0),
        ConvShape("fc8", batch, 4096, 1, 1, 1000, 1, 1, 1, 0),
    ]


def alexnet_bn_param_numels() -> List[int]:
    """21 tensors: 8 weights, batch-norm scale and shift for the 5 convolutions, 3 FC biases."""
    sizes: List[int] = []
    for i, cs in enumerate(alexnet_bn_convs(1)):
        sizes.append(cs.weight_numel)
        sizes += [cs.k, cs.k] if i < 5 else [cs.k]
    return sizes


def alexnet_grouped_convs(batch: int) -> List[ConvShape]:
    """The original AlexNet of the paper's scaling-ratio table (61 million parameters, 1.5 billion operations per
    image): the second, fourth and fifth convolutions split into two groups; fully connected layers as above."""
    out = alexnet_bn_convs(batch)
    for i in (1, 3, 4):
        out[i] = replace(out[i], groups=2)
    return out


def alexnet_grouped_param_numels() -> List[int]:
    """The original AlexNet's 16 tensors: a weight and a bias per layer."""
    sizes: List[int] = []
    for cs in alexnet_grouped_convs(1):
        sizes += [cs.weight_numel, cs.k]
    return sizes


def resnet50_v15_extra_shapes(batch: int) -> List[ConvShape]:
    """The shapes the "v1.5" form of ResNet-50 has and the original does not: the stride 2 of stages 3, 4, 5 sits on the
    3x3 convolution instead of the first 1x1, which then runs at stride 1 on the larger map.  Not the network the paper
    trains (its 7.72 G operations per image are the original's); listed as a second workload."""
    out = []
    for stage, (cin, mid, hw) in enumerate([(256, 128, 56), (512, 256, 28), (1024, 512, 14)], start=3):
        out.append(ConvShape(f"v15_res{stage}a_1x1a", batch, cin, hw, hw, mid, 1, 1, 1, 0))
        out.append(ConvShape(f"v15_res{stage}a_3x3s2", batch, mid, hw, hw, mid, 3, 3, 2, 1))
    return out


def tiny_cnn_convs(batch: int = 16) -> List[ConvShape]:
    """The two convolutions of the tiny whole-path parity network (3x32x32 input)."""
    return [
        ConvShape("tiny_conv1", batch, 3, 32, 32, 16, 3, 3, 1, 1),
        ConvShape("tiny_conv2", batch, 16, 16, 16, 32, 3, 3, 1, 1),
    ]


def he_std(cs: ConvShape) -> float:
    """He-normal standard deviation sqrt(2 / fan_in), fan_in = C*R*S."""
    return float(np.sqrt(2.0 / (cs.c * cs.r * cs.s)))


def poly_total_iters(epochs: int = 90, images: int = 1_280_000, batch: int = 32768) -> int:
    """Iterations of a run: epochs * images / batch ("Scaling Efficiency of Large Batches"), rounded up."""
    return -(-epochs * images // batch)
