"""CPU oracle (test infrastructure only): a residual network of bottleneck blocks, forward and backward.

The paper trains ResNet-50 ("ImageNet training with ResNet-50") and gives no layer-level description; the
structure here is the one of the network it names (the original variant, whose operation and parameter counts
match the numbers the paper prints): a stem convolution with batch normalisation and ReLU, a max pool with
overlapping windows, stages of bottleneck blocks (1x1 -> 3x3 -> 1x1, each followed by batch normalisation, ReLU
after the first two; the block's input -- through a strided 1x1 projection with batch normalisation where the
shape changes -- is added before the last ReLU; the stride of a stage's first block sits on its first 1x1),
global average pool, a fully connected classifier with bias, softmax cross-entropy averaged over the batch.
Every piece is the textbook definition in numpy float64; the convolutions go through ``oracle.c``; values are
stored as float32 between layers, as a GPU worker stores them.  Layout NCHW.

Mixed precision (``forward_backward_bf16``): the paper's fastest runs train in reduced precision with float32
master weights ("State-of-the-art results") and say no more about it; the reading taken here is the usual one.
Activations and their gradients are stored as bf16 (rounded to nearest even wherever the float32 trace rounds to
float32), the convolutions see the filters rounded to bf16, and everything a parameter owns (scale, shift,
statistics, every gradient of a parameter) as well as the pooled features, the classifier and the loss stay
float32.

``pair=True`` (both precisions): a value is rounded where it is stored, and a worker that computes the output of a
block with a projection as relu(bn(c3) + bn(projection)) in one pass never stores the projection's batch-norm
output; with ``pair`` that value enters the sum as computed.  Nothing else changes (the gradient that arrives at it is
the block output's stored gradient either way).

``Config`` fixes the sizes: ResNet-50 is Config(stem=(64, 7, 2, 3), widths=(64, 128, 256, 512),
blocks=(3, 4, 6, 3), classes=1000); tests use a few-channel version of the same graph.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

from . import NCHW, batchnorm, conv2d_bwd_data, conv2d_bwd_weight, conv2d_fwd, round_to_bf16
from .tiny_cnn import fc, global_avgpool, global_avgpool_bwd, softmax_xent


@dataclass(frozen=True)
class Config:
    stem: Tuple[int, int, int, int]          # filters, window, stride, pad
    widths: Tuple[int, ...]                  # bottleneck width per stage (block output = 4 * width)
    blocks: Tuple[int, ...]                  # blocks per stage
    classes: int
    in_channels: int = 3
    eps: float = 1e-5


# ---------------------------------------------------------------- max pool with any window / stride / pad
def maxpool(x, window: int, stride: int, pad: int):
    """Max over window x window taps, padding taps never win.  Returns (y, idx) where idx is the tap
    (row * window + column) of the first maximum in row-major order of the window."""
    x = np.asarray(x, dtype=np.float64)
    n, c, h, w = x.shape
    ph = (h + 2 * pad - window) // stride + 1
    pw = (w + 2 * pad - window) // stride + 1
    y = np.full((n, c, ph, pw), -np.inf)
    idx = np.zeros((n, c, ph, pw), dtype=np.int64)
    for p in range(ph):
        for q in range(pw):
            for r in range(window):
                for s in range(window):
                    ih, iw = p * stride - pad + r, q * stride - pad + s
                    if 0 <= ih < h and 0 <= iw < w:
                        v = x[:, :, ih, iw]
                        better = v > y[:, :, p, q]
                        y[:, :, p, q] = np.where(better, v, y[:, :, p, q])
                        idx[:, :, p, q] = np.where(better, r * window + s, idx[:, :, p, q])
    return y, idx


def maxpool_bwd(idx, dy, x_hw: Tuple[int, int], window: int, stride: int, pad: int):
    """Every output's gradient goes to the input its maximum came from; overlapping windows add."""
    dy = np.asarray(dy, dtype=np.float64)
    n, c, ph, pw = dy.shape
    h, w = x_hw
    dx = np.zeros((n, c, h, w))
    ni, ci = np.meshgrid(np.arange(n), np.arange(c), indexing="ij")
    for p in range(ph):
        for q in range(pw):
            ih = p * stride - pad + idx[:, :, p, q] // window
            iw = q * stride - pad + idx[:, :, p, q] % window
            np.add.at(dx, (ni, ci, ih, iw), dy[:, :, p, q])
    return dx


# ---------------------------------------------------------------- parameters
def conv_list(cfg: Config) -> List[Tuple[str, int, int, int, int, int]]:
    """(name, in channels, filters, window, stride, pad) of every convolution in network order."""
    out = [("stem", cfg.in_channels, cfg.stem[0], cfg.stem[1], cfg.stem[2], cfg.stem[3])]
    ch = cfg.stem[0]
    for si, (wd, nb) in enumerate(zip(cfg.widths, cfg.blocks)):
        for bi in range(nb):
            stride = 2 if (bi == 0 and si > 0) else 1
            name = f"s{si}b{bi}"
            out.append((name + ".c1", ch, wd, 1, stride, 0))
            out.append((name + ".c2", wd, wd, 3, 1, 1))
            out.append((name + ".c3", wd, 4 * wd, 1, 1, 0))
            if ch != 4 * wd or stride != 1:
                out.append((name + ".proj", ch, 4 * wd, 1, stride, 0))
            ch = 4 * wd
    return out


def param_shapes(cfg: Config) -> Dict[str, Tuple[int, ...]]:
    """Name -> shape of every trainable tensor, in network order (filter, scale, shift per convolution;
    classifier weight and bias)."""
    shapes: Dict[str, Tuple[int, ...]] = {}
    for name, cin, k, r, _, _ in conv_list(cfg):
        shapes[name + ".w"] = (k, cin, r, r)
        shapes[name + ".gamma"] = (k,)
        shapes[name + ".beta"] = (k,)
    shapes["fc.w"] = (cfg.classes, 4 * cfg.widths[-1])
    shapes["fc.b"] = (cfg.classes,)
    return shapes


# ---------------------------------------------------------------- forward / backward
def _s(a):
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


class _Net:
    """Runs the graph once, keeping what the backward pass needs.  ``store`` rounds to float32 between
    layers (the trace a device is compared with) or keeps float64 (finite differences); ``bf16`` stores
    activations and their gradients as bf16 instead and hands the convolutions bf16 filters."""

    def __init__(self, cfg: Config, params, store: bool, bf16: bool = False, pair: bool = False):
        self.cfg, self.p, self.store, self.bf16, self.pair = cfg, params, store, bf16, pair
        self.t: Dict[str, np.ndarray] = {}
        self.g: Dict[str, np.ndarray] = {}

    def keep(self, a):
        return _s(a) if self.store else np.asarray(a, dtype=np.float64)

    def act(self, a):
        """An activation or the gradient of one, as it is stored between layers."""
        return round_to_bf16(np.asarray(a, dtype=np.float64)).astype(np.float64) if self.bf16 else self.keep(a)

    def filt(self, name):
        w = _f32(self.p[name + ".w"])
        return round_to_bf16(w) if self.bf16 else w

    def conv(self, x, name, stride, pad):
        if self.store:
            return self.act(conv2d_fwd(_f32(x), self.filt(name), stride, pad, NCHW))
        return _conv_f64(x, np.asarray(self.p[name + ".w"], dtype=np.float64), stride, pad)

    def conv_bn(self, x, name, stride, pad, relu, residual=None, stored=True):
        z = self.conv(x, name, stride, pad)
        y, _, _ = batchnorm.forward(z, self.p[name + ".gamma"], self.p[name + ".beta"], self.cfg.eps)
        if residual is not None:
            y = y + residual
        a = np.maximum(y, 0.0) if relu else y
        a = self.act(a) if stored else np.asarray(a, dtype=np.float64)     # not stored: handed on as computed, unrounded
        self.t[name + ".x"], self.t[name + ".z"], self.t[name + ".a"] = x, z, a
        self.t[name + ".y"] = y                # before the ReLU, unrounded: tests look at its distance from zero
        return a

    def conv_bn_bwd(self, name, da, stride, pad, need_dx=True):
        """``da``: gradient wrt the batch-norm output (after the ReLU mask where there is one)."""
        x, z = self.t[name + ".x"], self.t[name + ".z"]
        w = self.p[name + ".w"]
        dz, dgamma, dbeta = batchnorm.backward(z, da, self.p[name + ".gamma"], self.cfg.eps)
        dz = self.act(dz)
        self.g[name + ".gamma"], self.g[name + ".beta"] = self.keep(dgamma), self.keep(dbeta)
        r = w.shape[2]
        self.g[name + ".w"] = self.keep(conv2d_bwd_weight(_f32(x), _f32(dz), (r, r), stride, pad, NCHW))
        self.t[name + ".dz"] = dz
        if not need_dx:
            return None
        dx = self.act(conv2d_bwd_data(_f32(dz), self.filt(name), x.shape[2:], stride, pad, NCHW))
        self.t[name + ".dx"] = dx
        return dx

    def forward(self, x, labels):
        cfg = self.cfg
        a = self.conv_bn(self.act(x), "stem", cfg.stem[2], cfg.stem[3], relu=True)
        self.t["pool.in_hw"] = a.shape[2:]
        pooled, self.t["pool.idx"] = maxpool(a, 3, 2, 1)
        a = self.act(pooled)
        ch = cfg.stem[0]
        self.blocks: List[Tuple[str, int, bool]] = []
        for si, (wd, nb) in enumerate(zip(cfg.widths, cfg.blocks)):
            for bi in range(nb):
                stride = 2 if (bi == 0 and si > 0) else 1
                name = f"s{si}b{bi}"
                proj = ch != 4 * wd or stride != 1
                # (pair: the projection's batch-norm output goes straight into the block's sum and is never stored)
                sc = self.conv_bn(a, name + ".proj", stride, 0, relu=False, stored=not self.pair) if proj else a
                b = self.conv_bn(a, name + ".c1", stride, 0, relu=True)
                b = self.conv_bn(b, name + ".c2", 1, 1, relu=True)
                a = self.conv_bn(b, name + ".c3", 1, 0, relu=True, residual=sc)
                self.blocks.append((name, stride, proj))
                ch = 4 * wd
        self.t["gap.in"] = a
        pooled = self.keep(global_avgpool(a))
        self.t["fc.in"] = pooled
        logits = self.keep(fc(pooled, np.asarray(self.p["fc.w"], dtype=np.float64), np.asarray(self.p["fc.b"], dtype=np.float64)))
        self.t["logits"] = logits
        loss, dlogits = softmax_xent(logits, labels)
        self.t["loss"] = np.float64(loss)
        return loss, dlogits

    def backward(self, dlogits):
        d = self.keep(dlogits)
        self.g["fc.w"] = self.keep(d.T @ self.t["fc.in"])
        self.g["fc.b"] = self.keep(d.sum(axis=0))
        dpool = self.keep(d @ np.asarray(self.p["fc.w"], dtype=np.float64))
        last = self.t["gap.in"]
        da = self.act(global_avgpool_bwd(dpool, last.shape[2], last.shape[3]))         # gradient wrt the last block's output
        for name, stride, proj in reversed(self.blocks):
            out = self.t[name + ".c3.a"]
            d_pre = self.act(np.where(out > 0.0, da, 0.0))                            # through the block's last ReLU
            db = self.conv_bn_bwd(name + ".c3", d_pre, 1, 0)
            db = self.act(np.where(self.t[name + ".c2.a"] > 0.0, db, 0.0))
            db = self.conv_bn_bwd(name + ".c2", db, 1, 1)
            db = self.act(np.where(self.t[name + ".c1.a"] > 0.0, db, 0.0))
            d_in = self.conv_bn_bwd(name + ".c1", db, stride, 0)
            d_sc = self.conv_bn_bwd(name + ".proj", d_pre, stride, 0) if proj else d_pre
            da = self.act(d_in + d_sc)
        da = self.act(maxpool_bwd(self.t["pool.idx"], da, self.t["pool.in_hw"], 3, 2, 1))
        da = self.act(np.where(self.t["stem.a"] > 0.0, da, 0.0))
        self.conv_bn_bwd("stem", da, self.cfg.stem[2], self.cfg.stem[3], need_dx=False)


def _conv_f64(x, w, stride, pad):
    """Direct sum in float64 (the C routine takes float32 operands); only for finite differences."""
    n, c, h, wd = x.shape
    k, _, r, s = w.shape
    p = (h + 2 * pad - r) // stride + 1
    q = (wd + 2 * pad - s) // stride + 1
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    y = np.zeros((n, k, p, q))
    for i in range(r):
        for j in range(s):
            y += np.einsum("nchw,kc->nkhw", xp[:, :, i:i + (p - 1) * stride + 1:stride, j:j + (q - 1) * stride + 1:stride], w[:, :, i, j])
    return y


def forward_backward(x, labels, params, cfg: Config, pair: bool = False):
    """One forward and backward pass with float32 stores.  Returns (trace, grads): the trace holds
    "<conv>.z" (convolution output), "<conv>.y" (after batch norm and residual, before the ReLU, float64),
    "<conv>.a" (the stored activation), "<conv>.dz" / "<conv>.dx" (the stored gradients with respect to the
    convolution's output and input), "logits", "loss";
    grads has one entry per parameter name."""
    net = _Net(cfg, params, store=True, pair=pair)
    _, dlogits = net.forward(np.asarray(x, dtype=np.float32), labels)
    net.backward(dlogits)
    return net.t, net.g


def forward_backward_bf16(x, labels, params, cfg: Config, pair: bool = False):
    """The same pass with bf16 activations, activation gradients and convolution filters (see the module
    header); parameters and their gradients float32.  ``x`` is rounded to bf16 first.  Returns (trace, grads)."""
    net = _Net(cfg, params, store=True, bf16=True, pair=pair)
    _, dlogits = net.forward(np.asarray(x, dtype=np.float32), labels)
    net.backward(dlogits)
    return net.t, net.g


def loss_only(x, labels, params, cfg: Config) -> float:
    """Forward pass in float64 without the float32 stores (for finite differences)."""
    net = _Net(cfg, params, store=False)
    loss, _ = net.forward(np.asarray(x, dtype=np.float64), labels)
    return float(loss)
