"""CPU oracle (test infrastructure only): AlexNet with batch normalisation, forward and backward.

The paper trains "AlexNet-BN" ("Scaling up Batch Size": batch normalisation added after each convolution, which
is what lets LARS reach batch 32K) and gives no layer-level description; the structure is the network it names with
ungrouped filters: five convolutions, each followed by batch normalisation (batch statistics) and ReLU, 3x3
stride-2 max pools after the first, second and fifth, then three fully connected layers with bias, ReLU after the
first two, and softmax cross-entropy averaged over the batch.  Dropout and local response normalisation are not
part of this oracle (the batch-norm variant drops the latter; the former is a random mask the paper does not
discuss).  Every piece is the textbook definition in numpy float64; the convolutions go through ``oracle.c``;
values are stored as float32 between layers.  Layout NCHW.

``Config``: AlexNet-BN is Config(convs=((96, 11, 4, 0, True), (256, 5, 1, 2, True), (384, 3, 1, 1, False),
(384, 3, 1, 1, False), (256, 3, 1, 1, True)), fcs=(4096, 4096), classes=1000) on 227x227 images.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np

from . import NCHW, batchnorm, conv2d_bwd_data, conv2d_bwd_weight, conv2d_fwd
from .resnet import _conv_f64, maxpool, maxpool_bwd
from .tiny_cnn import softmax_xent


@dataclass(frozen=True)
class Config:
    convs: Tuple[Tuple[int, int, int, int, bool], ...]     # filters, window, stride, pad, 3x3 stride-2 pool after
    fcs: Tuple[int, ...]                                   # widths of the hidden fully connected layers
    classes: int
    in_channels: int = 3
    eps: float = 1e-5


def feature_shape(cfg: Config, hw: Tuple[int, int]) -> Tuple[int, int, int]:
    """(channels, height, width) of what the first fully connected layer sees."""
    h, w = hw
    c = cfg.in_channels
    for k, r, stride, pad, pool in cfg.convs:
        h, w = (h + 2 * pad - r) // stride + 1, (w + 2 * pad - r) // stride + 1
        if pool:
            h, w = (h - 3) // 2 + 1, (w - 3) // 2 + 1
        c = k
    return c, h, w


def param_shapes(cfg: Config, hw: Tuple[int, int]) -> Dict[str, Tuple[int, ...]]:
    """Name -> shape in network order: filter, scale, shift per convolution; weight [out, c, h, w] (the first) or
    [out, in], and bias per fully connected layer."""
    shapes: Dict[str, Tuple[int, ...]] = {}
    c = cfg.in_channels
    for i, (k, r, _, _, _) in enumerate(cfg.convs):
        shapes[f"conv{i + 1}.w"] = (k, c, r, r)
        shapes[f"conv{i + 1}.gamma"] = (k,)
        shapes[f"conv{i + 1}.beta"] = (k,)
        c = k
    fc, fh, fw = feature_shape(cfg, hw)
    widths = list(cfg.fcs) + [cfg.classes]
    n_conv = len(cfg.convs)
    for j, out in enumerate(widths):
        name = f"fc{n_conv + 1 + j}"
        shapes[name + ".w"] = (out, fc, fh, fw) if j == 0 else (out, widths[j - 1])
        shapes[name + ".b"] = (out,)
    return shapes


def _s(a):
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _run(x, labels, params, cfg: Config, store: bool):
    """Forward (and, with ``store``, backward).  ``store`` rounds to float32 between layers; without it the
    pass stays in float64 and only the loss is returned (finite differences)."""
    keep = _s if store else (lambda a: np.asarray(a, dtype=np.float64))
    t: Dict[str, np.ndarray] = {}
    a = keep(x)
    for i, (k, r, stride, pad, pool) in enumerate(cfg.convs):
        name = f"conv{i + 1}"
        w = params[name + ".w"]
        t[name + ".x"] = a
        z = keep(conv2d_fwd(_f32(a), _f32(w), stride, pad, NCHW)) if store else _conv_f64(a, np.asarray(w, dtype=np.float64), stride, pad)
        y, _, _ = batchnorm.forward(z, params[name + ".gamma"], params[name + ".beta"], cfg.eps)
        a = keep(np.maximum(y, 0.0))
        t[name + ".z"], t[name + ".y"], t[name + ".a"] = z, y, a
        if pool:
            t[name + ".pool_in_hw"] = a.shape[2:]
            pooled, t[name + ".pool_idx"] = maxpool(a, 3, 2, 0)
            a = keep(pooled)
            t[name + ".pooled"] = a
    n = a.shape[0]
    t["features"] = a
    a = a.reshape(n, -1)
    n_conv = len(cfg.convs)
    n_fc = len(cfg.fcs) + 1
    for j in range(n_fc):
        name = f"fc{n_conv + 1 + j}"
        w = np.asarray(params[name + ".w"], dtype=np.float64).reshape(params[name + ".w"].shape[0], -1)
        b = np.asarray(params[name + ".b"], dtype=np.float64)
        t[name + ".x"] = a
        z = keep(a @ w.T + b)
        t[name + ".z"] = z
        a = keep(np.maximum(z, 0.0)) if j < n_fc - 1 else z
        t[name + ".a"] = a
    t["logits"] = a
    loss, dlogits = softmax_xent(a, labels)
    t["loss"] = np.float64(loss)
    if not store:
        return t, None

    g: Dict[str, np.ndarray] = {}
    d = keep(dlogits)
    for j in reversed(range(n_fc)):
        name = f"fc{n_conv + 1 + j}"
        if j < n_fc - 1:
            d = keep(np.where(t[name + ".z"] > 0.0, d, 0.0))
        w = np.asarray(params[name + ".w"], dtype=np.float64)
        g[name + ".w"] = keep(d.T @ t[name + ".x"]).reshape(w.shape)
        g[name + ".b"] = keep(d.sum(axis=0))
        d = keep(d @ w.reshape(w.shape[0], -1))
    d = d.reshape(t["features"].shape)
    for i in reversed(range(len(cfg.convs))):
        k, r, stride, pad, pool = cfg.convs[i]
        name = f"conv{i + 1}"
        if pool:
            d = keep(maxpool_bwd(t[name + ".pool_idx"], d, t[name + ".pool_in_hw"], 3, 2, 0))
        d = keep(np.where(t[name + ".a"] > 0.0, d, 0.0))
        dz, dgamma, dbeta = batchnorm.backward(t[name + ".z"], d, params[name + ".gamma"], cfg.eps)
        dz = keep(dz)
        g[name + ".gamma"], g[name + ".beta"] = keep(dgamma), keep(dbeta)
        xin = t[name + ".x"]
        g[name + ".w"] = keep(conv2d_bwd_weight(_f32(xin), _f32(dz), (r, r), stride, pad, NCHW))
        if i > 0:
            d = keep(conv2d_bwd_data(_f32(dz), _f32(params[name + ".w"]), xin.shape[2:], stride, pad, NCHW))
    return t, g


def forward_backward(x, labels, params, cfg: Config):
    """One forward and backward pass with float32 stores.  Returns (trace, grads): the trace holds "<layer>.z",
    "<layer>.y" (batch-norm output before the ReLU, float64), "<layer>.a", "logits", "loss"."""
    return _run(np.asarray(x, dtype=np.float32), labels, params, cfg, store=True)


def loss_only(x, labels, params, cfg: Config) -> float:
    """Forward pass in float64 without the float32 stores (for finite differences)."""
    t, _ = _run(np.asarray(x, dtype=np.float64), labels, params, cfg, store=False)
    return float(t["loss"])
