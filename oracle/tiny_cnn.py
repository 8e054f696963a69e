"""CPU oracle (test infrastructure only): the tiny CNN whole-path case.

conv 3->16 k3 s1 p1, ReLU, maxpool 2x2, conv 16->32 k3 s1 p1, ReLU, global
average pool, FC 32->10 (weight and bias), softmax cross-entropy averaged over
the batch; then one LARS step over the four parameter tensors.  The paper does
not discuss these glue layers (they are implied by the networks it trains);
they are the textbook definitions, written with numpy in float64.  The
convolutions and the update go through ``oracle.c``.  Activations and
gradients are stored as float32 between layers, as a GPU worker stores them.

Layout is NCHW throughout.
"""
from __future__ import annotations

from typing import Dict

import numpy as np

from . import NCHW, conv2d_bwd_data, conv2d_bwd_weight, conv2d_fwd, lars_step


def relu(x):
    return np.maximum(x, 0.0)


def relu_bwd(x, dy):
    return np.where(x > 0.0, dy, 0.0)


def maxpool2(x):
    """2x2 window, stride 2; also returns the index (0..3, row-major in the window) of the first maximum."""
    n, c, h, w = x.shape
    win = x.reshape(n, c, h // 2, 2, w // 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(n, c, h // 2, w // 2, 4)
    idx = np.argmax(win, axis=-1)  # first maximal element
    return np.take_along_axis(win, idx[..., None], axis=-1)[..., 0], idx


def maxpool2_bwd(idx, dy, h, w):
    n, c, ph, pw = dy.shape
    win = np.zeros((n, c, ph, pw, 4), dtype=np.float64)
    np.put_along_axis(win, idx[..., None], dy[..., None], axis=-1)
    return win.reshape(n, c, ph, pw, 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(n, c, h, w)


def global_avgpool(x):
    return x.mean(axis=(2, 3))


def global_avgpool_bwd(dy, h, w):
    return np.broadcast_to(dy[:, :, None, None] / (h * w), dy.shape + (h, w)).copy()


def fc(x, wt, b):
    return x @ wt.T + b


def softmax_xent(logits, labels):
    """Mean cross-entropy and its gradient wrt the logits, (softmax - onehot) / N."""
    z = logits - logits.max(axis=1, keepdims=True)
    e = np.exp(z)
    sm = e / e.sum(axis=1, keepdims=True)
    n = logits.shape[0]
    loss = -np.mean(np.log(sm[np.arange(n), labels]))
    d = sm.copy()
    d[np.arange(n), labels] -= 1.0
    return loss, d / n


def _s(a):
    """Store as float32 (what sits in memory between layers), hand back as float64."""
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def forward_backward(x, labels, params: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    """One forward and backward pass.  ``params``: w1 [16,3,3,3], w2 [32,16,3,3], wf [10,32], bf [10].
    Returns every activation ("a_*"), every gradient ("d_*") and the loss."""
    w1, w2, wf, bf = (np.asarray(params[k], dtype=np.float32) for k in ("w1", "w2", "wf", "bf"))
    t: Dict[str, np.ndarray] = {}
    x = np.asarray(x, dtype=np.float32)
    t["a_c1"] = _s(conv2d_fwd(x, w1, 1, 1, NCHW))
    t["a_r1"] = _s(relu(t["a_c1"]))
    pooled, idx = maxpool2(t["a_r1"])
    t["a_p1"] = _s(pooled)
    t["a_c2"] = _s(conv2d_fwd(t["a_p1"], w2, 1, 1, NCHW))
    t["a_r2"] = _s(relu(t["a_c2"]))
    t["a_gap"] = _s(global_avgpool(t["a_r2"]))
    t["a_fc"] = _s(fc(t["a_gap"], wf.astype(np.float64), bf.astype(np.float64)))
    loss, dlogits = softmax_xent(t["a_fc"], labels)
    t["loss"] = np.float64(loss)
    t["d_fc"] = _s(dlogits)
    t["d_wf"] = _s(t["d_fc"].T @ t["a_gap"])
    t["d_bf"] = _s(t["d_fc"].sum(axis=0))
    t["d_gap"] = _s(t["d_fc"] @ wf.astype(np.float64))
    t["d_r2"] = _s(global_avgpool_bwd(t["d_gap"], 16, 16))
    t["d_c2"] = _s(relu_bwd(t["a_c2"], t["d_r2"]))
    t["d_w2"] = _s(conv2d_bwd_weight(t["a_p1"], t["d_c2"], (3, 3), 1, 1, NCHW))
    t["d_p1"] = _s(conv2d_bwd_data(t["d_c2"], w2, (16, 16), 1, 1, NCHW))
    t["d_r1"] = _s(maxpool2_bwd(idx, t["d_p1"], 32, 32))
    t["d_c1"] = _s(relu_bwd(t["a_c1"], t["d_r1"]))
    t["d_w1"] = _s(conv2d_bwd_weight(x, t["d_c1"], (3, 3), 1, 1, NCHW))
    return t


def loss_only(x, labels, params) -> float:
    """Forward pass in float64 without the float32 stores (for finite differences)."""
    f64 = {k: np.asarray(v, dtype=np.float64) for k, v in params.items()}
    # the C convolution takes float32 operands, so this path uses a numpy float64 direct sum
    def conv(xx, ww):
        n, c, h, w = xx.shape
        k = ww.shape[0]
        xp = np.pad(xx, ((0, 0), (0, 0), (1, 1), (1, 1)))
        y = np.zeros((n, k, h, w))
        for r in range(3):
            for s in range(3):
                y += np.einsum("nchw,kc->nkhw", xp[:, :, r:r + h, s:s + w], ww[:, :, r, s])
        return y
    a = relu(conv(np.asarray(x, dtype=np.float64), f64["w1"]))
    a, _ = maxpool2(a)
    a = relu(conv(a, f64["w2"]))
    logits = fc(global_avgpool(a), f64["wf"], f64["bf"])
    return float(softmax_xent(logits, labels)[0])


def train_step(x, labels, params, velocity, eta, momentum, weight_decay, lr):
    """Forward, backward and one LARS step.  Updates ``params`` and ``velocity`` (dicts of float32
    arrays) in place; returns the trace of ``forward_backward`` plus "trust" (float64 [4])."""
    t = forward_backward(x, labels, params)
    names = ["w1", "w2", "wf", "bf"]
    grads = [np.ascontiguousarray(t["d_" + k], dtype=np.float32) for k in names]
    trust, norms = lars_step([params[k] for k in names], grads, [velocity[k] for k in names],
                             eta, momentum, weight_decay, lr)
    t["trust"], t["norms"] = trust, norms
    return t
