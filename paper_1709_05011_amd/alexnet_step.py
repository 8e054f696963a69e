"""One whole training step of AlexNet with batch normalisation on the device: forward, backward and the LARS
update, every layer a call into the C library (this module only owns buffers and the order of calls; torch is used
for device memory).  The network is the paper's "AlexNet-BN" ("Scaling up Batch Size") with ungrouped filters:
convolutions each followed by batch norm and ReLU, 3x3 stride-2 max pools where configured, fully connected layers
with bias (the first as a whole-window convolution over the last feature map, the others as 1x1 convolutions over
one pixel), ReLU after all but the last, softmax cross-entropy, then LARS over all parameter tensors.  No dropout.
Layout NHWC, fp32.

AlexNet-BN: AlexNetStep(convs=((96, 11, 4, 0, True), (256, 5, 1, 2, True), (384, 3, 1, 1, False),
(384, 3, 1, 1, False), (256, 3, 1, 1, True)), fcs=(4096, 4096), classes=1000, batch=..., image_hw=(227, 227)).
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import torch

from . import larsconv as lc

NHWC = lc.LC_NHWC


class AlexNetStep:
    def __init__(self, convs: Sequence[Tuple[int, int, int, int, bool]], fcs: Sequence[int], classes: int, batch: int,
                 image_hw: Tuple[int, int], in_channels: int = 3, eps: float = 1e-5, device: str = "cuda:0"):
        lc.lib()                     # fails here, loudly, when the library has not been built
        self.dev, self.eps, self.batch, self.classes = device, eps, batch, classes
        f32 = dict(dtype=torch.float32, device=device)
        self.conv_layers: List[dict] = []
        self.fc_layers: List[dict] = []
        self.params: Dict[str, torch.Tensor] = {}
        h, w = image_hw
        c = in_channels
        need = 0
        for i, (k, r, stride, pad, pool) in enumerate(convs):
            name = f"conv{i + 1}"
            d = lc.ConvDesc(batch, c, h, w, k, r, r, stride, stride, pad, pad, lc.LC_F32, NHWC)
            p, q = lc.conv2d_out_shape(d)
            L = dict(name=name, desc=d, out_hw=(p, q), pool=pool,
                     z=torch.empty((batch, p, q, k), **f32), a=torch.empty((batch, p, q, k), **f32),
                     mean=torch.empty(k, **f32), invstd=torch.empty(k, **f32))
            self.params[name + ".w"] = torch.zeros((k, r, r, c), **f32)
            self.params[name + ".gamma"] = torch.ones(k, **f32)
            self.params[name + ".beta"] = torch.zeros(k, **f32)
            need = max(need, lc.batchnorm_workspace_bytes(batch, k, p, q, NHWC))
            L["stats_tiles"] = lc.conv2d_fwd_stats_count(d)
            h, w, c = p, q, k
            if pool:
                h, w = (h - 3) // 2 + 1, (w - 3) // 2 + 1
                L["pooled"] = torch.empty((batch, h, w, k), **f32)
                L["pool_idx"] = torch.empty((batch, h, w, k), dtype=torch.uint8, device=device)
            self.conv_layers.append(L)
        self._stats = torch.empty(max([L["stats_tiles"] * L["desc"].k * 2 for L in self.conv_layers] + [2]), **f32)
        widths = list(fcs) + [classes]
        n_conv = len(convs)
        for j, out in enumerate(widths):
            name = f"fc{n_conv + 1 + j}"
            # the first fully connected layer is a whole-window convolution over the last feature map
            d = lc.ConvDesc(batch, c, h, w, out, h, w, 1, 1, 0, 0, lc.LC_F32, NHWC)
            L = dict(name=name, desc=d, relu=j < len(widths) - 1, z=torch.empty((batch, out), **f32))
            if L["relu"]:
                L["a"] = torch.empty((batch, out), **f32)
            self.params[name + ".w"] = torch.zeros((out, h, w, c), **f32)
            self.params[name + ".b"] = torch.zeros(out, **f32)
            self.fc_layers.append(L)
            c, h, w = out, 1, 1
        for L in self.conv_layers + self.fc_layers:
            for p_ in (lc.LC_PASS_FWD, lc.LC_PASS_BWD_DATA, lc.LC_PASS_BWD_WEIGHT):
                need = max(need, lc.conv2d_workspace_bytes(L["desc"], p_))
        self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
        self.grads = {k: torch.zeros_like(v) for k, v in self.params.items()}
        self.velocity = {k: torch.zeros_like(v) for k, v in self.params.items()}
        names = list(self.params)
        self._lars = lc.LarsArgs([self.params[k] for k in names], [self.grads[k] for k in names], [self.velocity[k] for k in names])
        self._lars_ws = torch.empty(max(lc.lars_workspace_bytes(self._lars.numel), 256), dtype=torch.uint8, device=device)
        self.trust = torch.zeros(len(names), **f32)
        # the squared norm of every filter gradient comes out of its backward-weight pass and is handed to the update
        self.gsq = {L["name"] + ".w": torch.zeros(lc.conv2d_bwd_weight_sq_count(L["desc"]), dtype=torch.float64, device=device)
                    for L in self.conv_layers + self.fc_layers}
        self._gsq_list = [self.gsq.get(k) for k in names]
        self._gsq_counts = [0 if t is None else t.numel() for t in self._gsq_list]
        self.logits = self.fc_layers[-1]["z"]
        self.dlogits = torch.empty((batch, classes), **f32)
        self.loss = torch.zeros(1, **f32)
        self._rows = torch.empty(batch, **f32)

    def forward(self, x: torch.Tensor, labels: torch.Tensor) -> torch.Tensor:
        """x: [batch, h, w, channels] fp32, labels: [batch] int32.  Returns the loss (a device tensor of one float)."""
        n = self.batch
        a = x
        for L in self.conv_layers:
            name, d, (p, q) = L["name"], L["desc"], L["out_hw"]
            L["x"] = a
            tiles = L["stats_tiles"]
            if tiles:           # the batch-norm statistics come out of the convolution's epilogue
                lc.conv2d_fwd_stats(d, a, self.params[name + ".w"], L["z"], self._stats, self._ws)
                lc.batchnorm_fwd_pre(lc.LC_F32, L["z"], self.params[name + ".gamma"], self.params[name + ".beta"], None, L["a"], L["mean"],
                                     L["invstd"], n, d.k, p, q, self.eps, True, NHWC, self._stats, tiles, self._ws)
            else:
                lc.conv2d_fwd(d, a, self.params[name + ".w"], L["z"], self._ws)
                lc.batchnorm_fwd_ex(L["z"], self.params[name + ".gamma"], self.params[name + ".beta"], None, L["a"], L["mean"],
                                    L["invstd"], n, d.k, p, q, self.eps, True, NHWC, self._ws)
            a = L["a"]
            if L["pool"]:
                lc.maxpool_fwd(a, L["pooled"], L["pool_idx"], n, d.k, p, q, 3, 2, 0, NHWC)
                a = L["pooled"]
        for L in self.fc_layers:
            name, d = L["name"], L["desc"]
            L["x"] = a
            lc.conv2d_fwd(d, a, self.params[name + ".w"], L["z"], self._ws)
            lc.bias_add(L["z"], self.params[name + ".b"], n, d.k)
            a = L["z"]
            if L["relu"]:
                lc.relu_fwd(L["z"], L["a"], L["z"].numel())
                a = L["a"]
        lc.softmax_xent(self.logits, labels, self.loss, self.dlogits, self._rows, n, self.classes)
        return self.loss

    def backward(self) -> None:
        n = self.batch
        d_out: torch.Tensor = self.dlogits
        for L in reversed(self.fc_layers):
            name, d = L["name"], L["desc"]
            if L["relu"]:
                dz = torch.empty_like(L["z"])
                lc.relu_bwd(L["z"], d_out, dz, dz.numel())
                d_out = dz
            lc.bias_grad(d_out, self.grads[name + ".b"], n, d.k)
            lc.conv2d_bwd_weight_sq(d, L["x"], d_out, self.grads[name + ".w"], self.gsq[name + ".w"], self._ws)
            dx = torch.empty_like(L["x"])
            lc.conv2d_bwd_data(d, d_out, self.params[name + ".w"], dx, self._ws)
            d_out = dx
        for i in reversed(range(len(self.conv_layers))):
            L = self.conv_layers[i]
            name, d, (p, q) = L["name"], L["desc"], L["out_hw"]
            if L["pool"]:
                da = torch.empty_like(L["a"])
                lc.maxpool_bwd(d_out, L["pool_idx"], da, n, d.k, p, q, 3, 2, 0, NHWC)
                d_out = da
            dz = torch.empty_like(L["z"])
            lc.batchnorm_bwd_ex(L["z"], d_out, self.params[name + ".gamma"], self.params[name + ".beta"], L["mean"], L["invstd"], dz,
                                self.grads[name + ".gamma"], self.grads[name + ".beta"], n, d.k, p, q, True, NHWC, self._ws)
            lc.conv2d_bwd_weight_sq(d, L["x"], dz, self.grads[name + ".w"], self.gsq[name + ".w"], self._ws)
            if i > 0:
                dx = torch.empty_like(L["x"])
                lc.conv2d_bwd_data(d, dz, self.params[name + ".w"], dx, self._ws)
                d_out = dx

    def lars(self, eta: float, momentum: float, weight_decay: float, lr: float) -> None:
        lc.lars_step_pre(self._lars, eta, momentum, weight_decay, lr, self._gsq_list, self._gsq_counts, trust_out=self.trust,
                         workspace=self._lars_ws)

    def step(self, x: torch.Tensor, labels: torch.Tensor, eta: float, momentum: float, weight_decay: float, lr: float) -> torch.Tensor:
        loss = self.forward(x, labels)
        self.backward()
        self.lars(eta, momentum, weight_decay, lr)
        return loss
