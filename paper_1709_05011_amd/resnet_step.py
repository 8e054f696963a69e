"""One whole training step of a bottleneck residual network on the device: forward, backward and the LARS
update, every layer a call into the C library (this module only owns buffers and the order of calls; torch is
used for device memory).  The network is the one the paper trains in "ImageNet training with ResNet-50":
stem convolution + batch norm + ReLU, 3x3 stride-2 max pool, stages of 1x1 -> 3x3 -> 1x1 blocks with batch norm
after every convolution and the block input (through a strided 1x1 projection where the shape changes) added
before the block's last ReLU, global average pool, classifier with bias, softmax cross-entropy, then LARS over
all parameter tensors ("Scaling up Batch Size").  Layout NHWC.

dtype LC_F32: everything fp32.  dtype LC_BF16 (the mixed precision of the paper's fastest runs, "State-of-the-art
results"): activations and their gradients are stored as bf16, the convolutions read a bf16 copy of each filter
that the LARS update writes next to the fp32 master weights; scale, shift, statistics, all parameter gradients,
momentum, the pooled features, the classifier and the loss stay fp32.  Channel counts must then be multiples of 8.

ResNet-50: ResNetStep(stem=(64, 7, 2, 3), widths=(64, 128, 256, 512), blocks=(3, 4, 6, 3), classes=1000, ...).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import torch

from . import larsconv as lc
from . import synth

NHWC = lc.LC_NHWC


@dataclass
class _ConvBn:
    name: str
    desc: lc.ConvDesc
    out_hw: Tuple[int, int]
    relu: bool                       # ReLU fused into the batch norm (no residual at this layer)
    x: Optional[torch.Tensor] = None  # input of the convolution
    z: Optional[torch.Tensor] = None  # convolution output
    a: Optional[torch.Tensor] = None  # after batch norm (+ residual, + ReLU)
    mean: Optional[torch.Tensor] = None
    invstd: Optional[torch.Tensor] = None


class ResNetStep:
    def __init__(self, stem: Tuple[int, int, int, int], widths: Sequence[int], blocks: Sequence[int], classes: int, batch: int,
                 image_hw: Tuple[int, int], in_channels: int = 3, eps: float = 1e-5, device: str = "cuda:0", dtype: int = lc.LC_F32,
                 join_sums: bool = True, fuse_stats: bool = True, pair_bn: bool = True, side_wgrad: bool = True,
                 grid_grads: bool = True):
        lc.lib()                     # fails here, loudly, when the library has not been built
        self.join_sums = join_sums   # False: the block-output gradient and the batch-norm sums behind it as two plain calls
        # The filter gradient of a layer and the gradient of its input both need only dz, and nothing before lars_step reads a
        # filter gradient: with side_wgrad the backward-weight calls go to a second stream (default priority, a workspace of
        # its own), which joins the main one before lars_step.  Same kernels on the same operands: the results do not change.
        self._side = torch.cuda.Stream(device=device) if side_wgrad else None
        self._keep: List[torch.Tensor] = []     # the dz tensors the second stream still reads (held until the join)
        # grid_grads: the input gradients of a stage's first block (two 1x1 convolutions of stride 2) stay on their output grid
        # -- backward-data through a stride-1 descriptor of that grid -- and the pass that joins them at the previous block's
        # output reads them there (relu_add_bwd_bnsums_grid_t): the zeros between the grid pixels are neither written nor read
        self.grid_grads = grid_grads
        self.pair_bn = pair_bn       # False: a projection's batch norm writes its output, which the block's last batch norm then adds
        self.dev, self.eps, self.batch, self.classes = device, eps, batch, classes
        self.dtype = dtype
        self._act = torch.bfloat16 if dtype == lc.LC_BF16 else torch.float32        # storage type of activations
        self.image_hw, self.in_channels = image_hw, in_channels
        self.layers: Dict[str, _ConvBn] = {}
        self.order: List[str] = []
        h, w = image_hw
        h, w = self._add("stem", in_channels, stem[0], stem[1], stem[2], stem[3], h, w, relu=True)
        self.pool_in_hw = (h, w)
        h, w = (h + 2 - 3) // 2 + 1, (w + 2 - 3) // 2 + 1
        self.pool_out_hw = (h, w)
        ch = stem[0]
        self.blocks: List[Tuple[str, bool]] = []
        for si, (wd, nb) in enumerate(zip(widths, blocks)):
            for bi in range(nb):
                stride = 2 if (bi == 0 and si > 0) else 1
                name = f"s{si}b{bi}"
                proj = ch != 4 * wd or stride != 1
                h1, w1 = self._add(name + ".c1", ch, wd, 1, stride, 0, h, w, relu=True)
                self._add(name + ".c2", wd, wd, 3, 1, 1, h1, w1, relu=True)
                self._add(name + ".c3", wd, 4 * wd, 1, 1, 0, h1, w1, relu=False)
                if proj:
                    self._add(name + ".proj", ch, 4 * wd, 1, stride, 0, h, w, relu=False)
                self.blocks.append((name, proj))
                ch, h, w = 4 * wd, h1, w1
        self.final_ch, self.final_hw = ch, (h, w)
        self.fc_desc = lc.ConvDesc(batch, ch, 1, 1, classes, 1, 1, 1, 1, 0, 0, lc.LC_F32, NHWC)

        # parameters, gradients, momentum: filter [k, r, s, c], scale [k], shift [k] per convolution; classifier
        f32 = dict(dtype=torch.float32, device=device)
        self.params: Dict[str, torch.Tensor] = {}
        for name in self.order:
            d = self.layers[name].desc
            self.params[name + ".w"] = torch.zeros((d.k, d.r, d.s, d.c), **f32)
            self.params[name + ".gamma"] = torch.ones(d.k, **f32)
            self.params[name + ".beta"] = torch.zeros(d.k, **f32)
        self.params["fc.w"] = torch.zeros((classes, 1, 1, ch), **f32)
        self.params["fc.b"] = torch.zeros(classes, **f32)
        self.grads = {k: torch.zeros_like(v) for k, v in self.params.items()}
        self.velocity = {k: torch.zeros_like(v) for k, v in self.params.items()}
        # bf16 copies of the filters for the convolutions (kept in step by the update)
        self.lowp: Dict[str, torch.Tensor] = {}
        if dtype == lc.LC_BF16:
            for name in self.order:
                self.lowp[name + ".w"] = torch.zeros_like(self.params[name + ".w"], dtype=torch.bfloat16)
        names = list(self.params)
        self._lowp_list = [self.lowp.get(k) for k in names] if self.lowp else None
        self._lars = lc.LarsArgs([self.params[k] for k in names], [self.grads[k] for k in names], [self.velocity[k] for k in names],
                                 w_lowp=self._lowp_list)
        self._lars_ws = self._bytes(lc.lars_workspace_bytes(self._lars.numel))
        self.trust = torch.zeros(len(names), **f32)
        # the squared norm of every filter gradient comes out of its backward-weight pass in pieces and is handed to
        # the update, which then reads those gradients once instead of twice
        self.gsq: Dict[str, torch.Tensor] = {}
        for name in self.order + ["fc"]:
            d = self.fc_desc if name == "fc" else self.layers[name].desc
            self.gsq[name + ".w"] = torch.zeros(lc.conv2d_bwd_weight_sq_count(d), dtype=torch.float64, device=device)
        self._gsq_list = [self.gsq.get(k) for k in names]
        self._gsq_counts = [0 if t is None else t.numel() for t in self._gsq_list]

        # batch-norm statistics out of the forward convolution's epilogue, where the layer's plan has one: one buffer,
        # written by the convolution and read by the batch norm right behind it
        self.stats_tiles: Dict[str, int] = {name: (lc.conv2d_fwd_stats_count(self.layers[name].desc) if fuse_stats else 0)
                                            for name in self.order}
        most = max([t * self.layers[name].desc.k * 2 for name, t in self.stats_tiles.items()] + [2])
        self._stats = torch.empty(most, dtype=torch.float32, device=device)
        # a projection's statistics wait for the block's last convolution (batchnorm_fwd_pair_t takes both): a buffer of their own
        most_proj = max([t * self.layers[name].desc.k * 2 for name, t in self.stats_tiles.items() if name.endswith(".proj")] + [2])
        self._stats_proj = torch.empty(most_proj, dtype=torch.float32, device=device)

        # one workspace for every convolution pass and every batch norm
        need = 0
        for name in self.order:
            L = self.layers[name]
            for p in (lc.LC_PASS_FWD, lc.LC_PASS_BWD_DATA, lc.LC_PASS_BWD_WEIGHT):
                need = max(need, lc.conv2d_workspace_bytes(L.desc, p))
            need = max(need, lc.batchnorm_workspace_bytes(batch, L.desc.k, L.out_hw[0], L.out_hw[1], NHWC))
        for p in (lc.LC_PASS_FWD, lc.LC_PASS_BWD_DATA, lc.LC_PASS_BWD_WEIGHT):
            need = max(need, lc.conv2d_workspace_bytes(self.fc_desc, p))
        # a strided 1x1 layer seen from its output grid: the same filters, stride 1, input of the output's size
        self._grid_desc: Dict[str, "lc.ConvDesc"] = {}
        for name in self.order:
            d = self.layers[name].desc
            if d.r == 1 and d.s == 1 and d.pad_h == 0 and d.pad_w == 0 and d.stride_h == d.stride_w and d.stride_h > 1:
                p_, q_ = self.layers[name].out_hw
                gd = lc.ConvDesc(batch, d.c, p_, q_, d.k, 1, 1, 1, 1, 0, 0, self.dtype, NHWC)
                self._grid_desc[name] = gd
                need = max(need, lc.conv2d_workspace_bytes(gd, lc.LC_PASS_BWD_DATA))
        self._ws = self._bytes(need)
        self._ws_side = self._bytes(need) if self._side is not None else None

        # activations that the backward pass reads stay allocated; gradients of activations come and go
        for name in self.order:
            L = self.layers[name]
            shape = (batch, L.out_hw[0], L.out_hw[1], L.desc.k)
            L.z = torch.empty(shape, dtype=self._act, device=device)
            # (with pair_bn a projection's batch-norm output is never stored)
            L.a = None if pair_bn and name.endswith(".proj") else torch.empty(shape, dtype=self._act, device=device)
            L.mean, L.invstd = torch.empty(L.desc.k, **f32), torch.empty(L.desc.k, **f32)
        self.pool_out = torch.empty((batch, self.pool_out_hw[0], self.pool_out_hw[1], stem[0]), dtype=self._act, device=device)
        self.pool_idx = torch.empty(self.pool_out.shape, dtype=torch.uint8, device=device)
        self.gap = torch.empty((batch, ch), **f32)
        self.logits = torch.empty((batch, classes), **f32)
        self.dlogits = torch.empty((batch, classes), **f32)
        self.loss = torch.zeros(1, **f32)
        self._rows = torch.empty(batch, **f32)

    # ------------------------------------------------------------------ construction helpers
    def _bytes(self, n: int):
        return torch.empty(max(n, 256), dtype=torch.uint8, device=self.dev)

    def _add(self, name, cin, k, r, stride, pad, h, w, relu):
        d = lc.ConvDesc(self.batch, cin, h, w, k, r, r, stride, stride, pad, pad, self.dtype, NHWC)
        p, q = lc.conv2d_out_shape(d)
        self.layers[name] = _ConvBn(name, d, (p, q), relu)
        self.order.append(name)
        return p, q

    def _new(self, like: torch.Tensor) -> torch.Tensor:
        return torch.empty_like(like)

    def _filter(self, name: str) -> torch.Tensor:
        """the filter as the convolutions read it"""
        return self.lowp[name + ".w"] if self.lowp else self.params[name + ".w"]

    def load(self, host_params: Dict[str, "np.ndarray"]) -> None:
        """Set the parameters from host arrays in the device layout (filters [k, r, s, c]); in bf16 mode the filters'
        bf16 copies are rounded on the host (to nearest even) and uploaded beside them."""
        for k, v in host_params.items():
            self.params[k].copy_(torch.from_numpy(v).reshape(self.params[k].shape))
            if k in self.lowp:
                bits = synth.to_bf16_bits(v).reshape(self.params[k].shape)
                self.lowp[k].copy_(torch.from_numpy(bits.view("int16")).view(torch.bfloat16))

    # ------------------------------------------------------------------ layers
    def _conv_bn(self, name: str, x: torch.Tensor, residual: Optional[torch.Tensor] = None, relu_after_residual: bool = False):
        L = self.layers[name]
        L.x = x
        k, (p, q) = L.desc.k, L.out_hw
        tiles = self.stats_tiles[name]
        if tiles:
            lc.conv2d_fwd_stats(L.desc, x, self._filter(name), L.z, self._stats, self._ws)
            lc.batchnorm_fwd_pre(self.dtype, L.z, self.params[name + ".gamma"], self.params[name + ".beta"], residual, L.a, L.mean,
                                 L.invstd, self.batch, k, p, q, self.eps, L.relu or relu_after_residual, NHWC, self._stats, tiles,
                                 self._ws)
        else:
            lc.conv2d_fwd(L.desc, x, self._filter(name), L.z, self._ws)
            lc.batchnorm_fwd_t(self.dtype, L.z, self.params[name + ".gamma"], self.params[name + ".beta"], residual, L.a, L.mean,
                               L.invstd, self.batch, k, p, q, self.eps, L.relu or relu_after_residual, NHWC, self._ws)
        return L.a

    def _conv_only(self, name: str, x: torch.Tensor, stats: torch.Tensor) -> None:
        L = self.layers[name]
        L.x = x
        if self.stats_tiles[name]:
            lc.conv2d_fwd_stats(L.desc, x, self._filter(name), L.z, stats, self._ws)
        else:
            lc.conv2d_fwd(L.desc, x, self._filter(name), L.z, self._ws)

    def _conv_bn_pair(self, name: str, x: torch.Tensor, other: str) -> torch.Tensor:
        """The block's last convolution, then relu(bn(its output) + bn_other(the projection's output)) in one pass."""
        self._conv_only(name, x, self._stats)
        L, O = self.layers[name], self.layers[other]
        k, (p, q) = L.desc.k, L.out_hw
        t1, t2 = self.stats_tiles[name], self.stats_tiles[other]
        lc.batchnorm_fwd_pair_t(self.dtype, L.z, self.params[name + ".gamma"], self.params[name + ".beta"], self._stats if t1 else None, t1,
                                O.z, self.params[other + ".gamma"], self.params[other + ".beta"], self._stats_proj if t2 else None, t2,
                                L.a, L.mean, L.invstd, O.mean, O.invstd, self.batch, k, p, q, self.eps, True, NHWC, self._ws)
        return L.a

    def _conv_bn_bwd(self, name: str, da: torch.Tensor, need_dx: bool = True, presummed: bool = False,
                     on_grid: bool = False) -> Optional[torch.Tensor]:
        """``da``: gradient with respect to the layer's output -- of the fused ReLU's output where the layer has
        one, otherwise of the batch-norm output itself (the caller has applied the block's last ReLU).  ``presummed``: the
        call that made ``da`` has left the batch-norm backward sums in the workspace."""
        L = self.layers[name]
        k, (p, q) = L.desc.k, L.out_hw
        dz = self._new(L.z)
        if presummed:
            lc.batchnorm_bwd_presummed_t(self.dtype, L.z, da, self.params[name + ".gamma"], L.mean, L.invstd, dz,
                                         self.grads[name + ".gamma"], self.grads[name + ".beta"], self.batch, k, p, q, NHWC, self._ws)
        else:
            lc.batchnorm_bwd_t(self.dtype, L.z, da, self.params[name + ".gamma"], self.params[name + ".beta"], L.mean, L.invstd, dz,
                               self.grads[name + ".gamma"], self.grads[name + ".beta"], self.batch, k, p, q, L.relu, NHWC, self._ws)
        if self._side is not None:
            ev = torch.cuda.Event()
            ev.record()
            with torch.cuda.stream(self._side):
                self._side.wait_event(ev)
                lc.conv2d_bwd_weight_sq(L.desc, L.x, dz, self.grads[name + ".w"], self.gsq[name + ".w"], self._ws_side)
            self._keep.append(dz)
        else:
            lc.conv2d_bwd_weight_sq(L.desc, L.x, dz, self.grads[name + ".w"], self.gsq[name + ".w"], self._ws)
        if not need_dx:
            return None
        if on_grid:                      # the gradient at the pixels the strided layer reads, [n, p, q, c]; zero elsewhere (not stored)
            dx = torch.empty((self.batch, p, q, L.desc.c), dtype=self._act, device=self.dev)
            lc.conv2d_bwd_data(self._grid_desc[name], dz, self._filter(name), dx, self._ws)
            return dx
        dx = self._new(L.x)
        lc.conv2d_bwd_data(L.desc, dz, self._filter(name), dx, self._ws)
        return dx

    # ------------------------------------------------------------------ the step
    def forward(self, x: torch.Tensor, labels: torch.Tensor) -> torch.Tensor:
        """x: [batch, h, w, channels] in the step's storage type, labels: [batch] int32.  Returns the loss (a device
        tensor of one float)."""
        n = self.batch
        a = self._conv_bn("stem", x)
        c0 = self.layers["stem"].desc.k
        lc.maxpool_fwd_t(self.dtype, a, self.pool_out, self.pool_idx, n, c0, self.pool_in_hw[0], self.pool_in_hw[1], 3, 2, 1, NHWC)
        a = self.pool_out
        for name, proj in self.blocks:
            if proj and self.pair_bn:
                # the projection's convolution now, its batch norm together with the block's last one: relu(bn(c3) + bn(proj))
                self._conv_only(name + ".proj", a, self._stats_proj)
                b = self._conv_bn(name + ".c1", a)
                b = self._conv_bn(name + ".c2", b)
                a = self._conv_bn_pair(name + ".c3", b, name + ".proj")
                continue
            sc = self._conv_bn(name + ".proj", a) if proj else a
            b = self._conv_bn(name + ".c1", a)
            b = self._conv_bn(name + ".c2", b)
            a = self._conv_bn(name + ".c3", b, residual=sc, relu_after_residual=True)
        lc.global_avgpool_fwd_t(self.dtype, a, self.gap, n, self.final_ch, self.final_hw[0], self.final_hw[1], NHWC)
        lc.conv2d_fwd(self.fc_desc, self.gap, self.params["fc.w"], self.logits, self._ws)
        lc.bias_add(self.logits, self.params["fc.b"], n, self.classes)
        lc.softmax_xent(self.logits, labels, self.loss, self.dlogits, self._rows, n, self.classes)
        return self.loss

    def backward(self) -> None:
        n = self.batch
        lc.bias_grad(self.dlogits, self.grads["fc.b"], n, self.classes)
        lc.conv2d_bwd_weight_sq(self.fc_desc, self.gap, self.dlogits, self.grads["fc.w"], self.gsq["fc.w"], self._ws)
        dgap = self._new(self.gap)
        lc.conv2d_bwd_data(self.fc_desc, self.dlogits, self.params["fc.w"], dgap, self._ws)
        last = self.layers[self.blocks[-1][0] + ".c3"].a
        g1: torch.Tensor = self._new(last)
        g2: Optional[torch.Tensor] = None
        lc.global_avgpool_bwd_t(self.dtype, dgap, g1, n, self.final_ch, self.final_hw[0], self.final_hw[1], NHWC)
        gstride = 1                      # > 1: g1 and g2 hold the gradient on the stride grid only
        for bi in range(len(self.blocks) - 1, -1, -1):
            name, proj = self.blocks[bi]
            out = self.layers[name + ".c3"].a
            d_pre = self._new(out)
            # both arriving gradients through the block's last ReLU -- and, where the layer's channel count allows the
            # vector path, the sums of the batch-norm backward pass of the block's last convolution on the way
            L3 = self.layers[name + ".c3"]
            joined = self.join_sums and L3.desc.k % (8 if self.dtype == lc.LC_BF16 else 4) == 0
            if joined and gstride > 1:
                lc.relu_add_bwd_bnsums_grid_t(self.dtype, out, g1, g2, d_pre, L3.z, L3.mean, L3.invstd, n, L3.desc.k, L3.out_hw[0],
                                              L3.out_hw[1], gstride, NHWC, self._ws)
            elif joined:
                lc.relu_add_bwd_bnsums_t(self.dtype, out, g1, g2, d_pre, L3.z, L3.mean, L3.invstd, n, L3.desc.k, L3.out_hw[0],
                                         L3.out_hw[1], NHWC, self._ws)
            else:
                lc.relu_add_bwd_t(self.dtype, out, g1, g2, d_pre, out.numel())
            d = self._conv_bn_bwd(name + ".c3", d_pre, presummed=joined)
            d = self._conv_bn_bwd(name + ".c2", d)
            # this block's two input gradients stay on the stride grid when both come from strided 1x1 layers and the pass
            # that takes them (the previous block's output) is the joined one
            gstride = 1
            if self.grid_grads and proj and bi > 0 and (name + ".c1") in self._grid_desc and (name + ".proj") in self._grid_desc:
                Lp = self.layers[self.blocks[bi - 1][0] + ".c3"]
                if self.join_sums and Lp.desc.k % (8 if self.dtype == lc.LC_BF16 else 4) == 0:
                    gstride = self.layers[name + ".c1"].desc.stride_h
            g1 = self._conv_bn_bwd(name + ".c1", d, on_grid=gstride > 1)
            g2 = (self._conv_bn_bwd(name + ".proj", d_pre, on_grid=gstride > 1) if proj else d_pre)
        d_pool = self._new(self.pool_out)
        lc.relu_add_bwd_t(self.dtype, None, g1, g2, d_pool, d_pool.numel())   # the pool's output feeds the first block twice
        stem = self.layers["stem"]
        da = self._new(stem.a)
        lc.maxpool_bwd_t(self.dtype, d_pool, self.pool_idx, da, n, stem.desc.k, self.pool_in_hw[0], self.pool_in_hw[1], 3, 2, 1, NHWC)
        self._conv_bn_bwd("stem", da, need_dx=False)
        if self._side is not None:
            torch.cuda.current_stream().wait_stream(self._side)
            self._keep.clear()

    def lars(self, eta: float, momentum: float, weight_decay: float, lr: float) -> None:
        lc.lars_step_pre(self._lars, eta, momentum, weight_decay, lr, self._gsq_list, self._gsq_counts, trust_out=self.trust,
                         workspace=self._lars_ws)

    def step(self, x: torch.Tensor, labels: torch.Tensor, eta: float, momentum: float, weight_decay: float, lr: float) -> torch.Tensor:
        loss = self.forward(x, labels)
        self.backward()
        self.lars(eta, momentum, weight_decay, lr)
        return loss
