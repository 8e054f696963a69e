#!/usr/bin/env python3
"""Benchmark of the conv + LARS training hot path on one MI355X.

Default run (the driver's contract): one "step" = forward of all 53 ResNet-50 convolutions and the
classifier, backward-data and backward-weight of every layer (no backward-data for the first
layer: there is no gradient with respect to the image), then one lars_step over the 161 parameter
tensors, fp32, batch 256, NHWC, synthetic N(0,1) inputs resident in HBM.  Prints ONE JSON line:
images/s, plus "roofline" for the dominant kernel and "cpu_baseline" (the CPU oracle timed on the
host cores on a bounded sample).  After the timed region the same line also gets lars_step on rotating
parameter sets ("lars.cold"), the whole network step with its glue layers ("whole_step") and the bf16 form
of the step at batch 512 ("bf16_step"), each a short run of its own (--no-extras skips them).

    python bench.py [--steps K] [--warmup W]          # the headline line
    python bench.py --dtype bf16                      # the same step at batch 512 with bf16 operands
    python bench.py --model alexnet_bn                # AlexNet-BN shaped step (5 convs + 3 FC layers as convs, 21 tensors)
    python bench.py --sweep [--batch 128]             # every distinct ResNet-50 conv shape x 3 passes
    python bench.py --model alexnet                   # the original grouped AlexNet (61 M parameters), bias per layer
    python bench.py --lars resnet50|alexnet_bn        # lars_step alone, GB/s against HBM peak
    python bench.py --batch-curve                     # images/s against the per-GPU batch, 16 .. 512
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F32 = 157.3      # TFLOP/s, MI355X dense fp32 matrix
PEAK_MFMA_BF16 = 2500.0    # TFLOP/s, MI355X dense bf16 matrix
PEAK_HBM = 8000.0          # GB/s
LARS_BYTES_PER_PARAM = 28  # norm pass reads w, g (8 B); update reads w, g, v and writes w, v (20 B)
# HBM-side bytes per launch of the dominant kernel: counters cannot be read from inside this process, so the figure is
# parsed from the tracked rocprofv3 summaries (two --pmc runs, FETCH_SIZE then WRITE_SIZE, scaled by what the same
# counters read for a 1 GiB copy; the commands are in the files).  None when the file or the kernel's row is missing.
TRAFFIC_PROFILES = {("resnet50", "f32"): "resnet50_step_fp32_b256_hbm_traffic_and_mfma.txt",
                    ("alexnet_bn", "f32"): "alexnet_bn_step_fp32_b256_kernel_trace.txt",
                    ("resnet50", "bf16"): "resnet50_step_bf16_b512_kernel_trace.txt"}
TRAFFIC_BATCH = {"f32": 256, "bf16": 512}


def kernel_instance_name(label: str, bf16: bool) -> str:
    """Name rocprofv3 prints for the main-kernel instance behind one of this file's labels (conv_gemm_128x128 ...)."""
    bm, bn = label.rsplit("_", 1)[1].split("x")
    return f"conv_gemm_pk_kernel<{bm}, {bn}, false, {'true' if bf16 else 'false'}, true, false>"


def profile_traffic(model: str, dtype: str, label: str, batch: int):
    """Read + written bytes per launch of kernel `label` from the FETCH_SIZE / WRITE_SIZE tables of the tracked summary."""
    name = TRAFFIC_PROFILES.get((model, dtype))
    if name is None or batch != TRAFFIC_BATCH[dtype] or not label.startswith("conv_gemm_"):
        return None
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    want = kernel_instance_name(label, dtype == "bf16")
    section, found = None, {}
    for line in open(path):
        head = line.strip()
        if head.startswith("FETCH_SIZE"):
            section = "FETCH_SIZE"
        elif head.startswith("WRITE_SIZE"):
            section = "WRITE_SIZE"
        elif section and line.startswith(want) and section not in found:
            found[section] = float(line.split()[-1]) * 1e6          # the scaled_MB/launch column
    if len(found) != 2:
        return None
    return found["FETCH_SIZE"] + found["WRITE_SIZE"]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Layer:
    """Device buffers and descriptor of one convolution of the workload."""

    def __init__(self, cs, gen, torch, lc, first: bool, bf16: bool = False):
        dev = "cuda:0"
        self.cs = cs
        self.first = first
        self.desc = lc.ConvDesc(cs.n, cs.c, cs.h, cs.w, cs.k, cs.r, cs.s, cs.stride, cs.stride, cs.pad, cs.pad,
                                lc.LC_BF16 if bf16 else lc.LC_F32, lc.LC_NHWC, cs.groups)
        cg = cs.c // cs.groups
        std = (2.0 / (cg * cs.r * cs.s)) ** 0.5
        act = torch.bfloat16 if bf16 else torch.float32
        self.x = torch.randn((cs.n, cs.h, cs.w, cs.c), generator=gen, device=dev).to(act)
        self.w_master = torch.randn((cs.k, cs.r, cs.s, cg), generator=gen, device=dev) * std     # fp32 weights
        self.w = self.w_master.to(act) if bf16 else self.w_master                                # what the convolutions read
        self.dy = torch.randn((cs.n, cs.p, cs.q, cs.k), generator=gen, device=dev).to(act)
        self.y = torch.empty((cs.n, cs.p, cs.q, cs.k), device=dev, dtype=act)
        self.dx = None if first else torch.empty((cs.n, cs.h, cs.w, cs.c), device=dev, dtype=act)
        self.dw = torch.empty((cs.k, cs.r, cs.s, cg), device=dev)
        self.dw_sq = torch.empty(lc.conv2d_bwd_weight_sq_count(self.desc), dtype=torch.float64, device=dev)   # pieces of sum dw^2
        self.ws_bytes = max(lc.conv2d_workspace_bytes(self.desc, p) for p in range(3))


def make_workspace(nbytes, torch):
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda:0")


class Timer:
    """HIP events on the stream the kernels are launched on (torch's current stream): one event after every library call,
    a call's span running from the event behind the previous call to its own (one more event opens the chain).  Half the
    events of a pair per call -- each costs the command processor a few microseconds between kernels."""

    def __init__(self, torch):
        self.torch = torch
        self.spans = []          # (key, start, stop)
        self.step_starts = []    # index into spans of the first call of every timed step
        self.last = None         # the event behind the latest call

    def totals(self):
        out = {}
        for key, a, b in self.spans:
            ms, n = out.get(key, (0.0, 0))
            out[key] = (ms + a.elapsed_time(b), n + 1)
        return out


def timed(timer, key, fn):
    if timer is None:
        fn()
        return
    if timer.last is None:
        timer.last = timer.torch.cuda.Event(enable_timing=True)
        timer.last.record()
    fn()
    b = timer.torch.cuda.Event(enable_timing=True)
    b.record()
    timer.spans.append((key, timer.last, b))
    timer.last = b


def model_shapes(synth, model: str, batch: int):
    """(layer shapes in network order, number of leading layers followed by batch norm, weight decay)."""
    if model == "alexnet_bn":
        return synth.alexnet_bn_convs(batch), 5, 5e-4
    if model == "alexnet":          # the original grouped network of the paper's scaling-ratio table: a bias per layer, no batch norm
        return synth.alexnet_grouped_convs(batch), 0, 5e-4
    return synth.resnet50_convs(batch) + [synth.resnet50_fc(batch)], 53, 5e-5


def run_train_step(args):
    import torch
    from paper_1709_05011_amd import larsconv as lc
    from paper_1709_05011_amd import synth

    lc.lib()
    bf16 = args.dtype == "bf16"
    batch = args.batch or (512 if bf16 else 256)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(0x5EED0300)
    shapes, n_bn, weight_decay = model_shapes(synth, args.model, batch)
    layers = [Layer(cs, gen, torch, lc, i == 0, bf16) for i, cs in enumerate(shapes)]
    ws = make_workspace(max(l.ws_bytes for l in layers), torch)

    # parameter tensors: filter, batch-norm scale, batch-norm shift per convolution; weight and bias per FC layer
    # (ResNet-50: 161 tensors, AlexNet-BN: 21)
    pw, pg, pv, plow = [], [], [], []
    for i, l in enumerate(layers):
        k = l.cs.k
        extra = [torch.ones(k, device="cuda:0"), torch.zeros(k, device="cuda:0")] if i < n_bn else [torch.zeros(k, device="cuda:0")]
        pw += [l.w_master] + extra
        plow += [l.w] + [None] * len(extra)
        pg += [l.dw] + [torch.randn(k, generator=gen, device="cuda:0") * 1e-2 for _ in extra]
    pv = [torch.zeros_like(t) for t in pw]
    # the squared norm of every filter gradient comes out of its backward-weight pass (conv2d_bwd_weight_sq) and is handed
    # to the update (lars_step_pre), which then reads those gradients once instead of twice; --plain-norms: the plain calls
    fused_norms = not args.plain_norms
    psq, psq_n = [], []
    for i, l in enumerate(layers):
        n_extra = 2 if i < n_bn else 1
        psq += [l.dw_sq if fused_norms else None] + [None] * n_extra
        psq_n += [l.dw_sq.numel() if fused_norms else 0] + [0] * n_extra
    # bf16 run: fp32 master weights and momentum; lars_step also writes the bf16 weights the convolutions read
    largs = lc.LarsArgs(pw, pg, pv, w_lowp=plow if bf16 else None)
    expect = {"alexnet_bn": synth.alexnet_bn_param_numels, "alexnet": synth.alexnet_grouped_param_numels,
              "resnet50": synth.resnet50_param_numels}[args.model]()
    assert list(largs.numel) == list(expect), "parameter list does not match the model's"
    lws = make_workspace(lc.lars_workspace_bytes(largs.numel), torch)
    trust = torch.empty(largs.n, device="cuda:0")
    T = synth.poly_total_iters()
    lr = lc.lars_poly_lr(1.0, 1000, T)

    def gemm_kernel_of(l, pass_):
        """Which conv kernel instance a call ends in (mirrors the library's dispatch; labels only)."""
        cs = l.cs
        if pass_ == "bwd_weight":
            return "wgrad"
        # ResNet's first layer has a forward kernel of its own
        if ((cs.c, cs.k, cs.r, cs.s, cs.stride, cs.pad) == (3, 64, 7, 7, 2, 3) and cs.p % 16 == 0 and cs.q % 16 == 0
                and not os.environ.get("LARSCONV_NO_STEM_DIRECT")):
            return "conv_stem"
        n_gemm = cs.k if pass_ == "fwd" else cs.c
        k_gemm = cs.c if pass_ == "fwd" else cs.k
        rows = cs.n * cs.p * cs.q if pass_ == "fwd" or cs.stride > 1 else cs.n * cs.h * cs.w
        scatter = pass_ == "bwd_data" and cs.stride > 1
        # bf16 has two more tiles, each taken with three or more rounds of such tiles (and not by the strided 1x1
        # backward-data layers, whose scatter epilogue exists for the 128-row tiles of 64 and 128 columns only)
        special = bf16 and k_gemm >= 32 and not scatter
        big = False
        if special and n_gemm >= 256:
            tiles = -(-rows // 256) * -(-n_gemm // 256)            # 256x256 (eight waves): one block per compute unit
            rounds = -(-tiles // 256)
            nkt = -(-(k_gemm * cs.r * cs.s) // 32)
            fill = 70 if n_gemm <= 512 else 85
            big = tiles >= 256 and tiles * 100 >= rounds * 256 * fill and (n_gemm <= 512 or nkt >= 16)
        # 3x3 stride-1 pad-1 layers in bf16: the kernel that stages the activation slab once for all nine taps
        if (bf16 and cs.r == 3 and cs.s == 3 and cs.stride == 1 and cs.pad == 1 and k_gemm % 32 == 0 and not big
                and -(-rows // 128) * -(-n_gemm // (128 if n_gemm > 64 else 64)) >= 256):
            return "conv3x3_slab"
        if n_gemm <= 64:
            return "conv_gemm_256x64" if special and -(-rows // 256) >= 3 * 3 * 256 else "conv_gemm_128x64"
        if special and n_gemm >= 256:
            if big:
                return "conv_gemm_256x256"
            if -(-rows // 128) * -(-n_gemm // 256) >= 3 * 2 * 256:
                return "conv_gemm_128x256"
        return "conv_gemm_128x128"

    def step(timer=None):
        if timer is not None:
            timer.step_starts.append(len(timer.spans))
        for l in layers:
            timed(timer, ("fwd", gemm_kernel_of(l, "fwd"), l.cs.flops),
                  lambda l=l: lc.conv2d_fwd(l.desc, l.x, l.w, l.y, ws))
        for l in reversed(layers):
            if not l.first:
                timed(timer, ("bwd_data", gemm_kernel_of(l, "bwd_data"), l.cs.flops),
                      lambda l=l: lc.conv2d_bwd_data(l.desc, l.dy, l.w, l.dx, ws))
            if fused_norms:
                timed(timer, ("bwd_weight", "wgrad", l.cs.flops),
                      lambda l=l: lc.conv2d_bwd_weight_sq(l.desc, l.x, l.dy, l.dw, l.dw_sq, ws))
            else:
                timed(timer, ("bwd_weight", "wgrad", l.cs.flops),
                      lambda l=l: lc.conv2d_bwd_weight(l.desc, l.x, l.dy, l.dw, ws))
        if fused_norms:
            timed(timer, ("lars", "lars", 0), lambda: lc.lars_step_pre(largs, 0.001, 0.9, weight_decay, lr, psq, psq_n, trust_out=trust,
                                                                     workspace=lws))
        else:
            timed(timer, ("lars", "lars", 0), lambda: lc.lars_step(largs, 0.001, 0.9, weight_decay, lr, trust, lws))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    timer = Timer(torch)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(timer)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    # aggregate the per-call spans: totals per pass and per kernel instance, and per-pass time of every step
    per_pass, per_kernel = {}, {}
    bounds = timer.step_starts + [len(timer.spans)]
    per_step = []                                       # one {pass: ms} per timed step
    for si in range(len(bounds) - 1):
        acc = {}
        for (pass_, kern, flops), a, b in timer.spans[bounds[si]:bounds[si + 1]]:
            ms = a.elapsed_time(b)
            acc[pass_] = acc.get(pass_, 0.0) + ms
            p = per_pass.setdefault(pass_, [0.0, 0, 0])
            p[0] += ms; p[1] += 1; p[2] += flops
            q = per_kernel.setdefault(kern, [0.0, 0, 0])
            q[0] += ms; q[1] += 1; q[2] += flops
        per_step.append(acc)

    def med_min(vals):
        v = sorted(vals)
        return round(v[len(v) // 2], 4), round(v[0], 4)
    pass_ms = {}
    for pass_ in per_pass:
        m, lo = med_min([st[pass_] for st in per_step])
        pass_ms[pass_] = {"median": m, "min": lo}
    conv_ms = sum(per_pass[p][0] for p in ("fwd", "bwd_data", "bwd_weight"))
    conv_flops = sum(per_pass[p][2] for p in ("fwd", "bwd_data", "bwd_weight"))
    lars_ms = per_pass["lars"][0] / per_pass["lars"][1]
    lars_bpp = LARS_BYTES_PER_PARAM + (2 if bf16 else 0)       # + the bf16 copy of the filters (an upper bound: not the BN tensors)
    lars_gbps = lars_bpp * sum(largs.numel) / (lars_ms * 1e-3) / 1e9
    dom = max((k for k in per_kernel if k != "lars"), key=lambda k: per_kernel[k][0])
    dms, dn, dfl = per_kernel[dom]
    achieved = dfl / (dms * 1e-3) / 1e12
    # bf16: all three passes multiply on the bf16 matrix pipe (the filter gradient too, unless the comparison knob
    # LARSCONV_WGRAD_WIDEN sends it through the widening fp32 kernel)
    widened = dom == "wgrad" and os.environ.get("LARSCONV_WGRAD_WIDEN")
    peak = PEAK_MFMA_BF16 if bf16 and not widened else PEAK_MFMA_F32
    name = {"alexnet_bn": "AlexNet-BN", "alexnet": "AlexNet (grouped)", "resnet50": "ResNet-50"}[args.model]
    n_conv = sum(1 for l in layers if l.cs.h * l.cs.w > 1 and not (l.cs.r == l.cs.h and l.cs.s == l.cs.w and l.cs.pad == 0))
    n_fc = len(layers) - n_conv
    result = {
        "metric": f"{name} fwd+bwd+LARS images/sec/GPU",
        "value": round(batch / (ms_per_step * 1e-3), 2),
        "unit": "images/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.model}_train_step_{'bf16' if bf16 else 'fp32'}_batch{batch}_nhwc ({n_conv} convs + {n_fc} fc: fwd, "
                               f"bwd_data, bwd_weight; lars_step over {largs.n} tensors / {sum(largs.numel) / 1e6:.1f}M params)",
                   "batch": batch, "layout": "NHWC",
                   "lars": {"eta": 0.001, "momentum": 0.9, "weight_decay": weight_decay, "lr": lr}},
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": round(achieved, 2), "peak": peak,
                     "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                     "traffic": profile_traffic(args.model, "bf16" if bf16 else "f32", dom, batch),
                     "launches_per_step": dn // args.steps, "avg_launch_ms": round(dms / dn, 4),
                     "flops_per_launch": dfl / dn},
        "conv_tflops": {p: round(per_pass[p][2] / (per_pass[p][0] * 1e-3) / 1e12, 2) for p in ("fwd", "bwd_data", "bwd_weight")},
        "conv_tflops_all": round(conv_flops / (conv_ms * 1e-3) / 1e12, 2),
        "conv_frac_of_mfma_peak": round(conv_flops / (conv_ms * 1e-3) / 1e12 / peak, 4),
        # lars_step inside the step: its gradients were written a moment ago and part of the 307 MB working set is still
        # in the 256 MB Infinity Cache, so this is an effective rate, not achieved HBM bandwidth ("cold" below is)
        "lars": {"in_step": {"ms": round(lars_ms, 4), "GBps_effective": round(lars_gbps, 1),
                             "frac_of_hbm_peak_effective": round(lars_gbps / PEAK_HBM, 4),
                             "g_norms": "from backward-weight (24 bytes per parameter move)" if fused_norms else "computed by lars_step",
                             "note": "cache-assisted: g was just written by backward-weight"},
                 "bytes_per_param": lars_bpp},
        "pass_ms_per_step": pass_ms,
        "kernel_ms_per_step": {k: round(v[0] / args.steps, 3) for k, v in per_kernel.items()},
    }
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(args.model, args.cpu_batch)
    return result


def cpu_baseline(model: str, batch: int):
    """The oracle as it stands, timed on the host cores on a bounded sample: the same network (all
    layers x 3 passes + the LARS step over the model's parameter list) at a small batch."""
    import numpy as np
    import oracle
    from paper_1709_05011_amd import synth

    shapes, _, weight_decay = model_shapes(synth, model, batch)
    cache = {}

    def data(cs):
        key = cs.key()
        if key not in cache:
            cache[key] = (synth.normal((cs.n, cs.h, cs.w, cs.c), 1), synth.normal((cs.k, cs.r, cs.s, cs.c // cs.groups), 2),
                          synth.normal((cs.n, cs.p, cs.q, cs.k), 3))
        return cache[key]

    for cs in shapes:
        data(cs)
    sizes = {"alexnet_bn": synth.alexnet_bn_param_numels, "alexnet": synth.alexnet_grouped_param_numels,
             "resnet50": synth.resnet50_param_numels}[model]()
    w = [synth.normal((n,), 10) for n in sizes]
    g = [synth.normal((n,), 11, std=0.01) for n in sizes]
    v = [np.zeros(n, np.float32) for n in sizes]
    t0 = time.perf_counter()
    for i, cs in enumerate(shapes):
        x, wt, dy = data(cs)
        if cs.groups > 1:
            oracle.conv2d_fwd_grouped(x, wt, cs.groups, cs.stride, cs.pad, oracle.NHWC)
            oracle.conv2d_bwd_data_grouped(dy, wt, cs.groups, (cs.h, cs.w), cs.stride, cs.pad, oracle.NHWC)
            oracle.conv2d_bwd_weight_grouped(x, dy, cs.groups, (cs.r, cs.s), cs.stride, cs.pad, oracle.NHWC)
            continue
        oracle.conv2d_fwd(x, wt, cs.stride, cs.pad, oracle.NHWC)
        if i:
            oracle.conv2d_bwd_data(dy, wt, (cs.h, cs.w), cs.stride, cs.pad, oracle.NHWC)
        oracle.conv2d_bwd_weight(x, dy, (cs.r, cs.s), cs.stride, cs.pad, oracle.NHWC)
    t1 = time.perf_counter()
    oracle.lars_step(w, g, v, 0.001, 0.9, weight_decay, 0.5)
    t2 = time.perf_counter()
    return {"value": round(batch / (t2 - t0), 3), "unit": "images/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"whole {model} step ({len(shapes)} layers x fwd/bwd_data/bwd_weight + {len(sizes)}-tensor LARS) at batch {batch}: "
                      f"conv {t1 - t0:.1f} s, LARS {t2 - t1:.2f} s",
            "lars_GBps": round(LARS_BYTES_PER_PARAM * sum(sizes) / (t2 - t1) / 1e9, 2)}


def time_call(torch, fn, iters, warmup=5):
    for _ in range(warmup):
        fn()
    evs = []
    for _ in range(iters):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        evs.append((a, b))
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in evs)
    return ms[len(ms) // 2], ms[0]


def run_sweep(args):
    """Every distinct ResNet-50 convolution shape, each pass timed separately."""
    import torch
    from paper_1709_05011_amd import larsconv as lc
    from paper_1709_05011_amd import synth

    batch = args.batch or 128
    bf16 = args.dtype == "bf16"
    peak = PEAK_MFMA_BF16 if bf16 else PEAK_MFMA_F32
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(0x5EED0200)
    rows = []
    tot = {"fwd": [0.0, 0.0], "bwd_data": [0.0, 0.0], "bwd_weight": [0.0, 0.0]}
    roof_ms = 0.0
    # after the 20 distinct shapes of the network the paper trains: the six layers only the "v1.5" form of ResNet-50 has
    # (stride on the 3x3 convolution), labelled rows that do not enter the totals
    shape_list = [(cs, count, False) for cs, count in synth.resnet50_distinct_shapes(batch)]
    shape_list += [(cs, 1, True) for cs in synth.resnet50_v15_extra_shapes(batch)]
    for idx, (cs, count, extra) in enumerate(shape_list, start=1):
        if args.only and idx not in args.only:
            continue
        l = Layer(cs, gen, torch, lc, False, args.dtype == "bf16")
        ws = make_workspace(l.ws_bytes, torch)
        calls = {
            "fwd": lambda: lc.conv2d_fwd(l.desc, l.x, l.w, l.y, ws),
            "bwd_data": lambda: lc.conv2d_bwd_data(l.desc, l.dy, l.w, l.dx, ws),
            "bwd_weight": lambda: lc.conv2d_bwd_weight(l.desc, l.x, l.dy, l.dw, ws),
        }
        # each pass against its own roof: min(MFMA peak, arithmetic intensity x HBM peak), the intensity from the
        # bytes every pass must move at least once (both operands read, the result written; the filter gradient
        # is fp32 in both modes)
        es = 2 if bf16 else 4
        xb, yb, wb = cs.n * cs.c * cs.h * cs.w * es, cs.n * cs.k * cs.p * cs.q * es, cs.weight_numel * es
        # a strided 1x1 window reads only the pixels on the stride grid (backward-data still writes all of dx)
        xread = cs.n * cs.c * cs.p * cs.q * es if cs.r == 1 and cs.s == 1 and cs.stride > 1 else xb
        min_bytes = {"fwd": xread + wb + yb, "bwd_data": yb + wb + xb, "bwd_weight": xread + yb + cs.weight_numel * 4}
        row = {"shape": idx, "name": cs.name, "c": cs.c, "k": cs.k, "rs": cs.r, "stride": cs.stride, "hw": cs.h,
               "count": count, "gflop": round(cs.flops / 1e9, 2)}
        if extra:
            row["extra"] = "ResNet-50 v1.5 only; not in the totals"
        for p, fn in calls.items():
            if p == "bwd_data" and idx == 1:
                continue                      # the first layer's input gradient is never needed in a training step
            med, mn = time_call(torch, fn, args.iters)
            tf = cs.flops / (med * 1e-3) / 1e12
            roof = min(peak, cs.flops / min_bytes[p] * PEAK_HBM / 1e3)
            row[p + "_ms"] = round(med, 4)
            row[p + "_tflops"] = round(tf, 2)
            row[p + "_roof_tflops"] = round(roof, 1)
            row[p + "_frac_of_roof"] = round(tf / roof, 3)
            if not extra:
                tot[p][0] += med * count
                tot[p][1] += cs.flops * count
                roof_ms += cs.flops / (roof * 1e12) * 1e3 * count
        rows.append(row)
        log(json.dumps(row))
        del l, ws
        torch.cuda.empty_cache()
    summary = {p: round(v[1] / (v[0] * 1e-3) / 1e12, 2) for p, v in tot.items() if v[0] > 0}
    all_ms = sum(v[0] for v in tot.values())
    all_fl = sum(v[1] for v in tot.values())
    return {"sweep": "resnet50_distinct_conv_shapes", "batch": batch, "dtype": args.dtype, "layout": "NHWC",
            "weighted_tflops": summary, "weighted_tflops_all": round(all_fl / (all_ms * 1e-3) / 1e12, 2),
            "frac_of_mfma_peak": round(all_fl / (all_ms * 1e-3) / 1e12 / peak, 4),
            "roof": "per pass min(MFMA peak, flops / minimal bytes x 8 TB/s)", "ms_all": round(all_ms, 3),
            "ms_at_roof": round(roof_ms, 3), "frac_of_roof": round(roof_ms / all_ms, 4), "rows": rows}


def measure_lars(which: str, n_sets: int, iters: int):
    """lars_step alone over the model's parameter list; n_sets > 1 rotates over that many parameter sets so that no call
    finds its data in the caches (each call then also pays the write-back of what the previous call left dirty)."""
    import torch
    from paper_1709_05011_amd import larsconv as lc
    from paper_1709_05011_amd import synth

    sizes = {"alexnet_bn": synth.alexnet_bn_param_numels, "alexnet": synth.alexnet_grouped_param_numels,
             "resnet50": synth.resnet50_param_numels}[which]()
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(0x5EED0400)
    sets = []
    for _ in range(n_sets):
        w = [torch.randn(n, generator=gen, device="cuda:0") for n in sizes]
        g = [torch.randn(n, generator=gen, device="cuda:0") * 1e-2 for n in sizes]
        v = [torch.zeros(n, device="cuda:0") for n in sizes]
        sets.append(lc.LarsArgs(w, g, v))
    lws = make_workspace(lc.lars_workspace_bytes(sizes), torch)
    trust = torch.empty(len(sizes), device="cuda:0")
    state = {"i": 0}

    def call():
        a = sets[state["i"] % n_sets]
        state["i"] += 1
        lc.lars_step(a, 0.001, 0.9, 5e-5, 0.5, trust, lws)

    med, mn = time_call(torch, call, iters, warmup=max(2, n_sets))
    nbytes = LARS_BYTES_PER_PARAM * sum(sizes)
    return {"lars": which, "tensors": len(sizes), "params": sum(sizes), "rotating_sets": n_sets,
            "ms_median": round(med, 4), "ms_min": round(mn, 4), "GBps_median": round(nbytes / (med * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(nbytes / (med * 1e-3) / 1e9 / PEAK_HBM, 4), "bytes_per_param": LARS_BYTES_PER_PARAM}


def run_lars(args):
    return measure_lars(args.lars, args.rotate, args.iters)


def run_batchnorm(args):
    """Batch normalisation (training mode) over the outputs of the distinct ResNet-50 convolution shapes, forward and
    backward timed separately; GB/s by the algorithmic bytes (forward 12, backward 20 bytes per element)."""
    import torch
    from paper_1709_05011_amd import larsconv as lc
    from paper_1709_05011_amd import synth

    batch = args.batch or 256
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(0x5EED0500)
    rows, seen = [], set()
    tot = {"fwd": [0.0, 0.0], "bwd": [0.0, 0.0]}
    for cs, count in synth.resnet50_distinct_shapes(batch):
        key = (cs.k, cs.p, cs.q)
        if key in seen:
            continue
        seen.add(key)
        n, c, h, w = cs.n, cs.k, cs.p, cs.q
        x = torch.randn((n, h, w, c), generator=gen, device="cuda:0")
        dy = torch.randn((n, h, w, c), generator=gen, device="cuda:0")
        y, dx = torch.empty_like(x), torch.empty_like(x)
        g, b = torch.ones(c, device="cuda:0"), torch.zeros(c, device="cuda:0")
        m, s, dg, db = (torch.empty(c, device="cuda:0") for _ in range(4))
        ws = make_workspace(lc.batchnorm_workspace_bytes(n, c, h, w, lc.LC_NHWC), torch)
        f_med, _ = time_call(torch, lambda: lc.batchnorm_fwd(x, g, b, y, m, s, n, c, h, w, 1e-5, lc.LC_NHWC, ws), args.iters)
        b_med, _ = time_call(torch, lambda: lc.batchnorm_bwd(x, dy, g, m, s, dx, dg, db, n, c, h, w, lc.LC_NHWC, ws), args.iters)
        elems = x.numel()
        row = {"c": c, "hw": h, "MB": round(elems * 4 / 1e6, 1), "fwd_ms": round(f_med, 4), "bwd_ms": round(b_med, 4),
               "fwd_GBps": round(12 * elems / (f_med * 1e-3) / 1e9, 1), "bwd_GBps": round(20 * elems / (b_med * 1e-3) / 1e9, 1)}
        rows.append(row)
        log(json.dumps(row))
        tot["fwd"][0] += f_med; tot["fwd"][1] += 12 * elems
        tot["bwd"][0] += b_med; tot["bwd"][1] += 20 * elems
        del x, dy, y, dx, ws
        torch.cuda.empty_cache()
    out = {"batchnorm": "outputs of the distinct ResNet-50 convolution shapes", "batch": batch, "layout": "NHWC", "dtype": "f32",
           "bytes_per_element": {"fwd": 12, "bwd": 20}}
    for p_, (ms, nbytes) in tot.items():
        gbps = nbytes / (ms * 1e-3) / 1e9
        out[p_] = {"GBps": round(gbps, 1), "frac_of_hbm_peak": round(gbps / PEAK_HBM, 4)}
    out["rows"] = rows
    return out


def run_full_step(args):
    """The WHOLE ResNet-50 training step at batch 256, fp32: every convolution, batch norm, ReLU, pool, the
    classifier, the loss, all gradients and lars_step over the 161 tensors, each a call into the library
    (paper_1709_05011_amd/resnet_step.py only orders the calls).  Weights are random (He), images and labels
    synthetic.  This is a secondary mode: the headline metric times the convolution + LARS path."""
    import torch
    from paper_1709_05011_amd.alexnet_step import AlexNetStep
    from paper_1709_05011_amd.resnet_step import ResNetStep

    from paper_1709_05011_amd import larsconv as lc

    bf16 = args.dtype == "bf16"
    if bf16 and args.model != "resnet50":
        raise SystemExit("--full-step --dtype bf16 is built for --model resnet50")
    batch = args.batch or (512 if bf16 else 256)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(0x5EED0600)
    alex = args.model == "alexnet_bn"
    if alex:       # --model alexnet_bn: the whole AlexNet-BN step (five convolutions with batch norm, three pools, three FC layers)
        net = AlexNetStep(((96, 11, 4, 0, True), (256, 5, 1, 2, True), (384, 3, 1, 1, False), (384, 3, 1, 1, False),
                           (256, 3, 1, 1, True)), (4096, 4096), 1000, batch, (227, 227))
    else:
        net = ResNetStep((64, 7, 2, 3), (64, 128, 256, 512), (3, 4, 6, 3), 1000, batch, (224, 224),
                         dtype=lc.LC_BF16 if bf16 else lc.LC_F32, join_sums=not args.no_join, fuse_stats=not args.no_fused_stats,
                         pair_bn=not args.no_pair,
                         side_wgrad=not args.no_side_stream and not args.graph, grid_grads=not args.no_grid_grads)     # (replays of a captured step gain nothing from the second stream)
    side = 227 if alex else 224
    label = f"{'AlexNet-BN' if alex else 'ResNet-50'} whole training step (all layers + LARS), batch {batch}, {side}x{side}, NHWC"
    if bf16:
        label += ", bf16 activations and filters, fp32 master weights"
    metric = ("alexnet_bn" if alex else "resnet50") + "_whole_step_images_per_second"
    dtype_name = "bf16" if bf16 else "f32"
    for name, t in net.params.items():
        if name.endswith(".w"):
            fan = t[0].numel()
            t.copy_(torch.randn(t.shape, generator=gen, device="cuda:0") * (2.0 / fan) ** 0.5)
            if bf16 and name in net.lowp:
                net.lowp[name].copy_(t)             # input preparation; from the first update on lars_step writes these copies
    x = torch.randn((batch, side, side, 3), generator=gen, device="cuda:0")
    if bf16:
        x = x.to(torch.bfloat16)
    labels = torch.randint(0, 1000, (batch,), generator=gen, device="cuda:0", dtype=torch.int32)
    lr = 0.1
    for _ in range(args.warmup):
        net.step(x, labels, 0.001, 0.9, 1e-4, lr)
    torch.cuda.synchronize()
    if args.graph:
        # the library allocates nothing and never synchronizes: the whole step is captured once and replayed
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            net.step(x, labels, 0.001, 0.9, 1e-4, lr)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        return {"metric": metric, "value": round(batch / (ms * 1e-3), 1), "unit": "images/s",
                "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 3), "higher_is_better": True,
                "scaling": "weak", "vs_baseline": None, "dtype": dtype_name, "data": "synthetic",
                "config": {"workload": label + ", one HIP graph"},
                "loss": round(float(net.loss.item()), 4)}
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    phases = {"forward": 0.0, "backward": 0.0, "lars_step": 0.0}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ev[0].record()
        loss = net.forward(x, labels)
        ev[1].record()
        net.backward()
        ev[2].record()
        net.lars(0.001, 0.9, 1e-4, lr)
        ev[3].record()
        torch.cuda.synchronize()
        for k, (a, b) in zip(phases, ((0, 1), (1, 2), (2, 3))):
            phases[k] += ev[a].elapsed_time(ev[b])
    wall = time.perf_counter() - t0
    ms = wall * 1e3 / args.steps
    return {"metric": metric, "value": round(batch / (ms * 1e-3), 1), "unit": "images/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 3), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": dtype_name, "data": "synthetic",
            "config": {"workload": label},
            "phase_ms": {k: round(v / args.steps, 3) for k, v in phases.items()}, "loss": round(float(loss.item()), 4),
            "peak_memory_GB": round(torch.cuda.max_memory_allocated() / 1e9, 2)}


def run_batch_curve(args):
    """Images per second against the per-GPU batch (the paper's figure of per-GPU speed against batch size, "Benefits of
    Large-Batch Training": larger local batches make the matrix kernels more efficient): the headline step
    (convolutions + LARS) and the whole network step at every batch size of the list."""
    import copy
    import gc

    import torch

    points = []
    for b in (args.batches or [16, 32, 64, 128, 256, 512, 1024]):
        a = copy.copy(args)
        a.batch, a.steps, a.warmup, a.no_cpu, a.graph = b, 10, 5, True, False
        head = run_train_step(a)
        gc.collect()
        torch.cuda.empty_cache()
        point = {"batch": b, "conv_lars_images_per_s": head["value"], "conv_lars_ms": head["ms_per_step"],
                 "conv_tflops_all": head["conv_tflops_all"], "conv_frac_of_mfma_peak": head["conv_frac_of_mfma_peak"]}
        if args.dtype == "f32" and args.model != "alexnet":
            full = run_full_step(a)
            point.update({"whole_step_images_per_s": full["value"], "whole_step_ms": full["ms_per_step"]})
            gc.collect()
            torch.cuda.empty_cache()
        log(json.dumps(point))
        points.append(point)
    best = max(points, key=lambda p_: p_["conv_lars_images_per_s"])
    return {"batch_curve": args.model, "dtype": args.dtype, "layout": "NHWC", "points": points,
            "best_batch_conv_lars": best["batch"],
            "note": "the paper's M40 peaks at 512 images per GPU and runs out of memory at 1024"}


def run_copy_calibration(args):
    """A plain device-to-device copy of known size: what the FETCH_SIZE / WRITE_SIZE counters of rocprofv3 read
    for it gives the factor by which the counters of the other kernels are scaled."""
    import torch

    nbytes = 1 << 30
    src = torch.ones(nbytes // 4, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(args.iters):
        dst.copy_(src)
    torch.cuda.synchronize()
    return {"copy_calibration": True, "bytes_read_per_launch": nbytes, "bytes_written_per_launch": nbytes,
            "launches": args.iters, "kernel": "the elementwise copy kernel torch launches for Tensor.copy_"}


def add_secondary_measurements(res, args):
    """Beside the headline (convolutions + LARS of the step's layers): lars_step on rotating parameter sets (cold), and --
    for the default workload -- the whole network step with its glue layers and the bf16 form of the step, each a short
    run of its own after the timed region, so that one recorded line carries them all."""
    import copy
    import gc

    import torch

    def release():
        gc.collect()
        torch.cuda.empty_cache()

    release()
    cold = measure_lars(args.model, 4, 20)
    res["lars"]["cold"] = {"ms_median": cold["ms_median"], "ms_min": cold["ms_min"], "GBps": cold["GBps_median"],
                           "frac_of_hbm_peak": cold["frac_of_hbm_peak"], "rotating_sets": 4,
                           "note": "stand-alone on 4 rotating parameter sets: nothing in cache, and the previous call's "
                                   "dirty lines are written back while this one reads"}
    release()
    if args.dtype != "f32" or args.batch or args.model == "alexnet":
        return
    a = copy.copy(args)
    a.steps, a.warmup, a.graph, a.full_step = 5, 2, False, True
    full = run_full_step(a)
    res["whole_step"] = {"ms_per_step": full["ms_per_step"], "images_per_s": full["value"], "phase_ms": full["phase_ms"],
                         "steps": a.steps, "workload": full["config"]["workload"],
                         "note": "every layer of the network (batch norm, ReLU, pools, residual adds, classifier, loss) "
                                 "besides the convolutions and lars_step of the headline"}
    release()
    if args.model != "resnet50":
        return
    b = copy.copy(args)
    b.steps, b.warmup, b.dtype, b.no_cpu = 5, 2, "bf16", True
    bf = run_train_step(b)
    res["bf16_step"] = {"ms_per_step": bf["ms_per_step"], "images_per_s": bf["value"], "batch": 512, "steps": b.steps,
                        "conv_tflops": bf["conv_tflops"], "conv_tflops_all": bf["conv_tflops_all"],
                        "conv_frac_of_mfma_peak": bf["conv_frac_of_mfma_peak"], "roofline": bf["roofline"],
                        "lars_in_step": bf["lars"]["in_step"], "workload": bf["config"]["workload"]}
    release()
    c = copy.copy(args)
    c.steps, c.warmup, c.graph, c.full_step, c.dtype = 5, 2, False, True, "bf16"
    bfull = run_full_step(c)
    res["bf16_whole_step"] = {"ms_per_step": bfull["ms_per_step"], "images_per_s": bfull["value"], "batch": 512,
                              "phase_ms": bfull["phase_ms"], "steps": c.steps, "workload": bfull["config"]["workload"]}
    release()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--dtype", choices=["f32", "bf16"], default="f32",
                    help="bf16: BASELINE configs[4] (bf16 activations/weights, fp32 sums, fp32 master weights; batch 512)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--plain-norms", action="store_true",
                    help="conv2d_bwd_weight + lars_step instead of conv2d_bwd_weight_sq + lars_step_pre (the update reads every gradient twice)")
    ap.add_argument("--no-extras", action="store_true",
                    help="headline only: skip the cold lars_step, whole-step and bf16 legs that follow the timed region")
    ap.add_argument("--cpu-batch", type=int, default=4)
    ap.add_argument("--model", choices=["resnet50", "alexnet_bn", "alexnet"], default="resnet50",
                    help="network whose layer shapes and parameter list make the step (default: the metric's ResNet-50)")
    ap.add_argument("--sweep", action="store_true")
    ap.add_argument("--only", type=int, nargs="*", help="sweep: shape numbers to run")
    ap.add_argument("--iters", type=int, default=20, help="timed calls per measurement in the stand-alone modes (after 5 warm-up calls; median reported)")
    ap.add_argument("--lars", choices=["resnet50", "alexnet_bn", "alexnet"])
    ap.add_argument("--rotate", type=int, default=1)
    ap.add_argument("--batchnorm", action="store_true", help="batch-normalisation layers alone, GB/s against HBM peak")
    ap.add_argument("--full-step", action="store_true", help="the whole ResNet-50 step: all layers, loss, gradients, LARS")
    ap.add_argument("--no-join", action="store_true",
                    help="--full-step: the gradient at a block output and the batch-norm sums behind it as two plain calls")
    ap.add_argument("--no-fused-stats", action="store_true",
                    help="--full-step: batch norm sums its input itself instead of taking the sums from the convolution's epilogue")
    ap.add_argument("--no-pair", action="store_true",
                    help="with --full-step: the two batch norms at the output of a projection block as two plain passes")
    ap.add_argument("--no-grid-grads", action="store_true",
                    help="with --full-step: the input gradients of the strided 1x1 layers as full tensors (zeros between the grid pixels)")
    ap.add_argument("--no-side-stream", action="store_true",
                    help="with --full-step: the filter gradients on the main stream instead of a second one")
    ap.add_argument("--graph", action="store_true", help="--full-step: capture the step in a HIP graph and time replays")
    ap.add_argument("--copy-calib", action="store_true", help="run a 1 GiB device copy (counter calibration)")
    ap.add_argument("--batch-curve", action="store_true", help="images/s against the per-GPU batch (headline step and whole step)")
    ap.add_argument("--batches", type=int, nargs="*", help="--batch-curve: batch sizes (default 16 .. 1024)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the hot path built here has no multi-GPU part "
                 "(the gradient all-reduce between backward and lars_step is out of scope); run with --gpus 1")
    if args.copy_calib:
        res = run_copy_calibration(args)
    elif args.batch_curve:
        res = run_batch_curve(args)
    elif args.sweep:
        res = run_sweep(args)
    elif args.lars:
        res = run_lars(args)
    elif args.batchnorm:
        res = run_batchnorm(args)
    elif args.full_step:
        res = run_full_step(args)
    else:
        res = run_train_step(args)
        if not args.no_extras:
            add_secondary_measurements(res, args)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
