"""Pins for the residual-network oracle (oracle/resnet.py): max pool with overlapping windows and the whole
graph, against brute force, special cases, finite differences and torch's float64 autograd as a third opinion."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import resnet, tiny_cnn
from paper_1709_05011_amd import synth

MINI = resnet.Config(stem=(8, 3, 1, 1), widths=(4, 8), blocks=(2, 1), classes=10)
R50 = resnet.Config(stem=(64, 7, 2, 3), widths=(64, 128, 256, 512), blocks=(3, 4, 6, 3), classes=1000)


def _rand(shape, seed, std=1.0):
    return synth.normal(shape, seed, std).astype(np.float64)


# ------------------------------------------------------------------ max pool
@pytest.mark.parametrize("h,w,window,stride,pad", [(7, 6, 3, 2, 1), (9, 9, 3, 2, 0), (8, 8, 2, 2, 0), (5, 7, 3, 1, 1), (6, 6, 2, 1, 0)])
def test_maxpool_matches_element_loops(h, w, window, stride, pad):
    x = _rand((2, 3, h, w), 11 + h)
    y, idx = resnet.maxpool(x, window, stride, pad)
    ph, pw = (h + 2 * pad - window) // stride + 1, (w + 2 * pad - window) // stride + 1
    assert y.shape == (2, 3, ph, pw)
    for n in range(2):
        for c in range(3):
            for p in range(ph):
                for q in range(pw):
                    best, tap = None, None
                    for r in range(window):
                        for s in range(window):
                            ih, iw = p * stride - pad + r, q * stride - pad + s
                            if 0 <= ih < h and 0 <= iw < w and (best is None or x[n, c, ih, iw] > best):
                                best, tap = x[n, c, ih, iw], r * window + s
                    assert y[n, c, p, q] == best and idx[n, c, p, q] == tap


def test_maxpool_window2_stride2_is_the_tiny_cnn_pool():
    x = _rand((2, 4, 8, 6), 5)
    y, idx = resnet.maxpool(x, 2, 2, 0)
    y2, idx2 = tiny_cnn.maxpool2(x)
    assert np.array_equal(y, y2) and np.array_equal(idx, idx2)


def test_maxpool_ties_take_the_first_valid_tap():
    x = np.ones((1, 1, 6, 6))
    _, idx = resnet.maxpool(x, 3, 2, 1)
    assert idx[0, 0, 0, 0] == 4          # the corner window's first in-bounds tap is (1, 1)
    assert idx[0, 0, 0, 1] == 3          # top edge: row 0 is padding, column 0 is inside
    assert idx[0, 0, 1, 0] == 1          # left edge
    assert idx[0, 0, 1, 1] == 0


def test_maxpool_matches_torch_float64():
    x = _rand((2, 3, 11, 9), 21)
    y, _ = resnet.maxpool(x, 3, 2, 1)
    ref = F.max_pool2d(torch.from_numpy(x), 3, 2, 1).numpy()
    assert np.array_equal(y, ref)


def test_maxpool_bwd_conserves_and_matches_autograd():
    x = _rand((2, 3, 11, 9), 22)
    y, idx = resnet.maxpool(x, 3, 2, 1)
    dy = _rand(y.shape, 23)
    dx = resnet.maxpool_bwd(idx, dy, (11, 9), 3, 2, 1)
    assert abs(dx.sum() - dy.sum()) < 1e-12
    xt = torch.from_numpy(x).requires_grad_(True)
    F.max_pool2d(xt, 3, 2, 1).backward(torch.from_numpy(dy))
    assert np.allclose(dx, xt.grad.numpy(), rtol=0, atol=1e-14)


def test_maxpool_bwd_overlapping_windows_add():
    x = np.zeros((1, 1, 5, 5))
    x[0, 0, 1, 1] = 1.0                    # row 1 lies in the windows of outputs 0 (rows -1..1) and 1 (rows 1..3)
    y, idx = resnet.maxpool(x, 3, 2, 1)
    dy = np.arange(1.0, 1.0 + y.size).reshape(y.shape)
    dx = resnet.maxpool_bwd(idx, dy, (5, 5), 3, 2, 1)
    assert dx[0, 0, 1, 1] == dy[0, 0, 0, 0] + dy[0, 0, 0, 1] + dy[0, 0, 1, 0] + dy[0, 0, 1, 1]


# ------------------------------------------------------------------ structure
def test_resnet50_structure_matches_the_papers_counts():
    # "ImageNet training with ResNet-50": 25 M parameters; the model table's 25,557,032 in 161 tensors
    shapes = resnet.param_shapes(R50)
    assert len(shapes) == 161
    assert sum(int(np.prod(s)) for s in shapes.values()) == 25_557_032
    convs = resnet.conv_list(R50)
    assert len(convs) == 53
    ref = synth.resnet50_convs(1)
    ours = sorted((cin, k, r, st, pd) for _, cin, k, r, st, pd in convs)
    theirs = sorted((cs.c, cs.k, cs.r, cs.stride, cs.pad) for cs in ref)
    assert ours == theirs


# ------------------------------------------------------------------ whole graph
def _mini_problem(seed=3, batch=4, hw=16):
    shapes = resnet.param_shapes(MINI)
    params = {}
    for i, (name, shp) in enumerate(shapes.items()):
        if name.endswith(".gamma"):
            params[name] = (1.0 + 0.2 * synth.normal(shp, seed + i)).astype(np.float32)
        elif name.endswith(".beta") or name == "fc.b":
            params[name] = (0.2 * synth.normal(shp, seed + i)).astype(np.float32)
        else:
            fan = int(np.prod(shp[1:]))
            params[name] = synth.normal(shp, seed + i, std=(2.0 / fan) ** 0.5).astype(np.float32)
    x = synth.normal((batch, 3, hw, hw), seed + 1000).astype(np.float32)
    labels = synth.uniform_int(batch, seed + 2000, MINI.classes)
    return x, labels, params


def test_stored_trace_agrees_with_the_float64_forward():
    x, labels, params = _mini_problem()
    trace, _ = resnet.forward_backward(x, labels, params, MINI)
    assert abs(trace["loss"] - resnet.loss_only(x, labels, params, MINI)) < 1e-5


def test_gradients_match_directional_finite_differences():
    x, labels, params = _mini_problem(seed=7)
    _, grads = resnet.forward_backward(x, labels, params, MINI)
    assert set(grads) == set(params)
    for trial in range(3):
        direction = {k: synth.normal(v.shape, 900 + 31 * trial + i).astype(np.float64) for i, (k, v) in enumerate(params.items())}
        h = 1e-6
        plus = {k: params[k].astype(np.float64) + h * direction[k] for k in params}
        minus = {k: params[k].astype(np.float64) - h * direction[k] for k in params}
        fd = (resnet.loss_only(x, labels, plus, MINI) - resnet.loss_only(x, labels, minus, MINI)) / (2 * h)
        an = sum(float((grads[k] * direction[k]).sum()) for k in params)
        assert abs(fd - an) <= 2e-4 * max(abs(fd), abs(an), 1e-3), (trial, fd, an)


def test_single_parameter_finite_differences():
    x, labels, params = _mini_problem(seed=9)
    _, grads = resnet.forward_backward(x, labels, params, MINI)
    picks = [("stem.w", (2, 1, 0, 2)), ("s0b0.proj.w", (5, 3, 0, 0)), ("s0b1.c2.w", (1, 2, 1, 1)), ("s1b0.c1.gamma", (3,)),
             ("s1b0.c3.beta", (7,)), ("s0b0.c1.beta", (0,)), ("fc.w", (4, 9)), ("fc.b", (2,))]
    for name, where in picks:
        h = 1e-5
        plus = {k: v.astype(np.float64).copy() for k, v in params.items()}
        minus = {k: v.astype(np.float64).copy() for k, v in params.items()}
        plus[name][where] += h
        minus[name][where] -= h
        fd = (resnet.loss_only(x, labels, plus, MINI) - resnet.loss_only(x, labels, minus, MINI)) / (2 * h)
        an = float(grads[name][where])
        assert abs(fd - an) <= 1e-4 * max(abs(fd), abs(an)) + 1e-7, (name, fd, an)


def test_gradients_match_torch_autograd_float64():
    x, labels, params = _mini_problem(seed=13)
    _, grads = resnet.forward_backward(x, labels, params, MINI)
    tp = {k: torch.from_numpy(v.astype(np.float64)).requires_grad_(True) for k, v in params.items()}

    def cbn(a, name, stride, pad):
        z = F.conv2d(a, tp[name + ".w"], None, stride, pad)
        return F.batch_norm(z, None, None, tp[name + ".gamma"], tp[name + ".beta"], True, 0.0, MINI.eps)

    a = F.relu(cbn(torch.from_numpy(x.astype(np.float64)), "stem", MINI.stem[2], MINI.stem[3]))
    a = F.max_pool2d(a, 3, 2, 1)
    ch = MINI.stem[0]
    for si, (wd, nb) in enumerate(zip(MINI.widths, MINI.blocks)):
        for bi in range(nb):
            stride = 2 if (bi == 0 and si > 0) else 1
            name = f"s{si}b{bi}"
            sc = cbn(a, name + ".proj", stride, 0) if (ch != 4 * wd or stride != 1) else a
            b = F.relu(cbn(a, name + ".c1", stride, 0))
            b = F.relu(cbn(b, name + ".c2", 1, 1))
            a = F.relu(cbn(b, name + ".c3", 1, 0) + sc)
            ch = 4 * wd
    logits = a.mean(dim=(2, 3)) @ tp["fc.w"].T + tp["fc.b"]
    loss = F.cross_entropy(logits, torch.from_numpy(labels.astype(np.int64)))
    loss.backward()
    for k in params:
        ref = tp[k].grad.numpy()
        err = np.abs(grads[k] - ref).max() / max(np.abs(ref).max(), 1e-12)
        assert err < 2e-5, (k, err)


# ------------------------------------------------------------------ mixed precision (bf16 activations and filters)
def _is_bf16(a):
    return not np.any(np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) & np.uint32(0xFFFF))


def test_unstored_shortcut_changes_roundings_only():
    """pair=True hands the projection's batch-norm output on unrounded: in the float32 trace that moves the block outputs by
    float32 rounding at most, in the bf16 trace by a bf16 step at most and in a minority of elements; the projection's
    own trace entry is then the unrounded value, whose rounding is the stored one."""
    x, labels, params = _mini_problem(seed=23)
    t0, g0 = resnet.forward_backward(x, labels, params, MINI)
    t1, g1 = resnet.forward_backward(x, labels, params, MINI, pair=True)
    projs = [k[:-2] for k in t0 if k.endswith(".proj.a")]
    assert projs
    first = projs[0][:-len(".proj")]                                                          # (later blocks see changed inputs)
    assert np.array_equal(t0[first + ".proj.a"], t1[first + ".proj.a"].astype(np.float32))   # same value, stored or not
    for name in projs:
        blk = name[:-len(".proj")]
        d = np.abs(t0[blk + ".c3.a"] - t1[blk + ".c3.a"])
        assert d.max() <= 1e-5 * np.abs(t0[blk + ".c3.a"]).max()
    assert abs(t0["loss"] - t1["loss"]) <= 1e-6 * t0["loss"]
    b0, _ = resnet.forward_backward_bf16(x, labels, params, MINI)
    b1, _ = resnet.forward_backward_bf16(x, labels, params, MINI, pair=True)
    assert np.array_equal(b0[first + ".proj.z"], b1[first + ".proj.z"])
    assert np.array_equal(b0[first + ".proj.a"], oracle.round_to_bf16(b1[first + ".proj.a"]))
    a0, a1 = b0[first + ".c3.a"], b1[first + ".c3.a"]
    assert _is_bf16(a1) and 0.5 < np.mean(a0 == a1) < 1.0
    # the shortcut's value moves by half a bf16 step of its own size at most, the sum is then rounded once
    assert np.all(np.abs(a0 - a1) <= 2.0 ** -8 * np.abs(b1[first + ".proj.a"]) + 2.0 ** -7 * np.maximum(np.abs(a0), np.abs(a1)) + 1e-30)


def test_bf16_trace_stores_bf16_values_and_float32_parameter_gradients():
    x, labels, params = _mini_problem(seed=17)
    trace, grads = resnet.forward_backward_bf16(x, labels, params, MINI)
    stored = [k for k in trace if k.endswith((".z", ".a", ".dz", ".dx"))]
    assert len(stored) >= 4 * 5
    for k in stored:
        assert np.array_equal(trace[k], trace[k].astype(np.float32)) and _is_bf16(trace[k]), k
    assert not _is_bf16(grads["stem.w"]) and not _is_bf16(trace["logits"])           # these stay float32
    for k, g in grads.items():
        assert np.array_equal(g, g.astype(np.float32).astype(np.float64)), k
    # near the float32 trace, and not equal to it (a network this narrow, with 64 values per batch-norm channel
    # at the end, is sensitive: its gradients move by a fifth; the forward pass by a few per cent)
    t32, g32 = resnet.forward_backward(x, labels, params, MINI)
    assert 0.0 < abs(trace["loss"] - t32["loss"]) < 2e-2 * t32["loss"]
    assert 0.0 < np.linalg.norm(trace["logits"] - t32["logits"]) < 5e-2 * np.linalg.norm(t32["logits"])
    num = sum(float(((grads[k] - g32[k]) ** 2).sum()) for k in grads)
    den = sum(float((g32[k] ** 2).sum()) for k in grads)
    assert 0.0 < num < 0.5 ** 2 * den


@pytest.mark.parametrize("pair", [False, True], ids=["shortcut_stored", "shortcut_not_stored"])
def test_bf16_trace_matches_torch_with_rounding_at_the_same_places(pair):
    """An independent run of the same graph: torch float64 autograd, with torch's own bfloat16 cast applied (value
    replaced, gradient passed straight through) to every stored activation and to the filters, and a hook that
    rounds the gradient wherever the trace stores one.  The two differ only where float32 rounding of a stored
    gradient of a parameter moves a later value across a bf16 rounding boundary: isolated elements, one bf16 step.
    ``pair``: the projection's batch-norm output is not stored, so torch does not round it either."""
    x, labels, params = _mini_problem(seed=19)
    trace, grads = resnet.forward_backward_bf16(x, labels, params, MINI, pair=pair)
    tp = {k: torch.from_numpy(v.astype(np.float64)).requires_grad_(True) for k, v in params.items()}

    def rnd(t):
        return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)

    def store(t):                 # the value as stored (bf16), the gradient arriving at it rounded too
        u = t + (rnd(t) - t).detach()
        u.register_hook(rnd)
        return u

    def tap(t):                   # one consumer's view of a stored tensor: that consumer's gradient is stored rounded
        u = t * 1.0
        if u.requires_grad:       # the image itself has no gradient
            u.register_hook(rnd)
        return u

    seen = {}

    def cbn(a, name, stride, pad):
        wq = tp[name + ".w"] + (rnd(tp[name + ".w"]) - tp[name + ".w"]).detach()
        z = store(F.conv2d(tap(a), wq, None, stride, pad))
        seen[name + ".z"] = z
        return F.batch_norm(z, None, None, tp[name + ".gamma"], tp[name + ".beta"], True, 0.0, MINI.eps)

    a = store(F.relu(cbn(rnd(torch.from_numpy(x.astype(np.float64))), "stem", MINI.stem[2], MINI.stem[3])))
    a = store(F.max_pool2d(a, 3, 2, 1))
    ch = MINI.stem[0]
    for si, (wd, nb) in enumerate(zip(MINI.widths, MINI.blocks)):
        for bi in range(nb):
            stride = 2 if (bi == 0 and si > 0) else 1
            name = f"s{si}b{bi}"
            if ch != 4 * wd or stride != 1:
                sc = cbn(a, name + ".proj", stride, 0)
                sc = sc if pair else store(sc)
            else:
                sc = a
            b = store(F.relu(cbn(a, name + ".c1", stride, 0)))
            b = store(F.relu(cbn(b, name + ".c2", 1, 1)))
            a = store(F.relu(cbn(b, name + ".c3", 1, 0) + sc))
            seen[name + ".c3.a"] = a
            ch = 4 * wd
    logits = a.mean(dim=(2, 3)) @ tp["fc.w"].T + tp["fc.b"]
    loss = F.cross_entropy(logits, torch.from_numpy(labels.astype(np.int64)))
    loss.backward()
    assert abs(float(loss.detach()) - trace["loss"]) < 1e-3 * trace["loss"]
    for k, t in seen.items():
        same = np.mean(t.detach().numpy() == trace[k])
        assert same > 0.99, (k, same)
        assert np.abs(t.detach().numpy() - trace[k]).max() <= 2.0 ** -7 * np.abs(trace[k]).max(), k
    for k in params:
        ref = tp[k].grad.numpy()
        err = np.abs(grads[k] - ref).max() / max(np.abs(ref).max(), 1e-12)
        assert err < 1e-5, (k, err)
