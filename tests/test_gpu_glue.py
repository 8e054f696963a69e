"""GPU parity of the glue layers (ReLU, 2x2 max pooling, global average pooling, bias, softmax cross-entropy)
through the C ABI against the numpy float64 definitions in oracle/tiny_cnn.py, in both layouts, and the tiny CNN
run END TO END on the device: every layer, forward and backward, and the LARS step, with nothing computed on the
host in between.  Tolerances: pooling and ReLU move values (exact, indices identical); averages, softmax and the
whole network <= 1e-4 tensor-scaled (fp32 on the device against float64)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import tiny_cnn
from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _dev(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a)).to(gu.DEV).to(dtype).contiguous()


def _lay(a, layout):      # NCHW numpy -> the layout under test
    return np.ascontiguousarray(a.transpose(0, 2, 3, 1)) if layout == lc.LC_NHWC else np.ascontiguousarray(a)


def _unlay(a, layout):
    return a.transpose(0, 3, 1, 2) if layout == lc.LC_NHWC else a


def _empty(shape, layout, dtype=torch.float32):
    n, c, h, w = shape
    return torch.empty((n, h, w, c) if layout == lc.LC_NHWC else shape, dtype=dtype, device=gu.DEV)


def test_relu_forward_and_backward():
    x = synth.normal((3, 5, 7, 11), 7000)
    x.reshape(-1)[::17] = 0.0                          # exact zeros take the "not positive" branch
    dy = synth.normal(x.shape, 7001)
    xd, dyd = _dev(x), _dev(dy)
    y, dx = torch.empty_like(xd), torch.empty_like(xd)
    lc.relu_fwd(xd, y, x.size)
    lc.relu_bwd(xd, dyd, dx, x.size)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(y.cpu().numpy(), tiny_cnn.relu(x.astype(np.float64)).astype(np.float32))
    np.testing.assert_array_equal(dx.cpu().numpy(), tiny_cnn.relu_bwd(x, dy).astype(np.float32))


@pytest.mark.parametrize("layout", [lc.LC_NCHW, lc.LC_NHWC], ids=["nchw", "nhwc"])
def test_maxpool_forward_indices_and_backward(layout):
    n, c, h, w = 3, 5, 8, 12
    x = synth.normal((n, c, h, w), 7100)
    x[0, 0, 0:2, 0:2] = 1.5                            # a four-way tie: the first element wins
    x[1, 2, 2:4, 4:6] = np.array([[0.0, 2.0], [2.0, -1.0]])   # a two-way tie: the earlier one wins
    dy = synth.normal((n, c, h // 2, w // 2), 7101)
    want_y, want_idx = tiny_cnn.maxpool2(x.astype(np.float64))
    xd = _dev(_lay(x, layout))
    y, idx = _empty((n, c, h // 2, w // 2), layout), _empty((n, c, h // 2, w // 2), layout, torch.uint8)
    lc.maxpool2x2_fwd(xd, y, idx, n, c, h, w, layout)
    dx = _empty((n, c, h, w), layout)
    dx.fill_(float("nan"))
    lc.maxpool2x2_bwd(_dev(_lay(dy, layout)), idx, dx, n, c, h, w, layout)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(_unlay(y.cpu().numpy(), layout), want_y.astype(np.float32))
    np.testing.assert_array_equal(_unlay(idx.cpu().numpy(), layout), want_idx.astype(np.uint8))
    assert want_idx[0, 0, 0, 0] == 0 and want_idx[1, 2, 1, 2] == 1
    np.testing.assert_array_equal(_unlay(dx.cpu().numpy(), layout), tiny_cnn.maxpool2_bwd(want_idx, dy.astype(np.float64), h, w).astype(np.float32))


@pytest.mark.parametrize("layout", [lc.LC_NCHW, lc.LC_NHWC], ids=["nchw", "nhwc"])
def test_global_average_pool_forward_and_backward(layout):
    # 63 pixels: less than a wave; a case with more; channel counts that are multiples of four (NHWC: four channels per thread)
    for (n, c, hh, ww, seed) in ((4, 33, 9, 7, 7200), (4, 33, 16, 16, 7210), (6, 2048, 7, 7, 7220), (3, 8, 5, 3, 7230), (2, 24, 1, 1, 7240)):
        x = synth.normal((n, c, hh, ww), seed)
        dy = synth.normal((n, c), seed + 1)
        y = torch.empty((n, c), device=gu.DEV)
        lc.global_avgpool_fwd(_dev(_lay(x, layout)), y, n, c, hh, ww, layout)
        dx = _empty((n, c, hh, ww), layout)
        lc.global_avgpool_bwd(_dev(dy), dx, n, c, hh, ww, layout)
        torch.cuda.synchronize()
        assert gu.scaled_err(y.cpu().numpy(), tiny_cnn.global_avgpool(x.astype(np.float64))) <= 1e-6
        assert gu.scaled_err(_unlay(dx.cpu().numpy(), layout), tiny_cnn.global_avgpool_bwd(dy.astype(np.float64), hh, ww)) <= 1e-6


@pytest.mark.parametrize("rows,k", [(37, 10), (512, 1000), (3, 70), (1, 5), (129, 64)])
def test_bias_add_and_bias_gradient(rows, k):
    y = synth.normal((rows, k), 7300)
    b = synth.normal((k,), 7301)
    yd = _dev(y)
    lc.bias_add(yd, _dev(b), rows, k)
    db = torch.empty(k, device=gu.DEV)
    lc.bias_grad(_dev(y), db, rows, k)
    torch.cuda.synchronize()
    np.testing.assert_allclose(yd.cpu().numpy(), y.astype(np.float64) + b, rtol=1e-6, atol=1e-7)
    assert gu.scaled_err(db.cpu().numpy(), y.astype(np.float64).sum(axis=0)) <= 1e-6


@pytest.mark.parametrize("n,k", [(16, 10), (5, 1000), (70, 3)])
def test_softmax_cross_entropy(n, k):
    logits = synth.normal((n, k), 7400 + k, std=3.0)
    labels = synth.uniform_int(n, 7401 + k, k)
    loss, d = torch.empty(1, device=gu.DEV), torch.empty((n, k), device=gu.DEV)
    lc.softmax_xent(_dev(logits), _dev(labels.astype(np.int32), torch.int32), loss, d, torch.empty(n, device=gu.DEV), n, k)
    torch.cuda.synchronize()
    want_loss, want_d = tiny_cnn.softmax_xent(logits.astype(np.float64), labels)
    assert abs(loss.item() - want_loss) <= 1e-5 * abs(want_loss)
    assert gu.scaled_err(d.cpu().numpy(), want_d) <= 1e-5
    assert abs(d.cpu().numpy().sum()) < 1e-5           # the gradient of every row sums to zero


def test_tiny_cnn_end_to_end_on_the_device():
    batch = 16
    x = synth.normal((batch, 3, 32, 32), 0x5EED0100)
    labels = synth.uniform_int(batch, 0x5EED0101, 10)
    params = {
        "w1": synth.normal((16, 3, 3, 3), 0x5EED0102, std=float(np.sqrt(2 / 27))),
        "w2": synth.normal((32, 16, 3, 3), 0x5EED0103, std=float(np.sqrt(2 / 144))),
        "wf": synth.normal((10, 32), 0x5EED0104, std=float(np.sqrt(2 / 32))),
        "bf": np.zeros(10, dtype=np.float32),
    }
    before = {k: v.copy() for k, v in params.items()}
    vel = {k: np.zeros_like(v) for k, v in params.items()}
    t = tiny_cnn.train_step(x, labels, params, vel, 0.001, 0.9, 5e-4, 1.0)   # the oracle's trace; updates params, vel

    # ReLU masks and pooling indices are decisions taken on fp32 activations that differ between the two sides by
    # rounding (~1e-7): the comparison below is meaningful because no decision of the oracle's trace is that close
    assert min(np.min(np.abs(t["a_c1"])), np.min(np.abs(t["a_c2"]))) > 2e-6
    r1 = t["a_r1"].reshape(batch, 16, 16, 2, 16, 2).transpose(0, 1, 2, 4, 3, 5).reshape(batch, 16, 16, 16, 4)
    top2 = np.sort(r1, axis=-1)[..., 2:]
    assert np.min((top2[..., 1] - top2[..., 0])[top2[..., 0] > 0]) > 2e-5

    L = lc.LC_NCHW
    d1 = gu.desc_for((batch, 3, 32, 32), (16, 3, 3, 3), 1, 1, L)
    d2 = gu.desc_for((batch, 16, 16, 16), (32, 16, 3, 3), 1, 1, L)
    df = gu.desc_for((batch, 32, 1, 1), (10, 32, 1, 1), 1, 0, L)
    ws = gu.workspace(max(lc.conv2d_workspace_bytes(d, p) for d in (d1, d2, df) for p in range(3)))
    E = lambda *shape: torch.empty(shape, device=gu.DEV)
    xd, lab = _dev(x), _dev(labels.astype(np.int32), torch.int32)
    w1, w2, wf, bf = (_dev(before[k]) for k in ("w1", "w2", "wf", "bf"))
    # forward
    a_c1, a_r1 = E(batch, 16, 32, 32), E(batch, 16, 32, 32)
    a_p1, i_p1 = E(batch, 16, 16, 16), torch.empty((batch, 16, 16, 16), dtype=torch.uint8, device=gu.DEV)
    a_c2, a_r2, a_gap, a_fc = E(batch, 32, 16, 16), E(batch, 32, 16, 16), E(batch, 32), E(batch, 10)
    lc.conv2d_fwd(d1, xd, w1, a_c1, ws)
    lc.relu_fwd(a_c1, a_r1, a_c1.numel())
    lc.maxpool2x2_fwd(a_r1, a_p1, i_p1, batch, 16, 32, 32, L)
    lc.conv2d_fwd(d2, a_p1, w2, a_c2, ws)
    lc.relu_fwd(a_c2, a_r2, a_c2.numel())
    lc.global_avgpool_fwd(a_r2, a_gap, batch, 32, 16, 16, L)
    lc.conv2d_fwd(df, a_gap, wf, a_fc, ws)
    lc.bias_add(a_fc, bf, batch, 10)
    loss, d_fc = E(1), E(batch, 10)
    lc.softmax_xent(a_fc, lab, loss, d_fc, E(batch), batch, 10)
    # backward
    d_wf, d_bf, d_gap = E(10, 32), E(10), E(batch, 32)
    d_r2, d_c2, d_w2, d_p1 = E(batch, 32, 16, 16), E(batch, 32, 16, 16), E(32, 16, 3, 3), E(batch, 16, 16, 16)
    d_r1, d_c1, d_w1 = E(batch, 16, 32, 32), E(batch, 16, 32, 32), E(16, 3, 3, 3)
    lc.conv2d_bwd_weight(df, a_gap, d_fc, d_wf, ws)
    lc.bias_grad(d_fc, d_bf, batch, 10)
    lc.conv2d_bwd_data(df, d_fc, wf, d_gap, ws)
    lc.global_avgpool_bwd(d_gap, d_r2, batch, 32, 16, 16, L)
    lc.relu_bwd(a_c2, d_r2, d_c2, d_c2.numel())
    lc.conv2d_bwd_weight(d2, a_p1, d_c2, d_w2, ws)
    lc.conv2d_bwd_data(d2, d_c2, w2, d_p1, ws)
    lc.maxpool2x2_bwd(d_p1, i_p1, d_r1, batch, 16, 32, 32, L)
    lc.relu_bwd(a_c1, d_r1, d_c1, d_c1.numel())
    lc.conv2d_bwd_weight(d1, xd, d_c1, d_w1, ws)
    # update
    w = [w1, w2, wf, bf]
    v = [torch.zeros_like(a) for a in w]
    args = lc.LarsArgs(w, [d_w1, d_w2, d_wf, d_bf], v)
    trust = E(4)
    lc.lars_step(args, 0.001, 0.9, 5e-4, 1.0, trust, gu.workspace(lc.lars_workspace_bytes(args.numel)))
    torch.cuda.synchronize()

    got = {"a_c1": a_c1, "a_r1": a_r1, "a_p1": a_p1, "a_c2": a_c2, "a_r2": a_r2, "a_gap": a_gap, "a_fc": a_fc, "d_fc": d_fc,
           "d_wf": d_wf, "d_bf": d_bf, "d_gap": d_gap, "d_r2": d_r2, "d_c2": d_c2, "d_w2": d_w2, "d_p1": d_p1, "d_r1": d_r1,
           "d_c1": d_c1, "d_w1": d_w1}
    for name, ten in got.items():
        err = gu.scaled_err(ten.cpu().numpy().reshape(t[name].shape), t[name])
        assert err <= TOL, (name, err)
    assert abs(loss.item() - float(t["loss"])) <= 1e-5 * float(t["loss"])
    tr = trust.cpu().numpy()
    assert np.all(np.abs(tr - t["trust"]) <= 1e-5 * t["trust"]), (tr, t["trust"])
    for i, k in enumerate(("w1", "w2", "wf", "bf")):
        assert gu.scaled_err(w[i].cpu().numpy().reshape(params[k].shape), params[k]) <= TOL, k
        if np.max(np.abs(vel[k])) > 0:
            assert gu.scaled_err(v[i].cpu().numpy().reshape(vel[k].shape), vel[k]) <= TOL, k


# ---------------------------------------------------------------- overlapping max pool, residual gradient
POOLS = {
    "resnet_stem_3x3_s2_p1": (2, 64, 16, 16, 3, 2, 1),
    "alexnet_3x3_s2_p0": (2, 6, 13, 13, 3, 2, 0),
    "ragged_3x3_s2_p1": (2, 5, 11, 9, 3, 2, 1),
    "odd_image_3x3_s2_p1_c8": (2, 8, 11, 9, 3, 2, 1),
    "odd_square_3x3_s2_p1_c12": (3, 12, 7, 7, 3, 2, 1),
    "one_pixel_3x3_s2_p1": (2, 4, 1, 1, 3, 2, 1),
    "one_row_3x3_s2_p1": (1, 4, 1, 6, 3, 2, 1),
    "stride1_3x3_p1": (1, 3, 7, 6, 3, 1, 1),
    "window2_stride2": (2, 4, 8, 6, 2, 2, 0),
    "window5_stride3_p2": (1, 2, 17, 14, 5, 3, 2),
}


@pytest.mark.parametrize("layout", [lc.LC_NCHW, lc.LC_NHWC], ids=["nchw", "nhwc"])
@pytest.mark.parametrize("name", list(POOLS))
def test_general_maxpool_forward_indices_and_backward(name, layout):
    from oracle import resnet as ores
    n, c, h, w, k, st, pd = POOLS[name]
    x = synth.normal((n, c, h, w), 7700)
    x[0, 0, 0:3, 0:3] = 2.5                             # ties inside and across windows: the first tap wins
    want_y, want_idx = ores.maxpool(x.astype(np.float64), k, st, pd)
    ph, pw = want_y.shape[2:]
    dy = synth.normal((n, c, ph, pw), 7701)
    xd = _dev(_lay(x, layout))
    y, idx = _empty((n, c, ph, pw), layout), _empty((n, c, ph, pw), layout, torch.uint8)
    dx = _empty((n, c, h, w), layout)
    dx.fill_(float("nan"))                              # every element must be written
    lc.maxpool_fwd(xd, y, idx, n, c, h, w, k, st, pd, layout)
    lc.maxpool_bwd(_dev(_lay(dy, layout)), idx, dx, n, c, h, w, k, st, pd, layout)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(_unlay(y.cpu().numpy(), layout), want_y.astype(np.float32))
    np.testing.assert_array_equal(_unlay(idx.cpu().numpy(), layout), want_idx.astype(np.uint8))
    want_dx = ores.maxpool_bwd(want_idx, dy.astype(np.float64), (h, w), k, st, pd)
    assert gu.scaled_err(_unlay(dx.cpu().numpy(), layout), want_dx) <= 1e-6       # at most four fp32 additions


def test_maxpool_3x3s2_gradient_is_the_same_in_both_layouts_bit_for_bit():
    """NHWC with four channels per thread takes one thread per 2x2 input patch for the 3x3 / stride 2 / padding 1 pool, NCHW
    one thread per input element; both add a pixel's windows in window order, so the sums are equal bit for bit."""
    from oracle import resnet as ores
    for (n, c, h, w, seed) in ((2, 64, 28, 28, 7750), (3, 8, 13, 10, 7751), (1, 4, 2, 3, 7752)):
        x = synth.normal((n, c, h, w), seed)
        _, idx_ref = ores.maxpool(x.astype(np.float64), 3, 2, 1)
        ph, pw = idx_ref.shape[2:]
        dy = synth.normal((n, c, ph, pw), seed + 10)
        res = {}
        for layout in (lc.LC_NCHW, lc.LC_NHWC):
            idx = _dev(_lay(idx_ref.astype(np.uint8), layout), torch.uint8)
            dx = _empty((n, c, h, w), layout)
            dx.fill_(float("nan"))
            lc.maxpool_bwd(_dev(_lay(dy, layout)), idx, dx, n, c, h, w, 3, 2, 1, layout)
            torch.cuda.synchronize()
            res[layout] = _unlay(dx.cpu().numpy(), layout)
        np.testing.assert_array_equal(res[lc.LC_NCHW], res[lc.LC_NHWC])
        assert np.all(np.isfinite(res[lc.LC_NHWC]))


def test_general_maxpool_with_window2_equals_the_2x2_pool():
    n, c, h, w = 2, 8, 12, 10
    xd = _dev(synth.normal((n, h, w, c), 7710))
    outs = []
    for general in (False, True):
        y = torch.empty((n, h // 2, w // 2, c), device=gu.DEV)
        idx = torch.empty((n, h // 2, w // 2, c), dtype=torch.uint8, device=gu.DEV)
        if general:
            lc.maxpool_fwd(xd, y, idx, n, c, h, w, 2, 2, 0, lc.LC_NHWC)
        else:
            lc.maxpool2x2_fwd(xd, y, idx, n, c, h, w, lc.LC_NHWC)
        torch.cuda.synchronize()
        outs.append((y.cpu().numpy(), idx.cpu().numpy()))
    np.testing.assert_array_equal(outs[0][0], outs[1][0])
    np.testing.assert_array_equal(outs[0][1], outs[1][1])


@pytest.mark.parametrize("count,two", [(4096 * 3, True), (4096 * 3, False), (1003, True), (7, False)])
def test_relu_add_bwd(count, two):
    y = synth.normal((count,), 7720)
    y[::13] = 0.0
    da, db = synth.normal((count,), 7721), synth.normal((count,), 7722)
    dx = torch.empty(count, device=gu.DEV)
    lc.relu_add_bwd(_dev(y), _dev(da), _dev(db) if two else None, dx, count)
    torch.cuda.synchronize()
    total = da.astype(np.float64) + (db.astype(np.float64) if two else 0.0)        # exact in float64
    np.testing.assert_array_equal(dx.cpu().numpy(), np.where(y > 0.0, total, 0.0).astype(np.float32))


def test_relu_add_bwd_without_mask_is_a_plain_sum():
    count = 4096 + 4
    da, db = synth.normal((count,), 7731), synth.normal((count,), 7732)
    dx = torch.empty(count, device=gu.DEV)
    lc.relu_add_bwd(None, _dev(da), _dev(db), dx, count)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(dx.cpu().numpy(), (da.astype(np.float64) + db.astype(np.float64)).astype(np.float32))
