"""The C-ABI library on a machine without a GPU: it loads, exports every function the header
declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import numpy as np

import pytest

from paper_1709_05011_amd import larsconv as lc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000000  # never dereferenced: every call below fails validation first


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "larsconv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"\b([a-z_0-9]+)\s*\([^;{]*\)\s*;", text)


def test_header_functions_are_exported():
    names = _declared_functions()
    assert set(names) == set(lc.EXPORTS)
    L = lc.lib()
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    assert lc.status_string(lc.LC_OK) == "ok"
    assert len({lc.status_string(i) for i in range(7)}) == 7
    assert lc.status_string(99) == "unknown status"


def test_out_shape_and_descriptor_validation():
    assert lc.conv2d_out_shape(lc.ConvDesc(1, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3)) == (112, 112)
    assert lc.conv2d_out_shape(lc.ConvDesc(1, 3, 227, 227, 96, 11, 11, 4, 4, 0, 0)) == (55, 55)
    assert lc.conv2d_out_shape(lc.ConvDesc(1, 256, 56, 56, 512, 1, 1, 2, 2, 0, 0)) == (28, 28)
    for bad in [lc.ConvDesc(0, 3, 8, 8, 4, 3, 3), lc.ConvDesc(1, 3, 8, 8, 4, 3, 3, 0, 1),
                lc.ConvDesc(1, 3, 8, 8, 4, 3, 3, 1, 1, -1, 0), lc.ConvDesc(1, 3, 2, 2, 4, 3, 3)]:
        with pytest.raises(lc.LarsConvError) as e:
            lc.conv2d_out_shape(bad)
        assert e.value.status == lc.LC_ERR_SHAPE
    with pytest.raises(lc.LarsConvError) as e:
        lc.conv2d_out_shape(lc.ConvDesc(1, 3, 8, 8, 4, 3, 3, dtype=7))
    assert e.value.status == lc.LC_ERR_UNSUPPORTED
    with pytest.raises(lc.LarsConvError) as e:
        lc.conv2d_out_shape(lc.ConvDesc(1, 3, 8, 8, 4, 3, 3, layout=2))
    assert e.value.status == lc.LC_ERR_UNSUPPORTED
    assert lc.lib().conv2d_out_shape(None, None, None) == lc.LC_ERR_NULL


def test_grouped_descriptor_validation():
    ok = lc.ConvDesc(2, 96, 27, 27, 256, 5, 5, 1, 1, 2, 2, groups=2)
    assert lc.conv2d_out_shape(ok) == (27, 27)
    assert lc.conv2d_out_shape(lc.ConvDesc(2, 96, 27, 27, 256, 5, 5, 1, 1, 2, 2, groups=0)) == (27, 27)       # 0 means 1
    for bad in [lc.ConvDesc(2, 96, 27, 27, 256, 5, 5, 1, 1, 2, 2, groups=5),      # does not divide c
                lc.ConvDesc(2, 96, 27, 27, 250, 5, 5, 1, 1, 2, 2, groups=4),      # does not divide k
                lc.ConvDesc(2, 96, 27, 27, 256, 5, 5, 1, 1, 2, 2, groups=-2)]:
        with pytest.raises(lc.LarsConvError) as e:
            lc.conv2d_out_shape(bad)
        assert e.value.status == lc.LC_ERR_SHAPE
        assert lc.conv2d_workspace_bytes(bad, lc.LC_PASS_FWD) == 0
    # a grouped call needs the slices of x and y plus the one-group call's scratch
    one = lc.ConvDesc(2, 48, 27, 27, 128, 5, 5, 1, 1, 2, 2)
    for p in (lc.LC_PASS_FWD, lc.LC_PASS_BWD_DATA, lc.LC_PASS_BWD_WEIGHT):
        need = lc.conv2d_workspace_bytes(ok, p)
        assert need >= 2 * 27 * 27 * (48 + 128) * 4 + lc.conv2d_workspace_bytes(one, p)
    L = lc.lib()
    P = ctypes.c_void_p(FAKE)
    d = ok.c_struct()
    need = lc.conv2d_workspace_bytes(ok, lc.LC_PASS_FWD)
    assert L.conv2d_fwd(ctypes.byref(d), None, P, P, P, need, None) == lc.LC_ERR_NULL
    assert L.conv2d_fwd(ctypes.byref(d), P, P, P, None, need, None) == lc.LC_ERR_WORKSPACE
    assert L.conv2d_fwd(ctypes.byref(d), P, P, P, P, need - 1, None) == lc.LC_ERR_WORKSPACE
    assert L.conv2d_bwd_data(ctypes.byref(d), P, ctypes.c_void_p(FAKE + 2), P, P, 1 << 40, None) == lc.LC_ERR_ALIGN
    assert L.conv2d_bwd_weight(ctypes.byref(d), P, P, None, P, 1 << 40, None) == lc.LC_ERR_NULL


def test_workspace_queries():
    nhwc = lc.ConvDesc(8, 64, 14, 14, 64, 3, 3, 1, 1, 1, 1)
    assert lc.conv2d_workspace_bytes(nhwc, lc.LC_PASS_FWD) % 256 == 0          # partial tiles of the stream-K blocks
    assert lc.conv2d_workspace_bytes(nhwc, lc.LC_PASS_BWD_DATA) >= 64 * 64 * 9 * 4
    assert lc.conv2d_workspace_bytes(nhwc, lc.LC_PASS_BWD_WEIGHT) % 256 == 0
    nchw = lc.ConvDesc(8, 64, 14, 14, 64, 3, 3, 1, 1, 1, 1, layout=lc.LC_NCHW)
    assert lc.conv2d_workspace_bytes(nchw, lc.LC_PASS_FWD) >= 2 * 8 * 64 * 14 * 14 * 4
    assert lc.conv2d_workspace_bytes(lc.ConvDesc(0, 1, 1, 1, 1, 1, 1), lc.LC_PASS_FWD) == 0
    assert lc.lars_workspace_bytes([64, 0, 5000]) > 0
    assert lc.lars_workspace_bytes([]) == 0
    assert lc.lars_workspace_bytes([-1]) == 0


@pytest.mark.parametrize("fn", [lc.conv2d_fwd, lc.conv2d_bwd_data, lc.conv2d_bwd_weight])
def test_conv_calls_reject_bad_arguments_before_launch(fn):
    d = lc.ConvDesc(2, 8, 9, 9, 8, 3, 3, 1, 1, 1, 1, layout=lc.LC_NCHW)   # needs a workspace in every pass

    def status(*args, **kw):
        with pytest.raises(lc.LarsConvError) as e:
            fn(*args, stream=0, **kw)
        return e.value.status

    assert status(d, None, FAKE, FAKE) == lc.LC_ERR_NULL
    assert status(d, FAKE, FAKE, None) == lc.LC_ERR_NULL
    assert status(d, FAKE + 2, FAKE, FAKE, FAKE, workspace_bytes=1 << 30) == lc.LC_ERR_ALIGN
    assert status(d, FAKE, FAKE, FAKE, None, workspace_bytes=0) == lc.LC_ERR_WORKSPACE
    assert status(d, FAKE, FAKE, FAKE, FAKE, workspace_bytes=16) == lc.LC_ERR_WORKSPACE
    assert status(d, FAKE, FAKE, FAKE, FAKE + 64, workspace_bytes=1 << 30) == lc.LC_ERR_WORKSPACE
    assert status(lc.ConvDesc(2, 8, 9, 9, 8, 3, 3, 1, 1, 1, 1, dtype=5), FAKE, FAKE, FAKE) == lc.LC_ERR_UNSUPPORTED
    assert status(lc.ConvDesc(2, 8, 2, 2, 8, 3, 3), FAKE, FAKE, FAKE) == lc.LC_ERR_SHAPE
    assert status(lc.ConvDesc(1 << 20, 8, 64, 64, 8, 3, 3), FAKE, FAKE, FAKE) == lc.LC_ERR_UNSUPPORTED  # > 2^31 rows


def test_lars_step_rejects_bad_arguments_before_launch():
    L = lc.lib()
    arr = (ctypes.c_void_p * 2)(FAKE, FAKE)
    odd = (ctypes.c_void_p * 2)(FAKE, FAKE + 2)
    null = (ctypes.c_void_p * 2)(FAKE, None)
    numel = (ctypes.c_int64 * 2)(100, 5000)
    neg = (ctypes.c_int64 * 2)(100, -5)

    def call(w, g, v, n, ws, ws_bytes, count=2):
        return L.lars_step(count, w, g, v, n, 0.001, 0.9, 5e-4, 1.0, None, None, ws, ws_bytes, None)

    assert call(arr, arr, arr, numel, FAKE, 1 << 20, count=-1) == lc.LC_ERR_SHAPE
    assert call(arr, arr, arr, numel, None, 0, count=0) == lc.LC_OK            # empty list: no-op
    assert call(None, arr, arr, numel, FAKE, 1 << 20) == lc.LC_ERR_NULL
    assert call(arr, null, arr, numel, FAKE, 1 << 20) == lc.LC_ERR_NULL
    assert call(arr, arr, arr, neg, FAKE, 1 << 20) == lc.LC_ERR_SHAPE
    assert call(arr, arr, odd, numel, FAKE, 1 << 20) == lc.LC_ERR_ALIGN
    assert call(arr, arr, arr, numel, None, 0) == lc.LC_ERR_WORKSPACE
    assert call(arr, arr, arr, numel, FAKE, 8) == lc.LC_ERR_WORKSPACE
    assert call(arr, arr, arr, numel, FAKE + 8, 1 << 20) == lc.LC_ERR_WORKSPACE


def test_index_division_constants_match_plain_division():
    # the kernels divide pixel indices by the output width and height with a multiply-high and a shift;
    # the library checks its constants against plain division for every divisor up to the argument
    L = lc.lib()
    L.lc_selftest_division.restype = ctypes.c_int
    L.lc_selftest_division.argtypes = [ctypes.c_int]
    assert L.lc_selftest_division(20000) == 0


def test_warmup_poly_lr_host_arithmetic_matches_oracle():
    import oracle
    base, start, W, T = 3.2, 0.1, 195, 3516
    for t in (0, 1, 97, 194, 195, 196, 1000, 3515, 3516, 4000):
        want = oracle.warmup_poly_lr(float(np.float32(base)), float(np.float32(start)), t, W, T, 2.0)
        assert abs(lc.lars_warmup_poly_lr(base, start, t, W, T, 2.0) - want) <= 1e-6 * max(want, 1e-3)
    assert lc.lars_warmup_poly_lr(base, start, 50, 0, T, 2.0) == lc.lars_poly_lr(base, 50, T, 2.0)


def test_lars_step_ex_rejects_bad_arguments_before_launch():
    L = lc.lib()
    arr = (ctypes.c_void_p * 2)(FAKE, FAKE)
    numel = (ctypes.c_int64 * 2)(100, 5000)
    eta = (ctypes.c_float * 2)(0.1, 0.2)
    skip = (ctypes.c_uint8 * 2)(0, 1)
    need = lc.lars_workspace_bytes([100, 5000])
    call = lambda w, ws, nb: L.lars_step_ex(2, w, arr, arr, numel, 0.001, 0.9, 5e-5, 1.0, eta, None, skip, None, None, ws, nb, None)
    assert call(None, ctypes.c_void_p(FAKE), need) == lc.LC_ERR_NULL
    assert call(arr, None, need) == lc.LC_ERR_WORKSPACE
    assert call(arr, ctypes.c_void_p(FAKE), need - 1) == lc.LC_ERR_WORKSPACE


def test_lars_step_ex_static_rejects_bad_arguments_before_launch():
    # the entry point on the library's own fixed scratch array: same checks, and a list beyond the array is refused
    L = lc.lib()
    arr = (ctypes.c_void_p * 2)(FAKE, FAKE)
    odd = (ctypes.c_void_p * 2)(FAKE + 2, FAKE)
    numel = (ctypes.c_int64 * 2)(100, 5000)
    call = lambda n, w, g, nm: L.lars_step_ex_static(n, w, g, arr, nm, 0.001, 0.9, 5e-5, 1.0, None, None, None, None, None, None)
    assert call(2, None, arr, numel) == lc.LC_ERR_NULL
    assert call(2, arr, arr, None) == lc.LC_ERR_NULL
    assert call(-1, arr, arr, numel) == lc.LC_ERR_SHAPE
    assert call(2, odd, arr, numel) == lc.LC_ERR_ALIGN
    assert call(0, None, None, None) == lc.LC_OK
    big = (ctypes.c_int64 * 2)(100, 600_000_000)
    assert lc.lars_workspace_bytes([100, 600_000_000]) > lc.LARS_STATIC_SCRATCH_BYTES
    assert call(2, arr, arr, big) == lc.LC_ERR_WORKSPACE
    text = open(os.path.join(ROOT, "include", "larsconv.h")).read()
    assert re.search(r"#define\s+LARS_STATIC_SCRATCH_BYTES\s+\(\(size_t\)2\s*<<\s*20\)", text) and lc.LARS_STATIC_SCRATCH_BYTES == 2 << 20


def test_norms_for_free_entry_points_reject_bad_arguments_before_launch():
    L = lc.lib()
    P = ctypes.c_void_p(FAKE)
    d = lc.ConvDesc(8, 64, 14, 14, 64, 3, 3, 1, 1, 1, 1)
    ds = d.c_struct()
    assert lc.conv2d_bwd_weight_sq_count(d) > 0
    assert lc.conv2d_bwd_weight_sq_count(lc.ConvDesc(0, 64, 14, 14, 64, 3, 3)) == 0
    need = lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT)
    assert L.conv2d_bwd_weight_sq(ctypes.byref(ds), P, P, P, None, P, need, None) == lc.LC_ERR_NULL
    assert L.conv2d_bwd_weight_sq(ctypes.byref(ds), P, P, P, ctypes.c_void_p(FAKE + 4), P, need, None) == lc.LC_ERR_ALIGN
    assert L.conv2d_bwd_weight_sq(ctypes.byref(ds), P, P, P, P, P, need - 1, None) == lc.LC_ERR_WORKSPACE
    arr = (ctypes.c_void_p * 2)(FAKE, FAKE)
    numel = (ctypes.c_int64 * 2)(100, 5000)
    need = lc.lars_workspace_bytes([100, 5000])
    pieces = (ctypes.c_void_p * 2)(FAKE, None)
    counts = (ctypes.c_int64 * 2)(10, 0)
    call = lambda pc, ct, ws, nb: L.lars_step_pre(2, arr, arr, arr, numel, 0.001, 0.9, 5e-5, 1.0, None, None, None, pc, ct, None, None, ws, nb, None)
    assert call(pieces, None, P, need) == lc.LC_ERR_NULL                 # the two arrays come together
    assert call(pieces, (ctypes.c_int64 * 2)(-1, 0), P, need) == lc.LC_ERR_SHAPE
    assert call((ctypes.c_void_p * 2)(FAKE + 4, None), counts, P, need) == lc.LC_ERR_ALIGN
    assert call(pieces, counts, None, need) == lc.LC_ERR_WORKSPACE
    assert call(pieces, counts, P, need - 1) == lc.LC_ERR_WORKSPACE


def test_glue_layers_reject_bad_arguments_before_launch():
    L = lc.lib()
    P = ctypes.c_void_p(FAKE)
    odd = ctypes.c_void_p(FAKE + 2)
    assert L.relu_fwd(None, P, 10, None) == lc.LC_ERR_NULL
    assert L.relu_fwd(P, odd, 10, None) == lc.LC_ERR_ALIGN
    assert L.relu_fwd(P, P, 0, None) == lc.LC_OK                       # nothing to do, nothing launched
    assert L.relu_bwd(P, None, P, 10, None) == lc.LC_ERR_NULL
    assert L.maxpool2x2_fwd(P, P, P, 2, 3, 5, 4, lc.LC_NCHW, None) == lc.LC_ERR_SHAPE      # odd height
    assert L.maxpool2x2_fwd(P, P, None, 2, 3, 4, 4, lc.LC_NCHW, None) == lc.LC_ERR_NULL
    assert L.maxpool2x2_bwd(P, P, P, 2, 3, 4, 4, 7, None) == lc.LC_ERR_UNSUPPORTED         # unknown layout
    assert L.global_avgpool_fwd(P, P, 0, 3, 4, 4, lc.LC_NHWC, None) == lc.LC_ERR_SHAPE
    assert L.global_avgpool_bwd(None, P, 1, 3, 4, 4, lc.LC_NHWC, None) == lc.LC_ERR_NULL
    assert L.bias_add(P, P, 5, 0, None) == lc.LC_ERR_SHAPE
    assert L.bias_grad(P, None, 5, 3, None) == lc.LC_ERR_NULL
    assert L.softmax_xent(P, P, P, P, None, 4, 10, None) == lc.LC_ERR_NULL
    assert L.softmax_xent(P, P, P, P, P, 4, 0, None) == lc.LC_ERR_SHAPE


def test_batchnorm_rejects_bad_arguments_before_launch():
    L = lc.lib()
    P = ctypes.c_void_p(FAKE)
    need = lc.batchnorm_workspace_bytes(4, 8, 5, 5, lc.LC_NHWC)
    assert need > 0 and need % 256 == 0
    assert lc.batchnorm_workspace_bytes(0, 8, 5, 5, lc.LC_NHWC) == 0
    assert lc.batchnorm_workspace_bytes(4, 8, 5, 5, 9) == 0
    fwd = lambda x, ws, nb, eps=1e-5, lay=lc.LC_NHWC, n=4: L.batchnorm_fwd(x, P, P, P, P, P, n, 8, 5, 5, eps, lay, ws, nb, None)
    assert fwd(None, P, need) == lc.LC_ERR_NULL
    assert fwd(P, None, need) == lc.LC_ERR_WORKSPACE
    assert fwd(P, P, need - 1) == lc.LC_ERR_WORKSPACE
    assert fwd(P, P, need, lay=5) == lc.LC_ERR_UNSUPPORTED
    assert fwd(P, P, need, n=0) == lc.LC_ERR_SHAPE
    assert fwd(P, P, need, eps=-1.0) == lc.LC_ERR_SHAPE
    assert fwd(ctypes.c_void_p(FAKE + 2), P, need) == lc.LC_ERR_ALIGN
    assert L.batchnorm_bwd(P, P, P, P, P, P, P, None, 4, 8, 5, 5, lc.LC_NHWC, P, need, None) == lc.LC_ERR_NULL
    assert L.batchnorm_bwd(P, P, P, P, P, P, P, P, 4, 8, 5, 5, lc.LC_NHWC, P, 0, None) == lc.LC_ERR_WORKSPACE


def test_fused_layers_reject_bad_arguments_before_launch():
    L = lc.lib()
    P = ctypes.c_void_p(FAKE)
    need = lc.batchnorm_workspace_bytes(4, 8, 5, 5, lc.LC_NHWC)
    # forward: the residual is optional, everything else is not
    assert L.batchnorm_fwd_ex(P, P, None, None, P, P, P, 4, 8, 5, 5, 1e-5, 1, lc.LC_NHWC, P, need, None) == lc.LC_ERR_NULL
    assert L.batchnorm_fwd_ex(P, P, P, ctypes.c_void_p(FAKE + 1), P, P, P, 4, 8, 5, 5, 1e-5, 1, lc.LC_NHWC, P, need, None) == lc.LC_ERR_ALIGN
    assert L.batchnorm_fwd_ex(P, P, P, None, P, P, P, 4, 8, 5, 5, 1e-5, 1, lc.LC_NHWC, P, need - 1, None) == lc.LC_ERR_WORKSPACE
    # backward through the ReLU needs beta; without the ReLU it may be missing (then the workspace check is reached)
    assert L.batchnorm_bwd_ex(P, P, P, None, P, P, P, P, P, 4, 8, 5, 5, 1, lc.LC_NHWC, P, need, None) == lc.LC_ERR_NULL
    assert L.batchnorm_bwd_ex(P, P, P, None, P, P, P, P, P, 4, 8, 5, 5, 0, lc.LC_NHWC, P, 0, None) == lc.LC_ERR_WORKSPACE
    # pools: window 1..15, pad below the window, the window must fit
    pool = lambda win, st, pd, h=9, lay=lc.LC_NHWC, x=P: L.maxpool_fwd(x, P, P, 2, 4, h, 9, win, st, pd, lay, None)
    assert pool(3, 2, 1, x=None) == lc.LC_ERR_NULL
    assert pool(0, 2, 0) == lc.LC_ERR_SHAPE
    assert pool(16, 2, 0) == lc.LC_ERR_SHAPE
    assert pool(3, 0, 1) == lc.LC_ERR_SHAPE
    assert pool(3, 2, 3) == lc.LC_ERR_SHAPE
    assert pool(5, 1, 0, h=3) == lc.LC_ERR_SHAPE
    assert pool(3, 2, 1, lay=4) == lc.LC_ERR_UNSUPPORTED
    assert L.maxpool_bwd(P, None, P, 2, 4, 9, 9, 3, 2, 1, lc.LC_NHWC, None) == lc.LC_ERR_NULL
    # gradient at a block's output: y or db may be missing, not both
    assert L.relu_add_bwd(None, P, None, P, 16, None) == lc.LC_ERR_NULL
    assert L.relu_add_bwd(P, None, P, P, 16, None) == lc.LC_ERR_NULL
    assert L.relu_add_bwd(P, P, P, ctypes.c_void_p(FAKE + 2), 16, None) == lc.LC_ERR_ALIGN
    assert L.relu_add_bwd(P, P, P, P, 0, None) == lc.LC_OK


def test_typed_layers_reject_bad_arguments_before_launch():
    """The `_t` entry points: an unknown storage type, and for bf16 anything but NHWC with whole 16-byte channel groups."""
    L = lc.lib()
    P = ctypes.c_void_p(FAKE)
    BF = lc.LC_BF16
    need = lc.batchnorm_workspace_bytes(4, 16, 5, 5, lc.LC_NHWC)
    fwd = lambda dt, c=16, lay=lc.LC_NHWC, x=P, nb=need: L.batchnorm_fwd_t(dt, x, P, P, None, P, P, P, 4, c, 5, 5, 1e-5, 1, lay, P, nb, None)
    assert fwd(2) == lc.LC_ERR_UNSUPPORTED
    assert fwd(BF, c=12) == lc.LC_ERR_UNSUPPORTED
    assert fwd(BF, lay=lc.LC_NCHW) == lc.LC_ERR_UNSUPPORTED
    assert fwd(BF, x=None) == lc.LC_ERR_NULL
    assert fwd(BF, x=ctypes.c_void_p(FAKE + 8)) == lc.LC_ERR_ALIGN          # bf16 tensors: 16-byte aligned
    assert fwd(BF, nb=need - 1) == lc.LC_ERR_WORKSPACE
    assert fwd(lc.LC_F32, nb=need - 1) == lc.LC_ERR_WORKSPACE               # fp32: the checks of batchnorm_fwd_ex
    bwd = lambda dt, beta=P, relu=1, c=16: L.batchnorm_bwd_t(dt, P, P, P, beta, P, P, P, P, P, 4, c, 5, 5, relu, lc.LC_NHWC, P, 0, None)
    assert bwd(BF, beta=None) == lc.LC_ERR_NULL
    assert bwd(BF, c=4) == lc.LC_ERR_UNSUPPORTED
    assert bwd(BF) == lc.LC_ERR_WORKSPACE
    assert bwd(3) == lc.LC_ERR_UNSUPPORTED
    pool = lambda dt, c=8, lay=lc.LC_NHWC, idx=P, win=3: L.maxpool_fwd_t(dt, P, P, idx, 2, c, 9, 9, win, 2, 1, lay, None)
    assert pool(BF, c=4) == lc.LC_ERR_UNSUPPORTED
    assert pool(BF, lay=lc.LC_NCHW) == lc.LC_ERR_UNSUPPORTED
    assert pool(BF, idx=None) == lc.LC_ERR_NULL
    assert pool(BF, idx=ctypes.c_void_p(FAKE + 4)) == lc.LC_ERR_ALIGN
    assert pool(BF, win=16) == lc.LC_ERR_SHAPE
    assert pool(9) == lc.LC_ERR_UNSUPPORTED
    assert L.maxpool_bwd_t(BF, P, P, None, 2, 8, 9, 9, 3, 2, 1, lc.LC_NHWC, None) == lc.LC_ERR_NULL
    assert L.maxpool_bwd_t(BF, P, P, P, 2, 8, 9, 9, 3, 2, 3, lc.LC_NHWC, None) == lc.LC_ERR_SHAPE
    assert L.relu_add_bwd_t(BF, None, P, None, P, 16, None) == lc.LC_ERR_NULL
    assert L.relu_add_bwd_t(BF, P, P, P, P, 12, None) == lc.LC_ERR_UNSUPPORTED
    assert L.relu_add_bwd_t(BF, P, P, P, ctypes.c_void_p(FAKE + 8), 16, None) == lc.LC_ERR_ALIGN
    assert L.relu_add_bwd_t(BF, P, P, P, P, 0, None) == lc.LC_OK
    assert L.relu_add_bwd_t(lc.LC_F32, None, P, None, P, 16, None) == lc.LC_ERR_NULL
    assert L.global_avgpool_fwd_t(BF, P, P, 2, 12, 4, 4, lc.LC_NHWC, None) == lc.LC_ERR_UNSUPPORTED
    assert L.global_avgpool_fwd_t(BF, P, None, 2, 16, 4, 4, lc.LC_NHWC, None) == lc.LC_ERR_NULL
    assert L.global_avgpool_bwd_t(BF, P, P, 0, 16, 4, 4, lc.LC_NHWC, None) == lc.LC_ERR_SHAPE
    assert L.global_avgpool_bwd_t(BF, P, P, 2, 16, 4, 4, lc.LC_NCHW, None) == lc.LC_ERR_UNSUPPORTED
    assert L.global_avgpool_bwd_t(4, P, P, 2, 16, 4, 4, lc.LC_NHWC, None) == lc.LC_ERR_UNSUPPORTED


def test_joined_block_gradient_rejects_bad_arguments_before_launch():
    L = lc.lib()
    P = ctypes.c_void_p(FAKE)
    need = lc.batchnorm_workspace_bytes(4, 16, 5, 5, lc.LC_NHWC)
    join = lambda dt=lc.LC_BF16, y=P, db=P, c=16, lay=lc.LC_NHWC, nb=need, xb=P: L.relu_add_bwd_bnsums_t(dt, y, P, db, P, xb, P, P, 4, c, 5, 5,
                                                                                                       lay, P, nb, None)
    assert join(y=None) == lc.LC_ERR_NULL                         # the mask is required here
    assert join(xb=None) == lc.LC_ERR_NULL
    assert join(db=None, nb=0) == lc.LC_ERR_WORKSPACE             # one gradient is fine: the workspace check is reached
    assert join(nb=0) == lc.LC_ERR_WORKSPACE
    assert join(c=12) == lc.LC_ERR_UNSUPPORTED                    # bf16: whole groups of eight channels
    assert join(dt=lc.LC_F32, c=6) == lc.LC_ERR_UNSUPPORTED       # fp32: the vector path only
    assert join(lay=lc.LC_NCHW) == lc.LC_ERR_UNSUPPORTED
    assert join(dt=7) == lc.LC_ERR_UNSUPPORTED
    assert join(xb=ctypes.c_void_p(FAKE + 8)) == lc.LC_ERR_ALIGN
    grid = lambda dt=lc.LC_BF16, y=P, st=2, c=16, lay=lc.LC_NHWC, nb=need: L.relu_add_bwd_bnsums_grid_t(dt, y, P, P, P, P, P, P, 4, c, 5, 5, st,
                                                                                                       lay, P, nb, None)
    assert grid(y=None) == lc.LC_ERR_NULL
    assert grid(st=0) == lc.LC_ERR_SHAPE                          # the gradients' stride is at least 1
    assert grid(st=-2) == lc.LC_ERR_SHAPE
    assert grid(nb=0) == lc.LC_ERR_WORKSPACE                      # a valid stride reaches the workspace check
    assert grid(st=1, nb=0) == lc.LC_ERR_WORKSPACE
    assert grid(c=12) == lc.LC_ERR_UNSUPPORTED
    assert grid(lay=lc.LC_NCHW) == lc.LC_ERR_UNSUPPORTED
    assert grid(dt=7) == lc.LC_ERR_UNSUPPORTED
    pre = lambda dt=lc.LC_BF16, c=16, lay=lc.LC_NHWC, nb=need, dy=P: L.batchnorm_bwd_presummed_t(dt, P, dy, P, P, P, P, P, P, 4, c, 5, 5, lay,
                                                                                                   P, nb, None)
    assert pre(dy=None) == lc.LC_ERR_NULL
    assert pre(c=12) == lc.LC_ERR_UNSUPPORTED
    assert pre(dt=lc.LC_F32, lay=lc.LC_NCHW) == lc.LC_ERR_UNSUPPORTED
    assert pre(nb=0) == lc.LC_ERR_WORKSPACE
    assert pre(dt=9) == lc.LC_ERR_UNSUPPORTED
def test_statistics_entry_points_reject_bad_arguments_before_launch():
    L = lc.lib()
    P = ctypes.c_void_p(FAKE)
    d = lc.ConvDesc(4, 64, 14, 14, 128, 3, 3, 1, 1, 1, 1, lc.LC_F32, lc.LC_NHWC)
    count = lc.conv2d_fwd_stats_count(d)
    assert count == 2 * ((4 * 14 * 14 + 127) // 128)                       # two half tiles of 128 rows each
    big = lc.ConvDesc(64, 128, 28, 28, 512, 1, 1, 1, 1, 0, 0, lc.LC_BF16, lc.LC_NHWC)
    assert lc.conv2d_fwd_stats_count(big) in (2 * ((64 * 28 * 28 + 255) // 256), 2 * ((64 * 28 * 28 + 127) // 128))
    assert lc.conv2d_fwd_stats_count(lc.ConvDesc(4, 64, 14, 14, 128, 3, 3, 1, 1, 1, 1, lc.LC_F32, lc.LC_NCHW)) == 0
    assert lc.conv2d_fwd_stats_count(lc.ConvDesc(4, 64, 14, 14, 128, 3, 3, 1, 1, 1, 1, lc.LC_F32, lc.LC_NHWC, groups=2)) == 0
    assert lc.conv2d_fwd_stats_count(lc.ConvDesc(0, 64, 14, 14, 128, 3, 3, 1, 1, 1, 1, lc.LC_F32, lc.LC_NHWC)) == 0
    cs = d.c_struct()
    need = lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD)
    call = lambda desc, st, y=P: L.conv2d_fwd_stats(ctypes.byref(desc), P, P, y, st, P, need, None)
    assert call(cs, None) == lc.LC_ERR_NULL
    assert call(cs, ctypes.c_void_p(FAKE + 4)) == lc.LC_ERR_ALIGN
    assert call(cs, P, y=None) == lc.LC_ERR_NULL
    nchw = lc.ConvDesc(4, 64, 14, 14, 128, 3, 3, 1, 1, 1, 1, lc.LC_F32, lc.LC_NCHW).c_struct()
    assert call(nchw, P) == lc.LC_ERR_UNSUPPORTED
    assert L.conv2d_fwd_stats(None, P, P, P, P, P, need, None) == lc.LC_ERR_NULL
    bneed = lc.batchnorm_workspace_bytes(4, 128, 14, 14, lc.LC_NHWC)
    pre = lambda st, tiles, lay=lc.LC_NHWC, dt=lc.LC_F32, nb=bneed: L.batchnorm_fwd_pre(dt, P, P, P, None, P, P, P, 4, 128, 14, 14, 1e-5, 1,
                                                                                     lay, st, tiles, P, nb, None)
    assert pre(None, count) == lc.LC_ERR_NULL
    assert pre(P, 0) == lc.LC_ERR_UNSUPPORTED
    assert pre(P, count, lay=lc.LC_NCHW) == lc.LC_ERR_UNSUPPORTED
    assert pre(ctypes.c_void_p(FAKE + 4), count) == lc.LC_ERR_ALIGN
    assert pre(P, count, dt=5) == lc.LC_ERR_UNSUPPORTED
    assert pre(P, count, nb=256) == lc.LC_ERR_WORKSPACE
    # the two batch norms of a projection block in one pass: every argument is checked before anything is launched
    def pair(x=P, x2=P, y=P, g2=P, st=None, tiles=0, st2=None, tiles2=0, lay=lc.LC_NHWC, dt=lc.LC_F32, nb=bneed, m2=P):
        return L.batchnorm_fwd_pair_t(dt, x, P, P, st, tiles, x2, g2, P, st2, tiles2, y, P, P, m2, P, 4, 128, 14, 14, 1e-5, 1, lay, P, nb, None)
    assert pair(x2=None) == lc.LC_ERR_NULL
    assert pair(y=None) == lc.LC_ERR_NULL
    assert pair(x=None) == lc.LC_ERR_NULL
    assert pair(g2=None) == lc.LC_ERR_NULL
    assert pair(m2=None) == lc.LC_ERR_NULL
    assert pair(dt=5) == lc.LC_ERR_UNSUPPORTED
    assert pair(nb=256) == lc.LC_ERR_WORKSPACE
    assert pair(st2=P, tiles2=0) == lc.LC_ERR_UNSUPPORTED                  # pieces without a count
    assert pair(st2=ctypes.c_void_p(FAKE + 4), tiles2=count) == lc.LC_ERR_ALIGN
    assert pair(st2=P, tiles2=count, lay=lc.LC_NCHW) == lc.LC_ERR_UNSUPPORTED
    assert pair(x2=ctypes.c_void_p(FAKE + 2)) == lc.LC_ERR_ALIGN


def test_poly_lr_host_arithmetic():
    assert lc.lars_poly_lr(1.0, 0, 3516) == 1.0
    assert lc.lars_poly_lr(1.0, 3516, 3516) == 0.0
    assert abs(lc.lars_poly_lr(1.0, 1000, 3516) - (1 - 1000 / 3516) ** 2) < 1e-7
    assert abs(lc.lars_poly_lr(0.2, 879, 3516) - 0.1125) < 1e-8


def test_binding_has_no_fallback(monkeypatch):
    monkeypatch.setattr(lc, "_lib", None)
    monkeypatch.setattr(lc, "LIB_PATH", "/nonexistent/liblarsconv.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        lc.lib()
