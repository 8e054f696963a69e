"""Thin ctypes binding of liblarsconv.so: same names as the C ABI, argument marshalling only.

Every function takes objects exposing ``data_ptr()`` (torch tensors on the GPU) or plain integer
addresses, passes them through and raises :class:`LarsConvError` on a non-zero status.  Nothing is
computed here, and there is no fallback: if the HIP library has not been built, loading fails.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblarsconv.so")

LC_OK, LC_ERR_NULL, LC_ERR_SHAPE, LC_ERR_UNSUPPORTED, LC_ERR_WORKSPACE, LC_ERR_LAUNCH, LC_ERR_ALIGN = range(7)
LC_F32, LC_BF16 = 0, 1
LC_NCHW, LC_NHWC = 0, 1
LC_PASS_FWD, LC_PASS_BWD_DATA, LC_PASS_BWD_WEIGHT = 0, 1, 2

EXPORTS = ["conv2d_out_shape", "conv2d_workspace_bytes", "conv2d_fwd", "conv2d_bwd_data", "conv2d_bwd_weight",
           "conv2d_bwd_weight_sq_count", "conv2d_bwd_weight_sq",
           "lars_workspace_bytes", "lars_step", "lars_step_ex", "lars_step_pre", "lars_step_ex_static", "lars_poly_lr", "lars_warmup_poly_lr",
           "relu_fwd", "relu_bwd", "maxpool2x2_fwd", "maxpool2x2_bwd", "global_avgpool_fwd", "global_avgpool_bwd",
           "bias_add", "bias_grad", "softmax_xent", "maxpool_fwd", "maxpool_bwd", "relu_add_bwd",
           "batchnorm_workspace_bytes", "batchnorm_fwd", "batchnorm_bwd", "batchnorm_fwd_ex", "batchnorm_bwd_ex",
           "batchnorm_fwd_t", "batchnorm_bwd_t", "maxpool_fwd_t", "maxpool_bwd_t", "relu_add_bwd_t", "global_avgpool_fwd_t",
           "global_avgpool_bwd_t", "relu_add_bwd_bnsums_t", "relu_add_bwd_bnsums_grid_t", "batchnorm_bwd_presummed_t",
           "conv2d_fwd_stats_count", "conv2d_fwd_stats", "batchnorm_fwd_pre", "batchnorm_fwd_pair_t",
           "lc_status_string", "lc_last_error_detail"]


class LarsConvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = lib().lc_last_error_detail().decode() if status == LC_ERR_LAUNCH else ""
        super().__init__(f"{where}: {status_string(status)} (lc_status {status})" + (f": {detail}" if detail else ""))


class lc_conv_desc(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int) for f in
                ("n", "c", "h", "w", "k", "r", "s", "stride_h", "stride_w", "pad_h", "pad_w", "dtype", "layout", "groups")]


@dataclass(frozen=True)
class ConvDesc:
    n: int
    c: int
    h: int
    w: int
    k: int
    r: int
    s: int
    stride_h: int = 1
    stride_w: int = 1
    pad_h: int = 0
    pad_w: int = 0
    dtype: int = LC_F32
    layout: int = LC_NHWC
    groups: int = 1

    def c_struct(self) -> lc_conv_desc:
        return lc_conv_desc(self.n, self.c, self.h, self.w, self.k, self.r, self.s, self.stride_h, self.stride_w,
                            self.pad_h, self.pad_w, self.dtype, self.layout, self.groups)


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (run ``__graft_entry__.build()``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                               "(python -m paper_1709_05011_amd.build); there is no CPU fallback")
        # torch ships its own HIP runtime (same soname as the system one).  It must be the one in the
        # process before this library is loaded, or device pointers and streams handed over by torch
        # would belong to another runtime instance than the one the kernels are launched with.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        dp = ctypes.POINTER(lc_conv_desc)
        L.conv2d_out_shape.restype = i32
        L.conv2d_out_shape.argtypes = [dp, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.conv2d_workspace_bytes.restype = sz
        L.conv2d_workspace_bytes.argtypes = [dp, i32]
        for name in ("conv2d_fwd", "conv2d_bwd_data", "conv2d_bwd_weight"):
            fn = getattr(L, name)
            fn.restype = i32
            fn.argtypes = [dp, vp, vp, vp, vp, sz, vp]
        L.conv2d_bwd_weight_sq_count.restype = sz
        L.conv2d_bwd_weight_sq_count.argtypes = [dp]
        L.conv2d_bwd_weight_sq.restype = i32
        L.conv2d_bwd_weight_sq.argtypes = [dp, vp, vp, vp, vp, vp, sz, vp]
        L.lars_step_pre.restype = i32
        L.lars_step_pre.argtypes = [i32, vp, vp, vp, vp, ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                    vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.lars_workspace_bytes.restype = sz
        L.lars_workspace_bytes.argtypes = [i32, vp]
        L.lars_step.restype = i32
        L.lars_step.argtypes = [i32, vp, vp, vp, vp, ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                vp, vp, vp, sz, vp]
        L.lars_step_ex.restype = i32
        L.lars_step_ex.argtypes = [i32, vp, vp, vp, vp, ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                   vp, vp, vp, vp, vp, vp, sz, vp]
        L.lars_step_ex_static.restype = i32
        L.lars_step_ex_static.argtypes = [i32, vp, vp, vp, vp, ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                          vp, vp, vp, vp, vp, vp]
        L.lars_poly_lr.restype = ctypes.c_float
        L.lars_poly_lr.argtypes = [ctypes.c_float, ctypes.c_int64, ctypes.c_int64, ctypes.c_float]
        L.lars_warmup_poly_lr.restype = ctypes.c_float
        L.lars_warmup_poly_lr.argtypes = [ctypes.c_float, ctypes.c_float, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_float]
        L.relu_fwd.argtypes = [vp, vp, sz, vp]
        L.relu_bwd.argtypes = [vp, vp, vp, sz, vp]
        L.maxpool2x2_fwd.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp]
        L.maxpool2x2_bwd.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp]
        L.global_avgpool_fwd.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
        L.global_avgpool_bwd.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
        L.bias_add.argtypes = [vp, vp, sz, i32, vp]
        L.bias_grad.argtypes = [vp, vp, sz, i32, vp]
        L.softmax_xent.argtypes = [vp, vp, vp, vp, vp, i32, i32, vp]
        L.maxpool_fwd.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp]
        L.maxpool_bwd.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp]
        L.relu_add_bwd.argtypes = [vp, vp, vp, vp, sz, vp]
        for name in ("relu_fwd", "relu_bwd", "maxpool2x2_fwd", "maxpool2x2_bwd", "global_avgpool_fwd", "global_avgpool_bwd",
                     "bias_add", "bias_grad", "softmax_xent", "maxpool_fwd", "maxpool_bwd", "relu_add_bwd"):
            getattr(L, name).restype = i32
        L.batchnorm_workspace_bytes.restype = sz
        L.batchnorm_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
        L.batchnorm_fwd.restype = i32
        L.batchnorm_fwd.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, ctypes.c_float, i32, vp, sz, vp]
        L.batchnorm_bwd.restype = i32
        L.batchnorm_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, sz, vp]
        L.batchnorm_fwd_ex.restype = i32
        L.batchnorm_fwd_ex.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, ctypes.c_float, i32, i32, vp, sz, vp]
        L.batchnorm_bwd_ex.restype = i32
        L.batchnorm_bwd_ex.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, sz, vp]
        L.batchnorm_fwd_t.restype = i32
        L.batchnorm_fwd_t.argtypes = [i32] + L.batchnorm_fwd_ex.argtypes
        L.batchnorm_bwd_t.restype = i32
        L.batchnorm_bwd_t.argtypes = [i32] + L.batchnorm_bwd_ex.argtypes
        for name in ("maxpool_fwd", "maxpool_bwd", "relu_add_bwd", "global_avgpool_fwd", "global_avgpool_bwd"):
            fn = getattr(L, name + "_t")
            fn.restype = i32
            fn.argtypes = [i32] + getattr(L, name).argtypes
        L.relu_add_bwd_bnsums_t.restype = i32
        L.relu_add_bwd_bnsums_t.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, sz, vp]
        L.relu_add_bwd_bnsums_grid_t.restype = i32
        L.relu_add_bwd_bnsums_grid_t.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, sz, vp]
        L.batchnorm_bwd_presummed_t.restype = i32
        L.batchnorm_bwd_presummed_t.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, sz, vp]
        L.conv2d_fwd_stats_count.restype = sz
        L.conv2d_fwd_stats_count.argtypes = [dp]
        L.conv2d_fwd_stats.restype = i32
        L.conv2d_fwd_stats.argtypes = [dp, vp, vp, vp, vp, vp, sz, vp]
        L.batchnorm_fwd_pair_t.restype = i32
        L.batchnorm_fwd_pair_t.argtypes = [i32, vp, vp, vp, vp, sz, vp, vp, vp, vp, sz, vp, vp, vp, vp, vp, i32, i32, i32, i32, ctypes.c_float,
                                           i32, i32, vp, sz, vp]
        L.batchnorm_fwd_pre.restype = i32
        L.batchnorm_fwd_pre.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, ctypes.c_float, i32, i32, vp, sz, vp, sz, vp]
        L.lc_status_string.restype = ctypes.c_char_p
        L.lc_status_string.argtypes = [i32]
        L.lc_last_error_detail.restype = ctypes.c_char_p
        L.lc_last_error_detail.argtypes = []
        _lib = L
    return _lib


def _ptr(obj) -> Optional[int]:
    if obj is None:
        return None
    if hasattr(obj, "data_ptr"):
        return obj.data_ptr() or None
    return int(obj) or None


def _nbytes(ws) -> int:
    if ws is None:
        return 0
    return ws.numel() * ws.element_size()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if hasattr(stream, "cuda_stream"):
        return stream.cuda_stream or None
    return int(stream) or None


def _desc(desc) -> lc_conv_desc:
    return desc.c_struct() if isinstance(desc, ConvDesc) else desc


def _check(status: int, where: str) -> None:
    if status != LC_OK:
        raise LarsConvError(status, where)


def status_string(status: int) -> str:
    return lib().lc_status_string(status).decode()


lc_status_string = status_string


def lc_last_error_detail() -> str:
    return lib().lc_last_error_detail().decode()


def conv2d_out_shape(desc):
    p, q = ctypes.c_int(), ctypes.c_int()
    _check(lib().conv2d_out_shape(ctypes.byref(_desc(desc)), ctypes.byref(p), ctypes.byref(q)), "conv2d_out_shape")
    return p.value, q.value


def conv2d_workspace_bytes(desc, pass_: int) -> int:
    return int(lib().conv2d_workspace_bytes(ctypes.byref(_desc(desc)), pass_))


def conv2d_fwd(desc, x, w, y, workspace=None, stream=None, workspace_bytes: Optional[int] = None) -> None:
    nb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().conv2d_fwd(ctypes.byref(_desc(desc)), _ptr(x), _ptr(w), _ptr(y), _ptr(workspace), nb, _stream(stream)),
           "conv2d_fwd")


def conv2d_bwd_data(desc, dy, w, dx, workspace=None, stream=None, workspace_bytes: Optional[int] = None) -> None:
    nb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().conv2d_bwd_data(ctypes.byref(_desc(desc)), _ptr(dy), _ptr(w), _ptr(dx), _ptr(workspace), nb,
                                 _stream(stream)), "conv2d_bwd_data")


def conv2d_bwd_weight(desc, x, dy, dw, workspace=None, stream=None, workspace_bytes: Optional[int] = None) -> None:
    nb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().conv2d_bwd_weight(ctypes.byref(_desc(desc)), _ptr(x), _ptr(dy), _ptr(dw), _ptr(workspace), nb,
                                   _stream(stream)), "conv2d_bwd_weight")


def conv2d_bwd_weight_sq_count(desc) -> int:
    return int(lib().conv2d_bwd_weight_sq_count(ctypes.byref(_desc(desc))))


def conv2d_bwd_weight_sq(desc, x, dy, dw, dw_sq_pieces, workspace=None, stream=None, workspace_bytes: Optional[int] = None) -> None:
    nb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().conv2d_bwd_weight_sq(ctypes.byref(_desc(desc)), _ptr(x), _ptr(dy), _ptr(dw), _ptr(dw_sq_pieces), _ptr(workspace),
                                      nb, _stream(stream)), "conv2d_bwd_weight_sq")


def _i64_array(vals: Sequence[int]):
    return (ctypes.c_int64 * max(len(vals), 1))(*vals)


def _ptr_array(objs: Sequence):
    return (ctypes.c_void_p * max(len(objs), 1))(*[_ptr(o) for o in objs])


def lars_workspace_bytes(numel: Sequence[int]) -> int:
    return int(lib().lars_workspace_bytes(len(numel), _i64_array(list(numel))))


class LarsArgs:
    """Host-side pointer and size arrays of one parameter list, marshalled once and reusable."""

    def __init__(self, w: Sequence, g: Sequence, v: Sequence, numel: Optional[Sequence[int]] = None,
                 w_lowp: Optional[Sequence] = None):
        if numel is None:
            numel = [t.numel() for t in w]
        self.n = len(w)
        self.numel = list(numel)
        self.w, self.g, self.v = _ptr_array(w), _ptr_array(g), _ptr_array(v)
        self.numel_arr = _i64_array(self.numel)
        self.w_lowp = _ptr_array(w_lowp) if w_lowp is not None else None
        self._keep = (list(w), list(g), list(v), list(w_lowp) if w_lowp is not None else None)


def lars_step(args: LarsArgs, eta: float, momentum: float, weight_decay: float, lr: float, trust_out=None,
              workspace=None, stream=None, workspace_bytes: Optional[int] = None) -> None:
    nb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().lars_step(args.n, args.w, args.g, args.v, args.numel_arr, eta, momentum, weight_decay, lr,
                           _ptr(trust_out), args.w_lowp, _ptr(workspace), nb, _stream(stream)), "lars_step")


def _per_tensor_arrays(args: "LarsArgs", eta_per_tensor, weight_decay_per_tensor, skip):
    def farr(a):
        if a is None:
            return None
        if len(a) != args.n:
            raise ValueError("per-tensor array of the wrong length")
        return (ctypes.c_float * max(args.n, 1))(*[float(x) for x in a])
    if skip is not None and len(skip) != args.n:
        raise ValueError("skip list of the wrong length")
    sk = None if skip is None else (ctypes.c_uint8 * max(args.n, 1))(*[1 if x else 0 for x in skip])
    return farr(eta_per_tensor), farr(weight_decay_per_tensor), sk


def lars_step_ex(args: LarsArgs, eta: float, momentum: float, weight_decay: float, lr: float, eta_per_tensor=None,
                 weight_decay_per_tensor=None, skip=None, trust_out=None, workspace=None, stream=None,
                 workspace_bytes: Optional[int] = None) -> None:
    """lars_step with per-tensor coefficients (sequences of floats or None) and a skip list (sequence of 0/1 or None)."""
    e, b, sk = _per_tensor_arrays(args, eta_per_tensor, weight_decay_per_tensor, skip)
    nb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().lars_step_ex(args.n, args.w, args.g, args.v, args.numel_arr, eta, momentum, weight_decay, lr, e, b, sk,
                              _ptr(trust_out), args.w_lowp, _ptr(workspace), nb, _stream(stream)), "lars_step_ex")


def lars_step_pre(args: LarsArgs, eta: float, momentum: float, weight_decay: float, lr: float, g_sq_pieces: Sequence,
                  g_sq_counts: Sequence[int], eta_per_tensor=None, weight_decay_per_tensor=None, skip=None, trust_out=None,
                  workspace=None, stream=None, workspace_bytes: Optional[int] = None) -> None:
    """lars_step_ex with sum g^2 of some tensors handed over in pieces (None / 0 entries: computed from g)."""
    if len(g_sq_pieces) != args.n or len(g_sq_counts) != args.n:
        raise ValueError("per-tensor array of the wrong length")
    e, b, sk = _per_tensor_arrays(args, eta_per_tensor, weight_decay_per_tensor, skip)
    nb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().lars_step_pre(args.n, args.w, args.g, args.v, args.numel_arr, eta, momentum, weight_decay, lr, e, b, sk,
                               _ptr_array(g_sq_pieces), _i64_array([int(c) for c in g_sq_counts]), _ptr(trust_out), args.w_lowp,
                               _ptr(workspace), nb, _stream(stream)), "lars_step_pre")


LARS_STATIC_SCRATCH_BYTES = 2 << 20


def lars_step_ex_static(args: LarsArgs, eta: float, momentum: float, weight_decay: float, lr: float, eta_per_tensor=None,
                        weight_decay_per_tensor=None, skip=None, trust_out=None, stream=None) -> None:
    """lars_step_ex on the library's own fixed scratch array (no workspace argument, nothing allocated)."""
    e, b, sk = _per_tensor_arrays(args, eta_per_tensor, weight_decay_per_tensor, skip)
    _check(lib().lars_step_ex_static(args.n, args.w, args.g, args.v, args.numel_arr, eta, momentum, weight_decay, lr, e, b, sk,
                                     _ptr(trust_out), args.w_lowp, _stream(stream)), "lars_step_ex_static")


def lars_poly_lr(base_lr: float, it: int, max_iter: int, power: float = 2.0) -> float:
    return float(lib().lars_poly_lr(base_lr, it, max_iter, power))


def lars_warmup_poly_lr(base_lr: float, start_lr: float, it: int, warmup_iters: int, max_iter: int, power: float = 2.0) -> float:
    return float(lib().lars_warmup_poly_lr(base_lr, start_lr, it, warmup_iters, max_iter, power))


# ---- glue layers of the small whole-path network (argument marshalling only) ----

def relu_fwd(x, y, count: int, stream=None) -> None:
    _check(lib().relu_fwd(_ptr(x), _ptr(y), count, _stream(stream)), "relu_fwd")


def relu_bwd(x, dy, dx, count: int, stream=None) -> None:
    _check(lib().relu_bwd(_ptr(x), _ptr(dy), _ptr(dx), count, _stream(stream)), "relu_bwd")


def maxpool2x2_fwd(x, y, idx, n: int, c: int, h: int, w: int, layout: int, stream=None) -> None:
    _check(lib().maxpool2x2_fwd(_ptr(x), _ptr(y), _ptr(idx), n, c, h, w, layout, _stream(stream)), "maxpool2x2_fwd")


def maxpool2x2_bwd(dy, idx, dx, n: int, c: int, h: int, w: int, layout: int, stream=None) -> None:
    _check(lib().maxpool2x2_bwd(_ptr(dy), _ptr(idx), _ptr(dx), n, c, h, w, layout, _stream(stream)), "maxpool2x2_bwd")


def global_avgpool_fwd(x, y, n: int, c: int, h: int, w: int, layout: int, stream=None) -> None:
    _check(lib().global_avgpool_fwd(_ptr(x), _ptr(y), n, c, h, w, layout, _stream(stream)), "global_avgpool_fwd")


def global_avgpool_bwd(dy, dx, n: int, c: int, h: int, w: int, layout: int, stream=None) -> None:
    _check(lib().global_avgpool_bwd(_ptr(dy), _ptr(dx), n, c, h, w, layout, _stream(stream)), "global_avgpool_bwd")


def bias_add(y, b, rows: int, k: int, stream=None) -> None:
    _check(lib().bias_add(_ptr(y), _ptr(b), rows, k, _stream(stream)), "bias_add")


def bias_grad(dy, db, rows: int, k: int, stream=None) -> None:
    _check(lib().bias_grad(_ptr(dy), _ptr(db), rows, k, _stream(stream)), "bias_grad")


def softmax_xent(logits, labels, loss, dlogits, row_scratch, n: int, k: int, stream=None) -> None:
    _check(lib().softmax_xent(_ptr(logits), _ptr(labels), _ptr(loss), _ptr(dlogits), _ptr(row_scratch), n, k, _stream(stream)),
           "softmax_xent")


def maxpool_fwd(x, y, idx, n: int, c: int, h: int, w: int, window: int, stride: int, pad: int, layout: int, stream=None) -> None:
    _check(lib().maxpool_fwd(_ptr(x), _ptr(y), _ptr(idx), n, c, h, w, window, stride, pad, layout, _stream(stream)), "maxpool_fwd")


def maxpool_bwd(dy, idx, dx, n: int, c: int, h: int, w: int, window: int, stride: int, pad: int, layout: int, stream=None) -> None:
    _check(lib().maxpool_bwd(_ptr(dy), _ptr(idx), _ptr(dx), n, c, h, w, window, stride, pad, layout, _stream(stream)), "maxpool_bwd")


def relu_add_bwd(y, da, db, dx, count: int, stream=None) -> None:
    _check(lib().relu_add_bwd(_ptr(y), _ptr(da), _ptr(db), _ptr(dx), count, _stream(stream)), "relu_add_bwd")


# ---- batch normalisation (training mode) ----

def batchnorm_workspace_bytes(n: int, c: int, h: int, w: int, layout: int) -> int:
    return int(lib().batchnorm_workspace_bytes(n, c, h, w, layout))


def batchnorm_fwd(x, gamma, beta, y, save_mean, save_invstd, n: int, c: int, h: int, w: int, eps: float, layout: int,
                  workspace=None, stream=None) -> None:
    _check(lib().batchnorm_fwd(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(save_mean), _ptr(save_invstd), n, c, h, w, eps,
                               layout, _ptr(workspace), _nbytes(workspace), _stream(stream)), "batchnorm_fwd")


def batchnorm_bwd(x, dy, gamma, save_mean, save_invstd, dx, dgamma, dbeta, n: int, c: int, h: int, w: int, layout: int,
                  workspace=None, stream=None) -> None:
    _check(lib().batchnorm_bwd(_ptr(x), _ptr(dy), _ptr(gamma), _ptr(save_mean), _ptr(save_invstd), _ptr(dx), _ptr(dgamma),
                               _ptr(dbeta), n, c, h, w, layout, _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "batchnorm_bwd")


def batchnorm_fwd_ex(x, gamma, beta, residual, y, save_mean, save_invstd, n: int, c: int, h: int, w: int, eps: float, relu: bool,
                     layout: int, workspace=None, stream=None) -> None:
    _check(lib().batchnorm_fwd_ex(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(residual), _ptr(y), _ptr(save_mean), _ptr(save_invstd),
                                  n, c, h, w, eps, int(bool(relu)), layout, _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "batchnorm_fwd_ex")


def batchnorm_bwd_ex(x, dy, gamma, beta, save_mean, save_invstd, dx, dgamma, dbeta, n: int, c: int, h: int, w: int, relu: bool,
                     layout: int, workspace=None, stream=None) -> None:
    _check(lib().batchnorm_bwd_ex(_ptr(x), _ptr(dy), _ptr(gamma), _ptr(beta), _ptr(save_mean), _ptr(save_invstd), _ptr(dx),
                                  _ptr(dgamma), _ptr(dbeta), n, c, h, w, int(bool(relu)), layout, _ptr(workspace),
                                  _nbytes(workspace), _stream(stream)), "batchnorm_bwd_ex")


# ---- the same layers with the storage type as an argument (LC_BF16: NHWC, channels a multiple of 8) ----

def batchnorm_fwd_t(dtype: int, x, gamma, beta, residual, y, save_mean, save_invstd, n: int, c: int, h: int, w: int, eps: float,
                    relu: bool, layout: int, workspace=None, stream=None) -> None:
    _check(lib().batchnorm_fwd_t(dtype, _ptr(x), _ptr(gamma), _ptr(beta), _ptr(residual), _ptr(y), _ptr(save_mean),
                                 _ptr(save_invstd), n, c, h, w, eps, int(bool(relu)), layout, _ptr(workspace), _nbytes(workspace),
                                 _stream(stream)), "batchnorm_fwd_t")


def batchnorm_bwd_t(dtype: int, x, dy, gamma, beta, save_mean, save_invstd, dx, dgamma, dbeta, n: int, c: int, h: int, w: int,
                    relu: bool, layout: int, workspace=None, stream=None) -> None:
    _check(lib().batchnorm_bwd_t(dtype, _ptr(x), _ptr(dy), _ptr(gamma), _ptr(beta), _ptr(save_mean), _ptr(save_invstd), _ptr(dx),
                                 _ptr(dgamma), _ptr(dbeta), n, c, h, w, int(bool(relu)), layout, _ptr(workspace),
                                 _nbytes(workspace), _stream(stream)), "batchnorm_bwd_t")


def maxpool_fwd_t(dtype: int, x, y, idx, n: int, c: int, h: int, w: int, window: int, stride: int, pad: int, layout: int,
                  stream=None) -> None:
    _check(lib().maxpool_fwd_t(dtype, _ptr(x), _ptr(y), _ptr(idx), n, c, h, w, window, stride, pad, layout, _stream(stream)),
           "maxpool_fwd_t")


def maxpool_bwd_t(dtype: int, dy, idx, dx, n: int, c: int, h: int, w: int, window: int, stride: int, pad: int, layout: int,
                  stream=None) -> None:
    _check(lib().maxpool_bwd_t(dtype, _ptr(dy), _ptr(idx), _ptr(dx), n, c, h, w, window, stride, pad, layout, _stream(stream)),
           "maxpool_bwd_t")


def relu_add_bwd_t(dtype: int, y, da, db, dx, count: int, stream=None) -> None:
    _check(lib().relu_add_bwd_t(dtype, _ptr(y), _ptr(da), _ptr(db), _ptr(dx), count, _stream(stream)), "relu_add_bwd_t")


def global_avgpool_fwd_t(dtype: int, x, y, n: int, c: int, h: int, w: int, layout: int, stream=None) -> None:
    _check(lib().global_avgpool_fwd_t(dtype, _ptr(x), _ptr(y), n, c, h, w, layout, _stream(stream)), "global_avgpool_fwd_t")


def global_avgpool_bwd_t(dtype: int, dy, dx, n: int, c: int, h: int, w: int, layout: int, stream=None) -> None:
    _check(lib().global_avgpool_bwd_t(dtype, _ptr(dy), _ptr(dx), n, c, h, w, layout, _stream(stream)), "global_avgpool_bwd_t")


# ---- the gradient at a block's output together with the sums of the batch-norm backward pass behind it ----

def relu_add_bwd_bnsums_t(dtype: int, y, da, db, dx, x_bn, save_mean, save_invstd, n: int, c: int, h: int, w: int, layout: int,
                          workspace=None, stream=None) -> None:
    _check(lib().relu_add_bwd_bnsums_t(dtype, _ptr(y), _ptr(da), _ptr(db), _ptr(dx), _ptr(x_bn), _ptr(save_mean), _ptr(save_invstd),
                                       n, c, h, w, layout, _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "relu_add_bwd_bnsums_t")


def relu_add_bwd_bnsums_grid_t(dtype: int, y, da, db, dx, x_bn, save_mean, save_invstd, n: int, c: int, h: int, w: int, grad_stride: int,
                               layout: int, workspace=None, stream=None) -> None:
    _check(lib().relu_add_bwd_bnsums_grid_t(dtype, _ptr(y), _ptr(da), _ptr(db), _ptr(dx), _ptr(x_bn), _ptr(save_mean),
                                            _ptr(save_invstd), n, c, h, w, grad_stride, layout, _ptr(workspace), _nbytes(workspace),
                                            _stream(stream)),
           "relu_add_bwd_bnsums_grid_t")


def batchnorm_bwd_presummed_t(dtype: int, x, dy, gamma, save_mean, save_invstd, dx, dgamma, dbeta, n: int, c: int, h: int, w: int,
                              layout: int, workspace=None, stream=None) -> None:
    _check(lib().batchnorm_bwd_presummed_t(dtype, _ptr(x), _ptr(dy), _ptr(gamma), _ptr(save_mean), _ptr(save_invstd), _ptr(dx),
                                           _ptr(dgamma), _ptr(dbeta), n, c, h, w, layout, _ptr(workspace), _nbytes(workspace),
                                           _stream(stream)), "batchnorm_bwd_presummed_t")
# ---- batch-norm statistics out of the convolution's epilogue ----

def conv2d_fwd_stats_count(desc) -> int:
    return int(lib().conv2d_fwd_stats_count(ctypes.byref(_desc(desc))))


def conv2d_fwd_stats(desc, x, w, y, stats, workspace=None, stream=None, workspace_bytes: Optional[int] = None) -> None:
    nb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().conv2d_fwd_stats(ctypes.byref(_desc(desc)), _ptr(x), _ptr(w), _ptr(y), _ptr(stats), _ptr(workspace), nb,
                                  _stream(stream)), "conv2d_fwd_stats")


def batchnorm_fwd_pair_t(dtype: int, x, gamma, beta, stats, stats_tiles: int, x2, gamma2, beta2, stats2, stats_tiles2: int, y, save_mean,
                         save_invstd, save_mean2, save_invstd2, n: int, c: int, h: int, w: int, eps: float, relu: bool, layout: int,
                         workspace, stream=None) -> None:
    _check(lib().batchnorm_fwd_pair_t(dtype, _ptr(x), _ptr(gamma), _ptr(beta), _ptr(stats), stats_tiles, _ptr(x2), _ptr(gamma2), _ptr(beta2),
                                      _ptr(stats2), stats_tiles2, _ptr(y), _ptr(save_mean), _ptr(save_invstd), _ptr(save_mean2),
                                      _ptr(save_invstd2), n, c, h, w, eps, int(bool(relu)), layout, _ptr(workspace), _nbytes(workspace),
                                      _stream(stream)), "batchnorm_fwd_pair_t")


def batchnorm_fwd_pre(dtype: int, x, gamma, beta, residual, y, save_mean, save_invstd, n: int, c: int, h: int, w: int, eps: float,
                      relu: bool, layout: int, stats, stats_tiles: int, workspace=None, stream=None) -> None:
    _check(lib().batchnorm_fwd_pre(dtype, _ptr(x), _ptr(gamma), _ptr(beta), _ptr(residual), _ptr(y), _ptr(save_mean),
                                   _ptr(save_invstd), n, c, h, w, eps, int(bool(relu)), layout, _ptr(stats), stats_tiles,
                                   _ptr(workspace), _nbytes(workspace), _stream(stream)), "batchnorm_fwd_pre")
