"""CPU oracle (test infrastructure only): ctypes front end of ``oracle.c``.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares nothing with the HIP library
and never imports it.  See the header of ``oracle.c`` for what each function
computes and which passage of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

NCHW, NHWC = 0, 1


def build(force: bool = False) -> str:
    """Compile ``oracle.c`` with gcc (plain -O2, OpenMP across independent outputs only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Conv(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int) for f in
                ("n", "c", "h", "w", "k", "r", "s", "stride_h", "stride_w", "pad_h", "pad_w", "layout")]


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_poly_lr.restype = ctypes.c_double
        _lib.oracle_poly_lr.argtypes = [ctypes.c_double, ctypes.c_int64, ctypes.c_int64, ctypes.c_double]
        _lib.oracle_threads.restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(_load().oracle_threads())


def set_threads(t: int) -> None:
    _load().oracle_set_threads(ctypes.c_int(t))


def _desc(n, c, h, w, k, r, s, stride, pad, layout) -> _Conv:
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    return _Conv(n, c, h, w, k, r, s, sh, sw, ph, pw, layout)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _fp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def out_shape(h, w, r, s, stride, pad) -> Tuple[int, int]:
    d = _desc(1, 1, h, w, 1, r, s, stride, pad, NCHW)
    p, q = ctypes.c_int(), ctypes.c_int()
    if _load().oracle_conv2d_out_shape(ctypes.byref(d), ctypes.byref(p), ctypes.byref(q)) != 0:
        raise ValueError("invalid convolution shape")
    return p.value, q.value


def _dims(x_shape, w_shape, layout):
    if layout == NCHW:
        n, c, h, w = x_shape
        k, c2, r, s = w_shape
    else:
        n, h, w, c = x_shape
        k, r, s, c2 = w_shape
    if c != c2:
        raise ValueError("channel mismatch")
    return n, c, h, w, k, r, s


def _act_shape(n, c, h, w, layout):
    return (n, c, h, w) if layout == NCHW else (n, h, w, c)


def conv2d_fwd(x, wt, stride=1, pad=0, layout=NCHW) -> np.ndarray:
    """Forward convolution; returns float64 Y in the same layout."""
    x, wt = _f32(x), _f32(wt)
    n, c, h, w, k, r, s = _dims(x.shape, wt.shape, layout)
    d = _desc(n, c, h, w, k, r, s, stride, pad, layout)
    p, q = out_shape(h, w, r, s, (d.stride_h, d.stride_w), (d.pad_h, d.pad_w))
    y = np.empty(_act_shape(n, k, p, q, layout), dtype=np.float64)
    _load().oracle_conv2d_fwd(ctypes.byref(d), _fp(x), _fp(wt), _fp(y))
    return y


def conv2d_bwd_data(dy, wt, x_hw: Tuple[int, int], stride=1, pad=0, layout=NCHW) -> np.ndarray:
    """Gradient wrt the input of height/width ``x_hw``; returns float64 dX."""
    dy, wt = _f32(dy), _f32(wt)
    h, w = x_hw
    if layout == NCHW:
        n, k, p, q = dy.shape
        k2, c, r, s = wt.shape
    else:
        n, p, q, k = dy.shape
        k2, r, s, c = wt.shape
    d = _desc(n, c, h, w, k, r, s, stride, pad, layout)
    if k != k2 or (p, q) != out_shape(h, w, r, s, (d.stride_h, d.stride_w), (d.pad_h, d.pad_w)):
        raise ValueError("dy shape does not match")
    dx = np.empty(_act_shape(n, c, h, w, layout), dtype=np.float64)
    _load().oracle_conv2d_bwd_data(ctypes.byref(d), _fp(dy), _fp(wt), _fp(dx))
    return dx


def conv2d_bwd_weight(x, dy, rs: Tuple[int, int], stride=1, pad=0, layout=NCHW) -> np.ndarray:
    """Gradient wrt the filter of window ``rs``; returns float64 dW."""
    x, dy = _f32(x), _f32(dy)
    r, s = rs
    if layout == NCHW:
        n, c, h, w = x.shape
        n2, k, p, q = dy.shape
        wshape = (k, c, r, s)
    else:
        n, h, w, c = x.shape
        n2, p, q, k = dy.shape
        wshape = (k, r, s, c)
    d = _desc(n, c, h, w, k, r, s, stride, pad, layout)
    if n != n2 or (p, q) != out_shape(h, w, r, s, (d.stride_h, d.stride_w), (d.pad_h, d.pad_w)):
        raise ValueError("dy shape does not match")
    dw = np.empty(wshape, dtype=np.float64)
    _load().oracle_conv2d_bwd_weight(ctypes.byref(d), _fp(x), _fp(dy), _fp(dw))
    return dw


def _at(fn, d, a, b, coords):
    coords = np.ascontiguousarray(coords, dtype=np.int32)
    assert coords.ndim == 2 and coords.shape[1] == 4
    out = np.empty(coords.shape[0], dtype=np.float64)
    mag = np.empty(coords.shape[0], dtype=np.float64)
    fn(ctypes.byref(d), _fp(a), _fp(b), _fp(coords), ctypes.c_int64(coords.shape[0]), _fp(out), _fp(mag))
    return out, mag


def conv2d_fwd_at(x, wt, coords, stride=1, pad=0, layout=NCHW):
    """Y at ``coords`` rows (n,k,p,q); returns (values, sum of |terms|)."""
    x, wt = _f32(x), _f32(wt)
    n, c, h, w, k, r, s = _dims(x.shape, wt.shape, layout)
    return _at(_load().oracle_conv2d_fwd_at, _desc(n, c, h, w, k, r, s, stride, pad, layout), x, wt, coords)


def conv2d_bwd_data_at(dy, wt, x_hw, coords, stride=1, pad=0, layout=NCHW):
    """dX at ``coords`` rows (n,c,h,w)."""
    dy, wt = _f32(dy), _f32(wt)
    h, w = x_hw
    if layout == NCHW:
        n, k = dy.shape[0], dy.shape[1]
        _, c, r, s = wt.shape
    else:
        n, k = dy.shape[0], dy.shape[3]
        _, r, s, c = wt.shape
    return _at(_load().oracle_conv2d_bwd_data_at, _desc(n, c, h, w, k, r, s, stride, pad, layout), dy, wt, coords)


def conv2d_bwd_weight_at(x, dy, rs, coords, stride=1, pad=0, layout=NCHW):
    """dW at ``coords`` rows (k,c,r,s)."""
    x, dy = _f32(x), _f32(dy)
    r, s = rs
    if layout == NCHW:
        n, c, h, w = x.shape
        k = dy.shape[1]
    else:
        n, h, w, c = x.shape
        k = dy.shape[3]
    return _at(_load().oracle_conv2d_bwd_weight_at, _desc(n, c, h, w, k, r, s, stride, pad, layout), x, dy, coords)


def _grouped(fn: str, groups: int, d, a, b, out) -> None:
    _load()
    f = getattr(_lib, fn)
    f.restype = None
    f(ctypes.byref(d), ctypes.c_int(groups), _fp(a), _fp(b), _fp(out))


def conv2d_fwd_grouped(x, wt, groups: int, stride=1, pad=0, layout=NCHW) -> np.ndarray:
    """Grouped forward convolution: x has c channels, wt is [k][c/groups][r][s] (NHWC: [k][r][s][c/groups])."""
    x, wt = _f32(x), _f32(wt)
    if layout == NCHW:
        n, c, h, w = x.shape
        k, cg, r, s = wt.shape
    else:
        n, h, w, c = x.shape
        k, r, s, cg = wt.shape
    if groups < 1 or c % groups or k % groups or cg * groups != c:
        raise ValueError("groups must divide both channel counts and match the filter")
    d = _desc(n, c, h, w, k, r, s, stride, pad, layout)
    p, q = out_shape(h, w, r, s, (d.stride_h, d.stride_w), (d.pad_h, d.pad_w))
    y = np.empty(_act_shape(n, k, p, q, layout), dtype=np.float64)
    _grouped("oracle_conv2d_fwd_grouped", groups, d, x, wt, y)
    return y


def conv2d_bwd_data_grouped(dy, wt, groups: int, x_hw: Tuple[int, int], stride=1, pad=0, layout=NCHW) -> np.ndarray:
    dy, wt = _f32(dy), _f32(wt)
    h, w = x_hw
    if layout == NCHW:
        n, k, p, q = dy.shape
        k2, cg, r, s = wt.shape
    else:
        n, p, q, k = dy.shape
        k2, r, s, cg = wt.shape
    c = cg * groups
    d = _desc(n, c, h, w, k, r, s, stride, pad, layout)
    if groups < 1 or k != k2 or k % groups or (p, q) != out_shape(h, w, r, s, (d.stride_h, d.stride_w), (d.pad_h, d.pad_w)):
        raise ValueError("dy shape does not match")
    dx = np.empty(_act_shape(n, c, h, w, layout), dtype=np.float64)
    _grouped("oracle_conv2d_bwd_data_grouped", groups, d, dy, wt, dx)
    return dx


def conv2d_bwd_weight_grouped(x, dy, groups: int, rs: Tuple[int, int], stride=1, pad=0, layout=NCHW) -> np.ndarray:
    x, dy = _f32(x), _f32(dy)
    r, s = rs
    if layout == NCHW:
        n, c, h, w = x.shape
        n2, k, p, q = dy.shape
    else:
        n, h, w, c = x.shape
        n2, p, q, k = dy.shape
    if groups < 1 or c % groups or k % groups:
        raise ValueError("groups must divide both channel counts")
    cg = c // groups
    wshape = (k, cg, r, s) if layout == NCHW else (k, r, s, cg)
    d = _desc(n, c, h, w, k, r, s, stride, pad, layout)
    if n != n2 or (p, q) != out_shape(h, w, r, s, (d.stride_h, d.stride_w), (d.pad_h, d.pad_w)):
        raise ValueError("dy shape does not match")
    dw = np.empty(wshape, dtype=np.float64)
    _grouped("oracle_conv2d_bwd_weight_grouped", groups, d, x, dy, dw)
    return dw


def lars_step(w: Sequence[np.ndarray], g: Sequence[np.ndarray], v: Sequence[np.ndarray],
              eta: float, momentum: float, weight_decay: float, lr: float):
    """One LARS step over a list of tensors.  ``w`` and ``v`` (float32, contiguous) are updated
    in place.  Returns (trust ratios float64 [L], norms float64 [L,2] = (||w||, ||g||) before the step)."""
    L = len(w)
    for a in list(w) + list(v):
        if a.dtype != np.float32 or not a.flags["C_CONTIGUOUS"] or not a.flags["WRITEABLE"]:
            raise ValueError("w and v must be writable contiguous float32 arrays")
    g = [_f32(a) for a in g]
    numel = np.array([a.size for a in w], dtype=np.int64)
    if any(a.size != b.size or a.size != c.size for a, b, c in zip(w, g, v)):
        raise ValueError("size mismatch")
    arr = ctypes.c_void_p * max(L, 1)
    wp = arr(*[a.ctypes.data for a in w])
    gp = arr(*[a.ctypes.data for a in g])
    vp = arr(*[a.ctypes.data for a in v])
    trust = np.empty(L, dtype=np.float64)
    norms = np.empty((L, 2), dtype=np.float64)
    _load().oracle_lars_step(ctypes.c_int(L), wp, gp, vp, _fp(numel), ctypes.c_double(eta),
                             ctypes.c_double(momentum), ctypes.c_double(weight_decay), ctypes.c_double(lr),
                             _fp(trust), _fp(norms))
    return trust, norms


def lars_step_ex(w: Sequence[np.ndarray], g: Sequence[np.ndarray], v: Sequence[np.ndarray],
                 eta: float, momentum: float, weight_decay: float, lr: float,
                 eta_per_tensor=None, wd_per_tensor=None, skip=None):
    """lars_step with per-tensor trust coefficients / weight decays (None = the scalar) and a skip list
    (tensors that take trust ratio 1).  Returns (trust ratios, norms) like lars_step."""
    L = len(w)
    for a in list(w) + list(v):
        if a.dtype != np.float32 or not a.flags["C_CONTIGUOUS"] or not a.flags["WRITEABLE"]:
            raise ValueError("w and v must be writable contiguous float32 arrays")
    g = [_f32(a) for a in g]
    numel = np.array([a.size for a in w], dtype=np.int64)
    if any(a.size != b.size or a.size != c.size for a, b, c in zip(w, g, v)):
        raise ValueError("size mismatch")
    arr = ctypes.c_void_p * max(L, 1)
    wp = arr(*[a.ctypes.data for a in w])
    gp = arr(*[a.ctypes.data for a in g])
    vp = arr(*[a.ctypes.data for a in v])
    trust = np.empty(L, dtype=np.float64)
    norms = np.empty((L, 2), dtype=np.float64)
    e = None if eta_per_tensor is None else np.ascontiguousarray(eta_per_tensor, dtype=np.float64)
    b = None if wd_per_tensor is None else np.ascontiguousarray(wd_per_tensor, dtype=np.float64)
    s = None if skip is None else np.ascontiguousarray(skip, dtype=np.uint8)
    for a in (e, b, s):
        if a is not None and a.size != L:
            raise ValueError("per-tensor array of the wrong length")
    lib = _load()
    lib.oracle_lars_step_ex.restype = None
    lib.oracle_lars_step_ex(ctypes.c_int(L), wp, gp, vp, _fp(numel), ctypes.c_double(eta), ctypes.c_double(momentum),
                            ctypes.c_double(weight_decay), ctypes.c_double(lr),
                            None if e is None else _fp(e), None if b is None else _fp(b), None if s is None else _fp(s),
                            _fp(trust), _fp(norms))
    return trust, norms


def poly_lr(base_lr: float, it: int, max_iter: int, power: float = 2.0) -> float:
    return float(_load().oracle_poly_lr(base_lr, it, max_iter, power))


def warmup_poly_lr(base_lr: float, start_lr: float, it: int, warmup_iters: int, max_iter: int, power: float = 2.0) -> float:
    lib = _load()
    lib.oracle_warmup_poly_lr.restype = ctypes.c_double
    lib.oracle_warmup_poly_lr.argtypes = [ctypes.c_double, ctypes.c_double, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_double]
    return float(lib.oracle_warmup_poly_lr(base_lr, start_lr, it, warmup_iters, max_iter, power))


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Oracle-side rounding of a float64/float32 result to the nearest bf16 value (ties to even),
    returned as float32.  Written with Python integer arithmetic on the bit pattern."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    low = bits & np.uint64(0xFFFF)
    keep = bits >> np.uint64(16)
    up = (low > np.uint64(0x8000)) | ((low == np.uint64(0x8000)) & ((keep & np.uint64(1)) == np.uint64(1)))
    keep = keep + up.astype(np.uint64)
    return (keep.astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(f.shape)
