"""Helpers for the GPU parity tests: move seeded numpy inputs to the device, call the C ABI through
the binding, bring results back.  torch is used for device memory only."""
import numpy as np
import torch

from paper_1709_05011_amd import larsconv as lc

DEV = "cuda:0"


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def workspace(nbytes: int):
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=DEV)


def to_layout(a: np.ndarray, layout: int) -> np.ndarray:
    """NCHW-ordered test array -> the layout under test."""
    return np.ascontiguousarray(a if layout == lc.LC_NCHW else np.transpose(a, (0, 2, 3, 1)))


def from_layout(a: np.ndarray, layout: int) -> np.ndarray:
    return a if layout == lc.LC_NCHW else np.transpose(a, (0, 3, 1, 2))


def desc_for(x_shape, w_shape, stride, pad, layout, dtype=lc.LC_F32) -> lc.ConvDesc:
    n, c, h, w = x_shape
    k, _, r, s = w_shape
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    return lc.ConvDesc(n, c, h, w, k, r, s, sh, sw, ph, pw, dtype, layout)


def gpu_fwd(d: lc.ConvDesc, x_l: np.ndarray, w_l: np.ndarray) -> np.ndarray:
    p, q = lc.conv2d_out_shape(d)
    shape = (d.n, d.k, p, q) if d.layout == lc.LC_NCHW else (d.n, p, q, d.k)
    y = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
    ws = workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_FWD))
    lc.conv2d_fwd(d, dev(x_l), dev(w_l), y, ws)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def gpu_bwd_data(d: lc.ConvDesc, dy_l: np.ndarray, w_l: np.ndarray) -> np.ndarray:
    shape = (d.n, d.c, d.h, d.w) if d.layout == lc.LC_NCHW else (d.n, d.h, d.w, d.c)
    dx = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
    ws = workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_DATA))
    lc.conv2d_bwd_data(d, dev(dy_l), dev(w_l), dx, ws)
    torch.cuda.synchronize()
    return dx.cpu().numpy()


def gpu_bwd_weight(d: lc.ConvDesc, x_l: np.ndarray, dy_l: np.ndarray) -> np.ndarray:
    shape = (d.k, d.c, d.r, d.s) if d.layout == lc.LC_NCHW else (d.k, d.r, d.s, d.c)
    dw = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
    ws = workspace(lc.conv2d_workspace_bytes(d, lc.LC_PASS_BWD_WEIGHT))
    lc.conv2d_bwd_weight(d, dev(x_l), dev(dy_l), dw, ws)
    torch.cuda.synchronize()
    return dw.cpu().numpy()


def scaled_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max |ref|: the tensor-scaled relative error the tolerances are stated for."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape
    assert np.all(np.isfinite(got)), "output has NaN/Inf (unwritten element?)"
    scale = float(np.max(np.abs(ref))) if ref.size else 1.0
    return float(np.max(np.abs(got - ref))) / (scale if scale > 0 else 1.0) if ref.size else 0.0
