"""CPU oracle (test infrastructure only): batch normalisation in training mode.

The paper adds batch normalisation after each convolution of AlexNet ("Scaling up Batch Size") and trains
ResNet-50, which has it throughout; it says nothing else about the layer.  This is the textbook definition
with batch statistics: per channel c, over the m = n*h*w values of the batch,
    mean_c = sum(x)/m,  var_c = sum((x - mean_c)^2)/m   (biased),
    xhat = (x - mean_c)/sqrt(var_c + eps),  y = gamma_c*xhat + beta_c,
and its gradient
    dbeta_c = sum(dy),  dgamma_c = sum(dy*xhat),
    dx = gamma_c/sqrt(var_c + eps) * (dy - dbeta_c/m - xhat*dgamma_c/m).
No running statistics.  numpy float64 throughout; layout NCHW (tests transpose for NHWC).
"""
from __future__ import annotations

import numpy as np


def forward(x, gamma, beta, eps=1e-5):
    """Returns (y, mean [c], inv_std [c])."""
    x = np.asarray(x, dtype=np.float64)
    mean = x.mean(axis=(0, 2, 3))
    var = ((x - mean[None, :, None, None]) ** 2).mean(axis=(0, 2, 3))
    inv_std = 1.0 / np.sqrt(var + eps)
    xhat = (x - mean[None, :, None, None]) * inv_std[None, :, None, None]
    g = np.asarray(gamma, dtype=np.float64)[None, :, None, None]
    b = np.asarray(beta, dtype=np.float64)[None, :, None, None]
    return g * xhat + b, mean, inv_std


def backward(x, dy, gamma, eps=1e-5):
    """Returns (dx, dgamma [c], dbeta [c])."""
    x = np.asarray(x, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    m = x.shape[0] * x.shape[2] * x.shape[3]
    mean = x.mean(axis=(0, 2, 3))
    var = ((x - mean[None, :, None, None]) ** 2).mean(axis=(0, 2, 3))
    inv_std = 1.0 / np.sqrt(var + eps)
    xhat = (x - mean[None, :, None, None]) * inv_std[None, :, None, None]
    dbeta = dy.sum(axis=(0, 2, 3))
    dgamma = (dy * xhat).sum(axis=(0, 2, 3))
    g = np.asarray(gamma, dtype=np.float64)
    dx = (g * inv_std)[None, :, None, None] * (dy - dbeta[None, :, None, None] / m - xhat * dgamma[None, :, None, None] / m)
    return dx, dgamma, dbeta
