"""Training-mode BatchNorm of the conv1d sub-block: CPU oracle in float64 (numpy).

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and the smoke check / CPU-baseline legs); the GPU
product path never imports this module and this module never imports the GPU package.

The paper trains its Jasper encoder (Section 4.1.1: the ``train`` action on the CTC loss; Section 3: a
trainable module computes the gradient flows) and leaves the layer mathematics to the backend, so
the definition is the textbook batch normalisation over the batch and time axes of every channel,
written out plainly:

    N          = B * T                                   (elements per channel)
    mean[c]    = (1/N) sum_{b,t} z[b,c,t]
    var[c]     = (1/N) sum_{b,t} (z[b,c,t] - mean[c])^2   (biased)
    invstd[c]  = 1 / sqrt(var[c] + eps)
    zhat       = (z - mean[c]) * invstd[c]
    y          = relu?( gamma[c]*zhat + beta[c] + residual )

and its backward pass for an upstream gradient dy of y, with m = [y > 0] (1 without ReLU), g = dy*m:

    dres       = g
    dbeta[c]   = sum_{b,t} g
    dgamma[c]  = sum_{b,t} g * zhat
    dz         = gamma[c]*invstd[c] * ( g - dbeta[c]/N - zhat * dgamma[c]/N )

Nothing is rounded.  Pins: tests/test_bn_oracle_pins.py (closed-form statistics of arithmetic
progressions, zero mean / known variance of zhat, finite differences through the statistics, the two
orthogonality identities of dz, affine invariance, torch's CPU float64 batch_norm with autograd).
"""
from __future__ import annotations

import numpy as np


def bn_train_fwd(z, gamma, beta, eps, residual=None, relu=False):
    """(y, mean, invstd) of training-mode BatchNorm over axes (0, 2) of z [B, C, T]."""
    z = np.asarray(z, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    B, C, T = z.shape
    n = B * T
    mean = np.empty(C)
    var = np.empty(C)
    for c in range(C):
        zc = z[:, c, :]
        mean[c] = zc.sum() / n
        var[c] = ((zc - mean[c]) ** 2).sum() / n
    invstd = 1.0 / np.sqrt(var + float(eps))
    zhat = (z - mean[None, :, None]) * invstd[None, :, None]
    v = gamma[None, :, None] * zhat + beta[None, :, None]
    if residual is not None:
        v = v + np.asarray(residual, dtype=np.float64)
    y = np.where(v > 0, v, 0.0) if relu else v
    return y, mean, invstd


def bn_train_bwd(dy, z, y_saved, gamma, mean, invstd, relu=False):
    """(dz, dres, dgamma, dbeta) from the upstream gradient of y; mean / invstd are the saved statistics."""
    dy = np.asarray(dy, dtype=np.float64)
    z = np.asarray(z, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    mean = np.asarray(mean, dtype=np.float64)
    invstd = np.asarray(invstd, dtype=np.float64)
    B, C, T = z.shape
    n = B * T
    if relu:
        if y_saved is None:
            raise ValueError("relu backward needs the saved output")
        g = np.where(np.asarray(y_saved, dtype=np.float64) > 0, dy, 0.0)
    else:
        g = dy.copy()
    zhat = (z - mean[None, :, None]) * invstd[None, :, None]
    dbeta = np.empty(C)
    dgamma = np.empty(C)
    for c in range(C):
        dbeta[c] = g[:, c, :].sum()
        dgamma[c] = (g[:, c, :] * zhat[:, c, :]).sum()
    dz = (gamma * invstd)[None, :, None] * (g - dbeta[None, :, None] / n - zhat * dgamma[None, :, None] / n)
    return dz, g, dgamma, dbeta
