"""Float64 CPU oracle for the fixed-statistics ("frozen") batch normalization
mode and for the running-statistics update that feeds it.

TEST INFRASTRUCTURE ONLY, like the rest of this package: only the tests, the
smoke check and the benchmark's CPU-baseline leg may import it; it imports
nothing from the product.

What the paper fixes (MegDet, section 3.1 "Problems with Small Mini-Batch Size"
and the opening of section 3.3; Table 3, row "16-base" with BN size 0): the
usual detector keeps the statistics of every batch-normalization layer fixed to
values computed beforehand and never re-estimates them while fine-tuning.  The
layer is then the formula of Algorithm 1's last step with constants in place of
the mini-batch statistics:

    y = gamma * (x - m) / sqrt(s2 + eps) + beta        m, s2: fixed per channel

Readings taken where the paper is silent (each is pinned by a test):

  * "the batch normalization layer is fixed" is read as: statistics AND the
    affine parameters are constants of the layer, so its backward is
    dx = dy * gamma / sqrt(s2 + eps) and there is no dgamma / dbeta;
  * the paper never says how the fixed values are obtained from training
    batches.  The update here is the exponential moving average of the work the
    section builds on (Ioffe and Szegedy): after a training forward with pooled
    mean mu and biased variance sigma2 over M values per channel,
        m  <- (1 - momentum) * m  + momentum * mu
        s2 <- (1 - momentum) * s2 + momentum * sigma2 * (M / (M - 1) if unbiased else 1)
    `momentum` and `unbiased` are the caller's; nothing in the paper picks them.

Every function in this file is pinned by the CPU tests (closed forms, a
float64 library variance, finite differences, the training forward in the
limit where batch and fixed statistics coincide); nothing here is "parity
unpinned".
"""

from __future__ import annotations

import numpy as np


def _bcast(v, layout: str) -> np.ndarray:
    shape = [1, 1, 1, 1]
    if layout == "NCHW":
        shape[1] = -1
    elif layout == "NHWC":
        shape[3] = -1
    else:
        raise ValueError(f"unknown layout {layout!r}")
    return np.asarray(v, dtype=np.float64).reshape(shape)


def frozen_forward_ref(x, fixed_mean, fixed_var, gamma, beta, eps: float, layout: str = "NCHW") -> np.ndarray:
    """y = gamma (x - m) / sqrt(s2 + eps) + beta with fixed m, s2 (Algorithm 1, last step,
    statistics held constant as in section 3.3's description of earlier detectors)."""
    x = np.asarray(x, dtype=np.float64)
    m, s2 = _bcast(fixed_mean, layout), _bcast(fixed_var, layout)
    return _bcast(gamma, layout) * (x - m) / np.sqrt(s2 + float(eps)) + _bcast(beta, layout)


def frozen_backward_ref(dy, fixed_var, gamma, eps: float, layout: str = "NCHW") -> np.ndarray:
    """dx of the fixed-statistics layer: every factor but x is a constant."""
    dy = np.asarray(dy, dtype=np.float64)
    return dy * (_bcast(gamma, layout) / np.sqrt(_bcast(fixed_var, layout) + float(eps)))


def running_update_ref(batch_mean, batch_var_biased, M: int, momentum: float, unbiased: bool,
                       running_mean, running_var):
    """One exponential-moving-average step; returns the new (running_mean, running_var)."""
    mu = np.asarray(batch_mean, dtype=np.float64)
    s2 = np.asarray(batch_var_biased, dtype=np.float64)
    rm = np.asarray(running_mean, dtype=np.float64)
    rv = np.asarray(running_var, dtype=np.float64)
    if unbiased:
        if M < 2:
            raise ValueError("the unbiased variance needs at least two values per channel")
        s2 = s2 * (float(M) / float(M - 1))
    keep = 1.0 - float(momentum)
    return keep * rm + float(momentum) * mu, keep * rv + float(momentum) * s2
