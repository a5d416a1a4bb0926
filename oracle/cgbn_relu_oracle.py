"""Float64 CPU oracle for CGBN followed by a residual add and a ReLU, the way the
backbone of the paper's detector (ResNet-50, section 4) places its normalization
layers: BN -> ReLU inside a block, BN -> (+ shortcut) -> ReLU at a block's end.

TEST INFRASTRUCTURE ONLY, like the rest of this package: only the tests, the
smoke check and the benchmark's CPU-baseline leg may import it; it imports
nothing from the product.

The normalization itself is Algorithm 1 of section 3.3 (pooled statistics over
the whole mini-batch); this file only composes the plain definitions of
oracle/cgbn_oracle.py with the two elementwise operations around them:

    z = gamma * (x - mean) * invstd + beta             Algorithm 1, last step
    y = max(0, z + r)                                  r: the shortcut, or absent

    dz = dy where y > 0, else 0                        ReLU passes gradient where its output is positive
    dr = dz                                            the add passes it through
    dbeta, dgamma, dx: the CGBN backward applied to dz

The paper states none of this (it has no backward and does not discuss the
activation); the reading is the standard one: the ReLU's derivative at 0 is taken
as 0, and the mask is read off the stored output y, so that forward and backward
agree on it bit for bit.

Pinned by the CPU tests (closed forms, finite differences away from the kink,
the unfused composition); nothing here is "parity unpinned".
"""

from __future__ import annotations

import numpy as np

from . import cgbn_oracle as O


def cgbn_relu_forward_ref(x, gamma, beta, eps: float, layout: str = "NCHW", residual=None):
    """Returns (y, mean, invstd)."""
    z, mean, invstd = O.cgbn_forward_ref(x, gamma, beta, eps, layout)
    if residual is not None:
        z = z + np.asarray(residual, dtype=np.float64)
    return np.maximum(z, 0.0), mean, invstd


def cgbn_relu_backward_ref(dy, y, x, mean, invstd, gamma, layout: str = "NCHW"):
    """Returns (dx, dgamma, dbeta, dz); dz is also the gradient of the shortcut."""
    dy = np.asarray(dy, dtype=np.float64)
    dz = np.where(np.asarray(y, dtype=np.float64) > 0.0, dy, 0.0)
    dx, dgamma, dbeta = O.cgbn_backward_ref(dz, x, mean, invstd, gamma, layout)
    return dx, dgamma, dbeta, dz
