"""Float64 CPU oracle for Cross-GPU Batch Normalization (CGBN).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain, obviously-correct
statement of what the CGBN hot path computes.  Only the tests, the smoke check
and the benchmark's CPU-baseline leg may import it; the product path (the HIP
library and its Python binding) never does, and this module imports nothing
from the product.  Everything here is numpy float64; there is no blocking,
fusion or reordering beyond what the definitions below state.

What the paper fixes (MegDet, section 3.3 "Cross-GPU Batch Normalization",
Algorithm 1 and the normalisation formula in its last step):

  * n devices each hold a sub-batch B_i of the mini-batch B;
  * device sums s_i are reduced to the mini-batch mean mu_B, which is broadcast;
  * device "variance sums" v_i are then taken against that pooled mean and
    reduced to the mini-batch variance sigma^2_B;
  * y = gamma * (x - mu_B) / sqrt(sigma^2_B + eps) + beta.

Readings taken where the paper is silent or loose (each is pinned by a test):

  * statistics are per channel, pooled over (N, H, W) -- convolutional batch
    normalisation as in the work the section builds on;
  * v_i sums squared deviations from the POOLED mean (Algorithm 1 broadcasts
    the mean before the variance step), not from a device-local mean;
  * "averaging the sum values" means dividing the total by the pooled count
    M = N*H*W;
  * the variance is the biased one (divide by M); eps sits inside the root;
  * devices hold equal image counts, so shard k is images [k*N/K, (k+1)*N/K).

The paper has no backward pass.  The one here is the chain rule through the
pooled mean and variance of the formula in Algorithm 1's last step:

    dbeta_c  = sum dy
    dgamma_c = sum dy * xhat                       xhat = (x - mean_c) * invstd_c
    dx       = gamma_c * invstd_c * (dy - dbeta_c / M - xhat * dgamma_c / M)

with M the pooled count, i.e. both sums run over every shard.

Two formulations are given on purpose: the plain full-batch definition
(`cgbn_forward_ref`, `cgbn_backward_ref`) and a literal shard-by-shard walk of
Algorithm 1 (`cgbn_forward_alg1`, `cgbn_backward_sharded`) that also returns
the per-device partials.  Tests check that they agree, so "K-shard pooled
statistics equal whole-batch statistics" is tested and not assumed.

Every function in this file is pinned by the CPU tests (hand-worked examples,
closed forms, finite differences, brute force, a float64 library batch norm);
nothing here is "parity unpinned".
"""

from __future__ import annotations

import numpy as np

LAYOUTS = ("NCHW", "NHWC")


# --------------------------------------------------------------------------
# layout helpers (index bookkeeping only)
# --------------------------------------------------------------------------

def _channel_axis(layout: str) -> int:
    if layout == "NCHW":
        return 1
    if layout == "NHWC":
        return 3
    raise ValueError(f"unknown layout {layout!r}")


def _pooled_axes(layout: str) -> tuple:
    """Axes pooled for the statistics: everything but the channel axis."""
    ca = _channel_axis(layout)
    return tuple(a for a in range(4) if a != ca)


def _per_channel(v: np.ndarray, layout: str) -> np.ndarray:
    """Reshape a [C] vector so that it broadcasts against a 4-d tensor."""
    shape = [1, 1, 1, 1]
    shape[_channel_axis(layout)] = -1
    return np.asarray(v, dtype=np.float64).reshape(shape)


def _as_f64_4d(x) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    if x.ndim != 4:
        raise ValueError("expected a 4-d activation tensor")
    return x


def bf16_bits_to_f64(bits) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) exactly to float64.

    A bfloat16 is the upper half of an IEEE binary32, so widening is a shift;
    binary32 -> binary64 is exact.
    """
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def f64_to_bf16_bits_rne(v) -> np.ndarray:
    """Round float64 values to bfloat16 bit patterns, nearest-even.

    Used only to report what a bf16-storing implementation would ideally hold;
    parity itself is always judged against the unrounded float64 result.
    Rounding goes through binary32 first (as a kernel computing in fp32 does).
    """
    f = np.asarray(v, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = np.isnan(f)
    out = rounded.astype(np.uint16)
    out[nan] = np.uint16(0x7FC0)
    return out


# --------------------------------------------------------------------------
# plain definition (full mini-batch)
# --------------------------------------------------------------------------

def cgbn_forward_ref(x, gamma, beta, eps: float, layout: str = "NCHW"):
    """Training-mode batch normalisation over the whole mini-batch.

    Algorithm 1 as a whole: mean (steps 1-5), biased variance about that mean
    (steps 6-10), normalise + affine (step 11).  Returns (y, mean, invstd) in
    float64 with invstd = 1/sqrt(var + eps).
    """
    x = _as_f64_4d(x)
    axes = _pooled_axes(layout)
    M = x.size // x.shape[_channel_axis(layout)]
    mean = x.sum(axis=axes) / M
    dev = x - _per_channel(mean, layout)
    var = (dev * dev).sum(axis=axes) / M
    invstd = 1.0 / np.sqrt(var + float(eps))
    xhat = dev * _per_channel(invstd, layout)
    y = _per_channel(gamma, layout) * xhat + _per_channel(beta, layout)
    return y, mean, invstd


def cgbn_backward_ref(dy, x, mean, invstd, gamma, layout: str = "NCHW"):
    """Gradient of L = sum(dy * y) through the pooled mean and variance.

    Chain rule applied to the formula of Algorithm 1's last step, with `mean`
    and `invstd` the forward's pooled statistics.  Returns (dx, dgamma, dbeta).
    """
    dy = _as_f64_4d(dy)
    x = _as_f64_4d(x)
    axes = _pooled_axes(layout)
    M = x.size // x.shape[_channel_axis(layout)]
    xhat = (x - _per_channel(mean, layout)) * _per_channel(invstd, layout)
    dbeta = dy.sum(axis=axes)
    dgamma = (dy * xhat).sum(axis=axes)
    dx = (_per_channel(gamma, layout) * _per_channel(invstd, layout)) * (
        dy - _per_channel(dbeta, layout) / M - xhat * _per_channel(dgamma, layout) / M
    )
    return dx, dgamma, dbeta


# --------------------------------------------------------------------------
# literal Algorithm 1: K devices, each with its own sub-batch
# --------------------------------------------------------------------------

def _shards(N: int, K: int):
    if K < 1 or K > N or N % K != 0:
        raise ValueError("need 1 <= K <= N and N % K == 0")
    per = N // K
    return [slice(k * per, (k + 1) * per) for k in range(K)]


def cgbn_forward_alg1(x, K: int, gamma, beta, eps: float, layout: str = "NCHW"):
    """Algorithm 1 step by step with K devices = K contiguous image ranges.

    Returns (y, mean, invstd, s, v): `s[k, c]` the device sums (steps 1-3),
    `v[k, c]` the device sums of squared deviations from the pooled mean
    (steps 6-8).
    """
    x = _as_f64_4d(x)
    N = x.shape[0]
    C = x.shape[_channel_axis(layout)]
    axes = _pooled_axes(layout)
    M = x.size // C
    shards = _shards(N, K)

    # steps 1-3: each device sums its own sub-batch
    s = np.empty((K, C), dtype=np.float64)
    for k, sl in enumerate(shards):
        s[k] = x[sl].sum(axis=axes)
    # steps 4-5: reduce to the mini-batch mean, broadcast
    mean = s.sum(axis=0) / M
    # steps 6-8: each device sums squared deviations from the broadcast mean
    v = np.empty((K, C), dtype=np.float64)
    for k, sl in enumerate(shards):
        d = x[sl] - _per_channel(mean, layout)
        v[k] = (d * d).sum(axis=axes)
    # steps 9-10: reduce to the mini-batch variance, broadcast
    var = v.sum(axis=0) / M
    invstd = 1.0 / np.sqrt(var + float(eps))
    # step 11: every device normalises its own sub-batch
    y = np.empty_like(x)
    g = _per_channel(gamma, layout)
    b = _per_channel(beta, layout)
    for sl in shards:
        y[sl] = g * (x[sl] - _per_channel(mean, layout)) * _per_channel(invstd, layout) + b
    return y, mean, invstd, s, v


def cgbn_backward_sharded(dy, x, mean, invstd, gamma, K: int, layout: str = "NCHW"):
    """Backward with the two reductions taken device by device and then pooled.

    Returns (dx, dgamma, dbeta, a, b) with `a[k, c] = sum_{B_k} dy` and
    `b[k, c] = sum_{B_k} dy * xhat`.
    """
    dy = _as_f64_4d(dy)
    x = _as_f64_4d(x)
    N = x.shape[0]
    C = x.shape[_channel_axis(layout)]
    axes = _pooled_axes(layout)
    M = x.size // C
    shards = _shards(N, K)
    mu = _per_channel(mean, layout)
    istd = _per_channel(invstd, layout)

    a = np.empty((K, C), dtype=np.float64)
    b = np.empty((K, C), dtype=np.float64)
    for k, sl in enumerate(shards):
        xhat = (x[sl] - mu) * istd
        a[k] = dy[sl].sum(axis=axes)
        b[k] = (dy[sl] * xhat).sum(axis=axes)
    dbeta = a.sum(axis=0)
    dgamma = b.sum(axis=0)
    dx = np.empty_like(x)
    g = _per_channel(gamma, layout)
    for sl in shards:
        xhat = (x[sl] - mu) * istd
        dx[sl] = g * istd * (dy[sl] - _per_channel(dbeta, layout) / M
                             - xhat * _per_channel(dgamma, layout) / M)
    return dx, dgamma, dbeta, a, b


# --------------------------------------------------------------------------
# convenience: forward + backward in one call (used by the timing leg)
# --------------------------------------------------------------------------

def cgbn_forward_backward_ref(x, dy, gamma, beta, eps: float, layout: str = "NCHW"):
    """Plain definition, forward then backward.  Channels are independent, so
    callers may pass any channel subset of a larger problem."""
    y, mean, invstd = cgbn_forward_ref(x, gamma, beta, eps, layout)
    dx, dgamma, dbeta = cgbn_backward_ref(dy, x, mean, invstd, gamma, layout)
    return dict(y=y, mean=mean, invstd=invstd, dx=dx, dgamma=dgamma, dbeta=dbeta)
