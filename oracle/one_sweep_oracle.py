"""Float64 CPU oracle for the one-sweep statistics variant of CGBN's forward.

TEST INFRASTRUCTURE ONLY, like the rest of this package.

Algorithm 1 (MegDet, section 3.3) takes two passes over each device's sub-batch:
sums first, then squared deviations from the pooled mean, with a reduce after
each.  The variant here leaves Algorithm 1: every device summarises its sub-batch
in ONE pass as (count, mean, M2) -- M2 the sum of squared deviations from the
device's OWN mean -- and the summaries are merged pairwise,

    n    = n_a + n_b
    d    = mean_b - mean_a
    mean = mean_a + d * n_b / n
    M2   = M2_a + M2_b + d^2 * n_a * n_b / n        (Chan, Golub, LeVeque)

which yields exactly (in exact arithmetic) the pooled mean and the pooled biased
variance M2 / n of Algorithm 1, with one reduce instead of two.  The output
formula is Algorithm 1's last step, unchanged.

Pinned by the CPU tests against numpy's mean/variance, against the two-pass
oracle, and by hand; nothing here is "parity unpinned".
"""

from __future__ import annotations

import numpy as np

from . import cgbn_oracle as O


def merge(a, b):
    """Merge two summaries (n, mean[C], M2[C]) of disjoint sets."""
    na, ma, Ma = a
    nb, mb, Mb = b
    n = na + nb
    d = mb - ma
    return n, ma + d * (nb / n), Ma + Mb + d * d * (na * nb / n)


def shard_summary(xs, layout: str):
    """(count, mean, M2) per channel of one device's sub-batch, M2 about the device's own mean."""
    xs = np.asarray(xs, dtype=np.float64)
    axes = O._pooled_axes(layout)
    n = xs.size // xs.shape[O._channel_axis(layout)]
    mean = xs.sum(axis=axes) / n
    dev = xs - O._per_channel(mean, layout)
    return n, mean, (dev * dev).sum(axis=axes)


def cgbn_forward_one_sweep(x, K: int, gamma, beta, eps: float, layout: str = "NCHW"):
    """Returns (y, mean, invstd) from per-shard one-pass summaries merged in shard order."""
    x = np.asarray(x, dtype=np.float64)
    N = x.shape[0]
    if K < 1 or N % K:
        raise ValueError("need 1 <= K and N % K == 0")
    tot = None
    for sl in O._shards(N, K):
        s = shard_summary(x[sl], layout)
        tot = s if tot is None else merge(tot, s)
    n, mean, M2 = tot
    invstd = 1.0 / np.sqrt(M2 / n + float(eps))
    y = O._per_channel(gamma, layout) * ((x - O._per_channel(mean, layout)) * O._per_channel(invstd, layout)) \
        + O._per_channel(beta, layout)
    return y, mean, invstd
