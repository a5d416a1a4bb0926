"""Seeded synthetic inputs for the CGBN workloads.

This module only draws random numbers and lays them out in memory; it holds
none of the method's arithmetic and is the one piece shared by the tests of
the float64 oracle, the GPU parity tests and the benchmark.

The tensors stand in for the feature maps a ResNet-50 + FPN detector produces
on an image padded to 800 x 1344 (the paper trains such a detector on a public
detection dataset; only the tensor shapes and value statistics are taken, no
dataset item is reproduced).

Recipe.  For workload `i` the base seed is 171107240 + i.  Per-channel
parameters (mu_c, sigma_c, gamma_c, beta_c) come from one generator seeded
with (seed, 2**31 - 1).  The values of channel c come from a generator of
their own, seeded with (seed, c), which draws x[:, c] first and dy[:, c]
second, both in float32, in (n, h, w) order.  A channel's bits therefore do
not depend on which other channels are generated, nor on threading.
bfloat16 workloads round the float32 draw to nearest-even bfloat16 and return
the bit patterns as uint16.
"""

from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Optional, Sequence

import numpy as np

BASE_SEED = 171107240
_PARAM_STREAM = 2**31 - 1


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                 # seed offset
    N: int
    C: int
    H: int
    W: int
    layout: str                # "NCHW" | "NHWC"
    dtype: str                 # "f32" | "bf16"  (storage of x, y, dy, dx)
    K: int
    x_kind: str                # "normal" | "relu" | "offset"
    mu_range: tuple = (-1.0, 1.0)
    sigma_range: tuple = (0.5, 2.0)
    dy_sigma: float = 1.0
    eps: float = 1e-5

    @property
    def S(self) -> int:
        return self.N * self.C * self.H * self.W

    @property
    def M(self) -> int:
        return self.N * self.H * self.W

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    # tiny correctness case
    "cfg0": Workload("cfg0", 0, 4, 16, 32, 32, "NCHW", "f32", 2, "normal",
                     (-1.0, 1.0), (0.5, 2.0), 1.0),
    # detector stem level: stride-2 map of an 800x1344 image
    "cfg1": Workload("cfg1", 1, 16, 64, 400, 672, "NCHW", "f32", 8, "normal",
                     (-2.0, 2.0), (0.5, 3.0), 1e-2),
    # FPN P2 level after ReLU
    "cfg2": Workload("cfg2", 2, 16, 256, 200, 336, "NCHW", "f32", 8, "relu",
                     (-1.0, 1.0), (1.0, 1.0), 1e-2),
    # batch 256 over 128 devices, deep stage
    "cfg3": Workload("cfg3", 3, 256, 2048, 25, 42, "NCHW", "f32", 128, "normal",
                     (-2.0, 2.0), (0.5, 3.0), 1e-3),
    # bf16 storage, channels-last, large offset / tiny spread
    "cfg4": Workload("cfg4", 4, 64, 512, 50, 84, "NHWC", "bf16", 32, "offset",
                     (100.0, 100.0), (0.01, 0.01), 1.0),
    # the same offset statistics kept in float32, where the spread survives
    "cfg4b": Workload("cfg4b", 5, 64, 512, 50, 84, "NHWC", "f32", 32, "offset",
                      (100.0, 100.0), (0.01, 0.01), 1.0),
}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def channel_params(wl: Workload):
    """(mu, sigma, gamma, beta) as float32 [C] vectors."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([wl.seed, _PARAM_STREAM])))
    mu = rng.uniform(wl.mu_range[0], wl.mu_range[1], wl.C).astype(np.float32)
    sigma = rng.uniform(wl.sigma_range[0], wl.sigma_range[1], wl.C).astype(np.float32)
    gamma = rng.uniform(0.5, 1.5, wl.C).astype(np.float32)
    beta = (0.1 * rng.standard_normal(wl.C)).astype(np.float32)
    return mu, sigma, gamma, beta


def _draw_channel(wl: Workload, c: int, mu: float, sigma: float):
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([wl.seed, int(c)])))
    shape = (wl.N, wl.H, wl.W)
    x = rng.standard_normal(shape, dtype=np.float32)
    x *= np.float32(sigma)
    x += np.float32(mu)
    if wl.x_kind == "relu":
        np.maximum(x, np.float32(0.0), out=x)
    dy = rng.standard_normal(shape, dtype=np.float32)
    dy *= np.float32(wl.dy_sigma)
    return x, dy


def make_inputs(wl: Workload, channels: Optional[Sequence[int]] = None, threads: int = 8):
    """Draw x, dy (in `wl.layout`, restricted to `channels` if given), gamma, beta.

    Returns a dict with `x`, `dy` (float32, or uint16 bfloat16 bit patterns),
    `gamma`, `beta` (float32, restricted likewise) and `channels`.
    """
    mu, sigma, gamma, beta = channel_params(wl)
    chans = list(range(wl.C)) if channels is None else [int(c) for c in channels]
    nc = len(chans)
    store = np.float32 if wl.dtype == "f32" else np.uint16
    if wl.layout == "NCHW":
        x = np.empty((wl.N, nc, wl.H, wl.W), dtype=store)
        dy = np.empty_like(x)
    else:
        # filled channel-major, transposed to channels-last at the end
        x = np.empty((nc, wl.N, wl.H, wl.W), dtype=store)
        dy = np.empty_like(x)

    def fill(j):
        c = chans[j]
        xc, dyc = _draw_channel(wl, c, float(mu[c]), float(sigma[c]))
        if wl.dtype == "bf16":
            xc, dyc = f32_to_bf16_bits(xc), f32_to_bf16_bits(dyc)
        if wl.layout == "NCHW":
            x[:, j] = xc
            dy[:, j] = dyc
        else:
            x[j] = xc
            dy[j] = dyc

    if threads > 1 and nc > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(nc)))
    else:
        for j in range(nc):
            fill(j)
    if wl.layout == "NHWC":
        x = np.ascontiguousarray(x.transpose(1, 2, 3, 0))
        dy = np.ascontiguousarray(dy.transpose(1, 2, 3, 0))
    return dict(x=x, dy=dy, gamma=gamma[chans].copy(), beta=beta[chans].copy(),
                channels=chans, eps=wl.eps)
