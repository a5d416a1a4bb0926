"""Shared plumbing for the GPU tests: device memory via torch, calls through the
ctypes binding of the C ABI, results back as numpy.  No arithmetic of the method."""

from __future__ import annotations

import numpy as np
import torch

from oracle import cgbn_oracle as O
from paper_1711_07240_amd import cgbn as L

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    """Upload bytes as they are (uint16 bf16 bit patterns travel as int16)."""
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def to_host_f64(t: torch.Tensor, dtype: str) -> np.ndarray:
    a = t.cpu().numpy()
    if dtype == "bf16":
        return O.bf16_bits_to_f64(a.view(np.uint16))
    return a.astype(np.float64)


def dims(shape, layout):
    if layout == "NCHW":
        N, C, H, W = shape
    else:
        N, H, W, C = shape
    return N, C, H, W


class Problem:
    """One CGBN problem resident on the GPU."""

    def __init__(self, x, dy, gamma, beta, eps, layout, dtype, K):
        self.layout, self.dtype, self.K, self.eps = layout, dtype, K, eps
        self.N, self.C, self.H, self.W = dims(x.shape, layout)
        self.x, self.dy = to_dev(x), to_dev(dy)
        self.gamma, self.beta = to_dev(gamma.astype(np.float32)), to_dev(beta.astype(np.float32))
        C = self.C
        self.y = torch.empty_like(self.x)
        self.dx = torch.empty_like(self.x)
        f = dict(dtype=torch.float32, device=DEV)
        self.mean, self.invstd, self.mean_lo = (torch.empty(C, **f) for _ in range(3))
        self.dgamma, self.dbeta = torch.empty(C, **f), torch.empty(C, **f)
        self.new_workspace()

    def new_workspace(self):
        wb = L.cgbn_workspace_bytes(self.N, self.C, self.H, self.W, self.layout, self.dtype, self.K)
        assert wb > 0
        self.ws = torch.empty(wb, dtype=torch.uint8, device=DEV)

    @property
    def shape_args(self):
        return (self.N, self.C, self.H, self.W)

    def forward(self, y=None, use_mean_lo=True):
        L.cgbn_forward(self.x, *self.shape_args, self.layout, self.K, self.gamma, self.beta, self.eps,
                       self.y if y is None else y, self.mean, self.invstd, self.dtype,
                       self.mean_lo if use_mean_lo else None, self.ws)

    def backward(self, dx=None, use_mean_lo=True):
        L.cgbn_backward(self.dy, self.x, self.mean, self.invstd, self.gamma,
                        self.dx if dx is None else dx, self.dgamma, self.dbeta,
                        *self.shape_args, self.layout, self.K, self.dtype,
                        self.mean_lo if use_mean_lo else None, self.ws)

    def results(self):
        torch.cuda.synchronize()
        return dict(
            y=to_host_f64(self.y, self.dtype), dx=to_host_f64(self.dx, self.dtype),
            mean=self.mean.cpu().numpy().astype(np.float64),
            mean_lo=self.mean_lo.cpu().numpy().astype(np.float64),
            invstd=self.invstd.cpu().numpy().astype(np.float64),
            dgamma=self.dgamma.cpu().numpy().astype(np.float64),
            dbeta=self.dbeta.cpu().numpy().astype(np.float64))


def widen(a: np.ndarray, dtype: str) -> np.ndarray:
    """Stored input values as float64 (what the oracle reads)."""
    return O.bf16_bits_to_f64(a) if dtype == "bf16" else a.astype(np.float64)


# --------------------------------------------------------------------------
# the stated tolerances
# --------------------------------------------------------------------------

def rms(a):
    a = np.asarray(a, dtype=np.float64)
    return float(np.sqrt(np.mean(a * a))) if a.size else 0.0


def max_rel_err(got, ref, floor):
    """max |got-ref| / max(|ref|, floor): relative error with a floor, so that
    reference values near zero are judged against the tensor's scale."""
    ref = np.asarray(ref, dtype=np.float64)
    den = np.maximum(np.abs(ref), floor)
    den = np.where(den > 0, den, 1.0)
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref) / den)) if ref.size else 0.0


def check_against_oracle(got, ref, dtype, what="", sum_scale=None, skip=()):
    """fp32: max abs err <= 1e-4 on y, max rel err <= 1e-4 on the rest.
    bf16 storage: 2e-2 on everything, y and dx relative with the RMS floor.
    `sum_scale`: the size a channel's gradient sums have when nothing cancels (sqrt(M) * rms(dy)); if given it is
    a further floor for dgamma and dbeta, so that with a single channel a sum that happens to cancel to nearly
    zero is not judged against itself (the RMS over one channel is that channel's value).
    `skip`: outputs left out of the comparison (and absent from `got` / `ref` if the caller has none)."""
    tol = 1e-4 if dtype == "f32" else 2e-2
    report = {}
    if "y" in skip:
        pass
    elif dtype == "f32":
        report["y"] = float(np.max(np.abs(got["y"] - ref["y"]))) if ref["y"].size else 0.0
    else:
        report["y"] = max_rel_err(got["y"], ref["y"], max(rms(ref["y"]), 1e-30))
    sigma = 1.0 / ref["invstd"]
    report["mean"] = max_rel_err(got["mean"], ref["mean"], np.maximum(rms(ref["mean"]), sigma))
    report["invstd"] = max_rel_err(got["invstd"], ref["invstd"], rms(ref["invstd"]))
    for k in ("dgamma", "dbeta", "dx"):
        if k in skip:
            continue
        floor = max(rms(ref[k]), 1e-30)
        if sum_scale is not None and k != "dx":
            floor = max(floor, float(sum_scale))
        report[k] = max_rel_err(got[k], ref[k], floor)
    bad = {k: v for k, v in report.items() if not (v <= tol)}
    assert not bad, f"{what}: over tolerance {tol:g}: {bad} (all: {report})"
    return report
