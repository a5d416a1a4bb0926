"""GPU parity at the full sizes of the five workloads, in the launch
configuration the benchmark times.  Every element of every output is compared
with the float64 oracle (channels are independent, so the oracle takes them a
few at a time, on a pool of host threads); all channels are also checked through
properties and against a float64 library reduction on the device."""

import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from oracle import cgbn_oracle as O
from paper_1711_07240_amd import synth
from gpu_harness import DEV, Problem, check_against_oracle, widen

pytestmark = pytest.mark.gpu


def _chan(t, layout, idx):
    return t[:, idx] if layout == "NCHW" else t[..., idx]


def _as_f64_dev(t, dtype):
    if dtype == "bf16":
        return t.view(torch.bfloat16).to(torch.float64)
    return t.to(torch.float64)


# every workload on the path the library takes by itself; the two extremes of the single-launch kernels
# (few huge planes, many tiny ones) also on the multi-sweep kernels a shape falls back to
# (the channels-last workloads run on the multi-sweep kernels in any case: by default with the forward's statistics
# from one sweep over x, and once more with a sweep each for the sums and the squared deviations)
@pytest.mark.parametrize("name,fused,one_sweep", [("cfg1", 1, 1), ("cfg2", 1, 1), ("cfg3", 1, 1), ("cfg4", 1, 1), ("cfg4b", 1, 1),
                                                  ("cfg1", 0, 1), ("cfg3", 0, 1), ("cfg4", 1, 0), ("cfg4b", 1, 0), ("cfg1", 0, 0)],
                         ids=["cfg1", "cfg2", "cfg3", "cfg4", "cfg4b", "cfg1-sweeps", "cfg3-sweeps", "cfg4-two-pass", "cfg4b-two-pass",
                              "cfg1-sweeps-two-pass"])
def test_full_size(name, fused, one_sweep):
    from paper_1711_07240_amd import cgbn as L
    old = L.cgbn_get_tuning("fused"), L.cgbn_get_tuning("one_sweep_stats")
    L.cgbn_set_tuning("fused", fused)
    L.cgbn_set_tuning("one_sweep_stats", one_sweep)
    try:
        _full_size(name, fused)
    finally:
        L.cgbn_set_tuning("fused", old[0])
        L.cgbn_set_tuning("one_sweep_stats", old[1])


def _full_size(name, fused):
    from paper_1711_07240_amd import cgbn as L
    wl = synth.WORKLOADS[name]
    t0 = time.time()
    print(f"[case] {name}: generating {wl.S} elements x2 on the host", flush=True)
    d = synth.make_inputs(wl, threads=16)
    print(f"[case] {name}: generated in {time.time() - t0:.1f}s; running forward+backward", flush=True)
    p = Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    p.forward()
    p.backward()
    torch.cuda.synchronize()
    single = (L.cgbn_get_tuning("last_forward_fused"), L.cgbn_get_tuning("last_backward_fused"))
    assert single == ((1, 1) if fused and wl.layout == "NCHW" else (0, 0)), single
    print(f"[case] {name}: kernels done (single launch: {single})", flush=True)

    # ---- every channel, every element, against the oracle -----------------
    t0 = time.time()
    y_host, dx_host = p.y.cpu().numpy(), p.dx.cpu().numpy()
    small = {k: getattr(p, k).cpu().numpy().astype(np.float64) for k in ("mean", "invstd", "dgamma", "dbeta")}
    per_chunk = max(1, (8 << 20) // wl.M)                  # ~8M elements per tensor and chunk

    def compare(c0):
        cs = slice(c0, min(wl.C, c0 + per_chunk))
        ref = O.cgbn_forward_backward_ref(widen(_chan(d["x"], wl.layout, cs), wl.dtype),
                                          widen(_chan(d["dy"], wl.layout, cs), wl.dtype),
                                          d["gamma"][cs].astype(np.float64), d["beta"][cs].astype(np.float64),
                                          wl.eps, wl.layout)
        got = {k: v[cs] for k, v in small.items()}
        for k, host in (("y", y_host), ("dx", dx_host)):
            a = np.ascontiguousarray(_chan(host, wl.layout, cs))
            got[k] = O.bf16_bits_to_f64(a.view(np.uint16)) if wl.dtype == "bf16" else a.astype(np.float64)
        return check_against_oracle(got, ref, wl.dtype, f"{name} channels {cs.start}..{cs.stop - 1}")

    with ThreadPoolExecutor(max_workers=16) as pool:
        reports = list(pool.map(compare, range(0, wl.C, per_chunk)))
    worst = {k: max(r[k] for r in reports) for k in reports[0]}
    print(f"[ok] {name}: all {wl.C} channels, every element, {len(reports)} chunks in {time.time() - t0:.1f}s: "
          f"worst {worst}", flush=True)
    del y_host, dx_host

    # ---- all channels: properties + a float64 library reduction ----------
    tol = 1e-4 if wl.dtype == "f32" else 2e-2
    dims_ = (0, 2, 3) if wl.layout == "NCHW" else (0, 1, 2)
    M = wl.M
    step = max(1, min(wl.C, (1 << 27) // M))          # ~1 GiB of float64 per chunk
    mean = p.mean.double() + p.mean_lo.double()
    for c0 in range(0, wl.C, step):
        cs = slice(c0, min(wl.C, c0 + step))
        bshape = (1, -1, 1, 1) if wl.layout == "NCHW" else (1, 1, 1, -1)
        x64 = _as_f64_dev(_chan(p.x, wl.layout, cs), wl.dtype)
        var_t, mean_t = torch.var_mean(x64, dim=dims_, unbiased=False)
        sig = torch.sqrt(var_t + wl.eps)
        assert torch.all((mean[cs] - mean_t).abs() <= tol * torch.maximum(mean_t.abs(), sig)), name
        assert torch.all((p.invstd[cs].double() - 1 / sig).abs() <= tol / sig), name
        xhat = (x64 - mean_t.view(bshape)) / sig.view(bshape)
        del x64
        y64 = _as_f64_dev(_chan(p.y, wl.layout, cs), wl.dtype)
        # the normalised output has mean beta and biased variance gamma^2 var/(var+eps)
        ytol = 1e-4 if wl.dtype == "f32" else 2e-2 * (p.beta[cs].abs().double() + 1e-2)
        assert torch.all((y64.mean(dim=dims_) - p.beta[cs].double()).abs() <= ytol), name
        want_var = p.gamma[cs].double() ** 2 * var_t / (var_t + wl.eps)
        assert torch.all((y64.var(dim=dims_, unbiased=False) - want_var).abs()
                         <= 10 * tol * want_var + 1e-6), name
        del y64
        dy64 = _as_f64_dev(_chan(p.dy, wl.layout, cs), wl.dtype)
        db_t = dy64.sum(dim=dims_)
        dg_t = (dy64 * xhat).sum(dim=dims_)
        del xhat
        scale_b = torch.sqrt((db_t ** 2).mean())
        assert torch.all((p.dbeta[cs].double() - db_t).abs() <= tol * torch.maximum(db_t.abs(), scale_b)), name
        if name != "cfg4":
            scale_g = torch.sqrt((dg_t ** 2).mean())
            assert torch.all((p.dgamma[cs].double() - dg_t).abs()
                             <= tol * torch.maximum(dg_t.abs(), scale_g)), name
        else:
            assert torch.all(p.dgamma[cs] == 0), name        # xhat is exactly zero
        dx64 = _as_f64_dev(_chan(p.dx, wl.layout, cs), wl.dtype)
        # the gradient sums to zero over the pooled axes
        budget = (1e-5 if wl.dtype == "f32" else 4e-3) * dx64.abs().sum(dim=dims_) + 1e-12
        assert torch.all(dx64.sum(dim=dims_).abs() <= budget), name
        del dx64, dy64
    print(f"[ok] {name}: all {wl.C} channels pass the property and library checks", flush=True)


@pytest.mark.parametrize("layout,fused", [("NCHW", 1), ("NCHW", 0), ("NHWC", 1)], ids=["NCHW", "NCHW-sweeps", "NHWC"])
def test_more_than_2_to_31_elements(layout, fused):
    """A tensor of 2.36e9 elements (9.4 GB per tensor): 64-bit indexing end to end, on the single-launch kernels
    and on the multi-sweep ones.  Drawn on the device; the first, a middle and the last channel element by
    element against the oracle, the last one holding the elements with the highest addresses."""
    from oracle import cgbn_oracle as O
    from paper_1711_07240_amd import cgbn as L
    old = L.cgbn_get_tuning("fused")
    L.cgbn_set_tuning("fused", fused)
    try:
        _more_than_2_to_31(layout, fused)
    finally:
        L.cgbn_set_tuning("fused", old)


def _more_than_2_to_31(layout, fused):
    from oracle import cgbn_oracle as O
    from paper_1711_07240_amd import cgbn as L
    N, C, H, W, K, eps = 32, 128, 512, 1125, 8, 1e-5
    S = N * C * H * W
    assert S > 2 ** 31
    print(f"[case] {S} elements, {layout}", flush=True)
    shape = (N, C, H, W) if layout == "NCHW" else (N, H, W, C)
    bs = (1, -1, 1, 1) if layout == "NCHW" else (1, 1, 1, -1)
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(77)
    mu = torch.linspace(-2, 2, C, device=dev).view(bs)
    x = torch.empty(shape, device=dev).normal_(generator=gen).mul_(1.5).add_(mu)
    dy = torch.empty(shape, device=dev).normal_(generator=gen)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    gamma = torch.linspace(0.5, 1.5, C, device=dev)
    beta = torch.linspace(-0.1, 0.1, C, device=dev)
    f = dict(dtype=torch.float32, device=dev)
    mean, invstd, mean_lo, dgamma, dbeta = (torch.empty(C, **f) for _ in range(5))
    ws = torch.empty(L.cgbn_workspace_bytes(N, C, H, W, layout, "f32", K), dtype=torch.uint8, device=dev)
    L.cgbn_forward(x, N, C, H, W, layout, K, gamma, beta, eps, y, mean, invstd, "f32", mean_lo, ws)
    L.cgbn_backward(dy, x, mean, invstd, gamma, dx, dgamma, dbeta, N, C, H, W, layout, K, "f32", mean_lo, ws)
    torch.cuda.synchronize()
    assert L.cgbn_get_tuning("last_forward_fused") == (1 if fused and layout == "NCHW" else 0)
    err = ws[L.cgbn_workspace_error_offset(N, C, H, W, layout, "f32", K):][:4].view(torch.int32)
    assert int(err.item()) == 0
    for c in (0, C // 2 + 1, C - 1):
        sl = slice(c, c + 1)
        pick = (lambda t: t[:, sl]) if layout == "NCHW" else (lambda t: t[..., sl])
        xs, dys = (pick(t).cpu().numpy().astype(np.float64) for t in (x, dy))
        g1, b1 = gamma[sl].cpu().numpy().astype(np.float64), beta[sl].cpu().numpy().astype(np.float64)
        ref = O.cgbn_forward_backward_ref(xs, dys, g1, b1, eps, layout)
        got = dict(y=pick(y).cpu().numpy().astype(np.float64), dx=pick(dx).cpu().numpy().astype(np.float64),
                   mean=mean[sl].cpu().numpy().astype(np.float64), mean_lo=mean_lo[sl].cpu().numpy().astype(np.float64),
                   invstd=invstd[sl].cpu().numpy().astype(np.float64), dgamma=dgamma[sl].cpu().numpy().astype(np.float64),
                   dbeta=dbeta[sl].cpu().numpy().astype(np.float64))
        print(f"[ok] channel {c}: {check_against_oracle(got, ref, 'f32', f'{layout} channel {c}')}", flush=True)
