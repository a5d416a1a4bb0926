"""GPU parity of cgbn_forward_relu / cgbn_backward_relu through the C ABI against
the float64 oracle, element by element.  The backward's mask is read off the
stored output y, which both sides are given as the same bits."""

import dataclasses

import numpy as np
import pytest
import torch

import gpu_harness as G
from oracle import cgbn_oracle as O
from oracle import cgbn_relu_oracle as R
from paper_1711_07240_amd import cgbn as L
from paper_1711_07240_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=[1, 0], ids=["fused", "sweeps"])
def path(request):
    old = L.cgbn_get_tuning("fused")
    L.cgbn_set_tuning("fused", request.param)
    yield request.param
    L.cgbn_set_tuning("fused", old)


BASE = synth.WORKLOADS["cfg1"]
CASES = [
    ("nchw-f32-wave-odd", dict(N=4, C=5, H=37, W=53, K=2, layout="NCHW", dtype="f32")),
    ("nchw-f32-block-ragged", dict(N=2, C=3, H=150, W=131, K=1, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane1050", dict(N=8, C=24, H=25, W=42, K=4, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane600", dict(N=10, C=6, H=20, W=30, K=5, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane40000", dict(N=2, C=3, H=200, W=200, K=2, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane90000-two-tiles", dict(N=2, C=2, H=300, W=300, K=1, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane258-8mod16", dict(N=8, C=5, H=6, W=43, K=2, layout="NCHW", dtype="f32")),
    ("nchw-bf16-plane4100-8mod16", dict(N=4, C=3, H=50, W=82, K=4, layout="NCHW", dtype="bf16")),
    ("nchw-f32-plane1075-odd", dict(N=8, C=6, H=25, W=43, K=4, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane273-odd", dict(N=16, C=6, H=13, W=21, K=4, layout="NCHW", dtype="f32")),
    ("nchw-bf16-plane1050", dict(N=8, C=12, H=25, W=42, K=4, layout="NCHW", dtype="bf16")),
    ("nchw-f32-plane1050-n32", dict(N=32, C=6, H=25, W=42, K=8, layout="NCHW", dtype="f32")),
    ("nchw-bf16-plane1100-n56", dict(N=56, C=4, H=25, W=44, K=7, layout="NCHW", dtype="bf16")),
    ("nchw-f32-plane16800-two-per-group", dict(N=5, C=3, H=100, W=168, K=5, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane4200-spill-bwd", dict(N=10, C=3, H=50, W=84, K=5, layout="NCHW", dtype="f32")),
    ("nchw-bf16-plane16800-spill-fwd", dict(N=6, C=2, H=100, W=168, K=3, layout="NCHW", dtype="bf16")),
    ("nchw-f32-plane8198-spill-fwd-8byte", dict(N=4, C=2, H=2, W=4099, K=2, layout="NCHW", dtype="f32")),
    ("nchw-bf16-wave", dict(N=4, C=6, H=33, W=35, K=2, layout="NCHW", dtype="bf16")),
    ("nchw-bf16-block", dict(N=2, C=2, H=160, W=161, K=2, layout="NCHW", dtype="bf16")),
    ("nchw-bf16-plane2600", dict(N=6, C=4, H=50, W=52, K=3, layout="NCHW", dtype="bf16")),
    ("nchw-f32-plane17408", dict(N=10, C=3, H=68, W=64, K=5, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane21888-3-per-group-bwd", dict(N=9, C=3, H=72, W=76, K=3, layout="NCHW", dtype="f32")),
    ("nchw-bf16-plane10368", dict(N=15, C=2, H=72, W=72, K=5, layout="NCHW", dtype="bf16")),
    ("nchw-bf16-tiny-7x7", dict(N=8, C=64, H=7, W=7, K=4, layout="NCHW", dtype="bf16")),
    ("nchw-f32-tiny-3x3", dict(N=6, C=24, H=3, W=3, K=3, layout="NCHW", dtype="f32")),
    ("nchw-bf16-tiny-13x21-odd", dict(N=4, C=24, H=13, W=21, K=2, layout="NCHW", dtype="bf16")),
    ("nhwc-f32-c16", dict(N=4, C=16, H=19, W=23, K=2, layout="NHWC", dtype="f32")),
    ("nhwc-f32-c7-scalar", dict(N=2, C=7, H=13, W=11, K=2, layout="NHWC", dtype="f32")),
    ("nhwc-f32-c64", dict(N=4, C=64, H=21, W=19, K=2, layout="NHWC", dtype="f32")),
    ("nhwc-bf16-c512", dict(N=4, C=512, H=10, W=21, K=2, layout="NHWC", dtype="bf16")),
    ("nhwc-bf16-c10-scalar", dict(N=2, C=10, H=7, W=5, K=2, layout="NHWC", dtype="bf16")),
]


def _shortcut(wl, d):
    r = np.random.default_rng(wl.seed + 77)
    s = r.standard_normal(d["x"].shape).astype(np.float32)
    return synth.f32_to_bf16_bits(s) if wl.dtype == "bf16" else s


def _check(got, ref, dtype, what):
    tol = 1e-4 if dtype == "f32" else 2e-2
    rep = {}
    if dtype == "f32":
        rep["y"] = float(np.max(np.abs(got["y"] - ref["y"])))
    else:
        rep["y"] = G.max_rel_err(got["y"], ref["y"], G.rms(ref["y"]))
    sigma = 1.0 / ref["invstd"]
    rep["mean"] = G.max_rel_err(got["mean"], ref["mean"], np.maximum(G.rms(ref["mean"]), sigma))
    rep["invstd"] = G.max_rel_err(got["invstd"], ref["invstd"], G.rms(ref["invstd"]))
    for k in ("dgamma", "dbeta", "dx", "dz"):
        if k in got:
            rep[k] = G.max_rel_err(got[k], ref[k], max(G.rms(ref[k]), 1e-30))
    bad = {k: v for k, v in rep.items() if not (v <= tol)}
    assert not bad, f"{what}: over tolerance {tol:g}: {bad} (all: {rep})"
    return rep


# shapes the single-launch kernels must take when they are switched on
SINGLE_LAUNCH = {"nchw-f32-plane1050", "nchw-f32-plane600", "nchw-f32-plane40000", "nchw-f32-plane90000-two-tiles",
                 "nchw-bf16-plane2600", "nchw-f32-plane258-8mod16", "nchw-bf16-plane4100-8mod16",
                 "nchw-f32-plane1075-odd", "nchw-bf16-plane1050", "nchw-f32-plane1050-n32", "nchw-bf16-plane1100-n56"}


def run_relu_case(wl, what, with_shortcut):
    print(f"[case] relu {what} shortcut={with_shortcut}: N={wl.N} C={wl.C} H={wl.H} W={wl.W} {wl.layout} {wl.dtype} K={wl.K}",
          flush=True)
    d = synth.make_inputs(wl)
    p = G.Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    sc_host = _shortcut(wl, d) if with_shortcut else None
    sc = G.to_dev(sc_host) if with_shortcut else None
    dz = torch.empty_like(p.x) if with_shortcut else None
    L.cgbn_forward_relu(p.x, sc, *p.shape_args, wl.layout, wl.K, p.gamma, p.beta, wl.eps, p.y, p.mean, p.invstd,
                        wl.dtype, p.mean_lo, p.ws)
    L.cgbn_backward_relu(p.dy, p.y, p.x, p.mean, p.invstd, p.gamma, p.dx, dz, p.dgamma, p.dbeta, *p.shape_args,
                         wl.layout, wl.K, wl.dtype, p.mean_lo, p.ws)
    got = p.results()
    if what in SINGLE_LAUNCH:
        want = L.cgbn_get_tuning("fused")
        assert L.cgbn_get_tuning("last_forward_fused") == want and L.cgbn_get_tuning("last_backward_fused") == want
    if what == "nchw-f32-plane273-odd":
        # float planes with an odd element count need 4-byte accesses; the ReLU backward is not built for them (it
        # would not fit the register budget) except with 24 slots per plane: the forward stays one launch, the
        # backward takes the multi-sweep kernels
        assert L.cgbn_get_tuning("last_forward_fused") == L.cgbn_get_tuning("fused")
        assert L.cgbn_get_tuning("last_backward_fused") == 0
    if with_shortcut:
        got["dz"] = G.to_host_f64(dz, wl.dtype)
    xw, dyw = G.widen(d["x"], wl.dtype), G.widen(d["dy"], wl.dtype)
    g64, b64 = d["gamma"].astype(np.float64), d["beta"].astype(np.float64)
    y_ref, mean_ref, invstd_ref = R.cgbn_relu_forward_ref(
        xw, g64, b64, wl.eps, wl.layout, residual=G.widen(sc_host, wl.dtype) if with_shortcut else None)
    # the backward's mask comes from the y the library stored: the oracle is given the same bits
    dx_ref, dg_ref, db_ref, dz_ref = R.cgbn_relu_backward_ref(dyw, got["y"], xw, mean_ref, invstd_ref, g64, wl.layout)
    ref = dict(y=y_ref, mean=mean_ref, invstd=invstd_ref, dx=dx_ref, dgamma=dg_ref, dbeta=db_ref, dz=dz_ref)
    rep = _check(got, ref, wl.dtype, what)
    frac = float((got["y"] > 0).mean())
    assert 0.05 < frac < 0.95, f"the case does not exercise both sides of the ReLU ({frac:.2f} positive)"
    if with_shortcut:
        # bit-exact where it is a selection: dz is dy or 0
        assert np.array_equal(got["dz"], np.where(got["y"] > 0, dyw, 0.0))
    # The mask itself, against the oracle's OWN output rather than the stored one: wherever the value the ReLU
    # sees is not within rounding of the kink, the library's y is positive exactly where the oracle's is, and
    # the gradient it lets through is the one a backward masked by the oracle's own y lets through.
    pre = O.cgbn_forward_ref(xw, g64, b64, wl.eps, wl.layout)[0]
    if with_shortcut:
        pre = pre + G.widen(sc_host, wl.dtype)
    away = np.abs(pre) > 1e-3
    assert away.mean() > 0.99
    assert np.array_equal((got["y"] > 0)[away], (pre > 0)[away])
    if with_shortcut:
        assert np.array_equal(got["dz"][away], np.where(pre > 0, dyw, 0.0)[away])
    dx_own, dg_own, db_own, _ = R.cgbn_relu_backward_ref(dyw, np.maximum(pre, 0.0), xw, mean_ref, invstd_ref, g64, wl.layout)
    near = float(np.abs(dyw[~away]).sum())            # gradient that elements within rounding of the kink could move
    assert np.all(np.abs(got["dbeta"] - db_own) <= (1e-4 if wl.dtype == "f32" else 2e-2) * np.maximum(np.abs(db_own), G.rms(db_own)) + near)
    print(f"[ok] relu {what}: {rep}", flush=True)


@pytest.mark.parametrize("with_shortcut", [False, True], ids=["relu", "add-relu"])
@pytest.mark.parametrize("name,kw", CASES, ids=[c[0] for c in CASES])
def test_relu_small(name, kw, with_shortcut):
    run_relu_case(dataclasses.replace(BASE, name=name, **kw), name, with_shortcut)


def test_relu_in_place():
    """y over the shortcut, dshortcut over dy: the way a residual block reuses its buffers."""
    wl = dataclasses.replace(BASE, name="in-place", N=4, C=6, H=40, W=41, K=2)
    d = synth.make_inputs(wl)
    p = G.Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    sc = G.to_dev(_shortcut(wl, d))
    dz, buf, dybuf = torch.empty_like(p.x), sc.clone(), p.dy.clone()
    L.cgbn_forward_relu(p.x, sc, *p.shape_args, wl.layout, wl.K, p.gamma, p.beta, wl.eps, p.y, p.mean, p.invstd,
                        wl.dtype, p.mean_lo, p.ws)
    L.cgbn_backward_relu(p.dy, p.y, p.x, p.mean, p.invstd, p.gamma, p.dx, dz, p.dgamma, p.dbeta, *p.shape_args,
                         wl.layout, wl.K, wl.dtype, p.mean_lo, p.ws)
    dx2 = torch.empty_like(p.x)
    L.cgbn_forward_relu(p.x, buf, *p.shape_args, wl.layout, wl.K, p.gamma, p.beta, wl.eps, buf, p.mean, p.invstd,
                        wl.dtype, p.mean_lo, p.ws)
    L.cgbn_backward_relu(dybuf, buf, p.x, p.mean, p.invstd, p.gamma, dx2, dybuf, p.dgamma, p.dbeta, *p.shape_args,
                         wl.layout, wl.K, wl.dtype, p.mean_lo, p.ws)
    torch.cuda.synchronize()
    assert torch.equal(buf, p.y) and torch.equal(dybuf, dz) and torch.equal(dx2, p.dx)


def test_relu_argument_errors():
    wl = dataclasses.replace(BASE, name="err", N=2, C=2, H=4, W=4, K=1)
    d = synth.make_inputs(wl)
    p = G.Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    with pytest.raises(L.CgbnError) as e:       # the stored output is required
        L.cgbn_backward_relu(p.dy, None, p.x, p.mean, p.invstd, p.gamma, p.dx, None, p.dgamma, p.dbeta, *p.shape_args,
                             wl.layout, wl.K, wl.dtype, p.mean_lo, p.ws)
    assert e.value.code == 1
    with pytest.raises(L.CgbnError) as e:       # dx and dshortcut must differ
        L.cgbn_backward_relu(p.dy, p.y, p.x, p.mean, p.invstd, p.gamma, p.dx, p.dx, p.dgamma, p.dbeta, *p.shape_args,
                             wl.layout, wl.K, wl.dtype, p.mean_lo, p.ws)
    assert e.value.code == 11


@pytest.mark.parametrize("name", ["cfg1", "cfg3"])
def test_relu_full_size(name, path):
    """The bench's launch configuration: sampled channels element by element against the oracle, every
    channel's statistics and gradient sums against a float64 library reduction."""
    if path == 0:
        pytest.skip("the multi-sweep kernels at full size are covered by the plain CGBN tests; once is enough here")
    wl = synth.WORKLOADS[name]
    print(f"[case] relu full size {name}", flush=True)
    gen = torch.Generator(device=G.DEV)
    gen.manual_seed(wl.seed)
    shape = (wl.N, wl.C, wl.H, wl.W)
    mu, sigma, gamma, beta = (torch.from_numpy(a).to(G.DEV) for a in synth.channel_params(wl))
    x = torch.randn(shape, generator=gen, device=G.DEV) * sigma.view(1, -1, 1, 1) + mu.view(1, -1, 1, 1)
    sc = torch.randn(shape, generator=gen, device=G.DEV)
    dy = torch.randn(shape, generator=gen, device=G.DEV) * wl.dy_sigma
    y, dx, dz = torch.empty_like(x), torch.empty_like(x), torch.empty_like(x)
    f = dict(dtype=torch.float32, device=G.DEV)
    mean, invstd, mean_lo, dgamma, dbeta = (torch.empty(wl.C, **f) for _ in range(5))
    ws = torch.empty(L.cgbn_workspace_bytes(*shape, wl.layout, wl.dtype, wl.K), dtype=torch.uint8, device=G.DEV)
    L.cgbn_forward_relu(x, sc, *shape, wl.layout, wl.K, gamma, beta, wl.eps, y, mean, invstd, wl.dtype, mean_lo, ws)
    L.cgbn_backward_relu(dy, y, x, mean, invstd, gamma, dx, dz, dgamma, dbeta, *shape, wl.layout, wl.K, wl.dtype,
                         mean_lo, ws)
    torch.cuda.synchronize()
    assert L.cgbn_get_tuning("last_forward_fused") == 1 and L.cgbn_get_tuning("last_backward_fused") == 1
    err = ws[L.cgbn_workspace_error_offset(*shape, wl.layout, wl.dtype, wl.K):][:4].view(torch.int32)
    assert int(err.item()) == 0
    # every channel: dz is a selection (bit-exact); gradient sums against float64 library reductions of dz
    assert torch.equal(dz, torch.where(y > 0, dy, torch.zeros_like(dy)))
    xh = (x.double() - (mean.double() + mean_lo.double()).view(1, -1, 1, 1)) * invstd.double().view(1, -1, 1, 1)
    db64 = dz.double().sum(dim=(0, 2, 3))
    dg64 = (dz.double() * xh).sum(dim=(0, 2, 3))
    del xh
    assert G.max_rel_err(dbeta.cpu().numpy(), db64.cpu().numpy(), G.rms(db64.cpu().numpy())) <= 1e-4
    assert G.max_rel_err(dgamma.cpu().numpy(), dg64.cpu().numpy(), G.rms(dg64.cpu().numpy())) <= 1e-4
    g64, b64 = gamma.cpu().numpy().astype(np.float64), beta.cpu().numpy().astype(np.float64)
    for c in sorted({0, wl.C // 3, wl.C - 1}):
        sl = slice(c, c + 1)
        xs, ss, dys = (t[:, sl].cpu().numpy().astype(np.float64) for t in (x, sc, dy))
        ys = y[:, sl].cpu().numpy().astype(np.float64)
        y_ref, m_ref, i_ref = R.cgbn_relu_forward_ref(xs, g64[sl], b64[sl], wl.eps, wl.layout, residual=ss)
        dx_ref, dg_ref, db_ref, dz_ref = R.cgbn_relu_backward_ref(dys, ys, xs, m_ref, i_ref, g64[sl], wl.layout)
        got = dict(y=ys, mean=mean[sl].cpu().numpy().astype(np.float64), invstd=invstd[sl].cpu().numpy().astype(np.float64),
                   dx=dx[:, sl].cpu().numpy().astype(np.float64), dgamma=dgamma[sl].cpu().numpy().astype(np.float64),
                   dbeta=dbeta[sl].cpu().numpy().astype(np.float64), dz=dz[:, sl].cpu().numpy().astype(np.float64))
        ref = dict(y=y_ref, mean=m_ref, invstd=i_ref, dx=dx_ref, dgamma=dg_ref, dbeta=db_ref, dz=dz_ref)
        print(f"[ok] relu full size {name} channel {c}: {_check(got, ref, wl.dtype, f'{name} channel {c}')}", flush=True)
