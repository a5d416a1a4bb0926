"""GPU parity of the one-sweep statistics variant ("one_sweep_stats" = 1) through the C ABI:
same outputs as the two-pass path, to the same tolerances, against the float64 oracle."""

import dataclasses

import numpy as np
import pytest
import torch

import gpu_harness as G
from oracle import cgbn_oracle as O
from oracle import one_sweep_oracle as S
from paper_1711_07240_amd import cgbn as L
from paper_1711_07240_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def one_sweep():
    old = L.cgbn_get_tuning("fused"), L.cgbn_get_tuning("one_sweep_stats")
    L.cgbn_set_tuning("fused", 0)               # the variant lives in the multi-sweep path
    L.cgbn_set_tuning("one_sweep_stats", 1)
    yield
    L.cgbn_set_tuning("fused", old[0])
    L.cgbn_set_tuning("one_sweep_stats", old[1])


BASE = synth.WORKLOADS["cfg1"]
OFFSET = synth.WORKLOADS["cfg4b"]               # Normal(100, 0.01): |mean| >> sigma
CASES = [
    ("nchw-f32-wave-odd", BASE, dict(N=4, C=5, H=37, W=53, K=2, layout="NCHW", dtype="f32")),
    ("nchw-f32-block-ragged", BASE, dict(N=2, C=3, H=150, W=131, K=1, layout="NCHW", dtype="f32")),
    ("nchw-bf16-block", BASE, dict(N=2, C=2, H=160, W=161, K=2, layout="NCHW", dtype="bf16")),
    ("nhwc-f32-c16", BASE, dict(N=4, C=16, H=19, W=23, K=2, layout="NHWC", dtype="f32")),
    ("nhwc-f32-c7-scalar", BASE, dict(N=2, C=7, H=13, W=11, K=2, layout="NHWC", dtype="f32")),
    ("nhwc-f32-c256-long-shard", BASE, dict(N=2, C=256, H=60, W=70, K=1, layout="NHWC", dtype="f32")),
    ("nhwc-bf16-c512", BASE, dict(N=4, C=512, H=10, W=21, K=2, layout="NHWC", dtype="bf16")),
    ("nhwc-f32-many-shards", BASE, dict(N=96, C=8, H=5, W=7, K=96, layout="NHWC", dtype="f32")),
    ("offset-nhwc-f32", OFFSET, dict(N=8, C=64, H=12, W=21, K=4, layout="NHWC", dtype="f32")),
    ("offset-nchw-f32", OFFSET, dict(N=8, C=6, H=40, W=50, K=4, layout="NCHW", dtype="f32")),
    ("all-equal-bf16", synth.WORKLOADS["cfg4"], dict(N=4, C=64, H=9, W=10, K=2, layout="NHWC", dtype="bf16")),
]


@pytest.mark.parametrize("name,base,kw", CASES, ids=[c[0] for c in CASES])
def test_one_sweep_forward_then_backward(name, base, kw):
    wl = dataclasses.replace(base, name=name, **kw)
    print(f"[case] one-sweep {name}", flush=True)
    d = synth.make_inputs(wl)
    p = G.Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    p.forward()
    p.backward()
    got = p.results()
    assert L.cgbn_get_tuning("last_forward_fused") == 0
    xw, dyw = G.widen(d["x"], wl.dtype), G.widen(d["dy"], wl.dtype)
    g64, b64 = d["gamma"].astype(np.float64), d["beta"].astype(np.float64)
    y, mean, invstd = S.cgbn_forward_one_sweep(xw, wl.K, g64, b64, wl.eps, wl.layout)
    dx, dgamma, dbeta = O.cgbn_backward_ref(dyw, xw, mean, invstd, g64, wl.layout)
    ref = dict(y=y, mean=mean, invstd=invstd, dx=dx, dgamma=dgamma, dbeta=dbeta)
    print(f"[ok] one-sweep {name}: {G.check_against_oracle(got, ref, wl.dtype, name)}", flush=True)


@pytest.mark.parametrize("layout,dtype", [("NCHW", "f32"), ("NHWC", "f32"), ("NHWC", "bf16")])
@pytest.mark.parametrize("sigmas", [5.0, 50.0, 5000.0])
def test_first_value_far_from_the_mean_changes_nothing(layout, dtype, sigmas):
    """The sums are taken about a pivot, the channel's first stored value.  Wherever that value lies -- 5, 50 or
    5000 standard deviations from the channel's mean -- the statistics keep their accuracy, because a row's M2 is
    built from deviations about running means, never as a difference of sums about the pivot.  (One outlier does
    change the true statistics; the oracle sees the same data.)"""
    wl = dataclasses.replace(BASE, name=f"far-{sigmas}", N=8, C=8, H=24, W=36, K=4, layout=layout, dtype=dtype)
    d = synth.make_inputs(wl)
    x = G.widen(d["x"], dtype).astype(np.float32)
    for c in (1, 6):                                        # two of the channels get the outlier first value
        ch = x[:, c] if layout == "NCHW" else x[..., c]
        ch[(0, 0, 0)] = np.float32(ch.mean() + sigmas * ch.std())
    if dtype == "bf16":
        x = synth.f32_to_bf16_bits(x)
    p = G.Problem(x, d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    flag = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    p.forward()
    p.backward()
    L.cgbn_workspace_status(p.ws, flag)
    got = p.results()
    assert L.cgbn_get_tuning("last_forward_fused") == 0 and int(flag.item()) == 0
    xw, dyw = G.widen(x, dtype), G.widen(d["dy"], dtype)
    g64, b64 = d["gamma"].astype(np.float64), d["beta"].astype(np.float64)
    y, mean, invstd = S.cgbn_forward_one_sweep(xw, wl.K, g64, b64, wl.eps, wl.layout)
    dx, dgamma, dbeta = O.cgbn_backward_ref(dyw, xw, mean, invstd, g64, wl.layout)
    ref = dict(y=y, mean=mean, invstd=invstd, dx=dx, dgamma=dgamma, dbeta=dbeta)
    print(f"[ok] pivot {sigmas} sigma off, {layout} {dtype}: {G.check_against_oracle(got, ref, dtype, 'far pivot')}", flush=True)


def test_matches_the_two_pass_path_closely():
    """Both paths on the same data: statistics agree to a few float roundings."""
    wl = dataclasses.replace(BASE, name="both", N=4, C=64, H=31, W=33, K=2, layout="NHWC")
    d = synth.make_inputs(wl)
    p = G.Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    p.forward()
    torch.cuda.synchronize()
    m1, i1 = p.mean.clone(), p.invstd.clone()
    L.cgbn_set_tuning("one_sweep_stats", 0)
    p.forward()
    torch.cuda.synchronize()
    assert float(((p.mean - m1).abs() * p.invstd).max()) <= 1e-6
    assert float(((p.invstd - i1).abs() / p.invstd).max()) <= 2e-6


def test_relu_variant_uses_it_too():
    wl = dataclasses.replace(BASE, name="relu", N=4, C=16, H=19, W=23, K=2, layout="NHWC")
    d = synth.make_inputs(wl)
    p = G.Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    L.cgbn_forward_relu(p.x, None, *p.shape_args, wl.layout, wl.K, p.gamma, p.beta, wl.eps, p.y, p.mean, p.invstd,
                        wl.dtype, p.mean_lo, p.ws)
    torch.cuda.synchronize()
    y, mean, invstd = S.cgbn_forward_one_sweep(d["x"].astype(np.float64), wl.K, d["gamma"].astype(np.float64),
                                               d["beta"].astype(np.float64), wl.eps, wl.layout)
    assert np.max(np.abs(p.y.cpu().numpy() - np.maximum(y, 0.0))) <= 1e-4


def test_full_size_cfg4():
    """cfg4's shape, the one this variant is for: every element of y and every channel's statistics against the
    one-sweep oracle (per-shard summaries merged pairwise), channel chunk by channel chunk on host threads;
    every channel's statistics also against float64 library reductions on the device."""
    from concurrent.futures import ThreadPoolExecutor
    wl = synth.WORKLOADS["cfg4"]
    print("[case] one-sweep cfg4 full size", flush=True)
    d = synth.make_inputs(wl, threads=16)
    p = G.Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    p.forward()
    torch.cuda.synchronize()
    assert L.cgbn_get_tuning("last_forward_fused") == 0
    y_host = p.y.cpu().numpy()
    mean_host = (p.mean.double() + p.mean_lo.double()).cpu().numpy()
    invstd_host = p.invstd.cpu().numpy().astype(np.float64)
    per_chunk = max(1, (8 << 20) // wl.M)

    def compare(c0):
        cs = slice(c0, min(wl.C, c0 + per_chunk))
        y, mean, invstd = S.cgbn_forward_one_sweep(G.widen(np.ascontiguousarray(d["x"][..., cs]), wl.dtype), wl.K,
                                                   d["gamma"][cs].astype(np.float64), d["beta"][cs].astype(np.float64),
                                                   wl.eps, wl.layout)
        got_y = O.bf16_bits_to_f64(np.ascontiguousarray(y_host[..., cs]).view(np.uint16))
        e_y = G.max_rel_err(got_y, y, max(G.rms(y), 1e-30))
        e_m = G.max_rel_err(mean_host[cs], mean, np.maximum(G.rms(mean), 1.0 / invstd))
        e_i = G.max_rel_err(invstd_host[cs], invstd, G.rms(invstd))
        assert e_y <= 2e-2 and e_m <= 2e-2 and e_i <= 2e-2, (c0, e_y, e_m, e_i)
        return e_y, e_m, e_i

    with ThreadPoolExecutor(max_workers=16) as pool:
        errs = list(pool.map(compare, range(0, wl.C, per_chunk)))
    print(f"[ok] one-sweep cfg4: every element of y, worst (y, mean, invstd) = {tuple(max(e[i] for e in errs) for i in range(3))}",
          flush=True)
    x64 = p.x.view(torch.bfloat16).to(torch.float64)
    mean64 = x64.mean(dim=(0, 1, 2))
    var64 = x64.var(dim=(0, 1, 2), unbiased=False)
    istd64 = 1.0 / torch.sqrt(var64 + wl.eps)
    mean = p.mean.double() + p.mean_lo.double()
    assert float(((mean - mean64).abs() * istd64).max()) <= 1e-4
    assert float(((p.invstd.double() - istd64).abs() / istd64).max()) <= 1e-4
