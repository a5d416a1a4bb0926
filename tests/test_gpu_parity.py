"""GPU parity: libcgbn through its C ABI against the float64 oracle, element by
element, on seeded inputs.  Sizes here finish in seconds on the CPU side yet
span several workgroup tiles, ragged tails and every kernel variant."""

import numpy as np
import pytest
import torch

from oracle import cgbn_oracle as O
from paper_1711_07240_amd import cgbn as L
from paper_1711_07240_amd import synth
from gpu_harness import DEV, Problem, check_against_oracle, widen, to_dev, to_host_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=[(1, 1), (0, 1), (0, 0)], ids=["fused", "sweeps", "sweeps-two-pass"])
def path(request):
    """Every test runs three times: with the register-resident single-launch kernels
    (where the shape allows them), with the multi-sweep kernels only (their forward taking
    its statistics from one sweep over x, the default), and with the multi-sweep kernels
    and a sweep each for the sums and for the squared deviations.  Yields whether the
    single-launch kernels are on."""
    old = L.cgbn_get_tuning("fused"), L.cgbn_get_tuning("one_sweep_stats")
    L.cgbn_set_tuning("fused", request.param[0])
    L.cgbn_set_tuning("one_sweep_stats", request.param[1])
    yield request.param[0]
    L.cgbn_set_tuning("fused", old[0])
    L.cgbn_set_tuning("one_sweep_stats", old[1])


def oracle_all(x, dy, gamma, beta, eps, layout, dtype):
    return O.cgbn_forward_backward_ref(widen(x, dtype), widen(dy, dtype), gamma.astype(np.float64),
                                       beta.astype(np.float64), eps, layout)


def run_case(wl, what):
    print(f"[case] {what}: N={wl.N} C={wl.C} H={wl.H} W={wl.W} {wl.layout} {wl.dtype} K={wl.K}", flush=True)
    d = synth.make_inputs(wl)
    p = Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    p.forward()
    p.backward()
    got = p.results()
    ref = oracle_all(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype)
    rep = check_against_oracle(got, ref, wl.dtype, what)
    print(f"[ok] {what}: {rep}", flush=True)
    return p, d, got, ref


def test_cfg0_tiny_nchw_fp32():
    run_case(synth.WORKLOADS["cfg0"], "cfg0")


BASE = synth.WORKLOADS["cfg1"]          # Normal(mu_c, sigma_c) activations
SMALL = [
    # NCHW fp32: one wavefront per plane; odd plane length (planes start off 16-byte boundaries)
    ("nchw-f32-wave-odd", dict(N=4, C=5, H=37, W=53, K=2, layout="NCHW", dtype="f32")),
    # NCHW fp32: planes split into chunks, ragged last chunk
    ("nchw-f32-block-ragged", dict(N=2, C=3, H=150, W=131, K=1, layout="NCHW", dtype="f32")),
    ("nchw-f32-block-odd", dict(N=4, C=3, H=101, W=99, K=4, layout="NCHW", dtype="f32")),
    # planes of 1050 elements as in the batch-256 deep stage (every other plane 8-byte aligned)
    ("nchw-f32-plane1050", dict(N=8, C=24, H=25, W=42, K=4, layout="NCHW", dtype="f32")),
    ("nchw-bf16-wave", dict(N=4, C=6, H=33, W=35, K=2, layout="NCHW", dtype="bf16")),
    ("nchw-bf16-block", dict(N=2, C=2, H=160, W=161, K=2, layout="NCHW", dtype="bf16")),
    # NHWC: 4-channel vectors, narrow tiles, scalar path, two column tiles
    ("nhwc-f32-c16", dict(N=4, C=16, H=19, W=23, K=2, layout="NHWC", dtype="f32")),
    ("nhwc-f32-c12", dict(N=6, C=12, H=17, W=9, K=3, layout="NHWC", dtype="f32")),
    ("nhwc-f32-c7-scalar", dict(N=2, C=7, H=13, W=11, K=2, layout="NHWC", dtype="f32")),
    ("nhwc-f32-c1028", dict(N=2, C=1028, H=9, W=7, K=1, layout="NHWC", dtype="f32")),
    ("nhwc-bf16-c512", dict(N=4, C=512, H=10, W=21, K=2, layout="NHWC", dtype="bf16")),
    ("nhwc-bf16-c24", dict(N=4, C=24, H=31, W=17, K=4, layout="NHWC", dtype="bf16")),
    ("nhwc-bf16-c10-scalar", dict(N=2, C=10, H=7, W=5, K=2, layout="NHWC", dtype="bf16")),
    ("nhwc-bf16-c300-scalar-two-tiles", dict(N=2, C=300, H=6, W=5, K=1, layout="NHWC", dtype="bf16")),
    # small planes kept whole in registers: several register-slot counts per plane
    ("nchw-f32-plane600", dict(N=10, C=6, H=20, W=30, K=5, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane702", dict(N=6, C=5, H=26, W=27, K=2, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane1100", dict(N=8, C=4, H=25, W=44, K=4, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane1398", dict(N=6, C=4, H=6, W=233, K=3, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane2900", dict(N=4, C=5, H=50, W=58, K=2, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane5000", dict(N=5, C=3, H=50, W=100, K=5, layout="NCHW", dtype="f32")),
    ("nchw-bf16-plane2600", dict(N=6, C=4, H=50, W=52, K=3, layout="NCHW", dtype="bf16")),
    # small planes of 16m + 8 bytes (8-byte accesses; every other plane starts off a 16-byte boundary; the last
    # plane ends exactly at the end of the tensor)
    ("nchw-f32-plane6-8mod16", dict(N=6, C=3, H=2, W=3, K=3, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane258-8mod16", dict(N=8, C=5, H=6, W=43, K=2, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane7938-8mod16", dict(N=4, C=3, H=63, W=126, K=2, layout="NCHW", dtype="f32")),
    ("nchw-bf16-plane84-8mod16", dict(N=6, C=4, H=6, W=14, K=2, layout="NCHW", dtype="bf16")),
    ("nchw-bf16-plane4100-8mod16", dict(N=4, C=3, H=50, W=82, K=4, layout="NCHW", dtype="bf16")),
    # small planes whose byte size is not a multiple of 8 (4-byte accesses in the single-launch kernels)
    ("nchw-f32-plane1075-odd", dict(N=8, C=6, H=25, W=43, K=4, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane15-odd", dict(N=6, C=5, H=3, W=5, K=2, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane8181-odd", dict(N=4, C=3, H=81, W=101, K=2, layout="NCHW", dtype="f32")),
    ("nchw-bf16-plane1050", dict(N=8, C=12, H=25, W=42, K=4, layout="NCHW", dtype="bf16")),
    ("nchw-bf16-plane6-", dict(N=4, C=3, H=2, W=3, K=2, layout="NCHW", dtype="bf16")),
    # small planes, enough images per unit that whole planes live in LDS beside those in registers
    ("nchw-f32-plane1050-n32", dict(N=32, C=6, H=25, W=42, K=8, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane600-n48", dict(N=48, C=3, H=20, W=30, K=4, layout="NCHW", dtype="f32")),
    ("nchw-bf16-plane1100-n56", dict(N=56, C=4, H=25, W=44, K=7, layout="NCHW", dtype="bf16")),
    # ... with 4-byte accesses (bf16 25x42 planes are 2100 bytes; fp32 13x21 planes 1092)
    ("nchw-bf16-plane1050-n64", dict(N=64, C=3, H=25, W=42, K=8, layout="NCHW", dtype="bf16")),
    ("nchw-f32-plane273-n80", dict(N=80, C=4, H=13, W=21, K=8, layout="NCHW", dtype="f32")),
    # planes a few slots too long for a wavefront's registers: one plane per wavefront, the last slots in LDS
    # (50x84 floats: backward; 100x168 bf16 and 90x100 floats: forward; 22x191 and 2x4099 floats: 8-byte accesses)
    ("nchw-f32-plane4200-spill-bwd", dict(N=10, C=3, H=50, W=84, K=5, layout="NCHW", dtype="f32")),
    ("nchw-bf16-plane16800-spill-fwd", dict(N=6, C=2, H=100, W=168, K=3, layout="NCHW", dtype="bf16")),
    ("nchw-f32-plane9000-spill-fwd", dict(N=5, C=2, H=90, W=100, K=1, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane4202-spill-bwd-8byte", dict(N=6, C=3, H=22, W=191, K=2, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane8198-spill-fwd-8byte", dict(N=4, C=2, H=2, W=4099, K=2, layout="NCHW", dtype="f32")),
    ("nchw-bf16-plane9200-spill-bwd", dict(N=8, C=2, H=92, W=100, K=4, layout="NCHW", dtype="bf16")),
    # planes of at most half a tile: the same channel's planes of two consecutive images share a workgroup
    # (100x168 floats: forward; 100x168 bf16, above: backward; an odd image count leaves the last unit one plane)
    ("nchw-f32-plane16800-two-per-group", dict(N=5, C=3, H=100, W=168, K=5, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane12600-two-per-group", dict(N=8, C=2, H=75, W=168, K=2, layout="NCHW", dtype="f32")),
    ("nchw-bf16-plane30000-two-per-group", dict(N=3, C=2, H=150, W=200, K=1, layout="NCHW", dtype="bf16")),
    # large planes: tiles that spill past the registers into LDS slots, ragged last tile
    ("nchw-f32-plane40000", dict(N=2, C=3, H=200, W=200, K=2, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane77500", dict(N=2, C=2, H=250, W=310, K=1, layout="NCHW", dtype="f32")),
    ("nchw-bf16-plane90000", dict(N=2, C=2, H=300, W=300, K=2, layout="NCHW", dtype="bf16")),
    # channels-last: several equal pieces per shard, long shards, few pixels
    ("nhwc-f32-c64", dict(N=4, C=64, H=19, W=23, K=2, layout="NHWC", dtype="f32")),
    ("nhwc-f32-c32-long-shards", dict(N=3, C=32, H=37, W=41, K=3, layout="NHWC", dtype="f32")),
    ("nhwc-f32-c96-few-pixels", dict(N=2, C=96, H=3, W=5, K=2, layout="NHWC", dtype="f32")),
    ("nhwc-f32-c256-long-shard", dict(N=2, C=256, H=60, W=70, K=1, layout="NHWC", dtype="f32")),
    ("nhwc-bf16-c128", dict(N=4, C=128, H=33, W=35, K=2, layout="NHWC", dtype="bf16")),
    ("nhwc-bf16-c64-long-shard", dict(N=2, C=64, H=50, W=41, K=2, layout="NHWC", dtype="bf16")),
    # three or four whole planes per workgroup in workgroup-wide slots, image counts that are not multiples of them,
    # planes that end inside a slot; and planes of 10-31 KB that stay one or two to a wavefront
    ("nchw-f32-plane17408", dict(N=10, C=3, H=68, W=64, K=5, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane21888-3-per-group-bwd", dict(N=9, C=3, H=72, W=76, K=3, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane26240-3-per-group-bwd", dict(N=8, C=2, H=80, W=82, K=2, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane30976", dict(N=7, C=2, H=88, W=88, K=7, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane40000-4-per-group-fwd", dict(N=6, C=3, H=100, W=100, K=3, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane48000-3-per-group-fwd", dict(N=5, C=2, H=120, W=100, K=5, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane10000", dict(N=16, C=3, H=50, W=50, K=4, layout="NCHW", dtype="f32")),
    ("nchw-f32-plane14400", dict(N=12, C=2, H=60, W=60, K=4, layout="NCHW", dtype="f32")),
    ("nchw-bf16-plane20000-4-per-group-bwd", dict(N=9, C=2, H=100, W=100, K=3, layout="NCHW", dtype="bf16")),
    ("nchw-bf16-plane10368", dict(N=15, C=2, H=72, W=72, K=5, layout="NCHW", dtype="bf16")),
    # tiny NCHW planes, C a multiple of 8: a run of planes of consecutive channels per workgroup (multi-sweep path);
    # odd element counts in bf16, planes shorter than a 16-byte vector, a ragged last channel group, one pixel
    ("nchw-bf16-tiny-7x7", dict(N=8, C=64, H=7, W=7, K=4, layout="NCHW", dtype="bf16")),
    ("nchw-f32-tiny-7x7", dict(N=6, C=40, H=7, W=7, K=3, layout="NCHW", dtype="f32")),
    ("nchw-bf16-tiny-13x21-odd", dict(N=4, C=24, H=13, W=21, K=2, layout="NCHW", dtype="bf16")),
    ("nchw-bf16-tiny-2x2", dict(N=8, C=16, H=2, W=2, K=2, layout="NCHW", dtype="bf16")),
    ("nchw-f32-tiny-1x3", dict(N=4, C=8, H=1, W=3, K=2, layout="NCHW", dtype="f32")),
    ("nchw-f32-tiny-1x1", dict(N=16, C=32, H=1, W=1, K=4, layout="NCHW", dtype="f32")),
    ("nchw-bf16-tiny-1x1", dict(N=16, C=8, H=1, W=1, K=8, layout="NCHW", dtype="bf16")),
    ("nchw-bf16-tiny-ragged-group", dict(N=3, C=264, H=5, W=5, K=3, layout="NCHW", dtype="bf16")),
    ("nchw-f32-tiny-2KiB", dict(N=4, C=16, H=16, W=32, K=2, layout="NCHW", dtype="f32")),
    ("nchw-bf16-tiny-14x14-c1024", dict(N=2, C=1024, H=14, W=14, K=2, layout="NCHW", dtype="bf16")),
    # degenerate shapes
    ("one-image-per-shard", dict(N=6, C=4, H=8, W=8, K=6, layout="NCHW", dtype="f32")),
    ("single-image", dict(N=1, C=3, H=20, W=20, K=1, layout="NCHW", dtype="f32")),
    ("one-pixel-planes", dict(N=8, C=5, H=1, W=1, K=4, layout="NCHW", dtype="f32")),
    ("one-pixel-nhwc", dict(N=8, C=8, H=1, W=1, K=2, layout="NHWC", dtype="f32")),
    ("one-channel", dict(N=2, C=1, H=64, W=65, K=2, layout="NHWC", dtype="f32")),
    # M = 2: dx is a difference of nearly equal terms unless eps is comparable to the variance
    ("two-values", dict(N=2, C=1, H=1, W=1, K=2, layout="NCHW", dtype="f32", eps=0.5)),
]


@pytest.mark.parametrize("name,kw", SMALL, ids=[s[0] for s in SMALL])
def test_small_shapes(name, kw):
    run_case(BASE.scaled(name=name, **kw), name)


LARGE_PLANES = [c for c in SMALL if c[0] in ("nchw-f32-plane40000", "nchw-f32-plane77500", "nchw-bf16-plane90000",
                                              "nchw-f32-block-ragged", "nchw-bf16-block", "nchw-f32-plane1050-n32",
                                              "nchw-f32-plane600-n48", "nchw-bf16-plane1100-n56", "nchw-f32-plane1100",
                                              "nchw-f32-plane16800-two-per-group", "nchw-bf16-plane30000-two-per-group")]


@pytest.mark.parametrize("name,kw", LARGE_PLANES, ids=[s[0] for s in LARGE_PLANES])
def test_large_planes_without_the_big_lds_variant(name, kw, path):
    """Shapes with few rows and shards take variants that keep more unit data in LDS (more slots of a large
    plane's tile, or further whole small planes); this runs the same shapes through the ordinary variants
    (the ones shapes with many rows or shards use)."""
    if path == 0:
        pytest.skip("multi-sweep path: no such variant")
    assert len(LARGE_PLANES) == 11
    L.cgbn_set_tuning("big_lds", 0)
    try:
        run_case(BASE.scaled(name=name, **kw), name + " (ordinary LDS split)")
    finally:
        L.cgbn_set_tuning("big_lds", 1)


@pytest.mark.parametrize("kind", ["relu", "offset-f32", "offset-bf16"])
def test_value_distributions_small(kind):
    if kind == "relu":
        wl = synth.WORKLOADS["cfg2"].scaled(N=4, C=16, H=40, W=56, K=2)
    elif kind == "offset-f32":
        wl = synth.WORKLOADS["cfg4b"].scaled(N=8, C=32, H=25, W=21, K=4)
    else:
        wl = synth.WORKLOADS["cfg4"].scaled(N=8, C=32, H=25, W=21, K=4)
    p, d, got, ref = run_case(wl, kind)
    if kind == "offset-bf16":
        # every stored x is exactly 100: mean exact, variance exactly zero, y = beta
        assert np.all(got["mean"] == 100.0)
        assert np.allclose(got["invstd"], wl.eps ** -0.5, rtol=1e-6)
        assert np.all(got["dgamma"] == 0.0)


@pytest.mark.parametrize("layout", ["NCHW", "NHWC"])
@pytest.mark.parametrize("scale", [1e-12, 1e12, 1e17])
def test_extreme_scales(scale, layout):
    """Activations of scale 1e-12 (variance far below eps), 1e12 and 1e17 (squared deviations near the top of float
    range, the limit the header states): the relative tolerances hold at every scale."""
    wl = BASE.scaled(N=6, C=8, H=33, W=47, K=3, layout=layout)
    d = synth.make_inputs(wl)
    x = (d["x"].astype(np.float64) * scale).astype(np.float32)
    p = Problem(x, d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    p.forward(); p.backward()
    ref = oracle_all(x, d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype)
    rep = check_against_oracle(p.results(), ref, wl.dtype, f"scale {scale:g}")
    print(f"[ok] scale {scale:g} {layout}: {rep}", flush=True)


def test_hand_examples_on_gpu():
    # the two hand-worked examples of tests/golden, through the HIP path
    from conftest import load_golden
    g = load_golden("hand_example_two_values.txt")
    x = np.array(g["x"], dtype=np.float32).reshape(2, 1, 1, 1)
    dy = np.array(g["dy"], dtype=np.float32).reshape(2, 1, 1, 1)
    p = Problem(x, dy, np.array(g["gamma"]), np.array(g["beta"]), g["eps"][0], "NCHW", "f32", 2)
    p.forward(); p.backward()
    r = p.results()
    assert np.allclose(r["y"].ravel(), g["y"], atol=1e-6) and np.allclose(r["dx"].ravel(), g["dx"], atol=1e-6)
    assert r["mean"][0] == g["mean"][0] and abs(r["invstd"][0] - g["invstd"][0]) < 1e-7
    assert abs(r["dgamma"][0] - g["dgamma"][0]) < 1e-6 and abs(r["dbeta"][0] - g["dbeta"][0]) < 1e-6
    g = load_golden("hand_example_pooled_variance.txt")
    x = np.array(g["x"], dtype=np.float32).reshape(4, 1, 1, 1)
    p = Problem(x, np.zeros_like(x), np.array(g["gamma"]), np.array(g["beta"]), g["eps"][0], "NHWC", "f32", 2)
    p.forward()
    r = p.results()
    assert np.allclose(r["y"].ravel(), g["y"], atol=1e-6) and abs(r["invstd"][0] - g["invstd"][0]) < 1e-7


@pytest.mark.parametrize("layout,dtype", [("NCHW", "f32"), ("NHWC", "f32"), ("NHWC", "bf16"), ("NCHW", "bf16")])
def test_step_entry_points_match_algorithm_1(layout, dtype):
    """Each step of Algorithm 1 on its own: the device sums s, v (and a, b of the
    backward) against the oracle's shard-by-shard walk."""
    wl = BASE.scaled(N=8, C=64, H=30, W=33, K=4, layout=layout, dtype=dtype)
    d = synth.make_inputs(wl)
    N, C, H, W, K = wl.N, wl.C, wl.H, wl.W, wl.K
    x64, dy64 = widen(d["x"], dtype), widen(d["dy"], dtype)
    g64, b64 = d["gamma"].astype(np.float64), d["beta"].astype(np.float64)
    y_r, mean_r, invstd_r, s_r, v_r = O.cgbn_forward_alg1(x64, K, g64, b64, wl.eps, layout)
    dx_r, dg_r, db_r, a_r, b_r = O.cgbn_backward_sharded(dy64, x64, mean_r, invstd_r, g64, K, layout)

    p = Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, layout, dtype, K)
    f64 = dict(dtype=torch.float64, device=DEV)
    s, v, a, b = (torch.empty(K * C, **f64) for _ in range(4))
    M = N * H * W
    L.cgbn_shard_sum(p.x, N, C, H, W, layout, K, dtype, s, p.ws)
    L.cgbn_reduce_mean(s, K, C, M, p.mean, p.mean_lo)
    L.cgbn_shard_sqdev(p.x, N, C, H, W, layout, K, dtype, p.mean, p.mean_lo, v, p.ws)
    L.cgbn_reduce_invstd(v, K, C, M, wl.eps, p.invstd)
    L.cgbn_normalize(p.x, N, C, H, W, layout, dtype, p.mean, p.mean_lo, p.invstd, p.gamma, p.beta, p.y)
    L.cgbn_backward_shard_sums(p.dy, p.x, N, C, H, W, layout, K, dtype, p.mean, p.mean_lo, p.invstd, a, b, p.ws)
    L.cgbn_backward_reduce(a, b, K, C, p.dbeta, p.dgamma)
    L.cgbn_backward_dx(p.dy, p.x, N, C, H, W, layout, dtype, p.mean, p.mean_lo, p.invstd, p.gamma,
                       p.dgamma, p.dbeta, p.dx)
    got = p.results()
    from gpu_harness import max_rel_err, rms
    tol = 1e-4 if dtype == "f32" else 2e-2
    for name, g_, r_ in (("s", s, s_r), ("v", v, v_r), ("a", a, a_r), ("b", b, b_r)):
        e = max_rel_err(g_.cpu().numpy().reshape(K, C), r_, rms(r_))
        assert e <= tol, (name, e)
    ref = dict(y=y_r, mean=mean_r, invstd=invstd_r, dx=dx_r, dgamma=dg_r, dbeta=db_r)
    check_against_oracle(got, ref, dtype, f"steps-{layout}-{dtype}")

    # the fused entry points compute the same thing (with the same kernels, or with the
    # register-resident ones): the outputs agree to float rounding
    q = Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, layout, dtype, K)
    q.forward(); q.backward()
    got2 = q.results()
    for k in ("y", "mean", "invstd", "dx", "dgamma", "dbeta"):
        assert np.allclose(got[k], got2[k], rtol=1e-2 if dtype == "bf16" else 2e-6, atol=1e-6), k
    assert np.allclose(got["mean"] + got["mean_lo"], got2["mean"] + got2["mean_lo"], rtol=2e-6, atol=2e-6)


def test_shard_count_changes_only_rounding_and_runs_are_reproducible():
    wl = BASE.scaled(N=12, C=8, H=24, W=40, K=1)
    d = synth.make_inputs(wl)
    ref = oracle_all(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype)
    outs = []
    for K in (1, 2, 3, 4, 6, 12):
        p = Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, K)
        p.forward(); p.backward()
        r = p.results()
        check_against_oracle(r, ref, wl.dtype, f"K={K}")
        p.y.zero_(); p.dx.zero_()
        p.forward(); p.backward()
        r2 = p.results()
        for k in r:
            assert np.array_equal(r[k], r2[k]), (K, k)      # bitwise reproducible
        outs.append(r)
    for r in outs[1:]:
        assert np.allclose(r["y"], outs[0]["y"], atol=2e-6)


@pytest.mark.parametrize("layout,dtype", [("NCHW", "f32"), ("NHWC", "bf16"), ("NHWC", "f32")])
def test_in_place(layout, dtype):
    wl = BASE.scaled(N=4, C=64, H=23, W=37, K=2, layout=layout, dtype=dtype)
    d = synth.make_inputs(wl)
    p = Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, layout, dtype, wl.K)
    p.forward(); p.backward()
    want = p.results()
    # dx written over dy, then y written over x
    p.backward(dx=p.dy)
    p.forward(y=p.x)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_f64(p.dy, dtype), want["dx"])
    assert np.array_equal(to_host_f64(p.x, dtype), want["y"])


def test_nan_stays_in_its_channel():
    wl = BASE.scaled(N=4, C=6, H=16, W=16, K=2)
    d = synth.make_inputs(wl)
    d["x"][1, 2, 3, 4] = np.nan
    p = Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    p.forward(); p.backward()
    r = p.results()
    assert np.all(np.isnan(r["y"][:, 2])) and np.isnan(r["mean"][2]) and np.all(np.isnan(r["dx"][:, 2]))
    keep = [0, 1, 3, 4, 5]
    assert np.all(np.isfinite(r["y"][:, keep])) and np.all(np.isfinite(r["dx"][:, keep]))
    clean = synth.make_inputs(wl)
    ref = oracle_all(clean["x"][:, keep], clean["dy"][:, keep], clean["gamma"][keep], clean["beta"][keep],
                     wl.eps, wl.layout, wl.dtype)
    got = {k: (v[:, keep] if v.ndim == 4 else v[keep]) for k, v in r.items()}
    check_against_oracle(got, ref, "f32", "nan-free channels")


@pytest.mark.parametrize("layout", ["NCHW", "NHWC"])
def test_infinity_stays_in_its_channel(layout):
    """+Inf in one channel: that channel's statistics and outputs are non-finite (Inf - Inf is NaN), nothing finite
    is invented, and every other channel is untouched."""
    wl = BASE.scaled(N=4, C=8, H=12, W=20, K=2, layout=layout)
    d = synth.make_inputs(wl)
    bad = 5
    if layout == "NCHW":
        d["x"][2, bad, 3, 4] = np.inf
        chan = lambda a, c: a[:, c]
    else:
        d["x"][2, 3, 4, bad] = np.inf
        chan = lambda a, c: a[..., c]
    p = Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    p.forward(); p.backward()
    r = p.results()
    assert not np.isfinite(r["mean"][bad]) and not np.any(np.isfinite(chan(r["y"], bad)))
    keep = [c for c in range(wl.C) if c != bad]
    clean = synth.make_inputs(wl)
    ref = oracle_all(chan(clean["x"], keep), chan(clean["dy"], keep), clean["gamma"][keep], clean["beta"][keep],
                     wl.eps, wl.layout, wl.dtype)
    got = {k: (chan(v, keep) if v.ndim == 4 else v[keep]) for k, v in r.items()}
    check_against_oracle(got, ref, "f32", "channels without the infinity")


def test_mean_lo_matters_only_for_offset_data_and_null_is_accepted():
    wl = synth.WORKLOADS["cfg4b"].scaled(N=4, C=16, H=20, W=21, K=2)
    d = synth.make_inputs(wl)
    ref = oracle_all(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype)
    p = Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    p.forward(use_mean_lo=False)
    p.backward(use_mean_lo=False)
    r = p.results()
    assert float(np.max(np.abs(r["y"] - ref["y"]))) <= 1e-4      # forward keeps the residual internally
    # mean + mean_lo reproduces the float64 mean far below float32 resolution
    p.forward(); p.backward()
    r = p.results()
    assert np.max(np.abs(r["mean"] + r["mean_lo"] - ref["mean"])) < 1e-9
    check_against_oracle(r, ref, "f32", "offset with mean_lo")


LIMITS = [
    # (name, shape, does the single-launch path take it): the limits of what a workgroup stages in LDS
    ("512-shards", dict(N=512, C=2, H=4, W=5, K=512, layout="NCHW", dtype="f32"), 1),
    ("520-shards-too-many", dict(N=520, C=2, H=4, W=5, K=520, layout="NCHW", dtype="f32"), 0),
    ("2048-rows", dict(N=2048, C=2, H=3, W=4, K=64, layout="NCHW", dtype="f32"), 1),
    ("2050-rows-too-many", dict(N=2050, C=2, H=3, W=4, K=2, layout="NCHW", dtype="f32"), 0),
    # small planes: 384 rows / 128 shards is the most the variant with planes in LDS stages
    ("384-rows-128-shards-lds-planes", dict(N=384, C=2, H=25, W=42, K=128, layout="NCHW", dtype="f32"), 1),
    ("390-rows-130-shards", dict(N=390, C=2, H=25, W=42, K=130, layout="NCHW", dtype="f32"), 1),
    # large planes, 4 tiles each in the forward: 96 images = 384 rows (variant with more data in LDS), 97 images = 388 rows
    ("large-planes-384-rows", dict(N=96, C=1, H=300, W=500, K=48, layout="NCHW", dtype="f32"), 1),
    # (its backward has 8 tiles per plane: 776 units per channel, more than workgroups fit the device at once)
    ("large-planes-388-rows", dict(N=97, C=1, H=300, W=500, K=1, layout="NCHW", dtype="f32"), (1, 0)),
    # channels-last: more partial rows than one combine pass of 64 lanes per shard
    ("nhwc-one-shard-many-pieces", dict(N=1, C=8, H=700, W=900, K=1, layout="NHWC", dtype="bf16"), 0),
]


@pytest.mark.parametrize("name,kw,fused", LIMITS, ids=[c[0] for c in LIMITS])
def test_limits_of_the_staging_areas(name, kw, fused, path):
    p, d, got, ref = run_case(BASE.scaled(name=name, **kw), name)
    if path:
        fwd, bwd = fused if isinstance(fused, tuple) else (fused, fused)
        assert L.cgbn_get_tuning("last_forward_fused") == fwd and L.cgbn_get_tuning("last_backward_fused") == bwd


CL_COMBINE = [
    # (name, shape, rows per shard wanted): channels-last row partials, many rows per shard (4 KiB pieces), shard counts
    # that give 4, 2 and 1 row lanes per shard in the combine step, and more shards than row lanes (two passes)
    ("k3-four-lanes-per-shard", dict(N=6, C=40, H=33, W=29, K=3, layout="NHWC", dtype="f32")),
    ("k5-two-lanes-per-shard", dict(N=10, C=24, H=21, W=23, K=5, layout="NHWC", dtype="bf16")),
    ("k8-two-lanes-odd-rows", dict(N=8, C=16, H=71, W=53, K=8, layout="NHWC", dtype="f32")),
    ("k12-one-lane-per-shard", dict(N=12, C=36, H=37, W=39, K=12, layout="NHWC", dtype="f32")),
    ("k20-two-passes", dict(N=20, C=24, H=45, W=47, K=20, layout="NHWC", dtype="bf16")),
    ("k1-sixteen-lanes", dict(N=2, C=72, H=41, W=37, K=1, layout="NHWC", dtype="f32")),
]


@pytest.mark.parametrize("name,kw", CL_COMBINE, ids=[c[0] for c in CL_COMBINE])
def test_channels_last_combine_lane_groups(name, kw, path):
    """The combine step of the channels-last kernels deals a shard's rows to 16 / K row lanes (a power of two)
    and joins their sums in lane order: every lane count, ragged rows per lane, both statistics variants (the
    `path` fixture's two multi-sweep settings)."""
    if path:
        pytest.skip("channels-last shapes take the multi-sweep kernels either way")
    wl = BASE.scaled(name=name, **kw)
    old = L.cgbn_get_tuning("piece_bytes")
    try:
        L.cgbn_set_tuning("piece_bytes", 4096)
        rps = L.cgbn_plan_get(wl.N, wl.C, wl.H, wl.W, wl.layout, wl.dtype, wl.K, "rps")
        assert rps >= 3, rps                      # several rows per row lane, or the case tests nothing
        run_case(wl, f"{name} rps={rps}")
    finally:
        L.cgbn_set_tuning("piece_bytes", old)


FEW_GROUPS = [
    # (shape, workgroups): large planes, one tile per plane -> 8 units per channel
    ("large-planes-8-units", dict(N=8, C=12, H=96, W=128, K=4, layout="NCHW", dtype="f32"), (8, 9, 13)),
    # small planes of 1050 floats, 64 images -> 2 units per channel forward, 4 backward
    ("small-planes-64-images", dict(N=64, C=10, H=25, W=42, K=16, layout="NCHW", dtype="f32"), (4, 5, 7)),
    ("small-planes-bf16", dict(N=96, C=6, H=25, W=44, K=8, layout="NCHW", dtype="bf16"), (4, 6)),
]


@pytest.mark.parametrize("name,kw,groups", FEW_GROUPS, ids=[c[0] for c in FEW_GROUPS])
def test_few_workgroups_walk_many_units(name, kw, groups, path):
    """The single-launch grid is persistent: with few workgroups each one takes several units of several
    channels in turn (registers, LDS slots and the staging area reused from unit to unit), and a grid that is
    not a whole number of channels leaves channels straddling two rounds."""
    if not path:
        pytest.skip("the multi-sweep kernels have no persistent grid")
    wl = BASE.scaled(name=name, **kw)
    d = synth.make_inputs(wl)
    ref = oracle_all(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype)
    old = L.cgbn_get_tuning("fused_groups")
    try:
        for g in groups:
            seen = []
            for stagger_us in (0, 3):       # 3: the channel slots start class by class, 3 us apart in all
                print(f"[case] {name}: {g} workgroups, start-up stagger {stagger_us} us", flush=True)
                L.cgbn_set_tuning("fused_groups", g)
                L.cgbn_set_tuning("stagger_us", stagger_us)
                p = Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
                p.forward(); p.backward()
                torch.cuda.synchronize()
                assert L.cgbn_get_tuning("last_forward_fused") == 1 and L.cgbn_get_tuning("last_backward_fused") == 1
                seen.append(p.results())
                check_against_oracle(seen[-1], ref, wl.dtype, f"{name} with {g} workgroups")
            for k in seen[0]:               # when a workgroup starts must not change a bit of the result
                assert np.array_equal(seen[0][k], seen[1][k]), (g, k)
    finally:
        L.cgbn_set_tuning("fused_groups", old)
        L.cgbn_set_tuning("stagger_us", 0)


@pytest.mark.parametrize("knob,value", [("spin_limit", 0), ("wait_us", 1)])
def test_bounded_wait_gives_up_cleanly(path, knob, value):
    """Failure handling of the single-launch kernels, forced from the host: with a
    poll limit of zero (or a time limit of a microsecond) a wait gives up unless the
    rows it needs are already there.  The grid must still drain, flag the error word
    and poison statistics with NaN rather than return numbers computed from an
    incomplete reduction."""
    if not path:
        pytest.skip("the multi-sweep kernels have no device-side waits")
    wl = BASE.scaled(N=8, C=64, H=96, W=128, K=4)
    d = synth.make_inputs(wl)
    p = Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    off = L.cgbn_workspace_error_offset(wl.N, wl.C, wl.H, wl.W, wl.layout, wl.dtype, wl.K)
    old = L.cgbn_get_tuning(knob)
    try:
        L.cgbn_set_tuning(knob, value)
        flag = torch.zeros(1, dtype=torch.int32, device=p.ws.device)
        p.forward()
        L.cgbn_workspace_status(p.ws, flag)          # the caller's way to learn of it: a device int, raised if the word is up
        torch.cuda.synchronize()
        gave_up = int(p.ws[off:off + 4].view(torch.int32).item())
        assert int(flag.item()) == gave_up
        r = p.results()
    finally:
        L.cgbn_set_tuning(knob, old)
    ref = oracle_all(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype)
    assert gave_up in (0, 1)
    any_nan = bool(np.isnan(r["y"]).any() or np.isnan(r["mean"]).any() or np.isnan(r["invstd"]).any())
    assert any_nan == bool(gave_up)
    # whatever is not NaN is right: never numbers from an incomplete reduction
    for k in ("mean", "invstd", "y"):
        fin = np.isfinite(r[k])
        assert np.allclose(r[k][fin], ref[k][fin], rtol=1e-4, atol=1e-4), k
    # and with the normal limit the same problem is clean
    p.forward(); p.backward()
    torch.cuda.synchronize()
    flag.fill_(7)
    L.cgbn_workspace_status(p.ws, flag)
    torch.cuda.synchronize()
    assert int(p.ws[off:off + 4].view(torch.int32).item()) == 0 and int(flag.item()) == 7    # a clean word leaves the flag alone
    check_against_oracle(p.results(), ref, wl.dtype, "after the forced give-up")
