"""GPU parity of the fixed-statistics entry points (cgbn_frozen_forward,
cgbn_frozen_backward, cgbn_update_running_stats), through the C ABI, against
the float64 oracle, element by element."""

import numpy as np
import pytest
import torch

import gpu_harness as G
from oracle import cgbn_oracle as O
from oracle import frozen_bn_oracle as F
from paper_1711_07240_amd import cgbn as L
from paper_1711_07240_amd import synth

pytestmark = pytest.mark.gpu

# (name, N, C, H, W, layout, dtype): several tiles and ragged tails of every map kernel variant
CASES = [
    ("nchw-large-plane", 2, 3, 67, 131, "NCHW", "f32"),
    ("nchw-odd-plane", 3, 5, 25, 42, "NCHW", "f32"),          # 1050 elements: 8-byte aligned every other plane
    ("nchw-tiny-plane", 4, 7, 3, 5, "NCHW", "f32"),
    ("nchw-bf16", 2, 6, 33, 65, "NCHW", "bf16"),
    ("nchw-bf16-odd", 3, 4, 7, 9, "NCHW", "bf16"),
    ("nhwc-vector", 4, 64, 9, 11, "NHWC", "f32"),
    ("nhwc-scalar-channels", 2, 37, 6, 7, "NHWC", "f32"),     # C not a multiple of the vector width
    ("nhwc-bf16", 4, 128, 13, 10, "NHWC", "bf16"),
    ("nhwc-bf16-scalar", 2, 10, 5, 3, "NHWC", "bf16"),
    ("one-pixel", 5, 8, 1, 1, "NCHW", "f32"),
    ("nchw-bf16-tiny-7x7", 4, 64, 7, 7, "NCHW", "bf16"),      # runs of tiny planes per workgroup (C a multiple of 8)
    ("nchw-f32-tiny-ragged-group", 2, 264, 3, 3, "NCHW", "f32"),
]


def _draw(N, C, H, W, layout, dtype, seed):
    r = np.random.default_rng(seed)
    shape = (N, C, H, W) if layout == "NCHW" else (N, H, W, C)
    bs = (1, -1, 1, 1) if layout == "NCHW" else (1, 1, 1, -1)
    mu, sg = r.uniform(-2, 2, C), r.uniform(0.5, 3, C)
    x = (r.standard_normal(shape) * sg.reshape(bs) + mu.reshape(bs)).astype(np.float32)
    dy = r.standard_normal(shape).astype(np.float32)
    if dtype == "bf16":
        x, dy = synth.f32_to_bf16_bits(x), synth.f32_to_bf16_bits(dy)
    fm = (mu + r.normal(0, 0.1, C)).astype(np.float32)
    fv = (sg * sg * r.uniform(0.8, 1.2, C)).astype(np.float32)
    gamma, beta = r.uniform(0.5, 1.5, C).astype(np.float32), r.normal(0, 0.1, C).astype(np.float32)
    return x, dy, fm, fv, gamma, beta


def _tolerance(dtype):
    # fp32: 1e-4 absolute on y (values of order 1), 1e-4 relative on dx; bf16 storage: 2e-2 relative with the RMS floor
    return 1e-4 if dtype == "f32" else 2e-2


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_frozen_forward_backward(case):
    name, N, C, H, W, layout, dtype = case
    print(f"[case] frozen {name}", flush=True)
    eps = 1e-5
    x, dy, fm, fv, gamma, beta = _draw(N, C, H, W, layout, dtype, 4242)
    dx_, dy_ = G.to_dev(x), G.to_dev(dy)
    y_d, dx_d = torch.empty_like(dx_), torch.empty_like(dy_)
    fm_d, fv_d, g_d, b_d = (G.to_dev(a) for a in (fm, fv, gamma, beta))
    L.cgbn_frozen_forward(dx_, N, C, H, W, layout, dtype, fm_d, fv_d, g_d, b_d, eps, y_d)
    L.cgbn_frozen_backward(dy_, N, C, H, W, layout, dtype, fv_d, g_d, eps, dx_d)
    torch.cuda.synchronize()
    y_ref = F.frozen_forward_ref(G.widen(x, dtype), fm, fv, gamma, beta, eps, layout)
    dx_ref = F.frozen_backward_ref(G.widen(dy, dtype), fv, gamma, eps, layout)
    y, dx = G.to_host_f64(y_d, dtype), G.to_host_f64(dx_d, dtype)
    tol = _tolerance(dtype)
    if dtype == "f32":
        assert np.max(np.abs(y - y_ref)) <= tol
    else:
        assert G.max_rel_err(y, y_ref, G.rms(y_ref)) <= tol
    assert G.max_rel_err(dx, dx_ref, G.rms(dx_ref)) <= tol


def test_frozen_in_place():
    N, C, H, W, layout, dtype = 3, 5, 25, 42, "NCHW", "f32"
    x, dy, fm, fv, gamma, beta = _draw(N, C, H, W, layout, dtype, 7)
    xd, dyd = G.to_dev(x), G.to_dev(dy)
    fm_d, fv_d, g_d, b_d = (G.to_dev(a) for a in (fm, fv, gamma, beta))
    y_sep, dx_sep = torch.empty_like(xd), torch.empty_like(dyd)
    L.cgbn_frozen_forward(xd, N, C, H, W, layout, dtype, fm_d, fv_d, g_d, b_d, 1e-5, y_sep)
    L.cgbn_frozen_backward(dyd, N, C, H, W, layout, dtype, fv_d, g_d, 1e-5, dx_sep)
    L.cgbn_frozen_forward(xd, N, C, H, W, layout, dtype, fm_d, fv_d, g_d, b_d, 1e-5, xd)
    L.cgbn_frozen_backward(dyd, N, C, H, W, layout, dtype, fv_d, g_d, 1e-5, dyd)
    torch.cuda.synchronize()
    assert torch.equal(xd, y_sep) and torch.equal(dyd, dx_sep)


def test_frozen_equals_training_forward_at_the_batch_statistics():
    """With the fixed statistics set to what cgbn_forward measured, both modes give the same y up to rounding."""
    N, C, H, W, layout, dtype, K, eps = 4, 6, 31, 17, "NCHW", "f32", 2, 1e-5
    x, dy, _, _, gamma, beta = _draw(N, C, H, W, layout, dtype, 99)
    p = G.Problem(x, dy, gamma, beta, eps, layout, dtype, K)
    p.forward()
    torch.cuda.synchronize()
    var = (1.0 / p.invstd.double() ** 2 - eps).float()
    y2 = torch.empty_like(p.x)
    L.cgbn_frozen_forward(p.x, N, C, H, W, layout, dtype, p.mean, var, p.gamma, p.beta, eps, y2)
    torch.cuda.synchronize()
    assert float((y2 - p.y).abs().max()) <= 2e-5


@pytest.mark.parametrize("layout,dtype", [("NCHW", "f32"), ("NHWC", "bf16")])
@pytest.mark.parametrize("unbiased", [True, False])
def test_running_statistics_after_a_training_forward(layout, dtype, unbiased):
    N, C, H, W, K, eps, mom = 4, 64, 9, 11, 2, 1e-5, 0.1
    x, dy, fm, fv, gamma, beta = _draw(N, C, H, W, layout, dtype, 31)
    p = G.Problem(x, dy, gamma, beta, eps, layout, dtype, K)
    p.forward()
    rm_d, rv_d = G.to_dev(fm), G.to_dev(fv)
    M = N * H * W
    for _ in range(3):                                        # three steps on the same batch
        L.cgbn_update_running_stats(p.mean, p.mean_lo, p.invstd, eps, M, C, mom, unbiased, rm_d, rv_d)
    torch.cuda.synchronize()
    xw = G.widen(x, dtype)
    _, mean_ref, invstd_ref = O.cgbn_forward_ref(xw, gamma, beta, eps, layout)
    var_ref = 1.0 / invstd_ref ** 2 - eps
    rm, rv = fm.astype(np.float64), fv.astype(np.float64)
    for _ in range(3):
        rm, rv = F.running_update_ref(mean_ref, var_ref, M, mom, unbiased, rm, rv)
    # the statistics come out of float vectors (mean, invstd): 1e-4 relative, the tolerance of the statistics
    assert G.max_rel_err(rm_d.cpu().numpy(), rm, np.sqrt(rv)) <= 1e-4
    assert G.max_rel_err(rv_d.cpu().numpy(), rv, G.rms(rv)) <= 1e-4


def test_running_statistics_when_the_variance_vanishes():
    """A constant channel: var = 0, invstd = 1/sqrt(eps); the recovered variance must be ~0, not negative or noisy."""
    N, C, H, W, eps = 2, 4, 5, 5, 1e-5
    x = np.full((N, C, H, W), 100.0, dtype=np.float32)
    p = G.Problem(x, np.zeros_like(x), np.ones(C, np.float32), np.zeros(C, np.float32), eps, "NCHW", "f32", 2)
    p.forward()
    rm_d, rv_d = torch.zeros(C, device=G.DEV), torch.zeros(C, device=G.DEV)
    L.cgbn_update_running_stats(p.mean, p.mean_lo, p.invstd, eps, N * H * W, C, 1.0, True, rm_d, rv_d)
    torch.cuda.synchronize()
    assert torch.all(rm_d == 100.0)
    assert float(rv_d.min()) >= 0.0 and float(rv_d.max()) <= 3e-7 * eps * 10


def test_argument_errors():
    t = torch.zeros(64, device=G.DEV)
    with pytest.raises(L.CgbnError) as e:
        L.cgbn_update_running_stats(t, None, t, 1e-5, 10, 4, 1.5, True, t, t)
    assert e.value.code == 10
    with pytest.raises(L.CgbnError) as e:
        L.cgbn_update_running_stats(t, None, t, 1e-5, 1, 4, 0.1, True, t, t)
    assert e.value.code == 2
    with pytest.raises(L.CgbnError) as e:
        L.cgbn_frozen_forward(t, 1, 4, 2, 2, "NCHW", "f32", t, None, t, t, 1e-5, t)
    assert e.value.code == 1
    with pytest.raises(L.CgbnError) as e:
        L.cgbn_frozen_backward(t, 1, 4, 2, 2, "NCHW", "f32", t, t, 0.0, t)
    assert e.value.code == 5


def test_frozen_full_size_sampled():
    """cfg1's shape (the bench's launch configuration): 4 sampled channels element by element."""
    wl = synth.WORKLOADS["cfg1"]
    print("[case] frozen cfg1 full size", flush=True)
    g = torch.Generator(device=G.DEV)
    g.manual_seed(5)
    x = torch.randn((wl.N, wl.C, wl.H, wl.W), generator=g, device=G.DEV) * 2.0 + 0.5
    dy = torch.randn((wl.N, wl.C, wl.H, wl.W), generator=g, device=G.DEV)
    r = np.random.default_rng(3)
    fm, fv = r.normal(0.5, 0.2, wl.C).astype(np.float32), r.uniform(2, 6, wl.C).astype(np.float32)
    gamma, beta = r.uniform(0.5, 1.5, wl.C).astype(np.float32), r.normal(0, 0.1, wl.C).astype(np.float32)
    y, dx = torch.empty_like(x), torch.empty_like(dy)
    a = [G.to_dev(v) for v in (fm, fv, gamma, beta)]
    L.cgbn_frozen_forward(x, wl.N, wl.C, wl.H, wl.W, "NCHW", "f32", a[0], a[1], a[2], a[3], 1e-5, y)
    L.cgbn_frozen_backward(dy, wl.N, wl.C, wl.H, wl.W, "NCHW", "f32", a[1], a[2], 1e-5, dx)
    torch.cuda.synchronize()
    for c in (0, 21, 42, 63):
        xs, dys = x[:, c:c + 1].cpu().numpy().astype(np.float64), dy[:, c:c + 1].cpu().numpy().astype(np.float64)
        y_ref = F.frozen_forward_ref(xs, fm[c:c + 1], fv[c:c + 1], gamma[c:c + 1], beta[c:c + 1], 1e-5, "NCHW")
        dx_ref = F.frozen_backward_ref(dys, fv[c:c + 1], gamma[c:c + 1], 1e-5, "NCHW")
        assert np.max(np.abs(y[:, c:c + 1].cpu().numpy() - y_ref)) <= 1e-4
        assert G.max_rel_err(dx[:, c:c + 1].cpu().numpy(), dx_ref, G.rms(dx_ref)) <= 1e-4
