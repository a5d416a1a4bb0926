"""Pins for the float64 oracle: everything here runs on the CPU.

The oracle is checked against things other than itself: two hand-worked
examples (tests/golden), closed forms, invariants, central finite differences,
brute-force index loops, and a float64 library batch norm with autograd.
"""

import itertools
import math

import numpy as np
import pytest
import torch

from conftest import load_golden
from oracle import cgbn_oracle as O


def _rand(shape, seed, scale=1.0, shift=0.0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(shape) * scale + shift


def _to_layout(x_nchw, layout):
    return x_nchw if layout == "NCHW" else np.ascontiguousarray(x_nchw.transpose(0, 2, 3, 1))


def _from_layout(x, layout):
    return x if layout == "NCHW" else x.transpose(0, 3, 1, 2)


# --------------------------------------------------------------------------
# hand-worked examples
# --------------------------------------------------------------------------

@pytest.mark.parametrize("layout", O.LAYOUTS)
def test_hand_example_two_values(layout):
    g = load_golden("hand_example_two_values.txt")
    x = np.array(g["x"]).reshape(2, 1, 1, 1)
    dy = np.array(g["dy"]).reshape(2, 1, 1, 1)
    K = int(g["K"][0])
    gamma, beta, eps = np.array(g["gamma"]), np.array(g["beta"]), g["eps"][0]

    y, mean, invstd, s, v = O.cgbn_forward_alg1(x, K, gamma, beta, eps, layout)
    assert np.allclose(s[:, 0], g["s"], rtol=0, atol=1e-15)
    assert np.allclose(v[:, 0], g["v"], rtol=0, atol=1e-15)
    assert mean[0] == pytest.approx(g["mean"][0], abs=1e-15)
    assert invstd[0] == pytest.approx(g["invstd"][0], abs=1e-15)
    assert np.allclose(y.ravel(), g["y"], rtol=0, atol=1e-15)

    y2, mean2, invstd2 = O.cgbn_forward_ref(x, gamma, beta, eps, layout)
    assert np.allclose(y2.ravel(), g["y"], rtol=0, atol=1e-15)
    assert mean2[0] == pytest.approx(g["mean"][0], abs=1e-15)
    assert invstd2[0] == pytest.approx(g["invstd"][0], abs=1e-15)

    dx, dgamma, dbeta = O.cgbn_backward_ref(dy, x, mean, invstd, gamma, layout)
    assert np.allclose(dx.ravel(), g["dx"], rtol=0, atol=1e-15)
    assert dgamma[0] == pytest.approx(g["dgamma"][0], abs=1e-15)
    assert dbeta[0] == pytest.approx(g["dbeta"][0], abs=1e-15)

    dx3, dgamma3, dbeta3, a, b = O.cgbn_backward_sharded(dy, x, mean, invstd, gamma, K, layout)
    assert np.allclose(dx3.ravel(), g["dx"], rtol=0, atol=1e-15)
    assert np.allclose(a[:, 0], [1.0, 0.0], atol=1e-15)        # per-device sum of dy
    assert np.allclose(b[:, 0], [-0.5, 0.0], atol=1e-15)       # per-device sum of dy*xhat


@pytest.mark.parametrize("layout", O.LAYOUTS)
def test_hand_example_pooled_variance(layout):
    g = load_golden("hand_example_pooled_variance.txt")
    x = np.array(g["x"]).reshape(4, 1, 1, 1)
    gamma, beta, eps = np.array(g["gamma"]), np.array(g["beta"]), g["eps"][0]
    y, mean, invstd, s, v = O.cgbn_forward_alg1(x, int(g["K"][0]), gamma, beta, eps, layout)
    assert np.allclose(s[:, 0], g["s"], atol=1e-15)
    assert np.allclose(v[:, 0], g["v"], atol=1e-15)
    assert mean[0] == pytest.approx(g["mean"][0], abs=1e-15)
    var = 1.0 / invstd[0] ** 2 - eps
    assert var == pytest.approx(g["var"][0], abs=1e-12)
    assert abs(var - g["var_if_local_means_were_used"][0]) > 1.0   # the rejected reading
    assert invstd[0] == pytest.approx(g["invstd"][0], abs=1e-15)
    assert np.allclose(y.ravel(), g["y"], atol=1e-15)
    y2, _, invstd2 = O.cgbn_forward_ref(x, gamma, beta, eps, layout)
    assert invstd2[0] == pytest.approx(g["invstd"][0], abs=1e-15)
    assert np.allclose(y2.ravel(), g["y"], atol=1e-15)


# --------------------------------------------------------------------------
# brute force with explicit index arithmetic on flat buffers (both layouts)
# --------------------------------------------------------------------------

def _flat_index(layout, n, c, h, w, N, C, H, W):
    if layout == "NCHW":
        return ((n * C + c) * H + h) * W + w
    return ((n * H + h) * W + w) * C + c


def _brute_force(xf, dyf, gamma, beta, eps, layout, N, C, H, W, K):
    """math.fsum loops straight from the definitions; returns flat lists."""
    M = N * H * W
    per = N // K
    y = [0.0] * len(xf)
    dx = [0.0] * len(xf)
    mean, invstd, dgamma, dbeta = [], [], [], []
    s = [[0.0] * C for _ in range(K)]
    v = [[0.0] * C for _ in range(K)]
    a = [[0.0] * C for _ in range(K)]
    b = [[0.0] * C for _ in range(K)]
    for c in range(C):
        idx = [[_flat_index(layout, n, c, h, w, N, C, H, W)
                for n in range(k * per, (k + 1) * per) for h in range(H) for w in range(W)]
               for k in range(K)]
        for k in range(K):
            s[k][c] = math.fsum(xf[i] for i in idx[k])
        mu = math.fsum(s[k][c] for k in range(K)) / M
        for k in range(K):
            v[k][c] = math.fsum((xf[i] - mu) ** 2 for i in idx[k])
        var = math.fsum(v[k][c] for k in range(K)) / M
        istd = 1.0 / math.sqrt(var + eps)
        mean.append(mu)
        invstd.append(istd)
        for k in range(K):
            a[k][c] = math.fsum(dyf[i] for i in idx[k])
            b[k][c] = math.fsum(dyf[i] * (xf[i] - mu) * istd for i in idx[k])
        db = math.fsum(a[k][c] for k in range(K))
        dg = math.fsum(b[k][c] for k in range(K))
        dbeta.append(db)
        dgamma.append(dg)
        for k in range(K):
            for i in idx[k]:
                xh = (xf[i] - mu) * istd
                y[i] = gamma[c] * xh + beta[c]
                dx[i] = gamma[c] * istd * (dyf[i] - db / M - xh * dg / M)
    return dict(y=y, dx=dx, mean=mean, invstd=invstd, dgamma=dgamma, dbeta=dbeta,
                s=s, v=v, a=a, b=b)


@pytest.mark.parametrize("layout", O.LAYOUTS)
@pytest.mark.parametrize("N,C,H,W,K", [(4, 3, 2, 5, 2), (6, 2, 3, 3, 3), (2, 5, 1, 7, 1)])
def test_brute_force_both_layouts(layout, N, C, H, W, K):
    shape = (N, C, H, W) if layout == "NCHW" else (N, H, W, C)
    x = _rand(shape, 11, 1.7, 0.4)
    dy = _rand(shape, 12)
    gamma = _rand(C, 13, 0.3, 1.0)
    beta = _rand(C, 14, 0.2)
    eps = 1e-3
    bf = _brute_force(x.ravel().tolist(), dy.ravel().tolist(), gamma.tolist(), beta.tolist(),
                      eps, layout, N, C, H, W, K)
    y, mean, invstd, s, v = O.cgbn_forward_alg1(x, K, gamma, beta, eps, layout)
    dx, dgamma, dbeta, a, b = O.cgbn_backward_sharded(dy, x, mean, invstd, gamma, K, layout)
    tol = dict(rtol=1e-12, atol=1e-12)
    assert np.allclose(y.ravel(), bf["y"], **tol)
    assert np.allclose(dx.ravel(), bf["dx"], **tol)
    assert np.allclose(mean, bf["mean"], **tol)
    assert np.allclose(invstd, bf["invstd"], **tol)
    assert np.allclose(dgamma, bf["dgamma"], **tol)
    assert np.allclose(dbeta, bf["dbeta"], **tol)
    assert np.allclose(s, bf["s"], **tol) and np.allclose(v, bf["v"], **tol)
    assert np.allclose(a, bf["a"], **tol) and np.allclose(b, bf["b"], **tol)
    # the plain definition against the same brute force
    y2, mean2, invstd2 = O.cgbn_forward_ref(x, gamma, beta, eps, layout)
    dx2, dgamma2, dbeta2 = O.cgbn_backward_ref(dy, x, mean2, invstd2, gamma, layout)
    assert np.allclose(y2.ravel(), bf["y"], **tol)
    assert np.allclose(dx2.ravel(), bf["dx"], **tol)
    assert np.allclose(dgamma2, bf["dgamma"], **tol)
    assert np.allclose(dbeta2, bf["dbeta"], **tol)


# --------------------------------------------------------------------------
# invariants and closed forms
# --------------------------------------------------------------------------

@pytest.mark.parametrize("layout", O.LAYOUTS)
def test_normalised_moments_closed_form(layout):
    N, C, H, W = 8, 5, 6, 7
    shape = (N, C, H, W) if layout == "NCHW" else (N, H, W, C)
    x = _rand(shape, 21, 2.5, -3.0)
    eps = 0.37
    ones, zeros = np.ones(C), np.zeros(C)
    xhat, mean, invstd = O.cgbn_forward_ref(x, ones, zeros, eps, layout)
    axes = O._pooled_axes(layout)
    var = 1.0 / invstd ** 2 - eps
    assert np.allclose(xhat.mean(axis=axes), 0.0, atol=1e-13)
    # biased variance of the normalised output is sigma^2/(sigma^2+eps), not 1
    assert np.allclose((xhat ** 2).mean(axis=axes), var / (var + eps), rtol=1e-12)
    # against numpy's own moments
    assert np.allclose(mean, x.mean(axis=axes), rtol=1e-13)
    assert np.allclose(var, x.var(axis=axes), rtol=1e-12)


@pytest.mark.parametrize("layout", O.LAYOUTS)
def test_shard_count_does_not_change_the_result(layout):
    N, C, H, W = 12, 4, 3, 5
    shape = (N, C, H, W) if layout == "NCHW" else (N, H, W, C)
    x = _rand(shape, 31, 1.3, 0.7)
    dy = _rand(shape, 32)
    gamma, beta, eps = _rand(C, 33, 0.2, 1.0), _rand(C, 34), 1e-5
    y0, mean0, invstd0 = O.cgbn_forward_ref(x, gamma, beta, eps, layout)
    dx0, dg0, db0 = O.cgbn_backward_ref(dy, x, mean0, invstd0, gamma, layout)
    for K in (1, 2, 3, 4, 6, 12):
        y, mean, invstd, s, v = O.cgbn_forward_alg1(x, K, gamma, beta, eps, layout)
        assert s.shape == (K, C) and v.shape == (K, C)
        assert np.allclose(y, y0, rtol=1e-12, atol=1e-12)
        assert np.allclose(mean, mean0, rtol=1e-12, atol=1e-14)
        assert np.allclose(invstd, invstd0, rtol=1e-12)
        dx, dg, db, a, b = O.cgbn_backward_sharded(dy, x, mean, invstd, gamma, K, layout)
        assert np.allclose(dx, dx0, rtol=1e-11, atol=1e-12)
        assert np.allclose(dg, dg0, rtol=1e-11, atol=1e-12)
        assert np.allclose(db, db0, rtol=1e-11, atol=1e-12)
    for K in (0, 5, 13):
        with pytest.raises(ValueError):
            O.cgbn_forward_alg1(x, K, gamma, beta, eps, layout)


def test_device_local_variance_would_differ():
    # two devices with very different local means: pooled variance must contain
    # the between-device term
    x = np.concatenate([_rand((2, 1, 4, 4), 41, 1.0, -5.0), _rand((2, 1, 4, 4), 42, 1.0, 5.0)])
    _, _, invstd, _, v = O.cgbn_forward_alg1(x, 2, np.ones(1), np.zeros(1), 1e-9, "NCHW")
    var = 1.0 / invstd[0] ** 2 - 1e-9
    local = 0.5 * (x[:2].var() + x[2:].var())
    assert var == pytest.approx(x.var(), rel=1e-10)
    assert var > 10 * local


@pytest.mark.parametrize("layout", O.LAYOUTS)
def test_gradient_sums_closed_forms(layout):
    N, C, H, W = 6, 3, 4, 5
    shape = (N, C, H, W) if layout == "NCHW" else (N, H, W, C)
    x, dy = _rand(shape, 51, 0.8, 2.0), _rand(shape, 52)
    gamma, beta, eps = _rand(C, 53, 0.2, 1.0), _rand(C, 54), 0.05
    _, mean, invstd = O.cgbn_forward_ref(x, gamma, beta, eps, layout)
    dx, dgamma, dbeta = O.cgbn_backward_ref(dy, x, mean, invstd, gamma, layout)
    axes = O._pooled_axes(layout)
    xhat = (x - O._per_channel(mean, layout)) * O._per_channel(invstd, layout)
    var = 1.0 / invstd ** 2 - eps
    # sum of dx over the pooled axes vanishes
    assert np.allclose(dx.sum(axis=axes), 0.0, atol=1e-12)
    # sum of dx*xhat = gamma*invstd*dgamma*eps/(var+eps)
    assert np.allclose((dx * xhat).sum(axis=axes), gamma * invstd * dgamma * eps / (var + eps),
                       rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("layout", O.LAYOUTS)
@pytest.mark.parametrize("K", [1, 2, 4])
def test_backward_matches_central_differences(layout, K):
    N, C, H, W = 4, 2, 3, 3
    shape = (N, C, H, W) if layout == "NCHW" else (N, H, W, C)
    x, dy = _rand(shape, 61, 1.5, 0.3), _rand(shape, 62)
    gamma, beta, eps = _rand(C, 63, 0.3, 1.0), _rand(C, 64), 1e-2

    def loss(x_, g_, b_):
        y = O.cgbn_forward_alg1(x_, K, g_, b_, eps, layout)[0]
        return float((dy * y).sum())

    _, mean, invstd = O.cgbn_forward_ref(x, gamma, beta, eps, layout)
    dx, dgamma, dbeta = O.cgbn_backward_ref(dy, x, mean, invstd, gamma, layout)
    h = 1e-6
    fd = np.zeros_like(x)
    for idx in itertools.product(*[range(s) for s in x.shape]):
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        fd[idx] = (loss(xp, gamma, beta) - loss(xm, gamma, beta)) / (2 * h)
    assert np.allclose(dx, fd, rtol=1e-6, atol=1e-8)
    for c in range(C):
        e = np.zeros(C)
        e[c] = h
        fg = (loss(x, gamma + e, beta) - loss(x, gamma - e, beta)) / (2 * h)
        fb = (loss(x, gamma, beta + e) - loss(x, gamma, beta - e)) / (2 * h)
        assert dgamma[c] == pytest.approx(fg, rel=1e-7, abs=1e-8)
        assert dbeta[c] == pytest.approx(fb, rel=1e-7, abs=1e-8)


# --------------------------------------------------------------------------
# special cases
# --------------------------------------------------------------------------

def test_constant_channel():
    x = np.full((4, 2, 3, 3), 100.0)
    x[:, 1] = _rand((4, 3, 3), 71)
    gamma, beta, eps = np.array([1.3, 0.7]), np.array([0.25, -0.5]), 1e-5
    y, mean, invstd = O.cgbn_forward_ref(x, gamma, beta, eps)
    assert mean[0] == 100.0
    assert invstd[0] == pytest.approx(eps ** -0.5, rel=1e-15)
    assert np.all(y[:, 0] == 0.25)
    dy = _rand(x.shape, 72)
    dx, dgamma, dbeta = O.cgbn_backward_ref(dy, x, mean, invstd, gamma)
    assert dgamma[0] == 0.0
    M = 4 * 9
    assert np.allclose(dx[:, 0], gamma[0] * eps ** -0.5 * (dy[:, 0] - dy[:, 0].sum() / M), rtol=1e-13)


def test_two_element_closed_form():
    a, b = 3.25, -1.5
    x = np.array([a, b]).reshape(2, 1, 1, 1)
    eps = 0.5
    _, mean, invstd = O.cgbn_forward_ref(x, np.ones(1), np.zeros(1), eps)
    assert mean[0] == pytest.approx((a + b) / 2)
    assert 1.0 / invstd[0] ** 2 - eps == pytest.approx((a - b) ** 2 / 4, rel=1e-14)


def test_affine_equivariance_and_image_permutation():
    N, C, H, W = 6, 3, 4, 4
    x = _rand((N, C, H, W), 81, 2.0, 1.0)
    gamma, beta, eps = _rand(C, 82, 0.2, 1.0), _rand(C, 83), 1e-3
    y0, _, _ = O.cgbn_forward_ref(x, gamma, beta, eps)
    alpha, delta = 3.5, -7.0
    y1, _, _ = O.cgbn_forward_ref(alpha * x + delta, gamma, beta, eps * alpha ** 2)
    assert np.allclose(y0, y1, rtol=1e-11, atol=1e-12)
    perm = np.random.default_rng(84).permutation(N)
    y2 = O.cgbn_forward_alg1(x[perm], 3, gamma, beta, eps)[0]
    assert np.allclose(y2, y0[perm], rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------
# library routine: float64 training-mode batch norm + autograd
# --------------------------------------------------------------------------

@pytest.mark.parametrize("layout", O.LAYOUTS)
@pytest.mark.parametrize("shape,K", [((4, 16, 32, 32), 2), ((6, 5, 7, 3), 3), ((2, 1, 1, 1), 2)])
def test_against_library_batch_norm(layout, shape, K):
    N, C, H, W = shape
    x_nchw = _rand(shape, 91, 1.4, -0.6)
    dy_nchw = _rand(shape, 92)
    gamma, beta, eps = _rand(C, 93, 0.25, 1.0), _rand(C, 94, 0.1), 1e-5

    xt = torch.tensor(x_nchw, dtype=torch.float64, requires_grad=True)
    gt = torch.tensor(gamma, dtype=torch.float64, requires_grad=True)
    bt = torch.tensor(beta, dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.batch_norm(xt, None, None, gt, bt, training=True, eps=eps)
    (yt * torch.tensor(dy_nchw)).sum().backward()
    var_t = xt.detach().var(dim=(0, 2, 3), unbiased=False)

    x, dy = _to_layout(x_nchw, layout), _to_layout(dy_nchw, layout)
    y, mean, invstd, _, _ = O.cgbn_forward_alg1(x, K, gamma, beta, eps, layout)
    dx, dgamma, dbeta = O.cgbn_backward_ref(dy, x, mean, invstd, gamma, layout)
    tol = dict(rtol=1e-9, atol=1e-10)
    assert np.allclose(_from_layout(y, layout), yt.detach().numpy(), **tol)
    assert np.allclose(mean, xt.detach().mean(dim=(0, 2, 3)).numpy(), **tol)
    assert np.allclose(invstd, (1.0 / torch.sqrt(var_t + eps)).numpy(), **tol)
    assert np.allclose(_from_layout(dx, layout), xt.grad.numpy(), **tol)
    assert np.allclose(dgamma, gt.grad.numpy(), **tol)
    assert np.allclose(dbeta, bt.grad.numpy(), **tol)


# --------------------------------------------------------------------------
# bfloat16 helpers against the library's conversions
# --------------------------------------------------------------------------

def test_bf16_widening_and_rounding_match_library():
    rng = np.random.default_rng(101)
    bits = rng.integers(0, 2 ** 16, size=4096, dtype=np.uint16)
    bits = bits[((bits >> 7) & 0xFF) != 0xFF]          # finite only
    wide = O.bf16_bits_to_f64(bits)
    t = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(wide, t)

    vals = np.concatenate([rng.standard_normal(4096) * 3.0,
                           np.array([1.00390625, 1.01171875, 100.25, -100.75, 0.0, 2.0 ** -130])])
    got = O.f64_to_bf16_bits_rne(vals)
    want = torch.tensor(vals, dtype=torch.float64).to(torch.float32).to(torch.bfloat16)
    want = want.view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert O.f64_to_bf16_bits_rne(np.array([1.0 + 2.0 ** -8]))[0] == 0x3F80
    assert O.f64_to_bf16_bits_rne(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 0x3F82
