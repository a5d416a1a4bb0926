"""Pins for oracle/cgbn_relu_oracle.py: hand-worked values, finite differences of
the whole composed map (statistics included) away from the ReLU's kink, the
structure of the mask -- and planted mistakes these pins must catch."""

import os
import types

import numpy as np
import pytest

from oracle import cgbn_oracle as O
from oracle import cgbn_relu_oracle as R

LAYOUTS = ("NCHW", "NHWC")


def _shape(layout, N, C, H, W):
    return (N, C, H, W) if layout == "NCHW" else (N, H, W, C)


@pytest.mark.parametrize("layout", LAYOUTS)
def test_hand_example(layout):
    # one channel, two values -1 and 1: mean 0, biased variance 1; eps = 3 makes invstd exactly 1/2.
    # gamma = 2, beta = 1/2: z = (-1/2, 3/2); ReLU: (0, 3/2).  With shortcut (1, -2): z + r = (1/2, -1/2) -> (1/2, 0).
    x = np.array([-1.0, 1.0]).reshape(_shape(layout, 2, 1, 1, 1))
    y, mean, invstd = R.cgbn_relu_forward_ref(x, [2.0], [0.5], 3.0, layout)
    assert mean.item() == 0.0 and invstd.item() == 0.5
    np.testing.assert_array_equal(y.ravel(), [0.0, 1.5])
    r = np.array([1.0, -2.0]).reshape(x.shape)
    y2, _, _ = R.cgbn_relu_forward_ref(x, [2.0], [0.5], 3.0, layout, residual=r)
    np.testing.assert_array_equal(y2.ravel(), [0.5, 0.0])
    # backward of the first case with dy = (5, 7): only the second element passes: dz = (0, 7)
    # xhat = (-1/2, 1/2): dbeta = 7, dgamma = 7/2; dx = gamma*invstd*(dz - dbeta/2 - xhat*dgamma/2)
    #   = 1 * ((0, 7) - 7/2 - (-1/2, 1/2)*7/4) = (-3.5 + 0.875, 3.5 - 0.875) = (-2.625, 2.625)
    dy = np.array([5.0, 7.0]).reshape(x.shape)
    dx, dgamma, dbeta, dz = R.cgbn_relu_backward_ref(dy, y, x, mean, invstd, [2.0], layout)
    np.testing.assert_array_equal(dz.ravel(), [0.0, 7.0])
    assert dbeta.item() == 7.0 and dgamma.item() == 3.5
    np.testing.assert_array_equal(dx.ravel(), [-2.625, 2.625])


def _problem(layout, seed=3, with_residual=True):
    r = np.random.default_rng(seed)
    shape = _shape(layout, 3, 2, 3, 2)
    x = r.normal(0.3, 1.5, shape)
    res = r.normal(0, 1, shape) if with_residual else None
    gamma, beta = r.uniform(0.5, 1.5, 2), r.normal(0, 0.3, 2)
    dy = r.normal(0, 1, shape)
    return x, res, gamma, beta, dy


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("with_residual", [False, True])
def test_backward_matches_central_differences(layout, with_residual):
    eps, h = 1e-2, 1e-6
    x, res, gamma, beta, dy = _problem(layout, 3, with_residual)
    y, mean, invstd = R.cgbn_relu_forward_ref(x, gamma, beta, eps, layout, residual=res)
    z, _, _ = O.cgbn_forward_ref(x, gamma, beta, eps, layout)
    pre = z + (res if with_residual else 0.0)
    assert np.min(np.abs(pre)) > 1e-3, "a pre-activation sits on the kink: pick another seed"
    dx, dgamma, dbeta, dz = R.cgbn_relu_backward_ref(dy, y, x, mean, invstd, gamma, layout)
    loss = lambda xx, rr, g, b: float((dy * R.cgbn_relu_forward_ref(xx, g, b, eps, layout, residual=rr)[0]).sum())
    num = np.empty_like(x)
    for i in np.ndindex(x.shape):
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        num[i] = (loss(xp, res, gamma, beta) - loss(xm, res, gamma, beta)) / (2 * h)
    np.testing.assert_allclose(dx, num, rtol=2e-6, atol=2e-8)
    if with_residual:
        numr = np.empty_like(x)
        for i in np.ndindex(x.shape):
            rp, rm = res.copy(), res.copy()
            rp[i] += h
            rm[i] -= h
            numr[i] = (loss(x, rp, gamma, beta) - loss(x, rm, gamma, beta)) / (2 * h)
        np.testing.assert_allclose(dz, numr, rtol=2e-6, atol=2e-8)
    for c in range(2):
        gp, gm, bp, bm = gamma.copy(), gamma.copy(), beta.copy(), beta.copy()
        gp[c] += h; gm[c] -= h; bp[c] += h; bm[c] -= h
        np.testing.assert_allclose(dgamma[c], (loss(x, res, gp, beta) - loss(x, res, gm, beta)) / (2 * h), rtol=2e-6)
        np.testing.assert_allclose(dbeta[c], (loss(x, res, gamma, bp) - loss(x, res, gamma, bm)) / (2 * h), rtol=2e-6)


@pytest.mark.parametrize("layout", LAYOUTS)
def test_structure(layout):
    x, res, gamma, beta, dy = _problem(layout, 8)
    y, mean, invstd = R.cgbn_relu_forward_ref(x, gamma, beta, 1e-5, layout, residual=res)
    assert y.min() == 0.0 and (y == 0).any() and (y > 0).any()
    # statistics are those of x alone, whatever the shortcut holds
    ax = (0, 2, 3) if layout == "NCHW" else (0, 1, 2)
    np.testing.assert_allclose(mean, x.mean(axis=ax), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(invstd, 1 / np.sqrt(x.var(axis=ax) + 1e-5), rtol=1e-13)
    # no shortcut == a shortcut of zeros
    y0, _, _ = R.cgbn_relu_forward_ref(x, gamma, beta, 1e-5, layout)
    yz, _, _ = R.cgbn_relu_forward_ref(x, gamma, beta, 1e-5, layout, residual=np.zeros_like(x))
    np.testing.assert_array_equal(y0, yz)
    # the mask is read off y: nothing flows where y == 0, dy flows unchanged elsewhere
    dx, dgamma, dbeta, dz = R.cgbn_relu_backward_ref(dy, y, x, mean, invstd, gamma, layout)
    assert np.all(dz[y == 0] == 0) and np.array_equal(dz[y > 0], dy[y > 0])
    # with every output positive the layer is plain CGBN
    big = np.full_like(x, 100.0)
    yb, m2, i2 = R.cgbn_relu_forward_ref(x, gamma, beta, 1e-5, layout, residual=big)
    zb, _, _ = O.cgbn_forward_ref(x, gamma, beta, 1e-5, layout)
    np.testing.assert_array_equal(yb, zb + big)
    dxb, dgb, dbb, dzb = R.cgbn_relu_backward_ref(dy, yb, x, m2, i2, gamma, layout)
    dxp, dgp, dbp = O.cgbn_backward_ref(dy, x, m2, i2, gamma, layout)
    np.testing.assert_array_equal(dxb, dxp)
    np.testing.assert_array_equal(dzb, dy)


SRC = open(os.path.join(os.path.dirname(R.__file__), "cgbn_relu_oracle.py")).read()

MUTANTS = [
    ("shortcut dropped", "        z = z + np.asarray(residual, dtype=np.float64)", "        z = z"),
    ("shortcut subtracted", "z = z + np.asarray(residual", "z = z - np.asarray(residual"),
    ("ReLU dropped", "return np.maximum(z, 0.0), mean, invstd", "return z, mean, invstd"),
    ("ReLU turned into abs", "return np.maximum(z, 0.0), mean, invstd", "return np.abs(z), mean, invstd"),
    ("mask inverted", "> 0.0, dy, 0.0)", "> 0.0, 0.0, dy)"),
    ("mask dropped", "dz = np.where(np.asarray(y, dtype=np.float64) > 0.0, dy, 0.0)", "dz = dy"),
    ("mask lets the kink through", "dtype=np.float64) > 0.0, dy, 0.0)", "dtype=np.float64) >= 0.0, dy, 0.0)"),
    ("statistics' gradient taken from dy instead of dz", "O.cgbn_backward_ref(dz, x,", "O.cgbn_backward_ref(dy, x,"),
]


def _battery():
    calls = []
    for layout in LAYOUTS:
        calls += [lambda l=layout: test_hand_example(l), lambda l=layout: test_structure(l),
                  lambda l=layout: test_backward_matches_central_differences(l, True),
                  lambda l=layout: test_backward_matches_central_differences(l, False)]
    return calls


def _failures(module, monkeypatch):
    import sys
    monkeypatch.setattr(sys.modules[__name__], "R", module)
    n = 0
    for call in _battery():
        try:
            call()
        except Exception:
            n += 1
    return n


def test_real_oracle_passes_the_battery(monkeypatch):
    assert _failures(R, monkeypatch) == 0


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(what, old, new, monkeypatch):
    assert SRC.count(old) == 1, f"mutation site for {what!r} not found exactly once"
    mod = types.ModuleType("oracle.mutant_relu_oracle")
    mod.__package__ = "oracle"
    exec(compile(SRC.replace(old, new), "mutant_relu_oracle.py", "exec"), mod.__dict__)
    assert _failures(mod, monkeypatch) > 0, f"no pin notices: {what}"
