"""Pins for the fixed-statistics oracle (oracle/frozen_bn_oracle.py) against
things other than itself: closed forms, numpy's own mean/variance routines, the
(separately pinned) training forward in the limit where batch and fixed
statistics coincide, finite differences -- and planted mistakes that these pins
must catch."""

import os
import types

import numpy as np
import pytest

from oracle import cgbn_oracle as O
from oracle import frozen_bn_oracle as F

LAYOUTS = ("NCHW", "NHWC")


def _shape(layout, N, C, H, W):
    return (N, C, H, W) if layout == "NCHW" else (N, H, W, C)


def _axes(layout):
    return (0, 2, 3) if layout == "NCHW" else (0, 1, 2)


def _draw(layout, N=3, C=4, H=5, W=2, seed=5):
    r = np.random.default_rng(seed)
    x = r.normal(1.5, 2.0, _shape(layout, N, C, H, W))
    return r, x, r.uniform(0.5, 1.5, C), r.normal(0, 0.3, C)


# ---- forward ---------------------------------------------------------------

@pytest.mark.parametrize("layout", LAYOUTS)
def test_landmarks_closed_form(layout):
    """x = m gives beta; x = m +- sqrt(s2 + eps) gives beta +- gamma (s2 + eps = 4, so the root is exact)."""
    C = 3
    m, s2, eps = np.array([0.5, -2.0, 10.0]), np.array([3.0, 3.0, 3.0]), 1.0
    g, b = np.array([2.0, -1.0, 0.25]), np.array([0.1, 0.2, -0.3])
    x = np.empty(_shape(layout, 3, C, 1, 1))
    for n, off in enumerate((0.0, 2.0, -2.0)):
        x[n] = (m + off).reshape(x[n].shape)
    y = F.frozen_forward_ref(x, m, s2, g, b, eps, layout)
    np.testing.assert_allclose(y[0].ravel(), b, rtol=0, atol=1e-15)
    np.testing.assert_allclose(y[1].ravel(), b + g, rtol=0, atol=1e-15)
    np.testing.assert_allclose(y[2].ravel(), b - g, rtol=0, atol=1e-15)


@pytest.mark.parametrize("layout", LAYOUTS)
def test_equals_training_forward_when_the_fixed_statistics_are_the_batch_statistics(layout):
    r, x, g, b = _draw(layout)
    eps = 1e-3
    m = np.mean(x, axis=_axes(layout))            # numpy's routines, not the oracle's arithmetic
    s2 = np.var(x, axis=_axes(layout))
    y_train, _, _ = O.cgbn_forward_ref(x, g, b, eps, layout)
    np.testing.assert_allclose(F.frozen_forward_ref(x, m, s2, g, b, eps, layout), y_train, rtol=1e-12, atol=1e-12)


def test_channels_last_is_a_transposition():
    r, x, g, b = _draw("NCHW")
    m, s2 = r.normal(0, 1, 4), r.uniform(0.1, 2, 4)
    y = F.frozen_forward_ref(x, m, s2, g, b, 1e-5, "NCHW")
    yl = F.frozen_forward_ref(x.transpose(0, 2, 3, 1), m, s2, g, b, 1e-5, "NHWC")
    np.testing.assert_array_equal(yl, y.transpose(0, 2, 3, 1))


@pytest.mark.parametrize("layout", LAYOUTS)
def test_is_the_per_channel_affine_map(layout):
    """y = a x + d with a = gamma / sqrt(s2 + eps), d = beta - m a: the form an inference engine folds it to."""
    r, x, g, b = _draw(layout)
    m, s2, eps = r.normal(0, 1, 4), r.uniform(0.1, 2, 4), 1e-5
    a = g / np.sqrt(s2 + eps)
    d = b - m * a
    bc = (1, -1, 1, 1) if layout == "NCHW" else (1, 1, 1, -1)
    np.testing.assert_allclose(F.frozen_forward_ref(x, m, s2, g, b, eps, layout), x * a.reshape(bc) + d.reshape(bc),
                               rtol=1e-12, atol=1e-12)


def test_eps_sits_inside_the_root():
    x = np.full((1, 1, 1, 1), 3.0)
    y = F.frozen_forward_ref(x, [1.0], [0.0], [1.0], [0.0], 4.0, "NCHW")       # (3-1)/sqrt(0+4) = 1
    assert y.item() == 1.0


# ---- backward --------------------------------------------------------------

@pytest.mark.parametrize("layout", LAYOUTS)
def test_backward_is_the_derivative_of_the_forward(layout):
    r, x, g, b = _draw(layout, N=2, C=3, H=2, W=2)
    m, s2, eps = r.normal(0, 1, 3), r.uniform(0.1, 2, 3), 1e-2
    dy = r.normal(0, 1, x.shape)
    dx = F.frozen_backward_ref(dy, s2, g, eps, layout)
    h = 1e-3                                       # the map is affine: central differences are exact up to rounding
    num = np.empty_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        num[i] = ((F.frozen_forward_ref(xp, m, s2, g, b, eps, layout)
                   - F.frozen_forward_ref(xm, m, s2, g, b, eps, layout)) * dy).sum() / (2 * h)
    np.testing.assert_allclose(dx, num, rtol=1e-9, atol=1e-9)


def test_backward_closed_form():
    dy = np.array([1.0, -2.0, 4.0]).reshape(3, 1, 1, 1)
    dx = F.frozen_backward_ref(dy, [15.0], [3.0], 1.0, "NCHW")                 # 3 / sqrt(16)
    np.testing.assert_array_equal(dx.ravel(), np.array([0.75, -1.5, 3.0]))


# ---- running statistics ----------------------------------------------------

def test_momentum_one_gives_the_batch_statistics_with_numpys_variance():
    r = np.random.default_rng(11)
    x = r.normal(3, 2, (5, 3, 4, 2))
    M = 5 * 4 * 2
    mu, s2 = x.mean(axis=(0, 2, 3)), x.var(axis=(0, 2, 3))
    rm, rv = F.running_update_ref(mu, s2, M, 1.0, True, np.zeros(3), np.ones(3))
    np.testing.assert_allclose(rm, mu, rtol=1e-15)
    np.testing.assert_allclose(rv, x.var(axis=(0, 2, 3), ddof=1), rtol=1e-13)
    _, rvb = F.running_update_ref(mu, s2, M, 1.0, False, np.zeros(3), np.ones(3))
    np.testing.assert_allclose(rvb, x.var(axis=(0, 2, 3), ddof=0), rtol=1e-15)


def test_momentum_zero_changes_nothing():
    rm, rv = F.running_update_ref([5.0], [7.0], 10, 0.0, True, [1.25], [2.5])
    assert rm.item() == 1.25 and rv.item() == 2.5


def test_hand_example():
    # M = 5: unbiased factor 5/4.  momentum 0.25: m = 0.75*2 + 0.25*10 = 4 ; s2 = 0.75*8 + 0.25*(4*5/4) = 7.25
    rm, rv = F.running_update_ref([10.0], [4.0], 5, 0.25, True, [2.0], [8.0])
    assert rm.item() == 4.0 and rv.item() == 7.25
    _, rvb = F.running_update_ref([10.0], [4.0], 5, 0.25, False, [2.0], [8.0])
    assert rvb.item() == 7.0


def test_repeated_updates_follow_the_geometric_closed_form():
    mu, s2, M, mom = np.array([1.0, -3.0]), np.array([2.0, 0.5]), 9, 0.1
    rm, rv = np.array([10.0, 10.0]), np.array([4.0, 4.0])
    rm0, rv0 = rm.copy(), rv.copy()
    for _ in range(25):
        rm, rv = F.running_update_ref(mu, s2, M, mom, True, rm, rv)
    decay = (1 - mom) ** 25
    np.testing.assert_allclose(rm, mu + decay * (rm0 - mu), rtol=1e-12)
    np.testing.assert_allclose(rv, s2 * 9 / 8 + decay * (rv0 - s2 * 9 / 8), rtol=1e-12)


def test_unbiased_needs_two_values():
    with pytest.raises(ValueError):
        F.running_update_ref([0.0], [0.0], 1, 0.1, True, [0.0], [1.0])


# ---- do these pins bite? ----------------------------------------------------

SRC = open(os.path.join(os.path.dirname(F.__file__), "frozen_bn_oracle.py")).read()

MUTANTS = [
    ("eps outside the root (forward)", "/ np.sqrt(s2 + float(eps)) + _bcast(beta, layout)",
     "/ (np.sqrt(s2) + float(eps)) + _bcast(beta, layout)"),
    ("beta dropped", "/ np.sqrt(s2 + float(eps)) + _bcast(beta, layout)", "/ np.sqrt(s2 + float(eps))"),
    ("mean not subtracted", "_bcast(gamma, layout) * (x - m) /", "_bcast(gamma, layout) * x /"),
    ("standard deviation passed for the variance", "return _bcast(gamma, layout) * (x - m) / np.sqrt(s2 + float(eps))",
     "return _bcast(gamma, layout) * (x - m) / (s2 + float(eps))"),
    ("gamma dropped from dx", "return dy * (_bcast(gamma, layout) / np.sqrt(", "return dy * (1.0 / np.sqrt("),
    ("eps dropped from dx", "np.sqrt(_bcast(fixed_var, layout) + float(eps)))", "np.sqrt(_bcast(fixed_var, layout)))"),
    ("channels-last axis off by one", "    elif layout == \"NHWC\":\n        shape[3] = -1", "    elif layout == \"NHWC\":\n        shape[2] = -1"),
    ("unbiased factor inverted", "s2 = s2 * (float(M) / float(M - 1))", "s2 = s2 * (float(M - 1) / float(M))"),
    ("unbiased factor ignored", "    if unbiased:\n        if M < 2:", "    if False:\n        if M < 2:"),
    ("momentum weights swapped", "return keep * rm + float(momentum) * mu, keep * rv + float(momentum) * s2",
     "return float(momentum) * rm + keep * mu, float(momentum) * rv + keep * s2"),
    ("running variance updated with the mean's weight only", "keep * rv + float(momentum) * s2", "rv + float(momentum) * s2"),
]


def _battery():
    calls = [test_channels_last_is_a_transposition, test_eps_sits_inside_the_root, test_backward_closed_form,
             test_momentum_one_gives_the_batch_statistics_with_numpys_variance, test_momentum_zero_changes_nothing,
             test_hand_example, test_repeated_updates_follow_the_geometric_closed_form]
    for layout in LAYOUTS:
        calls += [lambda l=layout: test_landmarks_closed_form(l),
                  lambda l=layout: test_equals_training_forward_when_the_fixed_statistics_are_the_batch_statistics(l),
                  lambda l=layout: test_is_the_per_channel_affine_map(l),
                  lambda l=layout: test_backward_is_the_derivative_of_the_forward(l)]
    return calls


def _failures(module, monkeypatch):
    import sys
    monkeypatch.setattr(sys.modules[__name__], "F", module)
    n = 0
    for call in _battery():
        try:
            call()
        except Exception:
            n += 1
    return n


def test_real_oracle_passes_the_battery(monkeypatch):
    assert _failures(F, monkeypatch) == 0


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(what, old, new, monkeypatch):
    assert SRC.count(old) == 1, f"mutation site for {what!r} not found exactly once"
    mod = types.ModuleType("mutant_frozen_oracle")
    exec(compile(SRC.replace(old, new), "mutant_frozen_oracle.py", "exec"), mod.__dict__)
    assert _failures(mod, monkeypatch) > 0, f"no pin notices: {what}"
