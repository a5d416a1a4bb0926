"""Pins for oracle/one_sweep_oracle.py: the pairwise merge against numpy's own mean and
variance of the union, a hand-worked merge, the two-pass oracle, and planted mistakes."""

import os
import types

import numpy as np
import pytest

from oracle import cgbn_oracle as O
from oracle import one_sweep_oracle as S

LAYOUTS = ("NCHW", "NHWC")


def test_hand_worked_merge():
    # {1, 3}: n=2, mean=2, M2=2.   {5, 7, 9}: n=3, mean=7, M2=8.   union {1,3,5,7,9}: mean 5, M2 = 16+4+0+4+16 = 40
    n, mean, M2 = S.merge((2, np.array([2.0]), np.array([2.0])), (3, np.array([7.0]), np.array([8.0])))
    assert n == 5 and mean.item() == 5.0 and M2.item() == 40.0


def test_merge_matches_numpy_on_the_union():
    r = np.random.default_rng(2)
    a, b = r.normal(3, 2, (7, 4)), r.normal(-1, 0.5, (11, 4))
    sa = (7, a.mean(axis=0), ((a - a.mean(axis=0)) ** 2).sum(axis=0))
    sb = (11, b.mean(axis=0), ((b - b.mean(axis=0)) ** 2).sum(axis=0))
    n, mean, M2 = S.merge(sa, sb)
    u = np.concatenate([a, b])
    assert n == 18
    np.testing.assert_allclose(mean, u.mean(axis=0), rtol=1e-13)
    np.testing.assert_allclose(M2 / n, u.var(axis=0), rtol=1e-13)


@pytest.mark.parametrize("layout", LAYOUTS)
def test_shard_summary_against_numpy(layout):
    r = np.random.default_rng(4)
    x = r.normal(1, 3, (3, 5, 4, 2) if layout == "NCHW" else (3, 4, 2, 5))
    ax = (0, 2, 3) if layout == "NCHW" else (0, 1, 2)
    n, mean, M2 = S.shard_summary(x, layout)
    assert n == 24
    np.testing.assert_allclose(mean, x.mean(axis=ax), rtol=1e-13)
    np.testing.assert_allclose(M2, x.var(axis=ax) * n, rtol=1e-13)


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("K", [1, 2, 3, 6])
def test_equals_the_two_pass_definition(layout, K):
    r = np.random.default_rng(7)
    shape = (6, 3, 4, 5) if layout == "NCHW" else (6, 4, 5, 3)
    bs = (1, -1, 1, 1) if layout == "NCHW" else (1, 1, 1, -1)
    # shards with very different means: the d^2 term carries most of the variance
    x = r.normal(0, 1, shape) + np.arange(6).reshape(6, 1, 1, 1) * 10.0 + np.array([0.0, 100.0, -50.0]).reshape(bs)
    g, b = r.uniform(0.5, 1.5, 3), r.normal(0, 0.2, 3)
    y1, m1, i1 = S.cgbn_forward_one_sweep(x, K, g, b, 1e-5, layout)
    y2, m2, i2 = O.cgbn_forward_ref(x, g, b, 1e-5, layout)
    np.testing.assert_allclose(m1, m2, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(i1, i2, rtol=1e-12)
    np.testing.assert_allclose(y1, y2, rtol=1e-10, atol=1e-10)


SRC = open(os.path.join(os.path.dirname(S.__file__), "one_sweep_oracle.py")).read()
MUTANTS = [
    ("between-set term dropped", "return n, ma + d * (nb / n), Ma + Mb + d * d * (na * nb / n)", "return n, ma + d * (nb / n), Ma + Mb"),
    ("between-set term weighted by the sum of counts", "d * d * (na * nb / n)", "d * d * (na + nb)"),
    ("mean moved by the wrong weight", "ma + d * (nb / n)", "ma + d * (na / n)"),
    ("M2 about zero instead of the shard mean", "dev = xs - O._per_channel(mean, layout)", "dev = xs"),
    ("unbiased variance", "invstd = 1.0 / np.sqrt(M2 / n + float(eps))", "invstd = 1.0 / np.sqrt(M2 / (n - 1) + float(eps))"),
    ("eps outside the root", "invstd = 1.0 / np.sqrt(M2 / n + float(eps))", "invstd = 1.0 / (np.sqrt(M2 / n) + float(eps))"),
]


def _battery():
    calls = [test_hand_worked_merge, test_merge_matches_numpy_on_the_union]
    for layout in LAYOUTS:
        calls += [lambda l=layout: test_shard_summary_against_numpy(l),
                  lambda l=layout: test_equals_the_two_pass_definition(l, 3),
                  lambda l=layout: test_equals_the_two_pass_definition(l, 1)]
    return calls


def _failures(module, monkeypatch):
    import sys
    monkeypatch.setattr(sys.modules[__name__], "S", module)
    n = 0
    for call in _battery():
        try:
            call()
        except Exception:
            n += 1
    return n


def test_real_oracle_passes_the_battery(monkeypatch):
    assert _failures(S, monkeypatch) == 0


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(what, old, new, monkeypatch):
    assert SRC.count(old) == 1, f"mutation site for {what!r} not found exactly once"
    mod = types.ModuleType("oracle.mutant_one_sweep")
    mod.__package__ = "oracle"
    exec(compile(SRC.replace(old, new), "mutant_one_sweep.py", "exec"), mod.__dict__)
    assert _failures(mod, monkeypatch) > 0, f"no pin notices: {what}"
