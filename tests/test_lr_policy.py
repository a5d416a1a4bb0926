"""The learning-rate policy against what the paper states (section 3.2, section 4)
and against the properties that define a linear warmup."""

import math

import pytest

from paper_1711_07240_amd import lr_policy as P


def test_base_rate_and_linear_scaling():
    # section 4: 0.02 at mini-batch 16; section 3.2: rate scales with the batch
    assert P.scaled_lr(16) == 0.02
    assert math.isclose(P.scaled_lr(256), 0.32, rel_tol=1e-15)      # k = 16
    assert math.isclose(P.scaled_lr(2), 0.0025, rel_tol=1e-15)
    for k in (2, 3, 8):
        assert math.isclose(P.scaled_lr(16 * k), k * P.scaled_lr(16), rel_tol=1e-15)
    with pytest.raises(ValueError):
        P.scaled_lr(0)


def test_warmup_is_linear_with_constant_increment():
    r, rh, n = 0.02, 0.32, 500
    assert P.warmup_lr(0, n, r, rh) == r
    assert P.warmup_lr(n, n, r, rh) == rh and P.warmup_lr(10 * n, n, r, rh) == rh
    inc = [P.warmup_lr(i + 1, n, r, rh) - P.warmup_lr(i, n, r, rh) for i in range(n)]
    assert max(inc) - min(inc) < 1e-15 and math.isclose(inc[0], (rh - r) / n, rel_tol=1e-9)
    assert P.warmup_lr(3, 0, r, rh) == rh                           # no warmup at all
    assert math.isclose(P.warmup_lr(n // 2, n, r, rh), (r + rh) / 2, rel_tol=1e-15)


def test_normal_policy_steps():
    f = [P.policy_factor(e, "normal") for e in range(11)]
    assert f[:8] == [1.0] * 8
    assert all(math.isclose(v, 0.1) for v in f[8:10]) and math.isclose(f[10], 0.01)
    assert P.total_epochs("normal") == 11
    with pytest.raises(ValueError):
        P.policy_factor(11, "normal")


def test_long_policy_steps():
    f = [P.policy_factor(e, "long") for e in range(18)]
    assert f[:11] == [1.0] * 11
    assert all(math.isclose(v, 0.1) for v in f[11:14])
    assert all(math.isclose(v, 0.01) for v in f[14:17])
    assert math.isclose(f[17], 0.005)                               # halved at epoch 17
    assert P.total_epochs("long") == 18


def test_combined_schedule():
    ipe = 118000 // 256                                             # iterations per epoch at batch 256 on 118k images
    lr = lambda it: P.learning_rate(it, ipe, 256, "normal", warmup_iters=200)
    assert lr(0) == 0.02 and math.isclose(lr(200), 0.32) and math.isclose(lr(100), 0.17)
    assert math.isclose(lr(8 * ipe), 0.032) and math.isclose(lr(8 * ipe - 1), 0.32)
    assert math.isclose(lr(10 * ipe), 0.0032)
    with pytest.raises(ValueError):
        lr(11 * ipe)
