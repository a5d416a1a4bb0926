"""Do the pins bite?  Plausible mistakes are planted in a COPY of the oracle's
source (on the CPU, in memory) and the pin tests are run against the copy:
every mutant must be caught by at least one pin, and the real oracle by none."""

import os
import types

import pytest

import test_oracle_pins as T
from oracle import cgbn_oracle as O

SRC = open(os.path.join(os.path.dirname(O.__file__), "cgbn_oracle.py")).read()

MUTANTS = [
    ("unbiased variance", "var = (dev * dev).sum(axis=axes) / M", "var = (dev * dev).sum(axis=axes) / (M - 1)", 1),
    ("eps outside the root (plain)", "invstd = 1.0 / np.sqrt(var + float(eps))\n    xhat",
     "invstd = 1.0 / (np.sqrt(var) + float(eps))\n    xhat", 1),
    ("eps outside the root (Algorithm 1 walk)", "invstd = 1.0 / np.sqrt(var + float(eps))\n    # step 11",
     "invstd = 1.0 / (np.sqrt(var) + float(eps))\n    # step 11", 1),
    ("deviations from the device-local mean", "d = x[sl] - _per_channel(mean, layout)",
     "d = x[sl] - _per_channel(s[k] / (M // K), layout)", 1),
    ("mean divided by the image count", "mean = x.sum(axis=axes) / M", "mean = x.sum(axis=axes) / x.shape[0]", 1),
    ("mean of Algorithm 1 divided by the shard count", "mean = s.sum(axis=0) / M", "mean = s.sum(axis=0) / K", 1),
    ("beta dropped", "y = _per_channel(gamma, layout) * xhat + _per_channel(beta, layout)",
     "y = _per_channel(gamma, layout) * xhat", 1),
    ("gamma dropped in step 11 of the walk", "y[sl] = g * (x[sl]", "y[sl] = (x[sl]", 1),
    ("dbeta term dropped from dx", "dy - _per_channel(dbeta, layout) / M - xhat * _per_channel(dgamma, layout) / M\n    )",
     "dy - xhat * _per_channel(dgamma, layout) / M\n    )", 1),
    ("sign of the dgamma term", "/ M - xhat * _per_channel(dgamma, layout) / M\n    )",
     "/ M + xhat * _per_channel(dgamma, layout) / M\n    )", 1),
    ("dgamma from x instead of xhat", "dgamma = (dy * xhat).sum(axis=axes)", "dgamma = (dy * x).sum(axis=axes)", 1),
    ("gamma dropped from dx", "dx = (_per_channel(gamma, layout) * _per_channel(invstd, layout)) * (",
     "dx = (_per_channel(invstd, layout)) * (", 1),
    ("per-shard count in the sharded backward", "dbeta = a.sum(axis=0)\n", "dbeta = a.sum(axis=0)\n    M = M // K\n", 1),
    ("sharded backward pools dgamma over one shard only", "dgamma = b.sum(axis=0)", "dgamma = b[0] * K", 1),
    ("channels-last axis off by one", "    if layout == \"NHWC\":\n        return 3", "    if layout == \"NHWC\":\n        return 2", 1),
    ("bfloat16 widened by the wrong shift", "<< np.uint32(16)\n    return b.view", "<< np.uint32(15)\n    return b.view", 1),
    ("bfloat16 rounding truncates", "rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)",
     "rounded = u >> np.uint32(16)", 1),
]


def battery():
    """The pin tests as zero-argument calls."""
    calls = []
    for layout in O.LAYOUTS:
        calls += [lambda l=layout: T.test_hand_example_two_values(l),
                  lambda l=layout: T.test_hand_example_pooled_variance(l),
                  lambda l=layout: T.test_brute_force_both_layouts(l, 4, 3, 2, 5, 2),
                  lambda l=layout: T.test_normalised_moments_closed_form(l),
                  lambda l=layout: T.test_shard_count_does_not_change_the_result(l),
                  lambda l=layout: T.test_gradient_sums_closed_forms(l),
                  lambda l=layout: T.test_backward_matches_central_differences(l, 2),
                  lambda l=layout: T.test_against_library_batch_norm(l, (6, 5, 7, 3), 3)]
    calls += [T.test_device_local_variance_would_differ, T.test_constant_channel, T.test_two_element_closed_form,
              T.test_affine_equivariance_and_image_permutation, T.test_bf16_widening_and_rounding_match_library]
    return calls


def failures(module, monkeypatch):
    monkeypatch.setattr(T, "O", module)
    n = 0
    for call in battery():
        try:
            call()
        except Exception:          # an assertion, or the mutant blowing up: either way it is caught
            n += 1
    return n


def test_real_oracle_passes_the_battery(monkeypatch):
    assert failures(O, monkeypatch) == 0


@pytest.mark.parametrize("what,old,new,count", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(what, old, new, count, monkeypatch):
    assert SRC.count(old) == count, f"mutation site for {what!r} not found exactly {count}x"
    mod = types.ModuleType("mutant_oracle")
    exec(compile(SRC.replace(old, new), "mutant_oracle.py", "exec"), mod.__dict__)
    assert failures(mod, monkeypatch) >= 1, f"no pin noticed: {what}"
