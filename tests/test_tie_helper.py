"""CPU checks of the ReLU-tie helper used by the GPU gradient tests: it must accept a gradient that differs from the
oracle's only by the decisions of units at the kink, find exactly those units, and refuse any other difference."""
import numpy as np
import pytest

import oracle
import synth
from gpu_helpers import assert_grads_match_up_to_relu_ties


@pytest.fixture(scope="module")
def probe():
    widths, blocks, hw, batch = (16, 16, 32), 1, 8, 6
    p, b = synth.resnet_init(1, widths, blocks, 10, perturb_bn=0.2)
    x, y = synth.image_pool(1, batch, 10, hw=hw)
    return oracle.GradientProbe(oracle.ResNetCifar(widths, blocks), p, b, x, y)


def _noisy(grads, rel=2e-6, seed=5):
    rng = np.random.default_rng(seed)
    return {k: v + rel * np.linalg.norm(v) / np.sqrt(v.size) * rng.standard_normal(v.shape) for k, v in grads.items()}


def test_planted_decisions_are_found(probe):
    margin = 5e-3                                   # a wide margin so that the small net has candidates at all
    units = probe.near_zero_units(margin)
    assert 12 <= len(units) <= 200, len(units)
    planted = {}
    for name, idx in units[1::5][:5]:               # a few of them, in several layers
        planted.setdefault(name, []).append(idx)
    n_planted = sum(len(v) for v in planted.values())
    got = _noisy(probe.grads(planted))
    with pytest.raises(AssertionError):             # plainly different from the oracle's gradient ...
        assert_grads_match_up_to_relu_ties(probe, got, 1e-4, margins=())
    assert assert_grads_match_up_to_relu_ties(probe, got, 1e-4, margins=(margin,)) == n_planted   # ... and explained by the units
    assert assert_grads_match_up_to_relu_ties(probe, _noisy(probe.grads()), 1e-4, margins=(margin,)) == 0


def test_other_differences_are_refused(probe):
    margin = 5e-3
    base = probe.grads()
    wrong = dict(base)
    wrong["s2.b0.conv1.weight"] = base["s2.b0.conv1.weight"] * 1.001          # a scale error in one tensor
    with pytest.raises(AssertionError):
        assert_grads_match_up_to_relu_ties(probe, wrong, 1e-4, margins=(margin,))
    wrong = dict(base)
    w = base["stem.conv.weight"].copy()
    w[:, 0, 0, :] = base["stem.conv.weight"][:, 2, 2, :]                       # taps swapped
    wrong["stem.conv.weight"] = w
    with pytest.raises(AssertionError):
        assert_grads_match_up_to_relu_ties(probe, wrong, 1e-4, margins=(margin,))
    # a unit outside the margin is never inverted: a decision planted there stays a mismatch
    far = [u for u in probe.near_zero_units(0.5) if u not in set(probe.near_zero_units(margin))][-1]
    with pytest.raises(AssertionError):
        assert_grads_match_up_to_relu_ties(probe, probe.grads({far[0]: [far[1]]}), 1e-4, margins=(margin,))
