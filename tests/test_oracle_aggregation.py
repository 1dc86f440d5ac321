"""Pins for the aggregation oracle (Eq. 4): closed forms and invariants."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth


def test_weights_from_tau_worked_values():
    # 8 fast workers with 32 steps, 2 slow with 16 (the 2:1 setting): 1/9 and 1/18.
    w = oracle.weights_from_tau([32] * 8 + [16] * 2)
    np.testing.assert_allclose(w[:8], 1.0 / 9.0, rtol=1e-15)
    np.testing.assert_allclose(w[8:], 1.0 / 18.0, rtol=1e-15)
    # tau_F = 32, tau_S = 1: 32/258 and 1/258.
    w = oracle.weights_from_tau([32] * 8 + [1] * 2)
    np.testing.assert_allclose(w, [32 / 258] * 8 + [1 / 258] * 2, rtol=1e-15)
    for tau in ([1], [3, 5, 7], [32] * 8 + [16] * 2):
        assert abs(oracle.weights_from_tau(tau).sum() - 1.0) < 1e-15
    # a worker with zero steps gets zero weight
    assert oracle.weights_from_tau([4, 0])[1] == 0.0
    with pytest.raises(ValueError):
        oracle.weights_from_tau([0, 0])


def test_exact_rational_result():
    x = np.array([[1, 2, 3], [5, 7, 11], [-2, 0, 4]], dtype=np.float64)
    tau = [3, 1, 4]
    w = oracle.weights_from_tau(tau)
    got = oracle.weighted_aggregate(x, w)
    for j in range(3):
        exact = sum(Fraction(t, sum(tau)) * Fraction(int(x[i, j])) for i, t in enumerate(tau))
        assert abs(got[j] - float(exact)) < 1e-14


def test_identical_replicas_dyadic_unit_and_uniform():
    base = synth.normal(1, 1, 1000).astype(np.float32)
    same = np.stack([base] * 4)
    np.testing.assert_array_equal(oracle.weighted_aggregate(same, [0.25] * 4), base.astype(np.float64))
    np.testing.assert_allclose(oracle.weighted_aggregate(same, [0.35, 0.35, 0.15, 0.15]), base, rtol=1e-15, atol=0)
    reps = synth.replicas(base, 5, 0)
    for i in range(5):
        e = np.zeros(5)
        e[i] = 1.0
        np.testing.assert_array_equal(oracle.weighted_aggregate(reps, e), reps[i].astype(np.float64))
    # uniform weights reduce to the arithmetic mean of local SGD
    np.testing.assert_allclose(oracle.weighted_aggregate(reps, [0.2] * 5), reps.astype(np.float64).mean(axis=0),
                               rtol=1e-14, atol=1e-300)
    np.testing.assert_array_equal(oracle.weighted_aggregate(reps[:1], [1.0]), reps[0].astype(np.float64))


def test_convex_hull_and_permutation():
    base = synth.normal(2, 1, 4096).astype(np.float32)
    reps = synth.replicas(base, 10, 1)
    w = oracle.weights_from_tau([32] * 8 + [16] * 2)
    out = oracle.weighted_aggregate(reps, w)
    assert np.all(out <= reps.max(axis=0) + 1e-12) and np.all(out >= reps.min(axis=0) - 1e-12)
    perm = np.array([9, 3, 5, 0, 1, 8, 2, 7, 6, 4])
    np.testing.assert_allclose(oracle.weighted_aggregate(reps[perm], w[perm]), out, rtol=1e-13, atol=1e-15)
    # a dropped term or a wrong weight is visible: compare with the matrix product
    np.testing.assert_allclose(out, w @ reps.astype(np.float64), rtol=1e-13, atol=1e-15)
