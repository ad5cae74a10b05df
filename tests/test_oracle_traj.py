"""Pins for the oracle's trajectory averaging (paper, "Trajectory averaging":
tau_out = (1/N) sum_i tau^(i); averaging N rollouts divides the residual
variance by N and leaves a deterministic bias unchanged)."""
from fractions import Fraction

import numpy as np


def test_mean_in_exact_rational_arithmetic(oracle):
    rng = np.random.default_rng(0)
    t = rng.standard_normal((7, 20, 2))
    want = np.empty((20, 2))
    for w in range(20):
        for c in range(2):
            want[w, c] = float(sum(Fraction(float(x)) for x in t[:, w, c]) / 7)
    np.testing.assert_allclose(oracle.traj_mean(t), want, rtol=0, atol=1e-14)


def test_closed_forms(oracle):
    rng = np.random.default_rng(1)
    one = rng.standard_normal((1, 20, 2))
    assert np.array_equal(oracle.traj_mean(one), one[0])                         # N = 1: the rollout itself
    same = np.repeat(one, 5, axis=0)
    np.testing.assert_allclose(oracle.traj_mean(same), one[0], rtol=1e-15)       # equal rollouts: unchanged
    t = rng.standard_normal((6, 20, 2))
    np.testing.assert_allclose(oracle.traj_mean(t[::-1]), oracle.traj_mean(t), rtol=1e-14)      # order does not matter
    np.testing.assert_allclose(oracle.traj_mean(3 * t + 2), 3 * oracle.traj_mean(t) + 2, rtol=1e-13)   # affine
    np.testing.assert_allclose(oracle.traj_mean(t.astype(np.float32)), t.astype(np.float32).astype(np.float64).mean(0), rtol=1e-14)
    # a waypoint moved in one rollout moves the mean by 1/N of it, and nothing else
    t2 = t.copy()
    t2[2, 7, 1] += 6.0
    diff = oracle.traj_mean(t2) - oracle.traj_mean(t)
    assert abs(diff[7, 1] - 1.0) < 1e-12 and np.abs(np.delete(diff.ravel(), 7 * 2 + 1)).max() < 1e-12


def test_variance_of_the_mean_falls_as_one_over_n(oracle):
    rng = np.random.default_rng(2)
    bias, sigma, trials = 0.3, 1.5, 4000
    for n in (1, 4, 16):
        means = np.array([oracle.traj_mean(bias + sigma * rng.standard_normal((n, 3))) for _ in range(trials)])
        assert abs(means.var() - sigma ** 2 / n) < 0.1 * sigma ** 2 / n
        assert abs(means.mean() - bias) < 4 * sigma / np.sqrt(n * trials * 3)    # the bias stays
