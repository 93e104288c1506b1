"""Pins of the oracle's Gaussian gradient noise (section "Nonconvex Problems": stochastic gradient =
exact gradient + Gaussian noise): distribution against scipy's normal law, moments, independence of
the two Box-Muller branches and of workers / iterations, the reach of the tails, and the element ->
draw mapping checked with the element-at-a-time Philox."""
import math

import numpy as np
import pytest
from scipy import stats

from oracle import tng_oracle as O
from oracle import tng_scalar as S


def test_noise_is_normal_with_the_requested_variance():
    n = 1 << 18
    for variance in (1.0, 0.01):
        z = O.gaussian_noise(seed=3, it=5, m=2, d=n, variance=variance)
        assert z.dtype == np.float64 and z.shape == (n,)
        sd = math.sqrt(variance)
        assert abs(z.mean()) < 5 * sd / math.sqrt(n)
        assert abs(z.var() / variance - 1.0) < 5 * math.sqrt(2.0 / n)
        assert abs(stats.kurtosis(z)) < 0.05 and abs(stats.skew(z)) < 0.03
        assert stats.kstest(z / sd, "norm").pvalue > 1e-3
        # u1 >= 2^-24 bounds the radius: |z| <= sqrt(48 ln 2) standard deviations
        assert np.abs(z).max() <= sd * math.sqrt(48 * math.log(2.0)) * (1 + 1e-6)
        assert np.abs(z).max() > 4.0 * sd


def test_branches_workers_and_iterations_are_uncorrelated():
    n = 1 << 16
    a = O.gaussian_noise(1, 0, 0, n, 1.0)
    pairs = a.reshape(-1, 2)
    assert abs(np.corrcoef(pairs[:, 0], pairs[:, 1])[0, 1]) < 5 / math.sqrt(n / 2)
    assert abs(np.corrcoef(a[:-1], a[1:])[0, 1]) < 5 / math.sqrt(n)
    for other in (O.gaussian_noise(1, 0, 1, n, 1.0), O.gaussian_noise(1, 1, 0, n, 1.0),
                  O.gaussian_noise(2, 0, 0, n, 1.0)):
        assert abs(np.corrcoef(a, other)[0, 1]) < 5 / math.sqrt(n)
    # same arguments, same numbers; a prefix of a longer draw is the shorter draw
    assert np.array_equal(a[:1001], O.gaussian_noise(1, 0, 0, 1001, 1.0))


def test_element_to_draw_mapping_with_the_scalar_generator():
    seed, it, m = (7 << 32) | 9, 4, 3
    z = O.gaussian_noise(seed, it, m, 23, 0.25)
    for e in range(23):
        pair = (e & 3) >> 1
        w1 = S.draw(seed, it, m, 2, 4 * (e >> 2) + 2 * pair)
        w2 = S.draw(seed, it, m, 2, 4 * (e >> 2) + 2 * pair + 1)
        u1 = ((w1 >> 8) + 1) / 2.0 ** 24
        u2 = (w2 >> 8) / 2.0 ** 24
        r = math.sqrt(-2.0 * math.log(u1))
        want = 0.5 * r * (math.cos(2 * math.pi * u2) if e % 2 == 0 else math.sin(2 * math.pi * u2))
        assert z[e] == pytest.approx(want, rel=1e-12, abs=1e-15)
    # Box-Muller radius: the two members of a pair lie on the circle of radius sigma sqrt(-2 ln u1)
    w1 = S.draw(seed, it, m, 2, 0)
    assert z[0] ** 2 + z[1] ** 2 == pytest.approx(0.25 * -2.0 * math.log(((w1 >> 8) + 1) / 2.0 ** 24), rel=1e-12)
