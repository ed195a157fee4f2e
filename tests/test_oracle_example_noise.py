"""Pins for the oracle's per-example form of the noise (second equation of the Algorithm section): the
draws are standard normal, independent between examples and from the once-per-step stream, scaled so
that a whole step's worth sums to variance sigma^2 C^2; and the stream words are those of the pinned
Philox function with the documented counter / key."""
import math

import numpy as np

import oracle


def test_scale_and_moments_of_a_whole_step():
    p, B, sigma, C = 120_000, 16, 1.3, 0.7
    acc = oracle.add_example_noise(np.zeros(p), sigma, C, B, 5, 2, 7, 0, B)
    # sum of B independent N(0, sigma^2 C^2 / B) draws per coordinate: N(0, sigma^2 C^2)
    assert abs(acc.mean()) < 0.01 * sigma * C
    assert abs(acc.std() / (sigma * C) - 1.0) < 0.01
    assert abs(np.mean((acc / (sigma * C)) ** 4) - 3.0) < 0.1          # normal kurtosis
    # a part of the step carries its share of the variance
    part = oracle.add_example_noise(np.zeros(p), sigma, C, B, 5, 2, 7, 4, 4)
    assert abs(part.std() / (sigma * C * math.sqrt(4 / B)) - 1.0) < 0.01


def test_examples_add_up_and_are_independent():
    p, B = 50_000, 8
    one = [oracle.add_example_noise(np.zeros(p), 1.0, 1.0, B, 9, 0, 3, j, 1) for j in range(B)]
    both = oracle.add_example_noise(np.zeros(p), 1.0, 1.0, B, 9, 0, 3, 2, 3)
    assert np.allclose(both, one[2] + one[3] + one[4], rtol=1e-12, atol=1e-15)
    # an accumulator that already holds something is added to, not overwritten
    base = np.linspace(-1, 1, p)
    assert np.allclose(oracle.add_example_noise(base, 1.0, 1.0, B, 9, 0, 3, 2, 3), base + both, rtol=1e-12)
    z = np.stack(one) * math.sqrt(B)                                        # unit variance each
    corr = np.corrcoef(z)
    assert np.abs(corr - np.eye(B)).max() < 0.02                            # ~4.5 standard errors at p = 50,000
    # and independent of the once-per-step stream of the same seed / step / tensor
    once = oracle.noise_normal(9, 0, 3, p)
    assert abs(np.corrcoef(once, z[0])[0, 1]) < 0.02
    assert not np.allclose(once, z[0])


def test_draws_come_from_the_documented_counter_and_key():
    seed, step, tid, j = 0x1234_5678_9ABC_DEF0, 6, 11, 5
    got = oracle.add_example_noise(np.zeros(8), 1.0, 1.0, 1, seed, step, tid, j, 1)
    for q in range(2):
        r = oracle.philox4x32_10([q, j, tid, step], [seed & 0xFFFFFFFF, (seed >> 32) ^ 0x50455245])
        u = [((int(w) >> 9) + 0.5) / 2 ** 23 for w in r]
        z = [math.sqrt(-2 * math.log(u[0])) * math.cos(2 * math.pi * u[1]), math.sqrt(-2 * math.log(u[0])) * math.sin(2 * math.pi * u[1]),
             math.sqrt(-2 * math.log(u[2])) * math.cos(2 * math.pi * u[3]), math.sqrt(-2 * math.log(u[2])) * math.sin(2 * math.pi * u[3])]
        assert np.allclose(got[4 * q: 4 * q + 4], z, rtol=1e-12)


def test_sigma_zero_adds_nothing():
    base = np.arange(10.0)
    assert np.array_equal(oracle.add_example_noise(base, 0.0, 1.0, 4, 1, 1, 1, 0, 4), base)
