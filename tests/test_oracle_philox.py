"""Pins for the oracle's noise generator: Philox4x32-10 integer stream, the uniform
mapping, Box-Muller, and the moments of the resulting normals (all on the CPU)."""
import math
import os

import numpy as np
import pytest
from scipy import stats

import oracle

M0, M1 = 0xD2511F53, 0xCD9E8D57
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def _kat_rows(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(t, 16) for t in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_published_known_answers(golden_dir):
    rows = _kat_rows(golden_dir)
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert oracle.philox4x32_10(ctr, key) == want


def _philox_bigint(ctr, key):
    """Arbitrary-precision evaluation of the round function (a second route; the
    published vectors above are the real pin)."""
    c = list(ctr)
    k = list(key)
    for r in range(10):
        if r:
            k = [(k[0] + W0) & MASK, (k[1] + W1) & MASK]
        p0, p1 = M0 * c[0], M1 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & MASK, p1 & MASK, ((p0 >> 32) ^ c[3] ^ k[1]) & MASK, p0 & MASK]
    return c


def test_philox_matches_bigint_on_random_counters():
    rng = np.random.default_rng(7)
    for _ in range(200):
        ctr = [int(v) for v in rng.integers(0, 2**32, 4)]
        key = [int(v) for v in rng.integers(0, 2**32, 2)]
        assert oracle.philox4x32_10(ctr, key) == _philox_bigint(ctr, key)
    # each counter / key word matters and is not interchangeable with another
    base = oracle.philox4x32_10([0, 0, 0, 0], [0, 0])
    seen = {tuple(base)}
    for pos in range(4):
        c = [0, 0, 0, 0]
        c[pos] = 1
        seen.add(tuple(oracle.philox4x32_10(c, [0, 0])))
    for pos in range(2):
        k = [0, 0]
        k[pos] = 1
        seen.add(tuple(oracle.philox4x32_10([0, 0, 0, 0], k)))
    assert len(seen) == 7


def test_stream_contract_counter_and_key_layout():
    """Element e of tensor t at (seed, step) is word e%4 of the call with
    counter (q lo, q hi, t, step lo) and key (seed lo, seed hi), q = e // 4."""
    seed, step, tid = 0x123456789ABCDEF, 0x1_0000_0005, 77
    raw = oracle.noise_raw(seed, step, tid, 23)
    for e in range(23):
        q = e // 4
        want = oracle.philox4x32_10([q & MASK, q >> 32, tid, step & MASK], [seed & MASK, seed >> 32])
        assert int(raw[e]) == want[e % 4]
    # a window further in equals the same elements of the stream from 0, and q's high word is used
    big = 4 * (2**32) + 8
    far = oracle.noise_raw(seed, step, tid, 8, first=big)
    for j in range(8):
        q = (big + j) // 4
        assert q >> 32 == 1
        want = oracle.philox4x32_10([q & MASK, q >> 32, tid, step & MASK], [seed & MASK, seed >> 32])
        assert int(far[j]) == want[(big + j) % 4]
    # ragged tail: a 7-element tensor is the prefix of the 8-element one
    assert np.array_equal(oracle.noise_raw(1, 2, 3, 7), oracle.noise_raw(1, 2, 3, 8)[:7])
    # distinct tensors / steps / seeds give distinct streams
    a = oracle.noise_raw(1, 2, 3, 64)
    for other in (oracle.noise_raw(2, 2, 3, 64), oracle.noise_raw(1, 3, 3, 64), oracle.noise_raw(1, 2, 4, 64)):
        assert not np.array_equal(a, other)


def test_uniform_and_box_muller_against_extended_precision():
    mp = pytest.importorskip("mpmath")
    mp.mp.dps = 40
    seed, step, tid = 5, 9, 2
    n = 4000
    raw = oracle.noise_raw(seed, step, tid, n)
    z = oracle.noise_normal(seed, step, tid, n)
    for e in range(0, n, 2):
        u0 = (mp.mpf(int(raw[e]) >> 9) + mp.mpf("0.5")) / mp.mpf(2) ** 23
        u1 = (mp.mpf(int(raw[e + 1]) >> 9) + mp.mpf("0.5")) / mp.mpf(2) ** 23
        assert 0 < u0 < 1 and 0 < u1 < 1
        r = mp.sqrt(-2 * mp.log(u0))
        assert abs(float(r * mp.cos(2 * mp.pi * u1)) - z[e]) <= 2e-14 * max(1.0, abs(z[e]))
        assert abs(float(r * mp.sin(2 * mp.pi * u1)) - z[e + 1]) <= 2e-14 * max(1.0, abs(z[e + 1]))


def test_box_muller_inverse_identities():
    """z0^2 + z1^2 = -2 ln u0 and the angle of (z0, z1) is 2 pi u1: catches swapped
    sin/cos, a wrong pair assignment, or a missing factor."""
    raw = oracle.noise_raw(11, 0, 0, 2000).astype(np.int64)
    z = oracle.noise_normal(11, 0, 0, 2000)
    u = ((raw >> 9) + 0.5) / 2.0**23
    u0, u1 = u[0::2], u[1::2]
    z0, z1 = z[0::2], z[1::2]
    assert np.allclose(z0 * z0 + z1 * z1, -2.0 * np.log(u0), rtol=1e-12, atol=0)
    ang = np.mod(np.arctan2(z1, z0), 2 * math.pi)
    d = np.abs(ang - 2 * math.pi * u1)
    d = np.minimum(d, 2 * math.pi - d)
    assert d.max() < 1e-9


def test_uniform_extremes_never_zero_or_one():
    # the mapping itself: numerator is an odd multiple of 2^-24
    for r, want in ((0, 2.0**-24), (MASK, 1 - 2.0**-24), (1 << 9, 1.5 * 2.0**-23)):
        u = ((r >> 9) + 0.5) / 2.0**23
        assert u == want and 0.0 < u < 1.0 and np.float32(u) == u


def test_normal_moments_and_distribution():
    p = 400_000
    z = oracle.noise_normal(0, 0, 0, p)
    assert abs(z.mean()) < 0.01
    assert abs(z.std() - 1.0) < 0.01
    assert abs(np.mean(z * z) - 1.0) < 0.01
    assert abs(stats.skew(z)) < 0.02 and abs(stats.kurtosis(z)) < 0.05
    assert stats.kstest(z, "norm").pvalue > 1e-3
    # neighbours (same call, adjacent calls) are uncorrelated
    for lag in (1, 2, 3, 4):
        assert abs(np.corrcoef(z[:-lag], z[lag:])[0, 1]) < 0.01
    # even and odd elements (cos and sin branches) are each standard normal
    assert abs(z[0::2].std() - 1) < 0.01 and abs(z[1::2].std() - 1) < 0.01


def test_noise_finalize_definition():
    rng = np.random.default_rng(3)
    acc = rng.standard_normal(10_003)
    # sigma = 0: plain division by |B|
    out = oracle.noise_finalize(acc, 0.0, 2.0, 64, 1, 2, 3)
    assert np.array_equal(out, acc / 64)
    # noise alone: std sigma*C/|B|, and it is exactly sigma*C*z/|B| with z the stream
    sigma, c, b = 1.3, 0.7, 32
    out = oracle.noise_finalize(np.zeros(200_000), sigma, c, b, 4, 5, 6)
    z = oracle.noise_normal(4, 5, 6, 200_000)
    assert np.allclose(out, sigma * c * z / b, rtol=1e-15, atol=0)
    assert abs(out.std() * b / (sigma * c) - 1) < 0.01
    assert abs(out.mean() * b / (sigma * c)) < 0.01
    # additive: out = acc/|B| + noise/|B|
    both = oracle.noise_finalize(acc, sigma, c, b, 4, 5, 6)
    assert np.allclose(both, acc / b + sigma * c * z[:acc.size] / b, rtol=1e-14, atol=1e-16)
