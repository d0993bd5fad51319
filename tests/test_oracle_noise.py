"""Pins for the oracle's noise stream (CPU only).

Philox words: known-answer vectors and an independent big-integer implementation.
Normal transform: binary64 Box-Muller through libm on the same uniforms, exhaustively over
all 2^23 inputs of ln and of sin/cos; sample moments; independence across stream coordinates.
"""
import math
import os

import numpy as np

from oracle import noise as N

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _philox_bigint(ctr, key):
    """Philox4x32-10 with Python integers, written from the SC'11 paper's round description."""
    c = list(ctr)
    k = list(key)
    for r in range(10):
        if r > 0:
            k[0] = (k[0] + 0x9E3779B9) % 2**32
            k[1] = (k[1] + 0xBB67AE85) % 2**32
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 // 2**32) ^ c[1] ^ k[0], p1 % 2**32, (p0 // 2**32) ^ c[3] ^ k[1], p0 % 2**32]
    return c


def test_philox_known_answers():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        v = [int(x, 16) for x in row]
        ctr, key, want = v[:4], v[4:6], v[6:]
        got = N.philox4x32_10(tuple(np.uint32(c) for c in ctr), key)
        assert [int(g) for g in got] == want
        assert _philox_bigint(ctr, key) == want


def test_philox_matches_bigint_on_random_inputs():
    rng = np.random.default_rng(5)
    ctr = rng.integers(0, 2**32, size=(4, 2000), dtype=np.uint32)
    key = (0x12345678, 0x9ABCDEF0)
    got = np.stack(N.philox4x32_10(tuple(ctr), key))
    for i in range(2000):
        assert _philox_bigint([int(x) for x in ctr[:, i]], key) == [int(x) for x in got[:, i]]


def test_uniform_is_exact_and_open():
    x = np.array([0, 0x1FF, 0x200, 0xFFFFFFFF], dtype=np.uint32)
    u = N.uniform_from_word(x)
    assert u.dtype == np.float32
    want = [(0 + 0.5) / 2**23, (0 + 0.5) / 2**23, (1 + 0.5) / 2**23, (2**23 - 0.5) / 2**23]
    assert [float(v) for v in u] == want
    assert 0.0 < float(u.min()) and float(u.max()) < 1.0


def test_ln_exhaustive_against_libm():
    words = np.arange(2**23, dtype=np.uint32) << np.uint32(9)
    u = N.uniform_from_word(words)
    got = N.neg2_ln(u).astype(np.float64)
    ref = -2.0 * np.log(u.astype(np.float64))
    assert np.all(got > 0.0)
    assert np.abs((got - ref) / ref).max() < 2.5e-7


def test_sincos_exhaustive_against_libm():
    words = np.arange(2**23, dtype=np.uint32) << np.uint32(9)
    ang = 2.0 * np.pi * N.uniform_from_word(words).astype(np.float64)
    c, s = N.sincos_2pi(words)
    assert np.abs(c - np.cos(ang)).max() < 2e-7
    assert np.abs(s - np.sin(ang)).max() < 2e-7


def test_normals_against_binary64_box_muller():
    rng = np.random.default_rng(11)
    x = rng.integers(0, 2**32, size=(4, 1_000_000), dtype=np.uint32)
    z = N.normals_from_words(*x)

    def ref(xa, xb):
        ua = ((xa >> 9).astype(np.float64) + 0.5) * 2.0**-23
        ub = ((xb >> 9).astype(np.float64) + 0.5) * 2.0**-23
        rho = np.sqrt(-2.0 * np.log(ua))
        return rho * np.cos(2 * np.pi * ub), rho * np.sin(2 * np.pi * ub)

    r = ref(x[0], x[1]) + ref(x[2], x[3])
    for got, want in zip(z, r):
        assert got.dtype == np.float32
        assert np.abs(got - want).max() < 2e-6


def test_noise_tensor_layout_and_moments():
    n = 1 << 20
    z = N.noise_tensor(3456, 7, 2, 5, n)
    assert z.shape == (n,) and z.dtype == np.float32
    # element 4j+i is output i of counter (j, tensor, step, k)
    j = 12345
    w = N.philox4x32_10((np.uint32(j), np.uint32(5), np.uint32(7), np.uint32(2)), (3456, 0))
    four = [float(v[0]) for v in N.normals_from_words(*[np.array([x]) for x in w])]
    assert four == [float(v) for v in z[4 * j:4 * j + 4]]
    se = 1.0 / math.sqrt(n)
    zz = z.astype(np.float64)
    assert abs(zz.mean()) < 4 * se
    assert abs(zz.var() - 1.0) < 4 * math.sqrt(2.0) * se
    assert abs((zz**3).mean()) < 4 * math.sqrt(15.0) * se
    assert abs((zz**4).mean() - 3.0) < 4 * math.sqrt(96.0) * se
    # a prefix of a longer tensor is the same stream (elements are addressable in isolation)
    assert np.array_equal(N.noise_tensor(3456, 7, 2, 5, 4096), z[:4096])


def test_streams_are_uncorrelated_across_coordinates():
    n = 1 << 18
    base = N.noise_tensor(1, 0, 0, 0, n).astype(np.float64)
    others = [N.noise_tensor(1, 0, 1, 0, n), N.noise_tensor(1, 1, 0, 0, n),
              N.noise_tensor(1, 0, 0, 1, n), N.noise_tensor(2, 0, 0, 0, n),
              N.noise_tensor(1 + 2**32, 0, 0, 0, n)]
    for o in others:
        assert not np.array_equal(o, base.astype(np.float32))
        assert abs(np.mean(base * o.astype(np.float64))) < 4.0 / math.sqrt(n)
    # even/odd outputs of one Box-Muller pair are uncorrelated too
    assert abs(np.mean(base[0::2] * base[1::2])) < 4.0 / math.sqrt(n / 2)


def test_kolmogorov_smirnov_against_normal_cdf():
    from scipy import stats
    z = N.noise_tensor(77, 3, 1, 9, 200_000).astype(np.float64)
    d, p = stats.kstest(z, "norm")
    assert p > 1e-3
