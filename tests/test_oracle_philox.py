"""Pins for the oracle's generator (CPU only).

What fixes it, independently of itself: the published Philox4x32-10
known-answer vectors; a scalar big-integer implementation written in a
different style; the distribution (moments, tail bound of a 24-bit
Box-Muller); and the closed form of Thm 5.4 for the expected |cosine| of a
Gaussian direction.
"""
import math
import os

import numpy as np

from oracle import philox

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            v = [int(t, 16) for t in line.split()]
            rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, want in rows:
        got = philox.philox4x32_10(*ctr, *key)
        assert [int(g) for g in got] == want


def _philox_scalar(ctr, key):
    """Independent scalar version: Python big integers, explicit round function."""
    c = list(ctr)
    k = list(key)

    def rnd(c, k):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        return [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]

    for i in range(10):
        c = rnd(c, k)
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def test_scalar_version_matches_known_answers():
    for ctr, key, want in _kat_rows():
        assert _philox_scalar(ctr, key) == want


def test_word_layout_row_quad_tag_seed():
    """word (row, col) = word col%4 of counter (row, col//4, tag, 0), key (seed_lo, seed_hi)."""
    seed = 0x0123456789ABCDEF
    w = philox.philox_words(seed, tag=1, rows=7, cols=10)
    assert w.shape == (7, 10) and w.dtype == np.uint32
    for row in (0, 3, 6):
        for col in (0, 1, 5, 9):
            ref = _philox_scalar([row, col // 4, 1, 0], [seed & 0xFFFFFFFF, seed >> 32])
            assert int(w[row, col]) == ref[col % 4]
    # different tag / seed change the stream; prefix property: fewer cols = same leading values
    assert not np.array_equal(w, philox.philox_words(seed, 0, 7, 10))
    assert not np.array_equal(w, philox.philox_words(seed + 1, 1, 7, 10))
    assert np.array_equal(w[:, :3], philox.philox_words(seed, 1, 7, 3))


def test_normal_is_box_muller_of_the_words():
    seed, tag = 42, 0
    w = philox.philox_words(seed, tag, 5, 8)
    z = philox.normal(seed, tag, 5, 8)
    assert z.dtype == np.float32
    for row in range(5):
        for q in range(2):
            x = [int(v) for v in w[row, 4 * q:4 * q + 4]]
            u = [((v >> 9) + 0.5) / 2 ** 23 for v in x]
            ref = [math.sqrt(-2 * math.log(u[0])) * math.cos(2 * math.pi * u[1]),
                   math.sqrt(-2 * math.log(u[0])) * math.sin(2 * math.pi * u[1]),
                   math.sqrt(-2 * math.log(u[2])) * math.cos(2 * math.pi * u[3]),
                   math.sqrt(-2 * math.log(u[2])) * math.sin(2 * math.pi * u[3])]
            np.testing.assert_allclose(z[row, 4 * q:4 * q + 4], np.float32(ref), rtol=0, atol=1e-7)
    # r not a multiple of 4: trailing words are simply dropped
    np.testing.assert_array_equal(philox.normal(seed, tag, 5, 3), z[:, :3])


def test_uniform_is_exact_in_fp32_and_open_interval():
    x = np.array([0, 1, 511, 512, 2 ** 31, 2 ** 32 - 1], dtype=np.uint32)
    u = philox._uniform(x)
    assert u.min() > 0.0 and u.max() < 1.0
    np.testing.assert_array_equal(u, u.astype(np.float32).astype(np.float64))


def test_normal_moments_and_tail():
    z = philox.normal(7, philox.TAG_G, 500_000, 8).astype(np.float64).ravel()   # 4e6 values
    n = z.size
    assert abs(z.mean()) < 5 / math.sqrt(n)
    assert abs(z.var() - 1.0) < 5 * math.sqrt(2.0 / n)
    assert abs(np.mean(z ** 3)) < 5 * math.sqrt(15.0 / n)
    assert abs(np.mean(z ** 4) - 3.0) < 5 * math.sqrt(96.0 / n)
    assert np.abs(z).max() <= math.sqrt(2 * 24 * math.log(2)) + 1e-6
    # columns are uncorrelated (sin/cos pairs share a radius but are orthogonal)
    Z = z.reshape(-1, 8)
    C = (Z.T @ Z) / Z.shape[0]
    assert np.abs(C - np.eye(8)).max() < 6 / math.sqrt(Z.shape[0])


def _beta(D):
    with open(os.path.join(GOLDEN, "beta_D.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            d, b = line.split()
            if int(d) == D:
                return float(b)
    raise KeyError(D)


def test_beta_closed_form_and_bounds():
    for D in (2, 3, 4, 16):
        b = math.gamma(D / 2) / (math.sqrt(math.pi) * math.gamma((D + 1) / 2))
        assert abs(b - _beta(D)) < 1e-12
        assert math.sqrt(2 / (math.pi * D)) <= b <= math.sqrt(2 / (math.pi * (D - 1)))


def test_expected_cosine_matches_thm_5_4():
    """E |<G, M>| / (|G| |M|) = beta_{d_out r} for a fixed M and G ~ N(0, I) of shape d_out x r.
    Here d_out = 8, r = 2, D = 16; draws are consecutive 8-row blocks of one stream
    plus blocks taken from many different seeds."""
    d_out, r, draws = 8, 2, 100_000
    M = np.arange(1, d_out * r + 1, dtype=np.float64).reshape(d_out, r) ** 1.5
    G = philox.normal(3, philox.TAG_G, d_out * draws, r).astype(np.float64).reshape(draws, d_out, r)
    cos = np.abs((G * M).sum(axis=(1, 2))) / (np.linalg.norm(G, axis=(1, 2)) * np.linalg.norm(M))
    se = cos.std() / math.sqrt(draws)
    assert abs(cos.mean() - _beta(16)) < 3.5 * se
    per_seed = []
    for s in range(400):
        g = philox.normal(1000 + s, philox.TAG_G, d_out, r).astype(np.float64)
        per_seed.append(abs((g * M).sum()) / (np.linalg.norm(g) * np.linalg.norm(M)))
    per_seed = np.array(per_seed)
    assert abs(per_seed.mean() - _beta(16)) < 3.5 * per_seed.std() / math.sqrt(per_seed.size)
