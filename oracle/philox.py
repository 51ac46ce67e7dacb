"""Oracle: counter-based Gaussian generator (test infrastructure only).

The paper only says that the Gaussian factor is generated from a stored
seed and regenerated at update time (Sec. 2.1 seed trick; Alg. 2, steps
"Generate R from s" and "Regenerate Delta using stored seed").  It does not
fix a generator, so this build's reading is:

  * integer stream: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), the
    public counter-based generator, with
        key     = (seed mod 2^32, seed div 2^32)
        counter = (row, col div 4, tag, 0)
    one call yields the four 32-bit words used for columns
    4*(col div 4) + {0,1,2,3} of that row;
  * uniform map: u(x) = ((x >> 9) + 1/2) * 2^-23, a 24-bit value that is
    exact in fp32 and lies strictly inside (0, 1);
  * normal map: Box-Muller, (z0, z1) = sqrt(-2 ln u(x0)) * (cos, sin)(2 pi u(x1)),
    (z2, z3) likewise from (x2, x3).

An element therefore depends only on (seed, tag, row, col): any tiling of
the matrix regenerates the same values.  The oracle evaluates the normal
map in fp64 and rounds once to fp32 (the values ARE fp32 numbers).

Pins (tests/test_oracle_philox.py): the published known-answer vectors of
Philox4x32-10, a second independently written scalar implementation,
moments and tail bound of the normal map, and the closed form of
Thm 5.4 (expected |cos| of a Gaussian direction = beta_D).
"""
import numpy as np

PHILOX_M0 = 0xD2511F53
PHILOX_M1 = 0xCD9E8D57
PHILOX_W0 = 0x9E3779B9
PHILOX_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)

TAG_G = 0        # left Gaussian factor of the perturbation (d_out x r)
TAG_OMEGA = 1    # token-space test matrix of Alg. 1 (N x r)
TAG_Q0 = 2       # feature-space start matrix (d_in x r), flagged variant
TAG_DENSE = 3    # dense Gaussian perturbation (non-linear-layer branch of Eq. 7)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten Philox rounds on arrays of 32-bit counter words.

    Inputs are broadcastable integer arrays (or scalars); returns four
    uint32 arrays.  Products are formed in 64 bits and split into high and
    low halves.
    """
    c0, c1, c2, c3 = np.broadcast_arrays(*[np.asarray(c, dtype=np.uint64) for c in (c0, c1, c2, c3)])
    k0 = np.uint64(int(k0) & 0xFFFFFFFF)
    k1 = np.uint64(int(k1) & 0xFFFFFFFF)
    m0 = np.uint64(PHILOX_M0)
    m1 = np.uint64(PHILOX_M1)
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + np.uint64(PHILOX_W0)) & _MASK
            k1 = (k1 + np.uint64(PHILOX_W1)) & _MASK
        p0 = m0 * c0            # < 2^64, no overflow
        p1 = m1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0), lo1, (hi0 ^ c3 ^ k1), lo0
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def philox_words(seed, tag, rows, cols):
    """uint32 words [rows][cols]: word (row, col) is word col%4 of the call
    with counter (row, col//4, tag, 0) and key (seed_lo, seed_hi)."""
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    k0, k1 = seed & 0xFFFFFFFF, seed >> 32
    nq = (cols + 3) // 4
    row = np.arange(rows, dtype=np.uint64)[:, None]
    quad = np.arange(nq, dtype=np.uint64)[None, :]
    x = philox4x32_10(row, quad, np.uint64(tag), np.uint64(0), k0, k1)
    words = np.stack(x, axis=-1).reshape(rows, 4 * nq)
    return np.ascontiguousarray(words[:, :cols])


def _uniform(x):
    return ((x >> np.uint32(9)).astype(np.float64) + 0.5) * 2.0 ** -23


def normal(seed, tag, rows, cols):
    """fp32 matrix [rows][cols] of N(0,1) values (Box-Muller on the Philox words)."""
    nq = (cols + 3) // 4
    w = philox_words(seed, tag, rows, 4 * nq).reshape(rows, nq, 4)
    out = np.empty((rows, nq, 4), dtype=np.float64)
    for a, b in ((0, 1), (2, 3)):
        rad = np.sqrt(-2.0 * np.log(_uniform(w[..., a])))
        ang = 2.0 * np.pi * _uniform(w[..., b])
        out[..., a] = rad * np.cos(ang)
        out[..., b] = rad * np.sin(ang)
    return np.ascontiguousarray(out.reshape(rows, 4 * nq)[:, :cols]).astype(np.float32)
