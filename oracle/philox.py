"""Philox-4x32-10 (Salmon et al., "Parallel random numbers: as easy as 1, 2, 3",
SC'11; constants as published with the Random123 library description) and the
Box-Muller Gaussian built on it.  Test infrastructure only.

The generator plays the part of the "random seed trick" (Section 3.5 of the
paper): the perturbation z_k of Section 3.4 is a pure function of
(seed, step, entry index) and is never stored.

Two implementations live here on purpose: `philox4x32_10_scalar` works on
Python integers one counter at a time and is the one to read against the
published round function; `philox4x32_10` is the same function on numpy uint64
lanes, used wherever more than a few thousand draws are needed.  Tests pin
both to the known-answer vectors and to each other.
"""
import math

import numpy as np

PHILOX_M0 = 0xD2511F53  # multiplier applied to counter word 0
PHILOX_M1 = 0xCD9E8D57  # multiplier applied to counter word 2
PHILOX_W0 = 0x9E3779B9  # Weyl increment of key word 0 (golden ratio)
PHILOX_W1 = 0xBB67AE85  # Weyl increment of key word 1 (sqrt 3 - 1)
MASK32 = 0xFFFFFFFF


def philox4x32_10_scalar(ctr, key):
    """ctr: 4 ints, key: 2 ints (each < 2**32) -> tuple of 4 ints.

    One round: (hi0, lo0) = M0 * c0 ; (hi1, lo1) = M1 * c2 ;
    c <- (hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0).  The key is bumped by the
    Weyl constants between rounds (nine bumps for ten rounds).
    """
    c0, c1, c2, c3 = (int(v) & MASK32 for v in ctr)
    k0, k1 = (int(v) & MASK32 for v in key)
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + PHILOX_W0) & MASK32
            k1 = (k1 + PHILOX_W1) & MASK32
        p0 = PHILOX_M0 * c0
        p1 = PHILOX_M1 * c2
        hi0, lo0 = p0 >> 32, p0 & MASK32
        hi1, lo1 = p1 >> 32, p1 & MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0), lo1, (hi0 ^ c3 ^ k1), lo0
    return c0, c1, c2, c3


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Vectorised twin of the scalar routine.  All arguments broadcast; values
    are taken modulo 2**32.  Returns four uint32 arrays."""
    m32 = np.uint64(MASK32)
    c0, c1, c2, c3, k0, k1 = np.broadcast_arrays(
        *(np.asarray(v, dtype=np.uint64) & m32 for v in (c0, c1, c2, c3, k0, k1)))
    c0, c1, c2, c3, k0, k1 = (a.copy() for a in (c0, c1, c2, c3, k0, k1))
    sh = np.uint64(32)
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + np.uint64(PHILOX_W0)) & m32
            k1 = (k1 + np.uint64(PHILOX_W1)) & m32
        p0 = np.uint64(PHILOX_M0) * c0
        p1 = np.uint64(PHILOX_M1) * c2
        hi0, lo0 = p0 >> sh, p0 & m32
        hi1, lo1 = p1 >> sh, p1 & m32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0), lo1, (hi0 ^ c3 ^ k1), lo0
    return tuple(a.astype(np.uint32) for a in (c0, c1, c2, c3))


def _split64(v):
    v = int(v) & 0xFFFFFFFFFFFFFFFF
    return v & MASK32, v >> 32


def zbar_words(seed, step, J):
    """Philox words behind the Gaussian of global entry index J (array).

    key = (lo32(seed), hi32(seed)); counter = (lo32(J>>2), hi32(J>>2),
    lo32(step), hi32(step)).  Four consecutive entries share one counter and
    take one Gaussian each from it.  Returns uint32 array [len(J), 4]."""
    J = np.asarray(J, dtype=np.uint64)
    q = J >> np.uint64(2)
    s_lo, s_hi = _split64(seed)
    t_lo, t_hi = _split64(step)
    r = philox4x32_10(q & np.uint64(MASK32), q >> np.uint64(32), t_lo, t_hi, s_lo, s_hi)
    return np.stack(r, axis=-1)


def box_muller_pair(ra, rb):
    """Two independent N(0,1) values from two 32-bit words, in fp64.

    u1 = ((ra >> 8) + 1) / 2**24 lies in (0, 1]; u2 = (rb >> 8) / 2**24 lies in
    [0, 1); both are exact in fp32.  Returns (rho cos theta, rho sin theta)
    with rho = sqrt(-2 ln u1), theta = 2 pi u2."""
    ra = np.asarray(ra, dtype=np.uint32)
    rb = np.asarray(rb, dtype=np.uint32)
    u1 = ((ra >> np.uint32(8)).astype(np.float64) + 1.0) * 2.0 ** -24
    u2 = (rb >> np.uint32(8)).astype(np.float64) * 2.0 ** -24
    rho = np.sqrt(-2.0 * np.log(u1))
    theta = 2.0 * math.pi * u2
    return rho * np.cos(theta), rho * np.sin(theta)


def zbar(seed, step, nnz_base, nnz):
    """The masked perturbation z_k restricted to one matrix: fp64 array [nnz].

    Entry j of the matrix has global index J = nnz_base + j.  Lane J & 3 picks
    which of the four Gaussians of the shared counter it takes:
    0 -> cos of pair (r0, r1), 1 -> sin of (r0, r1), 2 -> cos of (r2, r3),
    3 -> sin of (r2, r3)."""
    J = np.uint64(nnz_base) + np.arange(nnz, dtype=np.uint64)
    w = zbar_words(seed, step, J)
    a_cos, a_sin = box_muller_pair(w[:, 0], w[:, 1])
    b_cos, b_sin = box_muller_pair(w[:, 2], w[:, 3])
    lane = (J & np.uint64(3)).astype(np.int64)
    return np.choose(lane, [a_cos, a_sin, b_cos, b_sin])
