"""Pins for Box-Muller and for the estimator's scale: sample moments, the
range of the uniforms, and the two SPSA moment identities that hold for a
linear loss (Section 3.1: E (f+ - f-)^2 = 4 eps^2 |m . grad|^2; appendix lemma
on the surrogate-gradient norm: E |g z|^2 = (k + 2) |m . grad|^2)."""
import numpy as np

from oracle import philox


def test_uniform_ranges_and_extremes():
    ra = np.array([0, 0xFF, 0x100, 0xFFFFFFFF], dtype=np.uint32)
    rb = np.array([0, 0, 0, 0], dtype=np.uint32)
    c, s = philox.box_muller_pair(ra, rb)
    # u1 = 2^-24 for ra < 256 -> rho = sqrt(48 ln 2) = 5.768...; u1 = 1 -> rho = 0
    assert abs(c[0] - np.sqrt(48 * np.log(2.0))) < 1e-12 and c[0] == c[1]
    assert c[3] == 0.0 and np.all(s == 0.0)
    # theta = pi/2 when rb = 2^30
    c2, s2 = philox.box_muller_pair(np.uint32(0), np.uint32(1 << 30))
    assert abs(c2) < 1e-15 * 6 + 1e-15 and abs(s2 - np.sqrt(48 * np.log(2.0))) < 1e-12


def test_moments_one_million():
    z = philox.zbar(seed=12345, step=3, nnz_base=8, nnz=1_000_000)
    n = z.size
    assert np.all(np.abs(z) <= 5.77)
    assert abs(z.mean()) < 4.0 / np.sqrt(n)
    assert abs(z.var() - 1.0) < 4.0 * np.sqrt(2.0 / n)
    assert abs(np.mean(z ** 4) - 3.0) < 4.0 * np.sqrt(96.0 / n)
    assert abs(np.mean(z ** 3)) < 4.0 * np.sqrt(15.0 / n)
    # each of the four lanes is N(0,1) on its own, and lanes are uncorrelated
    lanes = z.reshape(-1, 4)
    for a in range(4):
        assert abs(lanes[:, a].var() - 1.0) < 5.0 * np.sqrt(2.0 / lanes.shape[0])
        for b in range(a + 1, 4):
            assert abs(np.mean(lanes[:, a] * lanes[:, b])) < 5.0 / np.sqrt(lanes.shape[0])


def test_steps_and_seeds_give_independent_streams():
    a = philox.zbar(1, 0, 0, 50_000)
    b = philox.zbar(1, 1, 0, 50_000)
    c = philox.zbar(2, 0, 0, 50_000)
    for u, v in ((a, b), (a, c), (b, c)):
        assert abs(np.mean(u * v)) < 5.0 / np.sqrt(u.size)
    assert np.array_equal(a, philox.zbar(1, 0, 0, 50_000))


def test_nnz_base_is_a_pure_offset():
    full = philox.zbar(9, 4, 0, 64)
    assert np.array_equal(philox.zbar(9, 4, 20, 44), full[20:])


def test_spsa_moment_identities_linear_loss():
    # f(w) = c . w on k coordinates: g = c . z exactly, so
    # E g^2 = |c|^2 and E g^2 |z|^2 = (k + 2) |c|^2.
    k, trials = 12, 40_000
    rng = np.random.default_rng(0)
    c = rng.standard_normal(k)
    z = philox.zbar(seed=77, step=0, nnz_base=0, nnz=k * trials).reshape(trials, k)
    # every trial uses its own block of entries = its own counters
    g = z @ c
    c2 = float(c @ c)
    m1 = g ** 2
    m2 = g ** 2 * np.sum(z ** 2, axis=1)
    assert abs(m1.mean() - c2) < 4.0 * m1.std() / np.sqrt(trials)
    assert abs(m2.mean() - (k + 2) * c2) < 4.0 * m2.std() / np.sqrt(trials)
    # a wrong scale (e.g. a missing factor 2 in -2 ln u) would be off by 2x:
    assert abs(m1.mean() / c2 - 1.0) < 0.05
