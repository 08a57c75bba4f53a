"""Pins for the oracle's counter-based generator: published known-answer
vectors, scalar-vs-vector agreement, and the counter/key layout."""
import os

import numpy as np

from oracle import philox

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(t, 16) for t in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    assert len(rows) == 3
    return rows


def test_scalar_known_answers():
    for ctr, key, out in _kat_rows():
        assert list(philox.philox4x32_10_scalar(ctr, key)) == out


def test_vector_known_answers():
    rows = _kat_rows()
    c = np.array([r[0] for r in rows], dtype=np.uint64)
    k = np.array([r[1] for r in rows], dtype=np.uint64)
    got = philox.philox4x32_10(c[:, 0], c[:, 1], c[:, 2], c[:, 3], k[:, 0], k[:, 1])
    got = np.stack(got, axis=-1)
    assert got.dtype == np.uint32
    assert got.tolist() == [r[2] for r in rows]


def test_scalar_equals_vector_on_random_counters():
    rng = np.random.default_rng(7)
    c = rng.integers(0, 2**32, size=(200, 4), dtype=np.uint64)
    k = rng.integers(0, 2**32, size=(200, 2), dtype=np.uint64)
    v = np.stack(philox.philox4x32_10(c[:, 0], c[:, 1], c[:, 2], c[:, 3], k[:, 0], k[:, 1]), -1)
    for i in range(200):
        assert tuple(v[i].tolist()) == philox.philox4x32_10_scalar(c[i].tolist(), k[i].tolist())


def test_zbar_counter_layout():
    # key = seed halves, counter = (J>>2 halves, step halves)
    seed, step = 0x0123456789ABCDEF, 0x00000002_00000005
    J = np.array([0, 1, 3, 4, 7, (1 << 34) + 9], dtype=np.uint64)
    w = philox.zbar_words(seed, step, J)
    for i, j in enumerate(J.tolist()):
        q = j >> 2
        want = philox.philox4x32_10_scalar(
            [q & 0xFFFFFFFF, q >> 32, 5, 2], [0x89ABCDEF, 0x01234567])
        assert tuple(w[i].tolist()) == want
    assert (w[0] == w[1]).all() and (w[1] == w[2]).all() and not (w[2] == w[3]).all()
