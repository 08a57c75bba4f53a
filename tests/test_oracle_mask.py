"""Pins for the synthetic mask and the tile-ordered sparse layout."""
import numpy as np
import pytest

from oracle import mask


def test_nnz_rounding_matches_workload_sizes():
    assert mask.nnz_for_density(256, 256, 1e-3) == 66
    assert mask.nnz_for_density(4096, 4096, 1e-3) == 16777
    assert mask.nnz_for_density(11008, 4096, 1e-3) == 45089
    assert mask.nnz_for_density(4096, 14336, 1e-2) == 587203
    assert mask.nnz_for_density(1024, 4096, 1e-4) == 419


def test_uniform_mask_basic():
    N, K, k = 256, 256, 66
    f = mask.mask_uniform(N, K, k, mask_seed=5)
    assert f.size == k and np.all(np.diff(f) > 0) and f[0] >= 0 and f[-1] < N * K
    assert np.array_equal(f, mask.mask_uniform(N, K, k, 5))
    assert not np.array_equal(f, mask.mask_uniform(N, K, k, 6))


def test_uniform_mask_is_first_k_distinct_draws_by_hand():
    # tiny range forces duplicates; recompute with the scalar generator
    from oracle.philox import philox4x32_10_scalar
    N, K, k, seed = 4, 8, 20, 0xABCDEF0123
    seen, d = [], 0
    while len(seen) < k:
        r = philox4x32_10_scalar([d & 0xFFFFFFFF, d >> 32, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        v = ((r[0] << 32) | r[1]) % (N * K)
        if v not in seen:
            seen.append(v)
        d += 1
    assert d > k  # duplicates did occur
    assert mask.mask_uniform(N, K, k, seed).tolist() == sorted(seen)


def test_uniform_mask_full_coverage():
    assert mask.mask_uniform(4, 8, 32, 1).tolist() == list(range(32))


def test_heavy_tail_structure():
    N, K = 1024, 512
    k = mask.nnz_for_density(N, K, 1e-2)
    f = mask.mask_heavy_tail(N, K, k, mask_seed=11)
    assert f.size == k and np.all(np.diff(f) > 0)
    rows = f // K
    counts = np.bincount(rows, minlength=N)
    H = -(-N // 100)
    hot = np.argsort(counts)[-H:]
    # the H busiest rows hold at least half of all entries, and are far denser
    assert counts[hot].sum() >= k // 2
    assert counts[hot].min() > 10 * np.median(counts)


def test_heavy_tail_mask_by_hand_with_the_scalar_generator():
    # ceil(N/100) hot rows from stream 1, floor(k/2) positions inside them from stream 2, the rest from
    # stream 3 over the whole matrix skipping what is taken: every draw recomputed one by one
    from oracle.philox import philox4x32_10_scalar
    N, K, k, seed = 150, 8, 31, 0x1234567899

    def stream(s, modulus):
        d = 0
        while True:
            r = philox4x32_10_scalar([d & 0xFFFFFFFF, d >> 32, s, 0], [seed & 0xFFFFFFFF, seed >> 32])
            yield ((r[0] << 32) | r[1]) % modulus
            d += 1

    def first_distinct(gen, want, taken=()):
        out, seen = [], set(taken)
        for v in gen:
            if v not in seen:
                seen.add(v)
                out.append(v)
                if len(out) == want:
                    return out

    H = 2
    hot = sorted(first_distinct(stream(1, N), H))
    inside = first_distinct(stream(2, H * K), k // 2)              # 15 of the 16 positions: duplicates are certain
    flat_hot = [hot[v // K] * K + v % K for v in inside]
    rest = first_distinct(stream(3, N * K), k - k // 2, taken=flat_hot)
    assert mask.mask_heavy_tail(N, K, k, seed).tolist() == sorted(flat_hot + rest)
    rows = np.array(sorted(flat_hot + rest)) // K
    assert sum(int(r in hot) for r in rows) >= k // 2


def test_uniform_mask_is_roughly_uniform():
    N, K = 512, 512
    f = mask.mask_uniform(N, K, 20000, 3)
    rows, cols = f // K, f % K
    for v, n in ((rows, N), (cols, K)):
        c = np.bincount(v // 64, minlength=n // 64)
        assert np.all(np.abs(c - c.mean()) < 5 * np.sqrt(c.mean()))


@pytest.mark.parametrize("N,K,k", [(256, 256, 66), (100, 128, 300), (130, 64, 0), (64, 64, 4096), (70, 192, 999)])
def test_tcsr_invariants_and_bruteforce(N, K, k):
    f = mask.mask_uniform(N, K, k, 21)
    tp, idx, perm = mask.tcsr_build(N, K, f)
    nt = mask.num_tiles(N, K)
    assert tp.dtype == np.uint32 and idx.dtype == np.uint32 and perm.dtype == np.uint32
    assert tp.size == nt + 1 and tp[0] == 0 and tp[-1] == k and np.all(np.diff(tp.astype(np.int64)) >= 0)
    assert np.array_equal(idx, f[perm].astype(np.uint32))
    assert sorted(idx.tolist()) == f.tolist()
    # brute force: python sort of explicit tuples
    ents = []
    for v in f.tolist():
        n, kk = divmod(v, K)
        t = (n // 64) * (K // 64) + kk // 64
        ents.append((t, (n % 64) * 64 + kk % 64, v))
    ents.sort()
    assert [e[2] for e in ents] == idx.tolist()
    for t in range(nt):
        for j in range(int(tp[t]), int(tp[t + 1])):
            assert ents[j][0] == t


def test_tcsr_tiles_of_a_band_are_contiguous_along_k():
    K = 256
    assert mask.tile_id(0, 0, K) == 0 and mask.tile_id(63, 63, K) == 0
    assert mask.tile_id(0, 64, K) == 1 and mask.tile_id(63, 255, K) == 3
    assert mask.tile_id(64, 0, K) == K // 64


def test_tcsr_rejects_duplicates():
    with pytest.raises(AssertionError):
        mask.tcsr_build(64, 64, np.array([3, 3, 5]))


def test_nnz_bases_are_padded_to_four():
    assert mask.nnz_bases([66, 16777, 5, 8]) == [0, 68, 68 + 16780, 68 + 16780 + 8]
