"""Synthetic stand-in for the sensitive mask m_k (Definition 3) and the
tile-ordered sparse layout that fixes the entry order j, hence which Gaussian
each sensitive weight receives.  Test infrastructure only.

The paper's mask is the top-k of squared gradients of a real model; no weights
or gradients exist here, so positions are seeded draws.  Two shapes:

* uniform: k distinct positions uniform over the matrix;
* heavy tail: motivated by the paper's finding that 0.1% of coordinates carry
  about half of the gradient norm (Figure 2): ceil(1% of rows) "hot" rows
  receive floor(k/2) of the entries, the rest are uniform.

Draw d of stream s is Philox-4x32-10 with key = mask seed (lo, hi) and
counter (lo32(d), hi32(d), s, 0); the value is (r0 * 2**32 + r1) mod range.
Duplicates are dropped in draw order until enough distinct values exist.

Tile order (TCSR): rows are cut into bands of 64, columns into tiles of 64;
tile id = (n // 64) * (K // 64) + k // 64, so the tiles of one band follow
each other along K.  Entries are sorted by (tile id, (n % 64) * 64 + k % 64);
tile_ptr is the exclusive prefix sum of the per-tile counts.  Position j in
this order is the entry index.
"""
import numpy as np

from .philox import philox4x32_10, MASK32

TILE_ROWS = 64      # rows per band
TILE_COLS = 64      # columns per tile


def nnz_for_density(N, K, density):
    """k = floor(density * N * K + 0.5)."""
    return int(np.floor(density * N * K + 0.5))


def _draws(mask_seed, stream, start, count, modulus):
    d = np.arange(start, start + count, dtype=np.uint64)
    k0 = int(mask_seed) & MASK32
    k1 = (int(mask_seed) >> 32) & MASK32
    r0, r1, _, _ = philox4x32_10(d & np.uint64(MASK32), d >> np.uint64(32), stream, 0, k0, k1)
    v = (r0.astype(np.uint64) << np.uint64(32)) | r1.astype(np.uint64)
    return (v % np.uint64(modulus)).astype(np.int64)


def _first_distinct(mask_seed, stream, want, modulus, exclude=None):
    """First `want` distinct draws of a stream (in draw order), skipping any
    value in `exclude`."""
    assert want <= modulus - (0 if exclude is None else len(exclude))
    chosen = []
    seen = set() if exclude is None else set(int(v) for v in exclude)
    start = 0
    while len(chosen) < want:
        batch = _draws(mask_seed, stream, start, max(1024, 2 * (want - len(chosen))), modulus)
        start += len(batch)
        for v in batch.tolist():
            if v not in seen:
                seen.add(v)
                chosen.append(v)
                if len(chosen) == want:
                    break
    return np.array(chosen, dtype=np.int64)


def mask_uniform(N, K, nnz, mask_seed):
    """Sorted flat positions n*K+k of nnz distinct uniform draws (stream 0)."""
    return np.sort(_first_distinct(mask_seed, 0, nnz, N * K))


def mask_heavy_tail(N, K, nnz, mask_seed):
    """Half of the entries inside ceil(N/100) hot rows, rest uniform."""
    H = -(-N // 100)
    hot = np.sort(_first_distinct(mask_seed, 1, H, N))                 # stream 1: rows
    n_hot = nnz // 2
    inside = _first_distinct(mask_seed, 2, n_hot, H * K)               # stream 2: (hot row, col)
    flat_hot = hot[inside // K] * K + inside % K
    rest = _first_distinct(mask_seed, 3, nnz - n_hot, N * K, exclude=flat_hot)  # stream 3
    return np.sort(np.concatenate([flat_hot, rest]))


def tile_id(n, k, K):
    n = np.asarray(n, dtype=np.int64)
    k = np.asarray(k, dtype=np.int64)
    return (n // TILE_ROWS) * (K // TILE_COLS) + k // TILE_COLS


def num_tiles(N, K):
    return (-(-N // TILE_ROWS)) * (K // TILE_COLS)


def tcsr_build(N, K, flat_sorted):
    """flat_sorted: ascending unique flat positions.  Returns
    (tile_ptr uint32 [ntiles+1], sp_idx uint32 [nnz] flat positions in tile
    order, perm uint32 [nnz] with sp_idx[j] == flat_sorted[perm[j]])."""
    assert K % TILE_COLS == 0
    flat = np.asarray(flat_sorted, dtype=np.int64)
    assert np.all(np.diff(flat) > 0), "mask positions must be unique and ascending"
    assert flat.size == 0 or (flat[0] >= 0 and flat[-1] < N * K)
    n, k = flat // K, flat % K
    t = tile_id(n, k, K)
    inner = (n % TILE_ROWS) * TILE_COLS + (k % TILE_COLS)
    perm = np.lexsort((inner, t))
    counts = np.bincount(t, minlength=num_tiles(N, K))
    tile_ptr = np.zeros(num_tiles(N, K) + 1, dtype=np.uint32)
    tile_ptr[1:] = np.cumsum(counts)
    return tile_ptr, flat[perm].astype(np.uint32), perm.astype(np.uint32)


def nnz_bases(nnz_list):
    """Running global entry offsets, each padded up to a multiple of 4 so that
    no two matrices share a Philox counter (z_k is one vector over all
    sensitive entries of the model, Section 3.4)."""
    bases, run = [], 0
    for z in nnz_list:
        bases.append(run)
        run += (int(z) + 3) // 4 * 4
    return bases
