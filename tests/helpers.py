"""Shared test plumbing: builds oracle-side matrices from the seeded inputs."""
import numpy as np

from oracle import mask as omask, quant as oquant
from oracle.zo import Matrix
from paper_2406_02913_amd import synth


def make_oracle_matrix(seed, M, N, K, group, density=1e-3, kind="uniform", nnz=None,
                       nnz_base=0, mask_seed=None, sigma=0.02):
    x = synth.activations(seed, M, K)
    W = synth.dense_weight(seed, N, K, sigma)
    t = synth.target(seed, M, N)
    k = omask.nnz_for_density(N, K, density) if nnz is None else nnz
    ms = seed + 1000 if mask_seed is None else mask_seed
    flat = (omask.mask_uniform if kind == "uniform" else omask.mask_heavy_tail)(N, K, k, ms)
    tile_ptr, sp_idx, perm = omask.tcsr_build(N, K, flat)
    codes, scales, sp_val = oquant.split_and_quantize(W, sp_idx.astype(np.int64), group)
    m = Matrix(x_bits=x, codes=codes, scales=scales, group=group, sp_idx=sp_idx,
               sp_val=sp_val, target_bits=t, nnz_base=nnz_base)
    m.tile_ptr = tile_ptr
    m.W = W
    m.flat_sorted = flat
    return m


def clone(m):
    c = Matrix(m.x_bits, m.codes, m.scales, m.group, m.sp_idx, m.sp_val.copy(), m.target_bits, m.nnz_base)
    for a in ("tile_ptr", "W", "flat_sorted"):
        if hasattr(m, a):
            setattr(c, a, getattr(m, a))
    return c
