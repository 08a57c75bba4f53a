"""Seeded synthetic inputs and the workload shape tables.

This module serves both the HIP path (tests, benchmark) and the CPU checker
with identical bits.  It holds none of the method's arithmetic: no
quantisation, no mask, no Philox, no loss -- only Gaussian activations,
Gaussian dense weights and Gaussian targets from numpy's own generator, and
the matrix shapes of the models the paper fine-tunes (Section 4: Llama2-7B,
Mistral-7B, OPT-6.7B).  numpy only; never imports torch or the native library.

Values are drawn in blocks of 2**20 elements, block b of a tensor using
numpy.random.default_rng([seed, tag, b]), so the result does not depend on how
many threads fill it.
"""
from concurrent.futures import ThreadPoolExecutor
import os

import numpy as np

_BLOCK = 1 << 20
TAG_X, TAG_W, TAG_T = 1, 2, 3


def _threads(threads=None):
    return threads or min(16, os.cpu_count() or 1)


def _fill_blocks(count, fill, threads=None):
    nblk = (count + _BLOCK - 1) // _BLOCK
    threads = _threads(threads)
    if nblk <= 1 or threads <= 1:
        for b in range(nblk):
            fill(b)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(nblk)))


def _normal_f32(seed, tag, count, sigma=1.0, threads=None):
    out = np.empty(count, dtype=np.float32)

    def fill(b):
        lo, hi = b * _BLOCK, min(count, (b + 1) * _BLOCK)
        rng = np.random.default_rng([int(seed), int(tag), b])
        rng.standard_normal(hi - lo, dtype=np.float32, out=out[lo:hi])
        if sigma != 1.0:
            out[lo:hi] *= np.float32(sigma)

    _fill_blocks(count, fill, threads)
    return out


def to_bf16_bits(v):
    """fp32 array -> uint16 bf16 bit patterns, round to nearest even."""
    u = np.ascontiguousarray(v, dtype=np.float32).view(np.uint32)
    return ((u + (((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF))) >> np.uint32(16)).astype(np.uint16)


def _normal_bf16_bits(seed, tag, count, threads=None):
    out = np.empty(count, dtype=np.uint16)

    def fill(b):
        lo, hi = b * _BLOCK, min(count, (b + 1) * _BLOCK)
        rng = np.random.default_rng([int(seed), int(tag), b])
        out[lo:hi] = to_bf16_bits(rng.standard_normal(hi - lo, dtype=np.float32))

    _fill_blocks(count, fill, threads)
    return out


def activations(seed, M, K):
    """x ~ N(0, 1), bf16 bit patterns [M, K]."""
    return _normal_bf16_bits(seed, TAG_X, M * K).reshape(M, K)


def dense_weight(seed, N, K, sigma=0.02):
    """W ~ N(0, sigma^2), fp32 [N, K] (out x in)."""
    return _normal_f32(seed, TAG_W, N * K, sigma).reshape(N, K)


def target(seed, M, N):
    """t ~ N(0, 1), bf16 bit patterns [M, N]."""
    return _normal_bf16_bits(seed, TAG_T, M * N).reshape(M, N)


# (name, N = out features, K = in features) of one decoder block's linears.
LLAMA2_7B_BLOCK = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                   ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
MISTRAL_7B_BLOCK = [("q", 4096, 4096), ("k", 1024, 4096), ("v", 1024, 4096), ("o", 4096, 4096),
                    ("gate", 14336, 4096), ("up", 14336, 4096), ("down", 4096, 14336)]
OPT_6_7B_BLOCK = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                  ("fc1", 16384, 4096), ("fc2", 4096, 16384)]

WORKLOADS = {
    # tiny single layer: 64 tokens, 256x256, group 32, 0.1% mask, 10 steps
    "c1": dict(block=[("lin", 256, 256)], layers=1, M=64, group=32, density=1e-3,
               mask="uniform", eps=1e-3, lr=1e-6, steps=10),
    # one Llama-2-7B decoder block, 16 x 256 tokens
    "c2": dict(block=LLAMA2_7B_BLOCK, layers=1, M=4096, group=128, density=1e-3,
               mask="uniform", eps=1e-3, lr=1e-6, steps=1),
    # all 32 blocks, heavy-tailed mask
    "c3": dict(block=LLAMA2_7B_BLOCK, layers=32, M=4096, group=128, density=1e-3,
               mask="heavy_tail", eps=1e-3, lr=1e-6, steps=100),
    # one Mistral-7B block, 16 x 512 tokens; densities 1e-4, 1e-3, 1e-2
    "c4": dict(block=MISTRAL_7B_BLOCK, layers=1, M=8192, group=128, density=1e-3,
               mask="uniform", eps=1e-3, lr=1e-6, steps=1),
    # OPT-6.7B block, decode-like token counts 1 / 16 / 64
    "c5": dict(block=OPT_6_7B_BLOCK, layers=1, M=16, group=128, density=1e-3,
               mask="uniform", eps=1e-3, lr=1e-6, steps=1),
    # the Llama stack at 16 tokens (memory-bound target)
    "c3m16": dict(block=LLAMA2_7B_BLOCK, layers=32, M=16, group=128, density=1e-3,
                  mask="heavy_tail", eps=1e-3, lr=1e-6, steps=100),
}


def matrix_seed(data_seed, layer, index):
    """One integer per (layer, matrix) so every matrix has its own streams."""
    return int(data_seed) * 1000003 + layer * 101 + index
