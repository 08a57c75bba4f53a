"""Pins for the oracle's non-uniform (look-up table) 4-bit format."""
import numpy as np

from oracle import layer, quant, philox
from paper_2406_02913_amd import synth


def test_sixteen_level_rows_are_lossless():
    # a row that takes 16 distinct fp16-exact values, each K/16 times: the equal-mass bins are the
    # levels themselves, so the table is the sorted levels, Dequantize(Q(W)) == W bit for bit and the
    # layer equals a plain matmul with the ORIGINAL weights
    rng = np.random.default_rng(1)
    N, K, M = 6, 128, 4
    W = np.empty((N, K), dtype=np.float32)
    levels = []
    for n in range(N):
        lv = np.sort(rng.choice(np.arange(-200, 200), size=16, replace=False)).astype(np.float32) * np.float32(2.0 ** -9)
        levels.append(lv)
        W[n] = rng.permutation(np.repeat(lv, K // 16))
    codes, lut, _ = quant.split_and_quantize_lut(W, np.zeros(0, dtype=np.int64))
    assert np.array_equal(lut.astype(np.float32), np.stack(levels))
    assert np.array_equal(quant.dequantize_lut(codes, lut), W.astype(np.float64))
    x = synth.activations(5, M, K)
    y = layer.linear_fwd(x, codes, None, 0, np.zeros(0, np.uint32), np.zeros(0, np.float32), lut=lut)
    assert np.array_equal(y, quant.bf16_bits_to_f64(x) @ W.astype(np.float64).T)


def test_centroids_are_the_bin_medians_and_codes_the_nearest():
    W = synth.dense_weight(8, 3, 64)
    codes, lut, _ = quant.split_and_quantize_lut(W, np.zeros(0, dtype=np.int64))
    for n in range(3):
        row = sorted(float(v) for v in W[n])
        for c in range(16):                      # K/16 = 4 per bin: ranks 2, 6, 10, ...
            assert float(lut[n, c]) == float(np.float16(row[4 * c + 2]))
        for k in range(64):
            d = [abs(float(W[n, k]) - float(lut[n, c])) for c in range(16)]
            assert codes[n, k] == d.index(min(d))            # list.index: the first (lowest) minimiser


def test_ties_go_to_the_lower_code_and_the_map_is_monotone():
    # levels -8..7 twice each (table = the levels); 0.5 is midway between 0 and 1 -> the lower one
    row = np.repeat(np.arange(-8, 8), 2).astype(np.float32)
    codes, lut, _ = quant.split_and_quantize_lut(row[None, :], np.zeros(0, dtype=np.int64))
    assert lut[0].tolist() == list(range(-8, 8))
    tie = row.copy()
    tie[30] = 6.5                                # replaces one 7: the table stays -8..7, 6.5 is midway 6 | 7
    c1, lut1, _ = quant.split_and_quantize_lut(tie[None, :], np.zeros(0, dtype=np.int64))
    assert lut1[0].tolist() == list(range(-8, 8)) and c1[0, 30] == 14 and c1[0, 31] == 15
    probe = row.copy()
    probe[:4] = [0.5, -0.5, 2.5, 100.0]
    c2, lut2, _ = quant.split_and_quantize_lut(probe[None, :], np.zeros(0, dtype=np.int64))
    # the four probes replace -8, -8, -7, -7: the order statistics shift, so look codes up directly
    t = lut2[0].astype(np.float64)
    for v, c in zip(probe[:4], c2[0, :4]):
        d = np.abs(float(v) - t)
        assert c == int(np.flatnonzero(d == d.min())[0])
    W = synth.dense_weight(9, 4, 256)
    codes, lut, _ = quant.split_and_quantize_lut(W, np.zeros(0, dtype=np.int64))
    dq = quant.dequantize_lut(codes, lut)
    for n in range(4):
        order = np.argsort(W[n], kind="stable")
        assert np.all(np.diff(dq[n, order]) >= 0)            # w1 <= w2  =>  dq(w1) <= dq(w2)
        assert np.all(np.diff(lut[n].astype(np.float64)) >= 0)
        inner = (W[n] >= lut[n, 0]) & (W[n] <= lut[n, 15])
        gap = np.diff(lut[n].astype(np.float64)).max()
        assert np.all(np.abs(dq[n] - W[n])[inner] <= 0.5 * gap + 1e-12)


def test_equal_mass_bins():
    # every code is used by about K/16 of a continuous row's elements (the table holds bin medians)
    W = synth.dense_weight(10, 2, 4096)
    codes, lut, _ = quant.split_and_quantize_lut(W, np.zeros(0, dtype=np.int64))
    for n in range(2):
        cnt = np.bincount(codes[n], minlength=16)
        assert cnt.sum() == 4096 and cnt[1:15].min() > 150 and cnt[1:15].max() < 400   # inner bins: ~256 each
        assert cnt[0] > 128 and cnt[15] > 128                                         # outer bins take the tails


def test_sparse_part_is_added_on_top_of_the_dense_code():
    # zero is not a centroid in general: on the mask the dense part dequantises to the centroid
    # nearest to zero and the sensitive value is added to it (w = w_dense + w_sparse)
    N, K, M = 8, 64, 3
    W = synth.dense_weight(11, N, K)
    idx = np.array([5, 64 + 9, 7 * 64 + 63], dtype=np.int64)
    codes, lut, sp_val = quant.split_and_quantize_lut(W, idx)
    assert np.array_equal(sp_val, W.reshape(-1)[idx])
    z = philox.zbar(3, 1, 0, idx.size)
    We = layer.effective_weight(codes, None, 0, idx, sp_val, z, +1, 1e-3, lut=lut)
    dq = quant.dequantize_lut(codes, lut)
    for j, f in enumerate(idx):
        n, k = divmod(int(f), K)
        c0 = dq[n, k]
        assert c0 == lut[n].astype(np.float64)[np.argmin(np.abs(lut[n].astype(np.float64)))]   # nearest to zero
        assert We[n, k] == c0 + (float(sp_val[j]) + float(np.float32(1e-3)) * z[j])
    off = np.ones(N * K, bool)
    off[idx] = False
    assert np.array_equal(We.reshape(-1)[off], dq.reshape(-1)[off])
    x = synth.activations(12, M, K)
    a = layer.linear_fwd(x, codes, None, 0, idx, sp_val, z, -1, 1e-3, lut=lut)
    b = layer.linear_fwd_addmm(x, codes, None, 0, idx, sp_val, z, -1, 1e-3, lut=lut)
    c = layer.linear_fwd_bruteforce(x, codes, None, 0, idx, sp_val, z, -1, 1e-3, lut=lut)
    assert np.allclose(a, b, rtol=0, atol=1e-12) and np.allclose(a, c, rtol=0, atol=1e-12)
