"""Host side of libszo against the oracle, bit for bit; export table; argument
validation (no kernel is launched by any test in this file)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import mask as omask, quant as oquant, philox as ophilox
from paper_2406_02913_amd import synth, szo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "szo.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(szo_[a-z0-9_]+)\s*\(", hdr))
    assert declared, "no declarations found"
    assert declared == set(szo.EXPORTS)
    for name in declared:
        assert getattr(szo.lib, name) is not None
    assert szo.szo_version() == 5
    assert szo.szo_workspace_bytes() >= 64 + 8 * 1024


def test_tile_type_rule_for_the_activation_range():
    # the fp16 tile converts bf16 activations exactly only up to the largest finite fp16
    assert szo.szo_choose_tile_dtype(0.0) == szo.TILE_F16
    assert szo.szo_choose_tile_dtype(65504.0) == szo.TILE_F16
    assert szo.szo_choose_tile_dtype(float(np.nextafter(np.float32(65504.0), np.float32(1e9)))) == szo.TILE_BF16
    assert szo.szo_choose_tile_dtype(float("inf")) == szo.TILE_BF16
    for bad in (-1.0, float("nan")):
        with pytest.raises(szo.SzoError) as e:
            szo.szo_choose_tile_dtype(bad)
        assert e.value.code == szo.EINVAL


def test_descriptor_layout_matches_header():
    # 3*8 + 2*4 + 8 + 8 + 8 pointers*8 + table pointer + format + reserved
    assert ctypes.sizeof(szo.LinearDesc) == 24 + 8 + 16 + 64 + 8 + 4 + 4 + 8
    assert szo.LinearDesc.x.offset == 48 and szo.LinearDesc.target.offset == 104
    assert szo.LinearDesc.lut.offset == 112 and szo.LinearDesc.format.offset == 120
    assert szo.LinearDesc.x_minus.offset == 128


@pytest.mark.parametrize("N,K,dens,seed", [(130, 64, 0.02, 21), (256, 1024, 1e-2, 22), (64, 4096, 1e-3, 23)])
def test_table_format_quantiser_bit_exact(N, K, dens, seed):
    from oracle import quant as oq
    from helpers import banded_codes
    W = synth.dense_weight(seed, N, K)
    k = int(dens * N * K + 0.5)
    flat = omask.mask_uniform(N, K, k, seed)
    _, sp_idx, _ = omask.tcsr_build(N, K, flat)
    codes, lut, sp_val = oq.split_and_quantize_lut(W, sp_idx.astype(np.int64))
    q, lut_c, sp_c = szo.szo_quantize_pack_lut(W, sp_idx)
    assert np.array_equal(q, oq.pack_codes(codes))
    assert np.array_equal(lut_c.view(np.uint16), lut.view(np.uint16))
    assert np.array_equal(sp_c, sp_val)
    qb, none = szo.szo_layout_weights(q, None, 0)
    assert none is None and np.array_equal(qb, banded_codes(q))
    W2 = W[:, :48]                                   # K % 32 != 0
    with pytest.raises(szo.SzoError):
        szo.szo_quantize_pack_lut(np.ascontiguousarray(W2), np.zeros(0, np.uint32))


def test_philox_host_known_answers_and_oracle():
    path = os.path.join(ROOT, "tests", "golden", "philox4x32_10_kat.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        assert szo.szo_philox4x32_10(w[0:4], w[4:6]).tolist() == w[6:10]
    rng = np.random.default_rng(1)
    for _ in range(50):
        c = rng.integers(0, 2**32, 4, dtype=np.uint64)
        k = rng.integers(0, 2**32, 2, dtype=np.uint64)
        assert tuple(szo.szo_philox4x32_10(c, k).tolist()) == ophilox.philox4x32_10_scalar(c.tolist(), k.tolist())


@pytest.mark.parametrize("N,K,k,seed", [(256, 256, 66, 5), (4, 64, 200, 9), (100, 128, 0, 1), (4096, 4096, 16777, 77)])
def test_uniform_mask_bit_exact(N, K, k, seed):
    assert np.array_equal(szo.szo_mask_generate(N, K, k, 0, seed), omask.mask_uniform(N, K, k, seed).astype(np.uint32))


@pytest.mark.parametrize("N,K,dens,seed", [(1024, 512, 1e-2, 11), (4096, 1024, 1e-3, 3), (130, 64, 0.02, 8)])
def test_heavy_tail_mask_bit_exact(N, K, dens, seed):
    k = omask.nnz_for_density(N, K, dens)
    assert np.array_equal(szo.szo_mask_generate(N, K, k, 1, seed), omask.mask_heavy_tail(N, K, k, seed).astype(np.uint32))


@pytest.mark.parametrize("N,K,k", [(256, 256, 66), (100, 128, 300), (130, 64, 0), (64, 64, 4096), (1000, 1024, 5000)])
def test_tcsr_bit_exact(N, K, k):
    flat = omask.mask_uniform(N, K, k, 21)
    tp, idx, perm = szo.szo_tcsr_build(N, K, flat)
    otp, oidx, operm = omask.tcsr_build(N, K, flat)
    assert szo.szo_num_tiles(N, K) == omask.num_tiles(N, K) == tp.size - 1
    assert np.array_equal(tp, otp) and np.array_equal(idx, oidx) and np.array_equal(perm, operm)


def test_tcsr_rejects_bad_input():
    out = np.zeros(16, np.uint32)
    f = lambda a: szo.lib.szo_tcsr_build(64, 64, np.asarray(a, np.uint32).ctypes.data, len(a),
                                         out.ctypes.data, out.ctypes.data, None)
    assert f([3, 3, 5]) == szo.EINVAL          # duplicate
    assert f([5, 3]) == szo.EINVAL             # not ascending
    assert f([64 * 64]) == szo.EINVAL          # out of range
    assert szo.lib.szo_tcsr_build(64, 100, out.ctypes.data, 0, out.ctypes.data, out.ctypes.data, None) == szo.EUNSUPPORTED
    assert szo.szo_num_tiles(64, 100) == 0


@pytest.mark.parametrize("N,K,G,k", [(64, 128, 32, 40), (96, 256, 64, 0), (40, 256, 128, 100), (512, 1024, 128, 524)])
def test_quantize_pack_bit_exact(N, K, G, k):
    W = synth.dense_weight(N * 7 + K, N, K)
    W[3, :G] = 0.0                                  # an all-zero group
    W[5, 0] = 3e-6                                  # a group whose scale is an fp16 subnormal
    W[5, 1:G] = 0.0
    flat = omask.mask_uniform(N, K, k, 2)
    _, sp_idx, _ = omask.tcsr_build(N, K, flat)
    q, s, v = szo.szo_quantize_pack(W, G, sp_idx)
    oc, os_, ov = oquant.split_and_quantize(W, sp_idx.astype(np.int64), G)
    assert np.array_equal(q, oquant.pack_codes(oc))
    assert np.array_equal(s.view(np.uint16), os_.view(np.uint16))
    assert np.array_equal(v, ov)


@pytest.mark.parametrize("N,K,G", [(64, 64, 32), (100, 256, 128), (513, 1152, 64)])
def test_banded_layout_places_every_code_and_scale_where_the_header_says(N, K, G):
    rng = np.random.default_rng(N + K)
    q = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    sc = rng.integers(0, 0x7C00, size=(N, K // G), dtype=np.uint16)
    qb, sb = szo.szo_layout_weights(q, sc, G)
    bands = (N + 63) // 64
    assert qb.size == szo.szo_qweight_bytes(N, K) == bands * 64 * K // 2
    assert sb.size == szo.szo_scales_count(N, K, G) == bands * 64 * (K // G)
    sb = sb.view(np.uint16)
    # element by element, from the formulas (not from the reshuffle in helpers)
    for n, k in zip(rng.integers(0, N, 300), rng.integers(0, K, 300)):
        B, r, T = n // 64, n % 64, k // 64
        assert qb[((B * (K // 64) + T) * 64 + r) * 32 + (k % 64) // 2] == q[n, k // 2]
        g = k // G
        assert sb[(B * (K // G) + g) * 64 + (r % 16) * 4 + r // 16] == sc[n, g]
    from helpers import banded_codes, banded_scales
    assert np.array_equal(qb, banded_codes(q)) and np.array_equal(sb, banded_scales(sc))
    if N % 64:      # padding rows: weight zero
        last = qb.reshape(bands, K // 64, 64, 32)[-1, :, N % 64:, :]
        assert (last == 0x88).all()
    assert szo.lib.szo_layout_weights(q.ctypes.data, sc.ctypes.data, N, K + 1, G, qb.ctypes.data, sb.ctypes.data) == szo.EINVAL
    assert szo.szo_qweight_bytes(64, 100) == 0


def test_half_conversion_matches_numpy_everywhere_it_matters():
    # scale = fp16(max/7): drive max through normals, subnormals, ties and overflow
    vals = np.concatenate([
        np.float32(7.0) * np.arange(0, 2048, dtype=np.float32) * np.float32(2.0 ** -25),   # subnormal grid incl. ties
        np.float32(7.0) * (np.float32(1.0) + np.arange(0, 4096, dtype=np.float32) * np.float32(2.0 ** -12)),
        np.random.default_rng(0).uniform(0, 1e-3, 4000).astype(np.float32),
        np.random.default_rng(1).uniform(0, 1e4, 4000).astype(np.float32)])
    W = np.zeros((vals.size, 32), dtype=np.float32)
    W[:, 0] = vals
    _, s, _ = szo.szo_quantize_pack(W, 32, np.zeros(0, np.uint32))
    want = (vals / np.float32(7.0)).astype(np.float16)
    assert np.array_equal(s[:, 0].view(np.uint16), want.view(np.uint16))


def test_quantize_rejects_overflowing_scale():
    W = np.full((1, 32), 1e6, dtype=np.float32)
    q = np.zeros(16, np.uint8); s = np.zeros(1, np.uint16)
    assert szo.lib.szo_quantize_pack(W.ctypes.data, 1, 32, 32, None, 0, q.ctypes.data, s.ctypes.data, None) == szo.EINVAL


def test_hot_calls_validate_before_touching_the_gpu():
    d = szo.LinearDesc(M=8, N=64, K=100, group=32, tile_dtype=0, nnz=0, nnz_base=0)
    assert szo.lib.szo_linear_fwd(ctypes.byref(d), 0, 0, 1, 1e-3, None) == szo.EINVAL        # K % group
    d.K = 96
    assert szo.lib.szo_linear_fwd(ctypes.byref(d), 0, 0, 1, 1e-3, None) == szo.EUNSUPPORTED  # K % 64
    d.K = 128
    assert szo.lib.szo_linear_fwd(ctypes.byref(d), 0, 0, 2, 1e-3, None) == szo.EINVAL        # sign
    assert szo.lib.szo_linear_fwd(ctypes.byref(d), 0, 0, 1, 1e-3, None) == szo.EINVAL        # null pointers
    d.group = 16
    assert szo.lib.szo_linear_fwd(ctypes.byref(d), 0, 0, 1, 1e-3, None) == szo.EUNSUPPORTED
    d.group, d.nnz_base = 32, 2
    assert szo.lib.szo_linear_fwd(ctypes.byref(d), 0, 0, 1, 1e-3, None) == szo.EINVAL        # nnz_base % 4
    d.nnz_base, d.tile_dtype = 0, 7
    assert szo.lib.szo_linear_fwd(ctypes.byref(d), 0, 0, 1, 1e-3, None) == szo.EINVAL
    assert szo.lib.szo_linear_fwd(None, 0, 0, 1, 1e-3, None) == szo.EINVAL
    d.tile_dtype, d.M = 0, 0
    assert szo.lib.szo_linear_fwd(ctypes.byref(d), 0, 0, 1, 1e-3, None) == szo.OK            # empty: no-op
    # table format: group is not looked at, the table pointer and the fp16 tile are required
    t = szo.LinearDesc(M=8, N=64, K=128, group=0, tile_dtype=1, nnz=0, nnz_base=0, format=szo.FORMAT_LUT)
    assert szo.lib.szo_linear_fwd(ctypes.byref(t), 0, 0, 1, 1e-3, None) == szo.EUNSUPPORTED  # bf16 tile
    t.tile_dtype = 0
    assert szo.lib.szo_linear_fwd(ctypes.byref(t), 0, 0, 1, 1e-3, None) == szo.EINVAL        # null pointers
    t.format = 2
    assert szo.lib.szo_linear_fwd(ctypes.byref(t), 0, 0, 1, 1e-3, None) == szo.EINVAL        # unknown format
    t.format, t.M = szo.FORMAT_LUT, 0
    assert szo.lib.szo_linear_fwd(ctypes.byref(t), 0, 0, 1, 1e-3, None) == szo.OK            # empty: no-op
    assert szo.lib.szo_mse_loss(None, None, 5, 1.0, None, None, None) == szo.EINVAL
    assert szo.lib.szo_sparse_update(None, None, 4, 2, 0, 0, None, 0.1, None) == szo.EINVAL
    assert szo.lib.szo_spsa_g(None, None, 0.1, None, None) == szo.EINVAL
    assert szo.lib.szo_zo_step(None, 1, 0, 0, 0.1, 0.1, None, None, 0, None) == szo.EINVAL
    # a layer without tokens may leave its activation pointers empty, but its sparse values are updated
    e = szo.LinearDesc(M=0, N=64, K=128, group=32, tile_dtype=0, nnz=8, nnz_base=0)
    buf = ctypes.create_string_buffer(64)
    assert szo.lib.szo_zo_step(ctypes.byref(e), 1, 0, 0, 0.1, 0.1, ctypes.addressof(buf), ctypes.addressof(buf), 0, None) == szo.EINVAL
    assert szo.lib.szo_debug_zbar(0, -1, 0, 0, None, None, None) == szo.EINVAL


def test_kernel_timing_calls_are_safe_without_any_launch():
    szo.szo_kernel_timing(True)
    assert szo.szo_kernel_timing_read() == (0.0, 0)
    szo.szo_kernel_timing(False)
    assert szo.lib.szo_kernel_timing_read(None, None) == szo.EINVAL
