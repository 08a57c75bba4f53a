"""Static decomposition w = w_sparse + w_dense (Section 3.4, first equation;
restated at the start of Appendix C.5) followed by 4-bit quantisation of the
dense part (Section 3.5, "Model weights").  Test infrastructure only.

The paper allows any post-training quantiser; the workloads here fix a plain
uniform symmetric one: per output row, per group of `group` consecutive input
columns, scale = fp16(max|w| / 7), code = clamp(rint(w / scale), -8, 7),
stored as code + 8 in a nibble (zero code 8).  Masked coordinates are set to
zero before the scales are taken, so w_dense is exactly zero on the mask and
"add the sparse part" equals "overwrite with the sparse part".

A second, non-uniform format (Appendix C.5, "Integration with weight
quantization method": a non-uniform quantiser is always dequantised first and
takes the SparseAdd form): per output row a table of 16 fp16 centroids, code =
index of the nearest centroid.  The paper fixes no codebook construction; the
reading here is the plainest deterministic one: the centroids of a row are the
16 order statistics of its dense part (mask zeroed) at ranks (2c+1)K/32, i.e.
the medians of 16 equal-mass bins, rounded to fp16.  Zero is then in general
not a centroid, so on the mask the dequantised dense part is a small non-zero
value and the sparse part is ADDED to it, as the decomposition says.
"""
import numpy as np


def bf16_bits_to_f64(bits):
    """uint16 bf16 bit patterns -> the exact values in fp64."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def f32_to_bf16_bits(v):
    """fp32 -> bf16 bit pattern, round to nearest even (finite inputs)."""
    u = np.asarray(v, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def split_and_quantize(W, flat_idx, group):
    """W: fp32 [N, K]; flat_idx: mask positions n*K+k (any order).

    Returns (codes uint8 [N, K] in 0..15, scales float16 [N, K/group],
    sp_val float32 [len(flat_idx)] in the order of flat_idx)."""
    W = np.asarray(W, dtype=np.float32)
    N, K = W.shape
    assert K % group == 0
    flat_idx = np.asarray(flat_idx, dtype=np.int64)
    sp_val = W.reshape(-1)[flat_idx].copy()
    dense = W.copy()
    dense.reshape(-1)[flat_idx] = np.float32(0.0)
    g = dense.reshape(N, K // group, group)
    maxabs = np.max(np.abs(g), axis=2)                       # fp32
    scales = (maxabs / np.float32(7.0)).astype(np.float16)    # fp32 divide, RNE to fp16
    s32 = scales.astype(np.float32)
    safe = np.where(s32 == 0, np.float32(1.0), s32)
    q = np.rint(g / safe[:, :, None])                         # fp32 divide, half-to-even
    q = np.where(s32[:, :, None] == 0, np.float32(0.0), q)
    q = np.clip(q, -8.0, 7.0).astype(np.int32)
    codes = (q + 8).astype(np.uint8).reshape(N, K)
    return codes, scales, sp_val


def pack_codes(codes):
    """[N, K] codes 0..15 -> [N, K/2] bytes, low nibble = even k."""
    codes = np.asarray(codes, dtype=np.uint8)
    return (codes[:, 0::2] | (codes[:, 1::2] << np.uint8(4))).astype(np.uint8)


def unpack_codes(packed):
    packed = np.asarray(packed, dtype=np.uint8)
    N, K2 = packed.shape
    out = np.empty((N, 2 * K2), dtype=np.uint8)
    out[:, 0::2] = packed & np.uint8(0x0F)
    out[:, 1::2] = packed >> np.uint8(4)
    return out


def dequantize(codes, scales, group):
    """Dequantize(Q(w_dense)) of Appendix C.5: (code - 8) * scale, in fp64.

    The product is exact: a 4-bit integer times an 11-bit significand."""
    codes = np.asarray(codes)
    N, K = codes.shape
    s = np.asarray(scales, dtype=np.float16).astype(np.float64)
    return (codes.astype(np.float64) - 8.0) * np.repeat(s, group, axis=1)


def split_and_quantize_lut(W, flat_idx):
    """Non-uniform 4-bit format.  W: fp32 [N, K], K % 32 == 0.

    Returns (codes uint8 [N, K] in 0..15, lut float16 [N, 16] non-decreasing
    along each row, sp_val float32 in the order of flat_idx)."""
    W = np.asarray(W, dtype=np.float32)
    N, K = W.shape
    assert K % 32 == 0
    flat_idx = np.asarray(flat_idx, dtype=np.int64)
    sp_val = W.reshape(-1)[flat_idx].copy()
    dense = W.copy()
    dense.reshape(-1)[flat_idx] = np.float32(0.0)
    ranks = (2 * np.arange(16) + 1) * (K // 32)
    lut = np.sort(dense, axis=1)[:, ranks].astype(np.float16)          # RNE to fp16
    codes = np.empty((N, K), dtype=np.uint8)
    for r0 in range(0, N, 128):                                        # row blocks only bound the memory used
        d = dense[r0:r0 + 128].astype(np.float64)
        t = lut[r0:r0 + 128].astype(np.float64)
        # nearest centroid; fp32 minus fp16 is exact in fp64; ties go to the lower index
        codes[r0:r0 + 128] = np.argmin(np.abs(d[:, :, None] - t[:, None, :]), axis=2)
    return codes, lut, sp_val


def dequantize_lut(codes, lut):
    """Dequantize(Q(w_dense)) for the non-uniform format: lut[n, code[n, k]], fp64."""
    codes = np.asarray(codes)
    t = np.asarray(lut, dtype=np.float16).astype(np.float64)
    return np.take_along_axis(t, codes.astype(np.int64), axis=1)
