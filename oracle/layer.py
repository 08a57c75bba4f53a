"""Linear layer with a sparse correction, and the stand-in loss.  Test
infrastructure only.

Forward (Appendix C.5): y = (Dequantize(Q(w_dense)) + w_sparse) x, i.e.
DenseMM(SparseAdd(w_sparse, Dequantize(Q(w_dense))), x).  The perturbed
forward of Definition 1 / Definition 4 evaluates the same expression at
w_sparse + sign * eps * z_k.  Shapes: x is [M, K], the weight is [N, K]
(out x in), y = x W^T is [M, N].

Mode "E" (exact) is the definition in fp64.  Mode "D" is identical except
that the effective weight is rounded to a 16-bit float after the sparse add
("f16" or "bf16"), with the sensitive value formed in fp32 the way a GPU
datapath would; it exists so that kernels can be gated to ~1e-5 against
something that isolates accumulation error from operand rounding.
"""
import numpy as np

from .quant import dequantize, dequantize_lut, f32_to_bf16_bits, bf16_bits_to_f64


def _round16(w32, tile_dtype):
    if tile_dtype == "f16":
        return w32.astype(np.float16).astype(np.float64)
    if tile_dtype == "bf16":
        return bf16_bits_to_f64(f32_to_bf16_bits(w32))
    raise ValueError(tile_dtype)


def effective_weight(codes, scales, group, sp_idx, sp_val, z=None, sign=0, eps=0.0,
                     mode="E", tile_dtype="f16", lut=None):
    """SparseAdd(w_sparse + sign*eps*z, Dequantize(Q(w_dense))) as a dense
    fp64 [N, K] matrix.  sp_idx are flat positions n*K+k, sp_val fp32.
    With `lut` (fp16 [N, 16]) the codes are of the non-uniform format and
    scales / group are not looked at."""
    dq = dequantize(codes, scales, group) if lut is None else dequantize_lut(codes, lut)
    N, K = dq.shape
    idx = np.asarray(sp_idx, dtype=np.int64)
    eps32 = np.float32(eps)
    if mode == "E":
        v = np.asarray(sp_val, dtype=np.float32).astype(np.float64)
        if z is not None and sign != 0:
            v = v + float(sign) * float(eps32) * np.asarray(z, dtype=np.float64)
        W = dq.copy()
        W.reshape(-1)[idx] += v
        return W
    if mode == "D":
        v32 = np.asarray(sp_val, dtype=np.float32).copy()
        if z is not None and sign != 0:
            v32 = v32 + (np.float32(sign) * eps32) * np.asarray(z, dtype=np.float64).astype(np.float32)
        w32 = dq.astype(np.float32)          # exact: 15 significant bits at most
        w32.reshape(-1)[idx] += v32
        return _round16(w32, tile_dtype)
    raise ValueError(mode)


def linear_fwd(x_bits, codes, scales, group, sp_idx, sp_val, z=None, sign=0, eps=0.0,
               mode="E", tile_dtype="f16", lut=None):
    """y = x W_eff^T in fp64.  x_bits: uint16 bf16 patterns [M, K]."""
    x = bf16_bits_to_f64(x_bits)
    W = effective_weight(codes, scales, group, sp_idx, sp_val, z, sign, eps, mode, tile_dtype, lut)
    return x @ W.T


def linear_fwd_addmm(x_bits, codes, scales, group, sp_idx, sp_val, z=None, sign=0, eps=0.0, lut=None):
    """The other association of Appendix C.5: SparseAddMM(DenseMM(Dequantize(
    Q(w_dense)), x), w_sparse, x) -- dense product first, then one rank-one
    column update per sensitive entry.  Must equal linear_fwd to fp64
    rounding."""
    x = bf16_bits_to_f64(x_bits)
    dq = dequantize(codes, scales, group) if lut is None else dequantize_lut(codes, lut)
    N, K = dq.shape
    y = x @ dq.T
    v = np.asarray(sp_val, dtype=np.float32).astype(np.float64)
    if z is not None and sign != 0:
        v = v + float(sign) * float(np.float32(eps)) * np.asarray(z, dtype=np.float64)
    idx = np.asarray(sp_idx, dtype=np.int64)
    for j in range(idx.size):
        n, k = divmod(int(idx[j]), K)
        y[:, n] += x[:, k] * v[j]
    return y


def linear_fwd_bruteforce(x_bits, codes, scales, group, sp_idx, sp_val, z=None, sign=0, eps=0.0, lut=None):
    """Triple loop over (m, n, k) in Python floats; tiny shapes only."""
    x = bf16_bits_to_f64(x_bits)
    M, K = x.shape
    N = codes.shape[0]
    if lut is None:
        s = np.asarray(scales, dtype=np.float16).astype(np.float64)
    extra = {}
    for j, f in enumerate(np.asarray(sp_idx, dtype=np.int64).tolist()):
        v = float(np.float32(sp_val[j]))
        if z is not None and sign != 0:
            v += sign * float(np.float32(eps)) * float(z[j])
        extra[f] = v
    y = np.zeros((M, N))
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                if lut is None:
                    w = (int(codes[n, k]) - 8) * float(s[n, k // group])
                else:
                    w = float(np.float16(lut[n, int(codes[n, k])]))
                acc += float(x[m, k]) * (w + extra.get(n * K + k, 0.0))
            y[m, n] = acc
    return y


def mse_loss(y, target_bits):
    """L = mean((y - t)^2) in fp64; the target is bf16 [M, N].  The paper only
    needs a scalar loss f (Definition 1); mean squared error against a seeded
    target is the workloads' stand-in for the language-model loss."""
    t = bf16_bits_to_f64(target_bits)
    d = np.asarray(y, dtype=np.float64) - t
    return float(np.mean(d * d))


def mse_grad_on_mask(x_bits, y, target_bits, sp_idx, K):
    """dL/dw at the mask positions for L = mean((x W^T - t)^2):
    dL/dW[n, k] = (2 / (M N)) * sum_m (y - t)[m, n] * x[m, k]."""
    x = bf16_bits_to_f64(x_bits)
    t = bf16_bits_to_f64(target_bits)
    r = (np.asarray(y, dtype=np.float64) - t) * (2.0 / y.size)
    idx = np.asarray(sp_idx, dtype=np.int64)
    n, k = idx // K, idx % K
    return np.einsum("mj,mj->j", r[:, n], x[:, k])
