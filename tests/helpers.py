"""Shared test plumbing: builds oracle-side matrices from the seeded inputs."""
import numpy as np

from oracle import mask as omask, quant as oquant
from oracle.zo import Matrix
from paper_2406_02913_amd import synth


def make_oracle_matrix(seed, M, N, K, group, density=1e-3, kind="uniform", nnz=None,
                       nnz_base=0, mask_seed=None, sigma=0.02, fmt="uniform"):
    x = synth.activations(seed, M, K)
    W = synth.dense_weight(seed, N, K, sigma)
    t = synth.target(seed, M, N)
    k = omask.nnz_for_density(N, K, density) if nnz is None else nnz
    ms = seed + 1000 if mask_seed is None else mask_seed
    flat = (omask.mask_uniform if kind == "uniform" else omask.mask_heavy_tail)(N, K, k, ms)
    tile_ptr, sp_idx, perm = omask.tcsr_build(N, K, flat)
    lut = None
    if fmt == "lut":
        codes, lut, sp_val = oquant.split_and_quantize_lut(W, sp_idx.astype(np.int64))
        scales = None
    else:
        codes, scales, sp_val = oquant.split_and_quantize(W, sp_idx.astype(np.int64), group)
    m = Matrix(x_bits=x, codes=codes, scales=scales, group=group, sp_idx=sp_idx,
               sp_val=sp_val, target_bits=t, nnz_base=nnz_base, lut=lut)
    m.tile_ptr = tile_ptr
    m.W = W
    m.flat_sorted = flat
    return m


def clone(m):
    c = Matrix(m.x_bits, m.codes, m.scales, m.group, m.sp_idx, m.sp_val.copy(), m.target_bits, m.nnz_base, m.lut,
               m.x_minus_bits)
    for a in ("tile_ptr", "W", "flat_sorted"):
        if hasattr(m, a):
            setattr(c, a, getattr(m, a))
    return c


def banded_codes(q_rowmajor):
    """Row-major packed codes [N, K/2] -> the banded device layout, written out from its definition:
    byte ((B*(K/64) + T)*64 + r)*32 + (k%64)/2, rows padded to 64 with code 8."""
    N, Kh = q_rowmajor.shape
    bands, T = (N + 63) // 64, Kh // 32
    pad = np.full((bands * 64, Kh), 0x88, dtype=np.uint8)
    pad[:N] = q_rowmajor
    return pad.reshape(bands, 64, T, 32).transpose(0, 2, 1, 3).reshape(-1)


def banded_scales(scales_rowmajor_bits):
    """Row-major fp16 bit patterns [N, K/group] -> banded layout: element (B*G + g)*64 + (r%16)*4 + r//16."""
    N, G = scales_rowmajor_bits.shape
    bands = (N + 63) // 64
    pad = np.zeros((bands * 64, G), dtype=np.uint16)
    pad[:N] = scales_rowmajor_bits
    out = np.empty((bands, G, 64), dtype=np.uint16)
    for r in range(64):
        out[:, :, (r % 16) * 4 + r // 16] = pad.reshape(bands, 64, G)[:, r, :]
    return out.reshape(-1)


def make_pair(seed, M, N, K, group, density=1e-3, kind="uniform", nnz=None, nnz_base=0, device="cuda", fmt="uniform"):
    """The same layer twice: oracle-side (numpy) and device-side (libszo host
    set-up + torch memory).  Asserts that mask, tile order, codes, scales and
    sparse values agree bit for bit before anything is computed."""
    from paper_2406_02913_amd import stack
    o = make_oracle_matrix(seed, M, N, K, group, density, kind, nnz, nnz_base, fmt=fmt)
    d = stack.build_linear(seed, M, N, K, group, density, kind, nnz, nnz_base, device=device, keep_host=True, fmt=fmt)
    h = d.host
    assert np.array_equal(h["flat"], o.flat_sorted.astype(np.uint32))
    assert np.array_equal(h["tile_ptr"], o.tile_ptr) and np.array_equal(h["sp_idx"], o.sp_idx)
    assert np.array_equal(h["qweight"], oquant.pack_codes(o.codes))
    assert np.array_equal(h["sp_val"], o.sp_val)
    assert np.array_equal(h["qweight_banded"], banded_codes(oquant.pack_codes(o.codes)))
    if fmt == "lut":
        assert np.array_equal(h["lut"].view(np.uint16), o.lut.view(np.uint16))
    else:
        assert np.array_equal(h["scales"].view(np.uint16), o.scales.view(np.uint16))
        assert np.array_equal(h["scales_banded"].view(np.uint16), banded_scales(o.scales.view(np.uint16)))
    return o, d


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def sigma_g(mats):
    """sqrt(sum |grad L on the mask|^2): the natural scale of g = z . grad L.  Small masks go through the
    oracle's mse_grad_on_mask; for large ones (its gather would take M x nnz doubles) the same formula
    dL/dW = (2 / (M N)) (y - t)^T x is evaluated as one dense product and read at the mask positions."""
    from oracle import layer
    from oracle.quant import bf16_bits_to_f64
    tot = 0.0
    for m in mats:
        y0 = layer.linear_fwd(m.x_bits, m.codes, m.scales, m.group, m.sp_idx, m.sp_val, lut=m.lut)
        M, K = m.x_bits.shape
        if M * m.sp_idx.size <= (1 << 27):
            grad = layer.mse_grad_on_mask(m.x_bits, y0, m.target_bits, m.sp_idx, K)
        else:
            r = (y0 - bf16_bits_to_f64(m.target_bits)) * (2.0 / y0.size)
            grad = (r.T @ bf16_bits_to_f64(m.x_bits)).reshape(-1)[m.sp_idx.astype(np.int64)]
        tot += float(np.sum(grad ** 2))
    return float(np.sqrt(tot))

class UpdateBound:
    """How far the sparse values may end up from the oracle's after some steps.  One step moves them by
    -lr g z (Section 3.4, fixed-parameter update rule), so an error dg on the SPSA scalar moves matrix i
    by lr |dg| ||z_i||, and the bar on g is |dg| <= 1e-2 max(|g|, sigma_g): for one step that is a
    relative error of 1e-2 max(|g|, sigma_g) / |g| on the update.  Both sides store fp32 values, so one
    ulp of the value per step comes on top."""

    def __init__(self, sg, lr):
        self.sg, self.lr, self.tol, self.steps = float(sg), float(np.float32(lr)), None, 0

    def add(self, r, extra_dg=0.0):
        """r: what the oracle's zo_step returned for this step (g and the per-matrix z); extra_dg: what
        the test allows on g beyond the bar (two activation sets: the losses' own error over 2 eps)."""
        dg = 1e-2 * max(abs(r["g"]), self.sg) + extra_dg
        if self.tol is None:
            self.tol = [0.0] * len(r["z"])
        for i, z in enumerate(r["z"]):
            self.tol[i] += self.lr * dg * float(np.linalg.norm(z))
        self.steps += 1

    def check(self, i, v_gpu, v_ref, v0):
        v_gpu, v_ref = np.asarray(v_gpu, dtype=np.float64), np.asarray(v_ref, dtype=np.float64)
        err = float(np.linalg.norm(v_gpu - v_ref))
        allowed = self.tol[i] + self.steps * float(np.linalg.norm(np.spacing(np.abs(v_ref).astype(np.float32))))
        moved = float(np.linalg.norm(v_ref - np.asarray(v0, dtype=np.float64)))
        assert err <= allowed, (i, err, allowed, moved)
        if self.lr > 0 and moved > 4 * allowed:       # the update is visible: the GPU's values moved too
            assert float(np.linalg.norm(v_gpu - np.asarray(v0, dtype=np.float64))) >= 0.5 * moved
