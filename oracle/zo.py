"""One sensitive-sparse ZO-SGD step.  Test infrastructure only.

SPSA (Definition 1): g = [f(w + eps z) - f(w - eps z)] / (2 eps), and the
surrogate gradient is g * z.  With the perturbation restricted to the fixed
sensitive coordinates (Definition 4; Section 3.4) only w_sparse moves:
w_sparse <- w_sparse - lr * g * z_k, the dense 4-bit part stays frozen.

Readings the paper leaves open: f is ONE scalar for the whole model, here the
sum over matrices of each matrix's mean squared error; z_k is one vector over
all sensitive entries, so matrix l uses global indices nnz_base_l + j;
eps = 0 is defined to give g = 0.
"""
from dataclasses import dataclass

import numpy as np

from .philox import zbar
from .layer import linear_fwd, mse_loss


@dataclass
class Matrix:
    x_bits: np.ndarray       # uint16 bf16 [M, K]
    codes: np.ndarray        # uint8 [N, K], 0..15
    scales: np.ndarray       # float16 [N, K/group]
    group: int
    sp_idx: np.ndarray       # uint32 [nnz] flat n*K+k, tile order
    sp_val: np.ndarray       # float32 [nnz]
    target_bits: np.ndarray  # uint16 bf16 [M, N]
    nnz_base: int = 0
    lut: np.ndarray = None   # float16 [N, 16]: non-uniform format (scales, group unused)
    x_minus_bits: np.ndarray = None   # uint16 bf16 [M, K]: activations seen by the -eps forward, if they
                                      # differ (below the first layer of a model they do); None = x_bits


def spsa_scalar(loss_plus, loss_minus, eps):
    """g of Definition 1; eps is the fp32 value the kernels receive."""
    e = float(np.float32(eps))
    if e == 0.0:
        return 0.0
    return (float(loss_plus) - float(loss_minus)) / (2.0 * e)


def model_loss(mats, seed, step, sign, eps, mode="E", tile_dtype="f16", zs=None,
               loss_fn=mse_loss):
    """f(w_sparse + sign*eps*z): the sum over matrices of loss_fn(y, target)."""
    total = 0.0
    for i, m in enumerate(mats):
        z = zs[i] if zs is not None else zbar(seed, step, m.nnz_base, m.sp_idx.size)
        x = m.x_minus_bits if (sign < 0 and m.x_minus_bits is not None) else m.x_bits
        y = linear_fwd(x, m.codes, m.scales, m.group, m.sp_idx, m.sp_val,
                       z=z, sign=sign, eps=eps, mode=mode, tile_dtype=tile_dtype, lut=m.lut)
        total += loss_fn(y, m.target_bits)
    return total


def zo_step(mats, seed, step, eps, lr, mode="E", tile_dtype="f16", loss_fn=mse_loss):
    """Two perturbed forwards, the SPSA scalar, the in-place sparse update.
    Returns dict(loss_plus, loss_minus, g, z=[per-matrix z_k])."""
    zs = [zbar(seed, step, m.nnz_base, m.sp_idx.size) for m in mats]
    lp = model_loss(mats, seed, step, +1, eps, mode, tile_dtype, zs, loss_fn)
    lm = model_loss(mats, seed, step, -1, eps, mode, tile_dtype, zs, loss_fn)
    g = spsa_scalar(lp, lm, eps)
    sparse_update(mats, zs, g, lr)
    return dict(loss_plus=lp, loss_minus=lm, g=g, z=zs)


def sparse_update(mats, zs, g, lr):
    """w_sparse <- w_sparse - lr * g * z_k, computed in fp64, stored fp32."""
    step_size = float(np.float32(lr)) * float(g)
    for m, z in zip(mats, zs):
        m.sp_val = (m.sp_val.astype(np.float64) - step_size * z).astype(np.float32)


def zo_step_inplace(mats, seed, step, eps, lr):
    """Same step written the MeZO way (Section 2.1, random-seed trick): perturb
    the stored fp32 values by +eps z, evaluate, by -2 eps z, evaluate, restore
    with +eps z, then update -- z regenerated from the seed each time.
    Returns dict(loss_plus, loss_minus, g, restored=[per-matrix values after
    the +eps, -2eps, +eps walk and before the update])."""
    e = np.float32(eps)

    def shift(c):
        for m in mats:
            z = zbar(seed, step, m.nnz_base, m.sp_idx.size)
            m.sp_val = (m.sp_val + (np.float32(c) * e) * z.astype(np.float32)).astype(np.float32)

    shift(+1.0)
    lp = model_loss(mats, seed, step, 0, 0.0)
    shift(-2.0)
    lm = model_loss(mats, seed, step, 0, 0.0)
    shift(+1.0)
    restored = [m.sp_val.copy() for m in mats]
    g = spsa_scalar(lp, lm, eps)
    zs = [zbar(seed, step, m.nnz_base, m.sp_idx.size) for m in mats]
    sparse_update(mats, zs, g, lr)
    return dict(loss_plus=lp, loss_minus=lm, g=g, restored=restored)
