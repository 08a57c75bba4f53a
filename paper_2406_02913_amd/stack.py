"""Device-resident state of a stack of sparse+int4 linear layers, built from the
seeded synthetic inputs with the library's own host set-up calls.  Plumbing
only: torch allocates and copies, every computation is a libszo call.
"""
from dataclasses import dataclass, field

import numpy as np
import torch

from . import synth, szo


def nnz_for_density(N, K, density):
    return int(np.floor(density * N * K + 0.5))


@dataclass
class DeviceLinear:
    name: str
    M: int
    N: int
    K: int
    group: int
    nnz: int
    nnz_base: int
    x: torch.Tensor
    qweight: torch.Tensor
    scales: torch.Tensor
    tile_ptr: torch.Tensor
    sp_idx: torch.Tensor
    sp_val: torch.Tensor
    target: torch.Tensor
    y: torch.Tensor = None
    lut: torch.Tensor = None          # fp16 [N,16]: non-uniform format (scales is None then)
    x_minus: torch.Tensor = None      # bf16 [M,K]: activations of the -eps forward, if they differ
    host: dict = field(default_factory=dict)

    def desc(self, tile_dtype=szo.TILE_F16, with_y=True):
        return szo.make_desc(self.M, self.N, self.K, self.group, self.nnz, self.nnz_base, self.x,
                             self.qweight, self.scales, self.tile_ptr, self.sp_idx, self.sp_val,
                             self.y if with_y else None, self.target, tile_dtype, self.lut, self.x_minus)


def _to_dev(a, device, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.view(dtype)
    return t.to(device)


def build_linear(seed, M, N, K, group, density=1e-3, kind="uniform", nnz=None, nnz_base=0,
                 device="cuda", keep_host=False, name="lin", y=None, mask_seed=None, sigma=0.02, fmt="uniform"):
    """Same recipe as the CPU checker's test helper: activations, dense weight
    and target from synth; mask, tile order and quantisation from libszo."""
    x = synth.activations(seed, M, K)
    W = synth.dense_weight(seed, N, K, sigma)
    t = synth.target(seed, M, N)
    k = nnz_for_density(N, K, density) if nnz is None else nnz
    ms = seed + 1000 if mask_seed is None else mask_seed
    flat = szo.szo_mask_generate(N, K, k, 0 if kind == "uniform" else 1, ms)
    tile_ptr, sp_idx, perm = szo.szo_tcsr_build(N, K, flat)
    lut = None
    if fmt == "lut":
        q, lut, sp_val = szo.szo_quantize_pack_lut(W, sp_idx)
        scales = None
    else:
        q, scales, sp_val = szo.szo_quantize_pack(W, group, sp_idx)
    q_banded, scales_banded = szo.szo_layout_weights(q, scales, group)
    if k == 0:      # keep non-null device pointers for empty arrays
        sp_idx_d = torch.zeros(4, dtype=torch.int32, device=device)
        sp_val_d = torch.zeros(4, dtype=torch.float32, device=device)
    else:
        sp_idx_d = _to_dev(sp_idx.view(np.int32), device)
        sp_val_d = _to_dev(sp_val, device)
    lin = DeviceLinear(
        name=name, M=M, N=N, K=K, group=group, nnz=k, nnz_base=nnz_base,
        x=_to_dev(x.view(np.int16), device, torch.bfloat16),
        qweight=_to_dev(q_banded, device),
        scales=None if scales is None else _to_dev(scales_banded.view(np.int16), device, torch.float16),
        lut=None if lut is None else _to_dev(lut.view(np.int16), device, torch.float16),
        tile_ptr=_to_dev(tile_ptr.view(np.int32), device),
        sp_idx=sp_idx_d, sp_val=sp_val_d,
        target=_to_dev(t.view(np.int16), device, torch.bfloat16),
        y=y if y is not None else torch.empty((M, N), dtype=torch.float32, device=device))
    if keep_host:
        lin.host = dict(x_bits=x, W=W, target_bits=t, flat=flat, tile_ptr=tile_ptr, sp_idx=sp_idx,
                        perm=perm, qweight=q, scales=scales, sp_val=sp_val,
                        qweight_banded=q_banded, scales_banded=scales_banded, lut=lut)
    return lin


def build_stack(workload, data_seed=0, device="cuda", M=None, layers=None, density=None,
                keep_host=False, progress=None, fmt="uniform"):
    """All matrices of a named workload (synth.WORKLOADS).  One y buffer, sized
    for the largest matrix, is shared by the whole stack."""
    cfg = dict(synth.WORKLOADS[workload]) if isinstance(workload, str) else dict(workload)
    M = cfg["M"] if M is None else M
    layers = cfg["layers"] if layers is None else layers
    density = cfg["density"] if density is None else density
    max_n = max(n for _, n, _ in cfg["block"])
    y = torch.empty((M, max_n), dtype=torch.float32, device=device)
    mats, base = [], 0
    for layer in range(layers):
        for i, (name, N, K) in enumerate(cfg["block"]):
            k = nnz_for_density(N, K, density)
            lin = build_linear(synth.matrix_seed(data_seed, layer, i), M, N, K, cfg["group"], density,
                               cfg["mask"], nnz=k, nnz_base=base, device=device, keep_host=keep_host,
                               name=f"L{layer}.{name}", y=y.view(-1)[:M * N].view(M, N), fmt=fmt)
            base += (k + 3) // 4 * 4
            mats.append(lin)
            if progress:
                progress(lin)
    return mats, cfg
