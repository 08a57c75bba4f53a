"""Seeded sweep over shapes, group sizes, densities, formats and tile configurations inside the
documented limits: every case is one forward per sign against the oracle, plus one fused step."""
import numpy as np
import pytest
import torch

from oracle import layer as olayer, philox as ophilox, zo as ozo
from paper_2406_02913_amd import szo
from helpers import make_pair, clone, rel_fro, sigma_g, UpdateBound

pytestmark = pytest.mark.gpu


def _cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        fmt = "lut" if rng.random() < 0.4 else "uniform"
        group = int(rng.choice([32, 64, 128]))
        K = int(rng.integers(1, 17)) * 64
        if K % group:
            K = (K + group - 1) // group * group
        M = int(rng.choice([1, 2, 15, 16, 17, 33, 64, 65, 100, 255, 256, 257, 300, 520]))
        N = int(rng.choice([1, 5, 63, 64, 65, 130, 255, 256, 257, 300, 511, 640]))
        dens = float(rng.choice([0.0, 1e-3, 1e-2, 5e-2]))
        kind = "heavy_tail" if (N >= 100 and dens <= 1e-2 and rng.random() < 0.5) else "uniform"   # hot rows hold k/2
        cfg = int(rng.choice([0, 1, 2, 3, 4, 5]))
        dt = "bf16" if (fmt == "uniform" and rng.random() < 0.25) else "f16"
        out.append((1000 + i, M, N, K, group, dens, kind, fmt, cfg, dt))
    return out


@pytest.fixture(autouse=True)
def _auto_tile_config():
    yield
    szo.szo_set_tile_config(0)


@pytest.mark.parametrize("case", _cases(96, 20240611), ids=lambda c: "-".join(str(v) for v in c[1:]))
def test_random_case(case):
    s, M, N, K, G, dens, kind, fmt, cfg, dtname = case
    dt = szo.TILE_BF16 if dtname == "bf16" else szo.TILE_F16
    o, d = make_pair(s, M, N, K, G, dens, kind=kind, nnz_base=4 * (s % 7), fmt=fmt)
    szo.szo_set_tile_config(cfg)
    seed, step, eps = 31 + s, s % 5, 1e-3
    z = ophilox.zbar(seed, step, o.nnz_base, o.sp_idx.size)
    scales = None if fmt == "lut" else o.scales
    for sign in (+1, -1):
        d.y.fill_(float("nan"))
        szo.szo_linear_fwd(d.desc(dt), seed, step, sign, eps)
        torch.cuda.synchronize()
        y = d.y.cpu().numpy()
        assert np.isfinite(y).all()
        yE = olayer.linear_fwd(o.x_bits, o.codes, scales, G, o.sp_idx, o.sp_val, z, sign, eps, "E", lut=o.lut)
        # relative to the outputs' natural size 0.02 sqrt(K) per element when the few outputs of a tiny
        # case happen to cancel (a 1 x 1 output can be anything)
        floor = 0.02 * np.sqrt(float(K) * M * N)
        assert np.linalg.norm(y - yE) <= 5e-3 * max(np.linalg.norm(yE), floor), (sign, rel_fro(y, yE))
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    om = clone(o)
    szo.szo_zo_step([d.desc(dt, with_y=False)], seed, step, eps, 1e-3, scal, ws, szo.STEP_FUSED_LOSS)
    lp, lm, g = scal.cpu().numpy()
    r = ozo.zo_step([om], seed, step, eps, 1e-3)
    assert abs(lp - r["loss_plus"]) <= 5e-3 * r["loss_plus"] and abs(lm - r["loss_minus"]) <= 5e-3 * r["loss_minus"]
    sg = sigma_g([o])
    # the bf16 tile cannot hold w + eps z to the estimator's 1e-2 budget (8-bit significand): 1e-1 there
    gtol = 1e-2 if dtname == "f16" else 1e-1
    assert abs(g - r["g"]) <= gtol * max(abs(r["g"]), sg), (g, r["g"])
    if o.sp_idx.size == 0:              # k = 0: the device side keeps a small placeholder array
        return
    # the update is -lr g z: it inherits g's error, which is bounded relative to max(|g|, sigma_g)
    bound = UpdateBound(sg, 1e-3)
    bound.add(r, extra_dg=(gtol - 1e-2) * max(abs(r["g"]), sg))
    bound.check(0, d.sp_val.cpu().numpy(), om.sp_val, o.sp_val)


@pytest.mark.parametrize("M,cfg,fmt", [(16, 0, "uniform"), (48, 5, "uniform"), (16, 0, "lut"), (300, 2, "uniform"), (300, 3, "lut")])
def test_every_weight_sensitive(M, cfg, fmt):
    """Density 1: the whole matrix lives in the sparse part (4096 entries per 64 x 64 tile), the dense codes
    are all the zero code (or, in the table format, whatever centroid is nearest to zero)."""
    N, K = 128, 256
    o, d = make_pair(2001, M, N, K, 128, 1.0, fmt=fmt)
    assert o.sp_idx.size == N * K
    szo.szo_set_tile_config(cfg)
    seed, step, eps = 3, 2, 1e-3
    z = ophilox.zbar(seed, step, 0, o.sp_idx.size)
    for sign in (+1, -1):
        szo.szo_linear_fwd(d.desc(), seed, step, sign, eps)
        torch.cuda.synchronize()
        yE = olayer.linear_fwd(o.x_bits, o.codes, None if fmt == "lut" else o.scales, 128, o.sp_idx, o.sp_val, z, sign, eps, "E", lut=o.lut)
        assert rel_fro(d.y.cpu().numpy(), yE) <= 5e-3
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    om = clone(o)
    szo.szo_zo_step([d.desc(with_y=False)], seed, step, eps, 1e-4, scal, ws, szo.STEP_FUSED_LOSS)
    r = ozo.zo_step([om], seed, step, eps, 1e-4)
    lp, lm, g = scal.cpu().numpy()
    sg = sigma_g([o])
    assert abs(lp - r["loss_plus"]) <= 5e-3 * r["loss_plus"] and abs(g - r["g"]) <= 1e-2 * max(abs(r["g"]), sg)
    bound = UpdateBound(sg, 1e-4)
    bound.add(r)
    bound.check(0, d.sp_val.cpu().numpy(), om.sp_val, o.sp_val)


def _dual_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        group = int(rng.choice([32, 64]))
        K = int(rng.choice([64, 192, 320, 448]))             # not a multiple of 128: never the few-token path
        M = int(rng.choice([1, 17, 100, 255, 256, 257, 300, 520, 700]))
        N = int(rng.choice([1, 5, 63, 64, 65, 127, 128, 129, 130, 255, 256, 257, 300, 511, 640]))
        dens = float(rng.choice([0.0, 1e-3, 1e-2, 5e-2]))
        kind = "heavy_tail" if (N >= 100 and dens <= 1e-2 and rng.random() < 0.5) else "uniform"
        dt = "bf16" if rng.random() < 0.25 else "f16"
        fmt = "lut" if (dt == "f16" and rng.random() < 0.35) else "uniform"
        out.append((3000 + i, M, N, K, group, dens, kind, dt, fmt))
    return out


@pytest.mark.parametrize("case", _dual_cases(32, 777), ids=lambda c: "-".join(str(v) for v in c[1:]))
def test_random_case_dual_sign_tiles(case):
    """Tile configuration 6 runs even a one-matrix step as the grouped launch with dual-sign tiles (both
    forwards of a 256 x 128 tile in one workgroup): one fused step per case against the oracle."""
    s, M, N, K, G, dens, kind, dtname, fmt = case
    dt = szo.TILE_BF16 if dtname == "bf16" else szo.TILE_F16
    o, d = make_pair(s, M, N, K, G, dens, kind=kind, nnz_base=4 * (s % 5), fmt=fmt)
    szo.szo_set_tile_config(6)
    seed, step, eps, lr = 11 + s, s % 3, 1e-3, 1e-3
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    om = clone(o)
    szo.szo_kernel_timing(True)
    szo.szo_zo_step([d.desc(dt, with_y=False)], seed, step, eps, lr, scal, ws, szo.STEP_FUSED_LOSS)
    _, launches = szo.szo_kernel_timing_read()
    szo.szo_kernel_timing(False)
    assert launches == 1
    lp, lm, g = scal.cpu().numpy()
    r = ozo.zo_step([om], seed, step, eps, lr)
    # every output carries an independent rounding error of ~1e-4 of its size (16-bit tile), which averages
    # down over the M N outputs of the mean
    ltol, gtol = (max(1e-5, 2e-3 / np.sqrt(M * N)), 1e-2) if dtname == "f16" else (5e-3, 1e-1)
    # relative to the loss's natural size (targets are N(0,1)): a 1 x 1 output can land next to its target
    assert abs(lp - r["loss_plus"]) <= ltol * max(r["loss_plus"], 1.0) and abs(lm - r["loss_minus"]) <= ltol * max(r["loss_minus"], 1.0)
    sg = sigma_g([o])
    assert abs(g - r["g"]) <= gtol * max(abs(r["g"]), sg), (g, r["g"], sg)
    if o.sp_idx.size:
        bound = UpdateBound(sg, lr)
        bound.add(r, extra_dg=(gtol - 1e-2) * max(abs(r["g"]), sg))
        bound.check(0, d.sp_val.cpu().numpy(), om.sp_val, o.sp_val)
