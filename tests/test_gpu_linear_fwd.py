"""GPU parity of the fused forward against the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import layer as olayer, philox as ophilox
from paper_2406_02913_amd import szo
from helpers import make_pair, rel_fro

pytestmark = pytest.mark.gpu

# (seed, M, N, K, group, density): tiny config, several tiles, ragged M and N, dense-ish masks
SHAPES = [
    (1, 64, 256, 256, 32, 1e-3),        # the tiny single-layer configuration
    (2, 100, 200, 320, 64, 1e-2),       # ragged M and N
    (3, 300, 384, 1024, 128, 1e-3),     # several tiles each way
    (4, 1, 128, 128, 128, 5e-2),        # a single token, dense mask
    (5, 257, 130, 192, 32, 0.0),        # k = 0: plain dequantise-then-matmul
    (6, 129, 513, 512, 128, 2e-2),      # one row past a tile boundary in both
    (7, 70, 192, 4160, 64, 1e-1),       # 65 column tiles (tile_ptr reload) and > 256 entries per tile
]
DTYPES = [(szo.TILE_F16, "f16", 2e-5), (szo.TILE_BF16, "bf16", 2e-5)]


def _run(d, sign, eps, seed, step, dt):
    d.y.fill_(float("nan"))
    szo.szo_linear_fwd(d.desc(dt), seed, step, sign, eps)
    torch.cuda.synchronize()
    return d.y.cpu().numpy()


@pytest.fixture(autouse=True)
def _auto_tile_config():
    yield
    szo.szo_set_tile_config(0)


@pytest.mark.parametrize("tile_cfg", [1, 2])
@pytest.mark.parametrize("dt,dtname,tol_d", DTYPES)
@pytest.mark.parametrize("shape", SHAPES)
def test_forward_matches_oracle(shape, dt, dtname, tol_d, tile_cfg):
    szo.szo_set_tile_config(tile_cfg)
    s, M, N, K, G, dens = shape
    o, d = make_pair(s, M, N, K, G, dens, nnz_base=8)
    seed, step, eps = 1234, 3, 1e-3
    z = ophilox.zbar(seed, step, 8, o.sp_idx.size)
    for sign in (+1, -1, 0):
        y = _run(d, sign, eps, seed, step, dt)
        assert np.isfinite(y).all()
        yD = olayer.linear_fwd(o.x_bits, o.codes, o.scales, G, o.sp_idx, o.sp_val, z, sign, eps, "D", dtname)
        yE = olayer.linear_fwd(o.x_bits, o.codes, o.scales, G, o.sp_idx, o.sp_val, z, sign, eps, "E")
        assert rel_fro(y, yD) <= tol_d, (sign, rel_fro(y, yD))
        assert rel_fro(y, yE) <= 5e-3, (sign, rel_fro(y, yE))
        # element-wise: fp32 accumulation of exact products over K terms
        scale = np.sqrt(K) * 0.02 * 4
        assert np.max(np.abs(y - yD)) <= 1e-4 * scale + 1e-6


def test_perturbation_difference_is_linear_in_z():
    # y(+) - y(-) = 2 eps x Z^T: checks the sign convention and that only masked entries move
    o, d = make_pair(7, 96, 256, 256, 32, 5e-3)
    seed, step, eps = 5, 1, 1e-2
    z = ophilox.zbar(seed, step, 0, o.sp_idx.size)
    yp = _run(d, +1, eps, seed, step, szo.TILE_F16).astype(np.float64)
    ym = _run(d, -1, eps, seed, step, szo.TILE_F16).astype(np.float64)
    from oracle.quant import bf16_bits_to_f64
    x = bf16_bits_to_f64(o.x_bits)
    Z = np.zeros((256, 256))
    Z.reshape(-1)[o.sp_idx.astype(np.int64)] = z
    want = 2 * float(np.float32(eps)) * x @ Z.T
    assert rel_fro(yp - ym, want) < 2e-2


def test_forward_is_deterministic_and_leaves_inputs_untouched():
    o, d = make_pair(8, 128, 256, 512, 128, 1e-2)
    before = d.sp_val.clone()
    a = _run(d, +1, 1e-3, 1, 0, szo.TILE_F16)
    b = _run(d, +1, 1e-3, 1, 0, szo.TILE_F16)
    assert np.array_equal(a, b)
    assert torch.equal(before, d.sp_val)


@pytest.mark.parametrize("tile_cfg", [1, 2])
def test_fused_loss_equals_separate_loss(tile_cfg):
    szo.szo_set_tile_config(tile_cfg)
    o, d = make_pair(9, 200, 384, 512, 128, 1e-2)
    ws = szo.new_workspace()
    seed, step, eps = 2, 2, 1e-3
    for dt in (szo.TILE_F16, szo.TILE_BF16):
        y = _run(d, -1, eps, seed, step, dt)
        acc = torch.zeros(2, dtype=torch.float64, device="cuda")
        szo.szo_mse_loss(d.y, d.target, d.M * d.N, 1.0 / (d.M * d.N), acc[0:1], ws)
        d.y.fill_(0)
        szo.szo_linear_fwd_mse(d.desc(dt), seed, step, -1, eps, 1.0 / (d.M * d.N), acc[1:2], ws)
        torch.cuda.synchronize()
        assert np.array_equal(d.y.cpu().numpy(), y)                 # y still written when requested
        a = acc.cpu().numpy()
        # the fused epilogue squares in fp32 and adds 16-term fp32 partials in fp64: per-term relative
        # rounding 2^-24, random in sign, so the sum of ~77k terms agrees to far better than 1e-8
        assert abs(a[0] - a[1]) <= 1e-8 * abs(a[0])
        assert abs(a[0] - olayer.mse_loss(y.astype(np.float64), o.target_bits)) <= 1e-12 * abs(a[0])
        acc2 = torch.zeros(1, dtype=torch.float64, device="cuda")
        szo.szo_linear_fwd_mse(d.desc(dt, with_y=False), seed, step, -1, eps, 1.0 / (d.M * d.N), acc2, ws)
        assert acc2.item() == a[1]                                  # no y, same loss, bit for bit
