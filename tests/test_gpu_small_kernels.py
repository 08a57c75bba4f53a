"""GPU parity for the Gaussian, the loss, the SPSA scalar and the update."""
import numpy as np
import pytest
import torch

from oracle import philox as ophilox, layer as olayer, zo as ozo
from paper_2406_02913_amd import synth, szo

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("base,nnz,seed,step", [(0, 1000, 1, 0), (68, 4099, 0xDEADBEEFCAFEF00D, 7),
                                                  ((1 << 34) + 8, 513, 3, (1 << 40) + 5)])
def test_philox_words_bit_exact_and_gaussian_close(base, nnz, seed, step):
    words = torch.empty(nnz * 4, dtype=torch.int32, device=DEV)
    z = torch.empty(nnz, dtype=torch.float32, device=DEV)
    szo.szo_debug_zbar(base, nnz, seed, step, words, z)
    torch.cuda.synchronize()
    J = np.uint64(base) + np.arange(nnz, dtype=np.uint64)
    want_w = ophilox.zbar_words(seed, step, J)
    assert np.array_equal(words.cpu().numpy().view(np.uint32).reshape(nnz, 4), want_w)
    want_z = ophilox.zbar(seed, step, base, nnz)
    err = np.abs(z.cpu().numpy().astype(np.float64) - want_z)
    assert err.max() < 2e-6, err.max()


def test_gaussian_extremes_on_device():
    # hunt a few million entries for the tails: |z| stays finite and bounded
    n = 4_000_000
    z = torch.empty(n, dtype=torch.float32, device=DEV)
    szo.szo_debug_zbar(0, n, 99, 1, None, z)
    assert torch.isfinite(z).all() and z.abs().max().item() <= 5.77
    assert abs(z.mean().item()) < 4 / np.sqrt(n) and abs(z.var().item() - 1) < 4 * np.sqrt(2 / n)


@pytest.mark.parametrize("count,off", [(1, 0), (7, 0), (4096, 0), (100_003, 0), (5_000_001, 0), (1001, 1), (70_000, 3)])
def test_mse_loss_matches_oracle_and_is_deterministic(count, off):
    rng = np.random.default_rng(count)
    y = rng.standard_normal(count + off).astype(np.float32)
    t = synth.to_bf16_bits(rng.standard_normal(count + off).astype(np.float32))
    yd = torch.from_numpy(y).to(DEV)[off:]
    td = torch.from_numpy(t.view(np.int16)).view(torch.bfloat16).to(DEV)[off:]
    ws = szo.new_workspace()
    acc = torch.full((1,), 0.5, dtype=torch.float64, device=DEV)
    scale = 1.0 / count
    szo.szo_mse_loss(yd, td, count, scale, acc, ws)
    szo.szo_mse_loss(yd, td, count, scale, acc, ws)        # accumulates; workspace returns to idle
    got = acc.item()
    want = 0.5 + 2 * olayer.mse_loss(y[off:].astype(np.float64), t[off:])
    assert abs(got - want) <= 1e-12 * max(1.0, abs(want))
    acc2 = torch.full((1,), 0.5, dtype=torch.float64, device=DEV)
    szo.szo_mse_loss(yd, td, count, scale, acc2, ws)
    szo.szo_mse_loss(yd, td, count, scale, acc2, ws)
    assert acc2.item() == got                               # bit-reproducible


def test_mse_zero_count_adds_nothing():
    ws = szo.new_workspace()
    acc = torch.full((1,), 1.25, dtype=torch.float64, device=DEV)
    szo.szo_mse_loss(None, None, 0, 1.0, acc, ws)
    assert acc.item() == 1.25


def test_spsa_scalar():
    lp = torch.tensor([2.5000001], dtype=torch.float64, device=DEV)
    lm = torch.tensor([2.4999999], dtype=torch.float64, device=DEV)
    g = torch.zeros(1, dtype=torch.float64, device=DEV)
    szo.szo_spsa_g(lp, lm, 1e-3, g)
    assert abs(g.item() - ozo.spsa_scalar(2.5000001, 2.4999999, 1e-3)) < 1e-12
    szo.szo_spsa_g(lp, lm, 0.0, g)
    assert g.item() == 0.0


@pytest.mark.parametrize("nnz,base", [(1, 0), (66, 0), (16777, 68), (45089, 16848), (3, 1 << 33)])
def test_sparse_update_matches_oracle(nnz, base):
    rng = np.random.default_rng(nnz)
    v0 = (0.02 * rng.standard_normal(nnz)).astype(np.float32)
    pad = torch.zeros(nnz + 8, dtype=torch.float32, device=DEV)
    pad[:nnz] = torch.from_numpy(v0)
    gval, lr, seed, step = -3.75, 1e-3, 11, 5
    g = torch.tensor([gval], dtype=torch.float64, device=DEV)
    szo.szo_sparse_update(pad, None, nnz, base, seed, step, g, lr)
    got = pad.cpu().numpy()
    z = ophilox.zbar(seed, step, base, nnz)
    want = (v0.astype(np.float64) - float(np.float32(lr)) * gval * z)
    delta_got = got[:nnz].astype(np.float64) - v0
    delta_want = want - v0
    assert np.all(got[nnz:] == 0)                                   # nothing past the end
    assert np.max(np.abs(got[:nnz] - want)) <= 2 * np.spacing(np.float32(0.1))
    assert np.linalg.norm(delta_got - delta_want) <= 1e-4 * np.linalg.norm(delta_want)


def test_update_and_forward_share_the_gaussian():
    # the update applied with g = 1, lr = -1 adds exactly z: compare with the debug kernel's z
    nnz, base = 1000, 24
    v = torch.zeros(nnz, dtype=torch.float32, device=DEV)
    g = torch.tensor([1.0], dtype=torch.float64, device=DEV)
    szo.szo_sparse_update(v, None, nnz, base, 5, 9, g, -1.0)
    z = torch.empty(nnz, dtype=torch.float32, device=DEV)
    szo.szo_debug_zbar(base, nnz, 5, 9, None, z)
    assert torch.equal(v, z)


def test_activation_absmax_and_the_fp16_tiles_saturation():
    """The fp16 tile truncates bf16 activations to fp16: beyond the largest finite fp16 they saturate at
    +-65504 (documented in the header).  szo_activation_absmax measures the range on the device and
    szo_choose_tile_dtype turns it into the tile type; the bf16 tile takes the same activations as they are."""
    from oracle import layer as olayer
    from oracle.quant import f32_to_bf16_bits
    from helpers import make_pair, rel_fro
    o, d = make_pair(151, 32, 256, 256, 128, 2e-3)
    out = torch.zeros(1, dtype=torch.float32, device="cuda")
    szo.szo_activation_absmax(d.x, d.M * d.K, out)
    xf = (o.x_bits.astype(np.uint32) << 16).view(np.float32)
    assert out.item() == float(np.abs(xf).max())
    assert szo.szo_choose_tile_dtype(out.item()) == szo.TILE_F16
    szo.szo_activation_absmax(d.x, 0, out)
    assert out.item() == 0.0
    # plant two outliers: 1e5 and -3e38 (both finite in bf16, both beyond fp16)
    xb = o.x_bits.copy()
    big = f32_to_bf16_bits(np.array([1.0e5, -3.0e38], dtype=np.float32))
    xb[3, 17], xb[20, 200] = big[0], big[1]
    d.x = torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).cuda()
    szo.szo_activation_absmax(d.x, d.M * d.K, out)
    assert out.item() == float(np.abs((big.astype(np.uint32) << 16).view(np.float32)).max())
    assert szo.szo_choose_tile_dtype(out.item()) == szo.TILE_BF16
    szo.szo_set_tile_config(2)                                     # the tiled kernel, both tile types
    # fp16 tile: the result is that of activations clamped to +-65504
    clamped = np.clip((xb.astype(np.uint32) << 16).view(np.float32), -65504.0, 65504.0)
    y_ref16 = clamped.astype(np.float64) @ olayer.effective_weight(o.codes, o.scales, o.group, o.sp_idx, o.sp_val).T
    szo.szo_linear_fwd(d.desc(szo.TILE_F16), 1, 0, 0, 0.0)
    y16 = d.y.cpu().numpy()
    assert np.isfinite(y16).all() and rel_fro(y16, y_ref16) <= 5e-3
    # bf16 tile: the activations as they are
    y_ref = olayer.linear_fwd(xb, o.codes, o.scales, o.group, o.sp_idx, o.sp_val)
    szo.szo_linear_fwd(d.desc(szo.TILE_BF16), 1, 0, 0, 0.0)
    ybf = d.y.cpu().numpy()
    assert np.isfinite(ybf).all() and rel_fro(ybf, y_ref) <= 1e-2
    szo.szo_set_tile_config(0)
    # NaN in, NaN out of the range scan
    xb[0, 0] = 0x7FC0
    szo.szo_activation_absmax(torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).cuda(), d.M * d.K, out)
    assert np.isnan(out.item())
