"""GPU parity of the few-token path (slices of 16, 32 or 48 token rows): dense product once, sparse
product per sign (the SparseAddMM association of Appendix C.5)."""
import numpy as np
import pytest
import torch

from oracle import layer as olayer, philox as ophilox, zo as ozo
from paper_2406_02913_amd import szo
from helpers import make_pair, clone, rel_fro, sigma_g, UpdateBound

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto_tile_config():
    yield
    szo.szo_set_tile_config(0)

# (seed, M, N, K, group, density)
SHAPES = [
    (11, 16, 256, 128, 128, 1e-2),      # one strip, one 128-column block (half a chunk: plain instantiation)
    (12, 16, 512, 1152, 128, 1e-3),     # 4.5 chunks of 256 columns: plain instantiation with a ragged last chunk
    (13, 1, 200, 256, 128, 5e-2),       # one token, ragged N, > 256 entries per band and chunk (several refills)
    (14, 7, 513, 2048, 128, 2e-3),      # ragged M and N, eight chunks
    (19, 16, 128, 1024, 128, 8e-2),     # ~1300 entries per band and chunk: the entry ring wraps inside a chunk
    (20, 3, 64, 4864, 128, 3e-3),       # 19 chunks, one band
    (21, 40, 320, 512, 128, 5e-3),      # 17..64 tokens: three passes of 16 token rows, the last one ragged
    (22, 64, 256, 384, 64, 1e-2),       # four passes, plain instantiation
    (15, 16, 320, 256, 32, 1e-2),       # group 32: scale applied per element
    (16, 9, 128, 384, 64, 2e-2),        # group 64
    (17, 16, 256, 256, 128, 0.0),       # k = 0
    (18, 16, 4096, 4096, 128, 1e-3),    # a full-size attention projection at 16 tokens
]


# configurations 4 and 5: 32 / 48 token rows per pass wherever there are more than 16 (otherwise only in large launches);
# configuration 7: the codes as a non-temporal stream (otherwise only in launches beyond the last-level cache)
@pytest.mark.parametrize("shape,cfg", [(sh, 0) for sh in SHAPES] + [(sh, c) for sh in SHAPES if sh[1] > 16 for c in (4, 5)] + [(sh, 7) for sh in SHAPES if sh[1] <= 16])
def test_few_token_forward_matches_oracle(shape, cfg):
    s, M, N, K, G, dens = shape
    szo.szo_set_tile_config(cfg)
    o, d = make_pair(s, M, N, K, G, dens, nnz_base=12)
    seed, step, eps = 77, 5, 1e-3
    z = ophilox.zbar(seed, step, 12, o.sp_idx.size)
    # fp32 accumulation of un-centred codes (|constant part| ~ 1e3 x the signal's terms) and fp16 sparse
    # values: a few 1e-4; the bar for y is 5e-3
    tol = 5e-4 if G == 128 else 1e-3
    for sign in (+1, -1, 0):
        d.y.fill_(float("nan"))
        szo.szo_linear_fwd(d.desc(), seed, step, sign, eps)
        torch.cuda.synchronize()
        y = d.y.cpu().numpy()
        assert np.isfinite(y).all()
        yE = olayer.linear_fwd(o.x_bits, o.codes, o.scales, G, o.sp_idx, o.sp_val, z, sign, eps, "E")
        assert rel_fro(y, yE) <= tol, (sign, rel_fro(y, yE))


def test_few_token_counters_seed_and_step_beyond_32_bits():
    """y(+) - y(-) = 2 eps x z^T isolates the regenerated Gaussians: entry index, seed and step all use
    their high words."""
    szo.szo_set_tile_config(0)
    base, seed, step, eps = (1 << 35) + 8, (1 << 40) + 77, (1 << 33) + 5, 0.05
    o, d = make_pair(23, 16, 192, 512, 128, 2e-2, nnz_base=base)
    z = ophilox.zbar(seed, step, base, o.sp_idx.size)
    ys = {}
    for sign in (+1, -1):
        szo.szo_linear_fwd(d.desc(), seed, step, sign, eps)
        ys[sign] = d.y.cpu().numpy().astype(np.float64)
    yp = olayer.linear_fwd(o.x_bits, o.codes, o.scales, 128, o.sp_idx, o.sp_val, z, +1, eps, "E")
    ym = olayer.linear_fwd(o.x_bits, o.codes, o.scales, 128, o.sp_idx, o.sp_val, z, -1, eps, "E")
    # z is held in fp16 (5e-4 relative) and the difference of two fp32 outputs carries their rounding
    assert rel_fro(ys[+1] - ys[-1], yp - ym) <= 3e-3
    # the same entries with the low words only give different Gaussians: the check can tell
    z_low = ophilox.zbar(77, 5, 8, o.sp_idx.size)
    assert np.abs(z - z_low).max() > 1.0


def test_few_token_path_agrees_with_the_tiled_kernel():
    o, d = make_pair(21, 16, 384, 512, 128, 1e-2)
    szo.szo_set_tile_config(0)
    szo.szo_linear_fwd(d.desc(), 3, 1, -1, 1e-3)
    a = d.y.cpu().numpy().copy()
    szo.szo_set_tile_config(1)
    szo.szo_linear_fwd(d.desc(), 3, 1, -1, 1e-3)
    b = d.y.cpu().numpy().copy()
    szo.szo_set_tile_config(0)
    assert rel_fro(a, b) < 1e-3 and not np.array_equal(a, b)      # two different kernels, same answer


def test_few_token_fused_loss_and_step():
    szo.szo_set_tile_config(0)
    o1, d1 = make_pair(31, 16, 512, 1152, 128, 2e-3, nnz_base=0)
    base2 = (o1.sp_idx.size + 3) // 4 * 4
    o2, d2 = make_pair(32, 16, 200, 256, 128, 1e-2, nnz_base=base2)
    ws = szo.new_workspace()
    # single-matrix fused loss, each sign
    for sign in (+1, -1):
        acc = torch.zeros(1, dtype=torch.float64, device="cuda")
        szo.szo_linear_fwd_mse(d1.desc(with_y=False), 9, 2, sign, 1e-3, 1.0 / (d1.M * d1.N), acc, ws)
        z = ophilox.zbar(9, 2, 0, o1.sp_idx.size)
        yE = olayer.linear_fwd(o1.x_bits, o1.codes, o1.scales, 128, o1.sp_idx, o1.sp_val, z, sign, 1e-3, "E")
        want = olayer.mse_loss(yE, o1.target_bits)
        assert abs(acc.item() - want) <= 1e-4 * want
    # single-matrix fused loss with more than 16 tokens: the partials of all 16-row passes add up
    o3, d3 = make_pair(33, 48, 384, 512, 128, 4e-3, nnz_base=64)
    acc = torch.zeros(1, dtype=torch.float64, device="cuda")
    szo.szo_linear_fwd_mse(d3.desc(with_y=False), 9, 2, -1, 1e-3, 1.0 / (d3.M * d3.N), acc, ws)
    z = ophilox.zbar(9, 2, 64, o3.sp_idx.size)
    yE = olayer.linear_fwd(o3.x_bits, o3.codes, o3.scales, 128, o3.sp_idx, o3.sp_val, z, -1, 1e-3, "E")
    want = olayer.mse_loss(yE, o3.target_bits)
    assert abs(acc.item() - want) <= 1e-4 * want
    # whole steps over two matrices
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    a, b = clone(o1), clone(o2)
    sg = sigma_g([o1, o2])
    descs = szo.desc_array([d1.desc(with_y=False), d2.desc(with_y=False)])
    bound = UpdateBound(sg, 1e-3)
    for s in range(4):
        szo.szo_zo_step(descs, 5, s, 1e-3, 1e-3, scal, ws, szo.STEP_FUSED_LOSS)
        lp, lm, g = scal.cpu().numpy()
        r = ozo.zo_step([a, b], 5, s, 1e-3, 1e-3)
        bound.add(r)
        assert abs(lp - r["loss_plus"]) <= 1e-4 * r["loss_plus"]
        assert abs(lm - r["loss_minus"]) <= 1e-4 * r["loss_minus"]
        assert abs(g - r["g"]) <= 1e-2 * max(abs(r["g"]), sg), (s, g, r["g"], sg)
    for i, (om, dd, o) in enumerate(((a, d1, o1), (b, d2, o2))):
        bound.check(i, dd.sp_val.cpu().numpy(), om.sp_val, o.sp_val)


def test_few_token_step_is_bit_reproducible():
    szo.szo_set_tile_config(0)
    outs = []
    for _ in range(2):
        _, d = make_pair(41, 16, 512, 1024, 128, 5e-3)
        ws = szo.new_workspace()
        scal = torch.zeros(3, dtype=torch.float64, device="cuda")
        for s in range(3):
            szo.szo_zo_step([d.desc(with_y=False)], 8, s, 1e-3, 1e-3, scal, ws, szo.STEP_FUSED_LOSS)
        outs.append((scal.cpu().numpy().copy(), d.sp_val.cpu().numpy().copy()))
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])


def test_non_temporal_code_stream_changes_no_bit():
    """Large one-slice launches load their codes with the non-temporal hint (a cache policy, not arithmetic);
    configuration 7 takes that instantiation at any size.  A step over three matrices (group 128, group 64,
    table format aside) must give the same scalars and the same updated values bit for bit either way."""
    outs = []
    for cfg in (0, 7):
        szo.szo_set_tile_config(cfg)
        ds_, base = [], 0
        for (sd, M, N, K, G, dens) in [(51, 16, 512, 1024, 128, 5e-3), (52, 9, 320, 768, 64, 1e-2), (53, 1, 200, 256, 128, 2e-2)]:
            o, d = make_pair(sd, M, N, K, G, dens, nnz_base=base)
            base += (o.sp_idx.size + 3) // 4 * 4
            ds_.append(d)
        ws = szo.new_workspace()
        scal = torch.zeros(3, dtype=torch.float64, device="cuda")
        descs = szo.desc_array([d.desc(with_y=False) for d in ds_])
        hist = []
        for s in range(3):
            szo.szo_zo_step(descs, 8, s, 1e-3, 1e-3, scal, ws, szo.STEP_FUSED_LOSS)
            hist.append(scal.cpu().numpy().copy())
        outs.append((np.array(hist), [d.sp_val.cpu().numpy().copy() for d in ds_]))
    szo.szo_set_tile_config(0)
    assert np.array_equal(outs[0][0], outs[1][0])
    assert all(np.array_equal(a, b) for a, b in zip(outs[0][1], outs[1][1]))


@pytest.mark.parametrize("cfg", [0, 7])
def test_one_full_size_block_at_16_tokens_two_steps(cfg):
    """The seven matrices of one Llama-2-7B block at their real sizes, in the grouped launch
    bench.py times (one forward launch, one update launch per step).  A whole stack streams more codes
    than the last-level cache holds and therefore runs the instantiation with the non-temporal code
    stream; configuration 7 selects it for this one block as well."""
    from paper_2406_02913_amd import synth
    szo.szo_set_tile_config(cfg)
    cfg = synth.WORKLOADS["c3m16"]
    os_, ds_, base = [], [], 0
    for i, (name, N, K) in enumerate(cfg["block"]):
        k = int(np.floor(cfg["density"] * N * K + 0.5))
        o, d = make_pair(100 + i, cfg["M"], N, K, cfg["group"], cfg["density"], kind=cfg["mask"], nnz=k, nnz_base=base)
        base += (k + 3) // 4 * 4
        os_.append(o)
        ds_.append(d)
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    descs = szo.desc_array([d.desc(with_y=False) for d in ds_])
    ref = [clone(o) for o in os_]
    sg = sigma_g(os_)
    lr = 1e-4
    bound = UpdateBound(sg, lr)
    for s in range(2):
        szo.szo_zo_step(descs, 17, s, cfg["eps"], lr, scal, ws, szo.STEP_FUSED_LOSS)
        lp, lm, g = scal.cpu().numpy()
        r = ozo.zo_step(ref, 17, s, cfg["eps"], lr)
        bound.add(r)
        assert abs(lp - r["loss_plus"]) <= 1e-4 * r["loss_plus"]
        assert abs(lm - r["loss_minus"]) <= 1e-4 * r["loss_minus"]
        assert abs(g - r["g"]) <= 1e-2 * max(abs(r["g"]), sg), (s, g, r["g"], sg)
    for i, (om, dd, o) in enumerate(zip(ref, ds_, os_)):
        bound.check(i, dd.sp_val.cpu().numpy(), om.sp_val, o.sp_val)


@pytest.mark.parametrize("cfg", [0, 4, 5])
def test_step_with_up_to_64_tokens_runs_as_slices(cfg):
    """17..64 tokens: the step streams the weights once per slice of 16 token rows, or of 32 / 48 in
    launches that are large (configurations 4 / 5 force that); matrices of different token counts may
    share a step, and the sparse values are updated exactly once."""
    szo.szo_set_tile_config(cfg)
    o1, d1 = make_pair(51, 64, 320, 512, 128, 2e-3, nnz_base=0)
    b2 = (o1.sp_idx.size + 3) // 4 * 4
    o2, d2 = make_pair(52, 40, 256, 384, 64, 5e-3, nnz_base=b2)          # ragged last slice, plain instantiation
    b3 = b2 + (o2.sp_idx.size + 3) // 4 * 4
    o3, d3 = make_pair(53, 16, 128, 256, 128, 1e-2, nnz_base=b3)
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    os_, ds_ = [o1, o2, o3], [d1, d2, d3]
    ref = [clone(o) for o in os_]
    sg = sigma_g(os_)
    descs = szo.desc_array([d.desc(with_y=False) for d in ds_])
    szo.szo_kernel_timing(True)
    bound = UpdateBound(sg, 1e-3)
    for s in range(3):
        szo.szo_zo_step(descs, 23, s, 1e-3, 1e-3, scal, ws, szo.STEP_FUSED_LOSS)
        lp, lm, g = scal.cpu().numpy()
        r = ozo.zo_step(ref, 23, s, 1e-3, 1e-3)
        bound.add(r)
        assert abs(lp - r["loss_plus"]) <= 1e-4 * r["loss_plus"]
        assert abs(lm - r["loss_minus"]) <= 1e-4 * r["loss_minus"]
        assert abs(g - r["g"]) <= 1e-2 * max(abs(r["g"]), sg), (s, g, r["g"], sg)
    _, launches = szo.szo_kernel_timing_read()
    szo.szo_kernel_timing(False)
    # few-token path: one launch per instantiation and step: group 128 and group 64 with 16 rows per pass,
    # or group 128 x 32 rows, group 64 x 32 rows and group 128 x 16 rows
    assert launches == (6 if cfg == 0 else 9)
    for i, (om, dd, o) in enumerate(zip(ref, ds_, os_)):
        bound.check(i, dd.sp_val.cpu().numpy(), om.sp_val, o.sp_val)
