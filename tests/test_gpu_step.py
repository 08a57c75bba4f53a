"""GPU parity of whole ZO steps (two forwards, losses, g, update)."""
import numpy as np
import pytest
import torch

from oracle import zo as ozo
from paper_2406_02913_amd import szo
from helpers import make_pair, clone, sigma_g, UpdateBound

pytestmark = pytest.mark.gpu


def _gpu_steps(devs, steps, seed, eps, lr, flags, dt=szo.TILE_F16, first=0):
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    out = []
    descs = szo.desc_array([d.desc(dt) for d in devs])
    for s in range(first, first + steps):
        szo.szo_zo_step(descs, seed, s, eps, lr, scal, ws, flags)
        out.append(scal.cpu().numpy().copy())
    return out


@pytest.fixture(autouse=True)
def _auto_tile_config():
    yield
    szo.szo_set_tile_config(0)


@pytest.mark.parametrize("tile_cfg", [0, 2])
@pytest.mark.parametrize("flags", [0, szo.STEP_FUSED_LOSS])
def test_tiny_configuration_ten_steps(flags, tile_cfg):
    szo.szo_set_tile_config(tile_cfg)
    # 64 tokens, 256x256, group 32, 66 sensitive entries, eps 1e-3, lr 1e-6, 10 steps
    o, d = make_pair(1, 64, 256, 256, 32, 1e-3)
    assert o.sp_idx.size == 66
    seed, eps, lr = 42, 1e-3, 1e-6
    got = _gpu_steps([d], 10, seed, eps, lr, flags)
    om = clone(o)
    sg = sigma_g([o])
    for s in range(10):
        r = ozo.zo_step([om], seed, s, eps, lr)
        lp, lm, g = got[s]
        assert abs(lp - r["loss_plus"]) <= 5e-3 * r["loss_plus"]
        assert abs(lm - r["loss_minus"]) <= 5e-3 * r["loss_minus"]
        assert abs(g - r["g"]) <= 1e-2 * max(abs(r["g"]), sg), (s, g, r["g"], sg)
    v = d.sp_val.cpu().numpy()
    # ten updates of ~1e-8 each on fp32 values of ~1e-2: allow the accumulated update 1% plus two ulps
    assert np.all(np.abs(v - om.sp_val) <= 1e-2 * np.abs(om.sp_val - o.sp_val) + 2 * np.spacing(np.abs(om.sp_val)))
    assert np.allclose(v, om.sp_val, rtol=1e-2, atol=0)


def test_larger_lr_update_direction_and_size():
    # with a visible step size the update itself is compared, not just the values
    o, d = make_pair(2, 96, 256, 320, 64, 5e-3)
    seed, eps, lr = 7, 1e-3, 1e-2
    _gpu_steps([d], 1, seed, eps, lr, 0)
    om = clone(o)
    r = ozo.zo_step([om], seed, 0, eps, lr)
    dv_gpu = d.sp_val.cpu().numpy().astype(np.float64) - o.sp_val
    dv_ref = om.sp_val.astype(np.float64) - o.sp_val
    sg = sigma_g([o])
    tol = 1e-2 * max(abs(r["g"]), sg) / max(abs(r["g"]), 1e-300)
    assert np.linalg.norm(dv_gpu - dv_ref) <= tol * np.linalg.norm(dv_ref) + 1e-9


def test_two_matrices_share_one_g_and_distinct_counters():
    o1, d1 = make_pair(3, 80, 128, 256, 32, 1e-2, nnz_base=0)
    base2 = (o1.sp_idx.size + 3) // 4 * 4
    o2, d2 = make_pair(4, 80, 256, 128, 64, 1e-2, nnz_base=base2)
    seed, eps, lr = 9, 1e-3, 1e-3
    got = _gpu_steps([d1, d2], 3, seed, eps, lr, szo.STEP_FUSED_LOSS)
    a, b = clone(o1), clone(o2)
    sg = sigma_g([o1, o2])
    bound = UpdateBound(sg, lr)
    for s in range(3):
        r = ozo.zo_step([a, b], seed, s, eps, lr)
        bound.add(r)
        assert abs(got[s][2] - r["g"]) <= 1e-2 * max(abs(r["g"]), sg)
    for i, (om, dd, o) in enumerate(((a, d1, o1), (b, d2, o2))):
        bound.check(i, dd.sp_val.cpu().numpy(), om.sp_val, o.sp_val)


def test_eps_zero_is_a_no_op():
    o, d = make_pair(5, 64, 128, 128, 32, 1e-2)
    before = d.sp_val.clone()
    got = _gpu_steps([d], 1, 1, 0.0, 1e-2, 0)
    assert got[0][2] == 0.0 and got[0][0] == got[0][1]
    assert torch.equal(before, d.sp_val)


def test_steps_are_bit_reproducible_and_resumable():
    o, da = make_pair(6, 64, 256, 256, 32, 5e-3)
    _, db = make_pair(6, 64, 256, 256, 32, 5e-3)
    ga = _gpu_steps([da], 6, 3, 1e-3, 1e-3, szo.STEP_FUSED_LOSS)
    gb = _gpu_steps([db], 3, 3, 1e-3, 1e-3, szo.STEP_FUSED_LOSS)
    saved = db.sp_val.cpu()
    _, dc = make_pair(6, 64, 256, 256, 32, 5e-3)
    dc.sp_val.copy_(saved)
    gc = _gpu_steps([dc], 3, 3, 1e-3, 1e-3, szo.STEP_FUSED_LOSS, first=3)
    assert all(np.array_equal(x, y) for x, y in zip(ga, gb + gc))
    assert torch.equal(da.sp_val, dc.sp_val)


def test_bf16_tile_is_available_and_less_accurate_on_g():
    # the 8-bit significand cannot hold w + eps*z to the estimator's budget; the fp16 tile can
    o, d16 = make_pair(1, 64, 256, 256, 32, 1e-3)
    _, dbf = make_pair(1, 64, 256, 256, 32, 1e-3)
    sg = sigma_g([o])
    e16, ebf = [], []
    for s in range(8):
        r = ozo.zo_step([clone(o)], 42, s, 1e-3, 0.0)
        g16 = _gpu_steps([d16], 1, 42, 1e-3, 0.0, 0, szo.TILE_F16, first=s)[0][2]
        gbf = _gpu_steps([dbf], 1, 42, 1e-3, 0.0, 0, szo.TILE_BF16, first=s)[0][2]
        e16.append(abs(g16 - r["g"]) / max(abs(r["g"]), sg))
        ebf.append(abs(gbf - r["g"]) / max(abs(r["g"]), sg))
    print("g error fp16 tile:", e16, "bf16 tile:", ebf)
    assert max(e16) <= 1e-2
    assert np.mean(ebf) > np.mean(e16)


def test_kernel_timing_counts_forward_launches_only():
    _, d = make_pair(3, 256, 256, 256, 32, 1e-3)        # a full row of 256-row tiles: the tiled path
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    szo.szo_set_tile_config(0)
    szo.szo_kernel_timing(True)
    for s in range(3):
        szo.szo_zo_step([d.desc(with_y=False)], 1, s, 1e-3, 1e-6, scal, ws, szo.STEP_FUSED_LOSS)
    ms, n = szo.szo_kernel_timing_read()
    szo.szo_kernel_timing(False)
    assert n == 6 and 0.0 < ms < 100.0          # two forwards per step on the tiled path
    szo.szo_zo_step([d.desc(with_y=False)], 1, 3, 1e-3, 1e-6, scal, ws, szo.STEP_FUSED_LOSS)
    assert szo.szo_kernel_timing_read() == (0.0, 0)


@pytest.mark.parametrize("dt", [szo.TILE_F16, szo.TILE_BF16])
def test_grouped_launch_of_a_step_equals_per_matrix_launches_bit_for_bit(dt):
    """Tile configuration 3 runs all forwards of a step (every matrix, both signs) as one grid driven
    by a descriptor table; configuration 2 launches them one by one.  Same tiles, same arithmetic,
    same order of the loss partials: identical scalars and identical updated values."""
    shapes = [(61, 300, 384, 1024, 128, 2e-3), (62, 257, 130, 192, 32, 0.0), (63, 129, 513, 512, 128, 2e-2),
              (64, 70, 192, 4160, 64, 1e-1)]
    results = []
    for cfg in (2, 3):
        szo.szo_set_tile_config(cfg)
        os_, ds_, base = [], [], 0
        for (sd, M, N, K, G, dens) in shapes:
            o, d = make_pair(sd, M, N, K, G, dens, nnz_base=base)
            base += (o.sp_idx.size + 3) // 4 * 4
            os_.append(o)
            ds_.append(d)
        ws = szo.new_workspace()
        scal = torch.zeros(3, dtype=torch.float64, device="cuda")
        descs = szo.desc_array([d.desc(dt, with_y=False) for d in ds_])
        hist = []
        szo.szo_kernel_timing(True)
        for s in range(3):
            szo.szo_zo_step(descs, 31, s, 1e-3, 1e-3, scal, ws, szo.STEP_FUSED_LOSS)
            hist.append(scal.cpu().numpy().copy())
        _, launches = szo.szo_kernel_timing_read()
        szo.szo_kernel_timing(False)
        assert launches == (3 if cfg == 3 else 3 * 2 * len(shapes))
        results.append((hist, [d.sp_val.cpu().numpy().copy() for d in ds_]))
        if cfg == 3:        # and both agree with the oracle
            ref = [clone(o) for o in os_]
            sg = sigma_g(os_)
            for s in range(3):
                r = ozo.zo_step(ref, 31, s, 1e-3, 1e-3)
                lp, lm, g = hist[s]
                assert abs(lp - r["loss_plus"]) <= (1e-6 if dt == szo.TILE_F16 else 1e-4) * r["loss_plus"]
                assert abs(g - r["g"]) <= (1e-2 if dt == szo.TILE_F16 else 1e-1) * max(abs(r["g"]), sg)
    szo.szo_set_tile_config(0)
    (h2, v2), (h3, v3) = results
    for a, b in zip(h2, h3):
        assert np.array_equal(a, b)
    for a, b in zip(v2, v3):
        assert np.array_equal(a, b)


def test_steps_on_a_side_stream_match_the_default_stream():
    outs = []
    for use_side in (False, True):
        szo.szo_set_tile_config(3)
        _, d = make_pair(71, 130, 320, 384, 64, 5e-3)
        ws = szo.new_workspace()
        scal = torch.zeros(3, dtype=torch.float64, device="cuda")
        torch.cuda.synchronize()
        st = torch.cuda.Stream() if use_side else torch.cuda.current_stream()
        for s in range(6):                       # more calls than staging buffers
            szo.szo_zo_step([d.desc(with_y=False)], 5, s, 1e-3, 1e-3, scal, ws, szo.STEP_FUSED_LOSS, st.cuda_stream)
        st.synchronize()
        outs.append((scal.cpu().numpy().copy(), d.sp_val.cpu().numpy().copy()))
    szo.szo_set_tile_config(0)
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])


def test_more_matrices_than_one_descriptor_table_holds():
    # 4100 layers (the tables of the grouped launches hold 4096): the step falls back to one launch per
    # matrix for the forwards and for the updates and still forms one g over all of them
    o, d = make_pair(12, 32, 64, 64, 32, 2e-2)
    n = 4100
    descs, mats = [], []
    for i in range(n):
        dd = d.desc(with_y=False)
        dd.nnz_base = 128 * i
        descs.append(dd)
        om = clone(o)
        om.nnz_base = 128 * i
        mats.append(om)
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    before = d.sp_val.clone()
    szo.szo_zo_step(descs, 21, 0, 1e-3, 0.0, scal, ws, szo.STEP_FUSED_LOSS)      # lr = 0: the shared values stay
    lp, lm, g = scal.cpu().numpy()
    r = ozo.zo_step(mats, 21, 0, 1e-3, 0.0)
    assert abs(lp - r["loss_plus"]) <= 5e-3 * r["loss_plus"] and abs(lm - r["loss_minus"]) <= 5e-3 * r["loss_minus"]
    assert abs(g - r["g"]) <= 1e-2 * max(abs(r["g"]), sigma_g(mats[:1]) * np.sqrt(n))
    assert torch.equal(before, d.sp_val)


def test_grouped_launch_with_128_row_tiles_for_steps_of_at_most_128_tokens():
    """Up to 128 tokens where the few-token path does not apply (here: one K is not a multiple of 128): a
    256-row tile would be mostly padding, so with the library choosing, a step that is large enough runs
    as one grid of 128x128 tiles; it must equal the per-matrix launches of the same tiles (configuration 1)
    bit for bit, and the oracle."""
    shapes = [(71, 100, 8192, 128, 128, 2e-3), (72, 128, 8200, 192, 64, 1e-3), (73, 65, 8192, 256, 32, 0.0)]
    results = []
    for cfg in (1, 0):
        szo.szo_set_tile_config(cfg)
        os_, ds_, base = [], [], 0
        for (sd, M, N, K, G, dens) in shapes:
            o, d = make_pair(sd, M, N, K, G, dens, nnz_base=base)
            base += (o.sp_idx.size + 3) // 4 * 4
            os_.append(o)
            ds_.append(d)
        ws = szo.new_workspace()
        scal = torch.zeros(3, dtype=torch.float64, device="cuda")
        descs = szo.desc_array([d.desc(with_y=False) for d in ds_])
        hist = []
        szo.szo_kernel_timing(True)
        for s in range(2):
            szo.szo_zo_step(descs, 37, s, 1e-3, 1e-3, scal, ws, szo.STEP_FUSED_LOSS)
            hist.append(scal.cpu().numpy().copy())
        _, launches = szo.szo_kernel_timing_read()
        szo.szo_kernel_timing(False)
        assert launches == (2 if cfg == 0 else 2 * 2 * len(shapes))
        results.append((hist, [d.sp_val.cpu().numpy().copy() for d in ds_]))
        if cfg == 0:
            ref = [clone(o) for o in os_]
            sg = sigma_g(os_)
            for s in range(2):
                r = ozo.zo_step(ref, 37, s, 1e-3, 1e-3)
                lp, lm, g = hist[s]
                assert abs(lp - r["loss_plus"]) <= 1e-6 * r["loss_plus"]
                assert abs(g - r["g"]) <= 1e-2 * max(abs(r["g"]), sg)
    (h1, v1), (h0, v0) = results
    for a, b in zip(h1, h0):
        assert np.array_equal(a, b)
    for a, b in zip(v1, v0):
        assert np.array_equal(a, b)


def test_one_dense_pass_flag_takes_the_slicing_path_at_any_token_count():
    """512 tokens run on the tiled kernel by default (two full forwards per layer); with
    SZO_STEP_ONE_DENSE_PASS the same step runs as slices whose dense product serves both signs.  Two
    different kernels and associations, the same losses, g and update; both agree with the oracle."""
    o1, d1 = make_pair(81, 512, 320, 512, 128, 2e-3, nnz_base=0)
    b2 = (o1.sp_idx.size + 3) // 4 * 4
    o2, d2 = make_pair(82, 300, 256, 256, 64, 5e-3, nnz_base=b2)
    seed, eps, lr = 17, 1e-3, 1e-3
    sg = sigma_g([o1, o2])
    outs = {}
    for flags in (szo.STEP_FUSED_LOSS, szo.STEP_FUSED_LOSS | szo.STEP_ONE_DENSE_PASS):
        da, db = make_pair(81, 512, 320, 512, 128, 2e-3, nnz_base=0)[1], make_pair(82, 300, 256, 256, 64, 5e-3, nnz_base=b2)[1]
        ws = szo.new_workspace()
        scal = torch.zeros(3, dtype=torch.float64, device="cuda")
        ref = [clone(o1), clone(o2)]
        szo.szo_kernel_timing(True)
        szo.szo_zo_step([da.desc(with_y=False), db.desc(with_y=False)], seed, 0, eps, lr, scal, ws, flags)
        _, launches = szo.szo_kernel_timing_read()
        szo.szo_kernel_timing(False)
        lp, lm, g = scal.cpu().numpy()
        r = ozo.zo_step(ref, seed, 0, eps, lr)
        assert abs(lp - r["loss_plus"]) <= 1e-4 * r["loss_plus"] and abs(lm - r["loss_minus"]) <= 1e-4 * r["loss_minus"]
        assert abs(g - r["g"]) <= 1e-2 * max(abs(r["g"]), sg)
        outs[flags] = (launches, g, da.sp_val.cpu().numpy(), db.sp_val.cpu().numpy())
    assert outs[szo.STEP_FUSED_LOSS][0] == 4                          # two matrices, two signs, tiled kernel
    assert outs[szo.STEP_FUSED_LOSS | szo.STEP_ONE_DENSE_PASS][0] == 2  # one launch per instantiation (group 128, group 64)
    ga, gb = outs[szo.STEP_FUSED_LOSS][1], outs[szo.STEP_FUSED_LOSS | szo.STEP_ONE_DENSE_PASS][1]
    assert abs(ga - gb) <= 2e-2 * max(abs(ga), sg)


def test_two_host_threads_each_with_its_own_stream_and_workspace():
    """The step's descriptor tables travel through per-thread pinned buffers: two host threads stepping
    different layers on different streams with different workspaces must not disturb each other."""
    import threading
    szo.szo_set_tile_config(0)
    cases = [(121, 300, 384, 512, 128, 2e-3), (122, 40, 512, 1152, 128, 2e-3)]      # tiled kernel | few-token kernel
    want = []
    for c in cases:                                    # reference: one after the other, default stream
        _, d = make_pair(*c)
        want.append((_gpu_steps([d], 6, 41, 1e-3, 1e-3, szo.STEP_FUSED_LOSS), d.sp_val.cpu().numpy().copy()))
    devs = [make_pair(*c)[1] for c in cases]
    wss = [szo.new_workspace() for _ in cases]
    scals = [torch.zeros(3, dtype=torch.float64, device="cuda") for _ in cases]
    streams = [torch.cuda.Stream() for _ in cases]
    torch.cuda.synchronize()
    got = [[], []]
    errors = []

    def worker(i):
        try:
            descs = szo.desc_array([devs[i].desc()])
            for s in range(6):
                szo.szo_zo_step(descs, 41, s, 1e-3, 1e-3, scals[i], wss[i], szo.STEP_FUSED_LOSS, streams[i].cuda_stream)
                streams[i].synchronize()
                got[i].append(scals[i].cpu().numpy().copy())
        except Exception as e:                          # surfaced in the main thread below
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not errors and all(not t.is_alive() for t in threads)
    for i in range(2):
        assert all(np.array_equal(a, b) for a, b in zip(got[i], want[i][0]))
        assert np.array_equal(devs[i].sp_val.cpu().numpy(), want[i][1])


@pytest.mark.parametrize("flags", [0, szo.STEP_FUSED_LOSS])
def test_empty_steps_and_empty_layers(flags):
    szo.szo_set_tile_config(0)
    ws = szo.new_workspace()
    scal = torch.full((3,), 7.0, dtype=torch.float64, device="cuda")
    szo.szo_zo_step([], 1, 0, 1e-3, 1e-3, scal, ws, flags)            # no layers: losses and g are zero
    assert scal.cpu().tolist() == [0.0, 0.0, 0.0]
    o, d = make_pair(131, 40, 256, 256, 128, 1e-2)
    empty = d.desc()
    empty.M = 0                                                        # a layer without tokens contributes nothing
    szo.szo_zo_step([d.desc(), empty], 1, 0, 1e-3, 0.0, scal, ws, flags)
    a = scal.cpu().numpy().copy()
    szo.szo_zo_step([d.desc()], 1, 0, 1e-3, 0.0, scal, ws, flags)
    assert np.array_equal(a, scal.cpu().numpy()) and a[0] > 0
    # every layer empty: both losses and g are zero, and the update (with g = 0) leaves the values alone
    before = d.sp_val.clone()
    e2 = d.desc()
    e2.N = 0
    scal.fill_(7.0)
    szo.szo_zo_step([empty, e2], 1, 0, 1e-3, 1e-2, scal, ws, flags)
    assert scal.cpu().tolist() == [0.0, 0.0, 0.0]
    assert torch.equal(before, d.sp_val)


@pytest.mark.parametrize("cfg", [0, 3])
def test_step_over_layers_of_both_tile_types(cfg):
    # an fp16-tile layer and a bf16-tile layer in one step: no grouped launch, one g
    szo.szo_set_tile_config(cfg)
    o1, d1 = make_pair(141, 300, 256, 256, 128, 5e-3, nnz_base=0)
    b2 = (o1.sp_idx.size + 3) // 4 * 4
    o2, d2 = make_pair(142, 300, 320, 512, 64, 5e-3, nnz_base=b2)
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    descs = szo.desc_array([d1.desc(szo.TILE_F16, with_y=False), d2.desc(szo.TILE_BF16, with_y=False)])
    szo.szo_zo_step(descs, 3, 0, 1e-3, 0.0, scal, ws, szo.STEP_FUSED_LOSS)
    lp, lm, g = scal.cpu().numpy()
    r = ozo.zo_step([clone(o1), clone(o2)], 3, 0, 1e-3, 0.0)
    assert abs(lp - r["loss_plus"]) <= 5e-3 * r["loss_plus"] and abs(lm - r["loss_minus"]) <= 5e-3 * r["loss_minus"]
    assert abs(g - r["g"]) <= 1e-1 * max(abs(r["g"]), sigma_g([o1, o2]))       # the bf16 layer's share of g is coarse


@pytest.mark.parametrize("dt,fmt", [(szo.TILE_F16, "uniform"), (szo.TILE_BF16, "uniform"), (szo.TILE_F16, "lut")])
def test_dual_sign_tiles_of_the_grouped_launch(dt, fmt):
    """With the library choosing the tiles, a step that fills the chip runs as one launch in which every
    workgroup computes both forwards of a 256 x 128 tile (weights dequantised once, written to two copies
    that differ at the sensitive entries).  Ragged shapes (M not a multiple of 256, N not of 128 or 64),
    a mask dense enough for tiles with more than 64 entries, and a matrix without entries; compared with
    the oracle and with the one-forward-per-workgroup launch (tile configuration 3), whose losses it must
    reproduce up to the order of the fp64 partial sums."""
    shapes = [(161, 2000, 3000, 256, 128, 2e-2), (162, 2048, 3104, 192, 64, 1e-3), (163, 1100, 1024, 128, 32, 0.0)]
    results = {}
    for cfg in (3, 0):
        szo.szo_set_tile_config(cfg)
        os_, ds_, base = [], [], 0
        for (sd, M, N, K, G, dens) in shapes:
            o, d = make_pair(sd, M, N, K, G, dens, nnz_base=base, fmt=fmt)
            base += (o.sp_idx.size + 3) // 4 * 4
            os_.append(o)
            ds_.append(d)
        ws = szo.new_workspace()
        scal = torch.zeros(3, dtype=torch.float64, device="cuda")
        descs = szo.desc_array([d.desc(dt, with_y=False) for d in ds_])
        hist = []
        szo.szo_kernel_timing(True)
        for s in range(2):
            szo.szo_zo_step(descs, 43, s, 1e-3, 1e-3, scal, ws, szo.STEP_FUSED_LOSS)
            hist.append(scal.cpu().numpy().copy())
        _, launches = szo.szo_kernel_timing_read()
        szo.szo_kernel_timing(False)
        assert launches == 2                                   # one grouped launch per step either way
        results[cfg] = (hist, [d.sp_val.cpu().numpy().copy() for d in ds_])
    szo.szo_set_tile_config(0)
    for a, b in zip(results[3][0], results[0][0]):
        assert abs(a[0] - b[0]) <= 1e-12 * a[0] and abs(a[1] - b[1]) <= 1e-12 * a[1], (a, b)
    ref = [clone(o) for o in os_]
    sg = sigma_g(os_)
    bound = UpdateBound(sg, 1e-3)
    for s in range(2):
        r = ozo.zo_step(ref, 43, s, 1e-3, 1e-3)
        bound.add(r)
        lp, lm, g = results[0][0][s]
        ltol, gtol = (1e-6, 1e-2) if dt == szo.TILE_F16 else (1e-4, 1e-1)
        assert abs(lp - r["loss_plus"]) <= ltol * r["loss_plus"] and abs(lm - r["loss_minus"]) <= ltol * r["loss_minus"]
        assert abs(g - r["g"]) <= gtol * max(abs(r["g"]), sg), (s, g, r["g"], sg)
    if dt == szo.TILE_F16:
        for i, (om, o) in enumerate(zip(ref, os_)):
            if o.sp_idx.size:
                bound.check(i, results[0][1][i], om.sp_val, o.sp_val)
