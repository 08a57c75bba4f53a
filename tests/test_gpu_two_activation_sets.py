"""szo_zo_step with a second set of activations for the -eps forward (desc.x_minus): inside a model the two
forwards of a layer see different inputs.  The few-token path then still reads the weights once for
both signs (one block of token rows per set); the tiled path simply reads x_minus in its second forward."""
import numpy as np
import pytest
import torch

from oracle import zo as ozo
from paper_2406_02913_amd import synth, szo
from helpers import make_pair, clone, sigma_g, UpdateBound

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto_tile_config():
    yield
    szo.szo_set_tile_config(0)


def _with_x_minus(o, d, seed):
    # other values AND twice the size (bf16 exponent + 1), so that a forward that read the wrong set shows in
    # its loss (two equally distributed sets would give almost equal mean squared errors)
    xm = (synth.activations(seed, d.M, d.K) + np.uint16(0x0080)).astype(np.uint16)
    o.x_minus_bits = xm
    d.x_minus = torch.from_numpy(xm.view(np.int16)).view(torch.bfloat16).cuda()
    return o, d


def _check_step(os_, ds_, flags, steps=2, seed=29, eps=1e-3, lr=1e-7, ltol=1e-4):
    # (with activations this different g is ~1e2-1e3: a small lr keeps the update a perturbation)
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    ref = [clone(o) for o in os_]
    sg = sigma_g(os_)
    descs = szo.desc_array([d.desc(with_y=not (flags & szo.STEP_FUSED_LOSS)) for d in ds_])
    out = []
    bound = UpdateBound(sg, lr)
    for s in range(steps):
        szo.szo_zo_step(descs, seed, s, eps, lr, scal, ws, flags)
        lp, lm, g = scal.cpu().numpy()
        r = ozo.zo_step(ref, seed, s, eps, lr)
        bound.add(r, extra_dg=ltol * (r["loss_plus"] + r["loss_minus"]) / (2 * eps))
        assert abs(lp - r["loss_plus"]) <= ltol * r["loss_plus"], (s, lp, r["loss_plus"])
        assert abs(lm - r["loss_minus"]) <= ltol * r["loss_minus"], (s, lm, r["loss_minus"])
        # L+ and L- now come from different activations: g is a difference of two unrelated losses divided
        # by 2 eps, so its error is that of the losses, not of their (cancelling) common part
        assert abs(g - r["g"]) <= 1e-2 * max(abs(r["g"]), sg) + ltol * (r["loss_plus"] + r["loss_minus"]) / (2 * eps)
        out.append((lp, lm, g))
    for i, (om, dd, oo) in enumerate(zip(ref, ds_, os_)):
        if oo.sp_idx.size:
            bound.check(i, dd.sp_val.cpu().numpy(), om.sp_val, oo.sp_val)
    return out


# (seed, M, N, K, group, density, format)
FEW = [(91, 1, 200, 256, 128, 2e-2, "uniform"), (92, 16, 512, 1152, 128, 2e-3, "uniform"),
       (93, 40, 320, 512, 64, 5e-3, "uniform"), (94, 23, 256, 384, 128, 1e-2, "lut"), (95, 100, 256, 256, 128, 1e-2, "uniform")]


@pytest.mark.parametrize("case", FEW)
def test_few_tokens_with_two_activation_sets(case):
    s, M, N, K, G, dens, fmt = case
    o, d = _with_x_minus(*make_pair(s, M, N, K, G, dens, fmt=fmt), seed=s + 500)
    szo.szo_kernel_timing(True)
    out = _check_step([o], [d], szo.STEP_FUSED_LOSS)
    _, launches = szo.szo_kernel_timing_read()
    szo.szo_kernel_timing(False)
    assert launches == 2                                   # one launch per step: the weights are read once for both signs
    assert abs(out[0][0] - out[0][1]) > 1e-3 * out[0][0]   # the two forwards really saw different inputs


@pytest.mark.parametrize("cfg", [2, 3])
def test_tiled_kernel_with_two_activation_sets(cfg):
    szo.szo_set_tile_config(cfg)
    o1, d1 = _with_x_minus(*make_pair(96, 300, 384, 320, 64, 2e-3, nnz_base=0), seed=601)
    b2 = (o1.sp_idx.size + 3) // 4 * 4
    o2, d2 = make_pair(97, 260, 256, 256, 128, 5e-3, nnz_base=b2)          # this layer: the same x for both
    _check_step([o1, o2], [d1, d2], szo.STEP_FUSED_LOSS, ltol=1e-5)
    o1, d1 = _with_x_minus(*make_pair(96, 300, 384, 320, 64, 2e-3, nnz_base=0), seed=601)
    o2, d2 = make_pair(97, 260, 256, 256, 128, 5e-3, nnz_base=b2)
    _check_step([o1, o2], [d1, d2], 0, ltol=1e-5)                          # separate loss kernel


def test_mixed_step_and_equal_sets_reduce_to_the_plain_step():
    # a step over a layer with two sets and a layer with one; and x_minus == x must give what no x_minus gives
    o1, d1 = _with_x_minus(*make_pair(98, 16, 256, 512, 128, 5e-3, nnz_base=0), seed=602)
    b2 = (o1.sp_idx.size + 3) // 4 * 4
    o2, d2 = make_pair(99, 48, 320, 256, 128, 5e-3, nnz_base=b2)
    _check_step([o1, o2], [d1, d2], szo.STEP_FUSED_LOSS)
    oa, da = make_pair(98, 16, 256, 512, 128, 5e-3)
    ob, db = make_pair(98, 16, 256, 512, 128, 5e-3)
    db.x_minus = db.x.clone()
    ws = szo.new_workspace()
    res = []
    for d in (da, db):
        scal = torch.zeros(3, dtype=torch.float64, device="cuda")
        szo.szo_zo_step([d.desc(with_y=False)], 5, 0, 1e-3, 1e-3, scal, ws, szo.STEP_FUSED_LOSS)
        res.append(scal.cpu().numpy().copy())
    sg = sigma_g([oa])
    assert abs(res[0][0] - res[1][0]) <= 1e-6 * res[0][0] and abs(res[0][1] - res[1][1]) <= 1e-6 * res[0][1]
    assert abs(res[0][2] - res[1][2]) <= 1e-2 * max(abs(res[0][2]), sg)


def test_misaligned_x_minus_is_rejected():
    import ctypes
    o, d = make_pair(98, 16, 256, 512, 128, 5e-3)
    desc = d.desc()
    desc.x_minus = d.x.data_ptr() + 2
    ws = szo.new_workspace()
    scal = torch.zeros(3, dtype=torch.float64, device="cuda")
    assert szo.lib.szo_zo_step(ctypes.byref(desc), 1, 0, 0, 1e-3, 1e-3, scal.data_ptr(), ws.data_ptr(), 1, None) == szo.EINVAL
