"""The single-layer calls are plain kernel launches on the caller's stream (fill kernels instead of memset
nodes, no host synchronisation, no allocation): a HIP graph captured around them must replay to the
same results as the eager calls, every time."""
import numpy as np
import pytest
import torch

from paper_2406_02913_amd import szo
from helpers import make_pair

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("flags", [0, szo.STEP_FUSED_LOSS])
def test_whole_step_call_refuses_a_capturing_stream(flags):
    """szo_zo_step stages descriptor tables through pinned host buffers that later calls reuse, so a
    captured step would replay stale tables: while the stream is capturing it must return
    SZO_EUNSUPPORTED with nothing enqueued (the captured graph stays empty and the values untouched)."""
    szo.szo_set_tile_config(0)
    _, d = make_pair(112, 16, 256, 256, 128, 5e-3)
    ws = szo.new_workspace()
    scal = torch.full((3,), 5.0, dtype=torch.float64, device="cuda")
    v0 = d.sp_val.clone()
    descs = szo.desc_array([d.desc()])
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        graph.capture_begin()
        with pytest.raises(szo.SzoError) as err:
            szo.szo_zo_step(descs, 1, 0, 1e-3, 1e-3, scal, ws, flags)
        scal.add_(1.0)                                                # something to replay
        graph.capture_end()
    assert err.value.code == szo.EUNSUPPORTED
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    assert scal.cpu().tolist() == [6.0, 6.0, 6.0] and torch.equal(v0, d.sp_val)
    szo.szo_zo_step(descs, 1, 0, 1e-3, 1e-3, scal, ws, flags)         # and the eager call still works
    torch.cuda.synchronize()
    assert scal[0].item() > 0 and not torch.equal(v0, d.sp_val)


@pytest.mark.parametrize("M", [16, 300])            # few-token kernel, tiled kernel
def test_forward_loss_g_update_replay_from_a_graph(M):
    szo.szo_set_tile_config(0)
    o, d = make_pair(111, M, 320, 512, 128, 5e-3)
    ws = szo.new_workspace()
    seed, eps, lr = 13, 1e-3, 1e-3
    scale = 1.0 / (M * 320)
    acc = torch.zeros(3, dtype=torch.float64, device="cuda")         # L+, L-, g
    step_dev = 4

    def body():
        acc.zero_()                                                   # a fill kernel, not a memset node
        szo.szo_linear_fwd_mse(d.desc(with_y=False), seed, step_dev, +1, eps, scale, acc[0:1], ws)
        szo.szo_linear_fwd(d.desc(), seed, step_dev, -1, eps)
        szo.szo_mse_loss(d.y, d.target, M * 320, scale, acc[1:2], ws)
        szo.szo_spsa_g(acc[0:1], acc[1:2], eps, acc[2:3])
        szo.szo_sparse_update(d.sp_val, d.sp_idx, d.nnz, d.nnz_base, seed, step_dev, acc[2:3], lr)

    v0 = d.sp_val.clone()
    body()                                                            # eager: also the warm-up before capture
    torch.cuda.synchronize()
    want_acc, want_v = acc.cpu().numpy().copy(), d.sp_val.cpu().numpy().copy()
    assert want_acc[2] != 0.0 and not np.array_equal(want_v, v0.cpu().numpy())

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    d.sp_val.copy_(v0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        graph.capture_begin()
        body()
        graph.capture_end()
    torch.cuda.synchronize()
    for rep in range(3):
        d.sp_val.copy_(v0)                                            # eager work between the replays
        acc.fill_(-1.0)
        d.y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(acc.cpu().numpy(), want_acc), rep
        assert np.array_equal(d.sp_val.cpu().numpy(), want_v), rep
