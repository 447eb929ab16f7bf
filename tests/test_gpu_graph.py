"""GPU: the library's calls only launch kernels (no allocation, no memset), so a forward +
backward step captures into a HIP graph as it is.  Replays are checked against the eager
result, several times, with eager work and synchronisations between them and with new input
values written into the captured buffers."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


def test_forward_backward_step_replays_from_a_graph():
    import torch

    import paper_2204_03643_amd as tv

    dev = torch.device("cuda:0")
    y, lam, g = workloads.config3(B=4, C=128)
    B, C, H, W = y.shape
    yt, lt, gt = (torch.from_numpy(a).to(dev) for a in (y, lam, g))
    xt, gy, gl = torch.empty_like(yt), torch.empty_like(yt), torch.empty_like(lt)
    rows = tv.rows_along(y.shape, -1)
    L = tv.tv_lambda(lt.data_ptr(), C, H)
    seg = torch.empty(B * C * H, dtype=torch.int64, device=dev)
    fwsb = tv.tv1d_fwd_workspace_bytes(rows, L)
    assert fwsb > 0
    fws = torch.empty(fwsb, dtype=torch.uint8, device=dev)
    bwsb = tv.tv1d_bwd_workspace_bytes(rows, L)
    bws = torch.empty(bwsb, dtype=torch.uint8, device=dev)

    def step():
        tv.tv1d_prox_fwd_ex(yt, xt, rows, L, seg=seg, ws=fws, ws_bytes=fwsb)
        tv.tv1d_prox_bwd_seg(gt, seg, gy, gl, rows, L, bws, bwsb)

    def eager():
        step()
        torch.cuda.synchronize()
        return xt.clone(), gy.clone(), gl.clone()

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                           # warm-up on the capture stream
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    rng = np.random.default_rng(91)
    for rep in range(4):
        if rep:                                          # new values in the captured buffers
            yt.copy_(torch.from_numpy(rng.normal(size=y.shape).astype(np.float32)))
            gt.copy_(torch.from_numpy(rng.normal(size=y.shape).astype(np.float32)))
            lt.copy_(torch.from_numpy((10 ** rng.uniform(-3, 1, size=C)).astype(np.float32)))
        ref = eager()
        for t in (xt, gy, gl, seg):
            t.zero_()                                    # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(xt, ref[0]) and torch.equal(gy, ref[1]) and torch.equal(gl, ref[2]), rep


@pytest.mark.parametrize("planes,H,W,K", [(16, 32, 32, 3),       # small batch: a plane per workgroup, both ways
                                          (40, 16, 16, 3),       # row-per-lane one-launch forward and reverse sweep
                                          (1600, 32, 32, 2),     # the same, two planes per wave
                                          (6, 64, 64, 2),        # a plane per workgroup, 8 x 8 threads x samples
                                          (5, 40, 56, 2),        # ... reverse sweep from the saved pass outputs
                                          (3, 100, 70, 2)])      # pass by pass both ways
def test_2d_step_replays_from_a_graph(planes, H, W, K):
    import torch

    import paper_2204_03643_amd as tv

    dev = torch.device("cuda:0")
    rng = np.random.default_rng(planes + H)
    y = np.maximum(rng.normal(size=(planes, H, W)), 0).astype(np.float32)
    g = rng.normal(size=(planes, H, W)).astype(np.float32)
    lam = (10 ** rng.uniform(-2, 0.3, size=4)).astype(np.float32)
    yt, lt, gt = (torch.from_numpy(a).to(dev) for a in (y, lam, g))
    xt, gy, gl = torch.empty_like(yt), torch.empty_like(yt), torch.empty_like(lt)
    L = tv.tv_lambda(lt.data_ptr(), lt.numel(), 1)
    wsb = tv.tv2d_workspace_bytes(planes, H, W, K)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)

    def step():
        tv.tv2d_prox_fwd(yt, xt, planes, H, W, L, K, ws, wsb)
        tv.tv2d_prox_bwd(gt, gy, gl, planes, H, W, L, K, ws, wsb)

    step()
    torch.cuda.synchronize()
    ref = (xt.clone(), gy.clone(), gl.clone())
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for t in (xt, gy, gl):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(xt, ref[0]) and torch.equal(gy, ref[1]) and torch.equal(gl, ref[2]), rep


def test_long_rows_and_large_planes_replay_from_a_graph():
    """Long rows with the multilevel start (averaging kernels, coarse levels, fine level) and the
    2D operator on planes beyond 32 x 32 (warm-started passes, transposing column kernels, split
    dL/dlam reduction): every replay must reproduce the eager result bit for bit."""
    import torch

    import paper_2204_03643_amd as tv

    dev = torch.device("cuda:0")
    rng = np.random.default_rng(17)
    n, n_rows = 2500, 9
    y1 = np.cumsum(rng.normal(scale=0.05, size=(n_rows, n)), axis=1).astype(np.float32)
    lam1 = (10 ** np.linspace(-2, 0.7, n_rows)).astype(np.float32)
    y1t, l1t = torch.from_numpy(y1).to(dev), torch.from_numpy(lam1).to(dev)
    x1t = torch.empty_like(y1t)
    r1 = tv.rows_along(y1.shape, -1)
    L1 = tv.tv_lambda(l1t.data_ptr(), n_rows, 1)
    fwsb = tv.tv1d_fwd_workspace_bytes(r1, L1)
    assert fwsb > 0
    fws = torch.empty(fwsb, dtype=torch.uint8, device=dev)

    planes, H, W, K = 3, 70, 48, 3
    y2 = rng.normal(size=(planes, H, W)).astype(np.float32)
    g2 = rng.normal(size=(planes, H, W)).astype(np.float32)
    y2t, g2t = torch.from_numpy(y2).to(dev), torch.from_numpy(g2).to(dev)
    l2t = torch.tensor([0.4], device=dev)
    x2t, gy2, gl2 = torch.empty_like(y2t), torch.empty_like(y2t), torch.empty_like(l2t)
    L2 = tv.tv_lambda(l2t.data_ptr(), 1, 1)
    wsb = tv.tv2d_workspace_bytes(planes, H, W, K)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)

    x1p = torch.empty_like(y1t)         # the plain call: the levels of a row live in that row of x

    def step():
        tv.tv1d_prox_fwd_ex(y1t, x1t, r1, L1, ws=fws, ws_bytes=fwsb)
        tv.tv1d_prox_fwd(y1t, x1p, r1, L1)
        tv.tv2d_prox_fwd(y2t, x2t, planes, H, W, L2, K, ws, wsb)
        tv.tv2d_prox_bwd(g2t, gy2, gl2, planes, H, W, L2, K, ws, wsb)

    step()
    torch.cuda.synchronize()
    assert torch.equal(x1p, x1t)
    ref = [t.clone() for t in (x1t, x2t, gy2, gl2)]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for t in (x1t, x2t, gy2, gl2):
            t.zero_()
        fws.fill_(0xff)
        x1p.view(torch.uint8).fill_(0xff if rep % 2 else 0x01)      # stale flags and levels must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip((x1t, x2t, gy2, gl2), ref):
            assert torch.equal(a, b), rep
        assert torch.equal(x1p, ref[0]), rep
