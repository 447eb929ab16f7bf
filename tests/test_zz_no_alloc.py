"""tv1d_prox_bwd_noalloc (the backward call for callers that cannot allocate: its dL/dlam
scratch is a static device array of the library) against tv1d_prox_bwd, through the C ABI, on two
calls in a row that share the array, the second with a smaller input."""
import numpy as np
import pytest

import oracle
import workloads
from gpuutil import lam_per_row, rows_view
from parity import check_batch

pytestmark = pytest.mark.gpu


def _both(y, lam, lam_div, g, axis=-1):
    import torch

    import paper_2204_03643_amd as tv

    dev = torch.device("cuda:0")
    yt, gt = (torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev) for a in (y, g))
    lt = torch.from_numpy(np.ascontiguousarray(lam, dtype=np.float32).ravel()).to(dev)
    rows = tv.rows_along(y.shape, axis)
    L = tv.tv_lambda(lt.data_ptr(), lt.numel(), lam_div)
    xt = torch.empty_like(yt)
    tv.tv1d_prox_fwd(yt, xt, rows, L)
    wsb = tv.tv1d_bwd_workspace_bytes(rows, L)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
    gy_a, gy_b = torch.full_like(gt, float("nan")), torch.full_like(gt, float("nan"))
    gl_a, gl_b = torch.full_like(lt, float("nan")), torch.full_like(lt, float("nan"))
    tv.tv1d_prox_bwd(gt, xt, gy_a, gl_a, rows, L, ws, wsb)
    torch.cuda.synchronize()
    # nothing is allocated on the device by the call: neither through torch (its own count may
    # only fall, when Python drops tensors of earlier tests meanwhile) nor behind its back (the
    # device's free memory does not shrink)
    before, free_before = torch.cuda.memory_allocated(), torch.cuda.mem_get_info()[0]
    tv.tv1d_prox_bwd_noalloc(gt, xt, gy_b, gl_b, rows, L)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() <= before and torch.cuda.mem_get_info()[0] >= free_before
    return tuple(t.cpu().numpy() for t in (xt, gy_a, gl_a, gy_b, gl_b))


def test_two_calls_share_the_static_scratch():
    # first call: 2^15 rows of 32 in 128 lambda slots (row-per-lane kernel, partial sums per 32 rows)
    y, lam, g = workloads.config3(B=8, C=128)
    x, gy_a, gl_a, gy_b, gl_b = _both(y, lam, 32, g)
    assert np.array_equal(gy_a, gy_b) and np.array_equal(gl_a, gl_b)
    yr, gr = rows_view(y, -1), rows_view(g, -1)
    check_batch(yr, lam_per_row(lam, len(yr), 32), gr, rows_view(x, -1), rows_view(gy_b, -1),
                gl_gpu=gl_b, lam_count=lam.size, lam_div=32, label="noalloc first call")
    # second call, smaller and of another shape: 100 rows of 300 samples, a lambda per row (one
    # term per row, long-row kernel); whatever the first call left in the array must not matter
    rng = np.random.default_rng(5)
    y2 = np.cumsum(rng.normal(scale=0.3, size=(100, 300)), axis=-1).astype(np.float32)
    g2 = rng.normal(size=y2.shape).astype(np.float32)
    lam2 = (10 ** rng.uniform(-2, 0.5, size=100)).astype(np.float32)
    x2, gy_a, gl_a, gy_b, gl_b = _both(y2, lam2, 1, g2)
    assert np.array_equal(gy_a, gy_b) and np.array_equal(gl_a, gl_b)
    check_batch(y2, lam2, g2, x2, gy_b, gl_gpu=gl_b, lam_count=100, lam_div=1, label="noalloc second call")
    # strided rows (columns), scalar lambda, no grad_lam wanted
    import torch

    import paper_2204_03643_amd as tv
    dev = torch.device("cuda:0")
    y3 = rng.normal(size=(3, 20, 50)).astype(np.float32)
    yt, gt = torch.from_numpy(y3).to(dev), torch.from_numpy(rng.normal(size=y3.shape).astype(np.float32)).to(dev)
    lt = torch.tensor([0.3], device=dev)
    rows, L = tv.rows_along(y3.shape, -2), tv.tv_lambda(lt.data_ptr(), 1, 1)
    xt, ga, gb = torch.empty_like(yt), torch.empty_like(yt), torch.empty_like(yt)
    tv.tv1d_prox_fwd(yt, xt, rows, L)
    tv.tv1d_prox_bwd(gt, xt, ga, None, rows, L, None, 0)
    tv.tv1d_prox_bwd_noalloc(gt, xt, gb, None, rows, L)
    torch.cuda.synchronize()
    assert torch.equal(ga, gb)


def test_too_many_rows_is_an_error():
    import torch

    import paper_2204_03643_amd as tv
    t = torch.zeros(64, device="cuda:0")
    rows = tv.tv_rows((1 << 20) + 1, 2, 1, 1, 2, 1)
    with pytest.raises(tv.TVError) as e:
        tv.tv1d_prox_bwd_noalloc(t, t, t, t, rows, tv.tv_lambda(t.data_ptr(), 1, 1))
    assert e.value.status == 8
