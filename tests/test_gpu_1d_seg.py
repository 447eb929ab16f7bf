"""GPU: the forward/backward pair that hands the segments over as a per-row code
(tv1d_prox_fwd_seg / tv1d_prox_bwd_seg) against the oracle and against the plain pair."""
import numpy as np
import pytest

import workloads
from gpuutil import lam_per_row, rows_view, run_1d
from parity import check_batch

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _row_per_lane_kernels(lane_per_row):
    yield


def _codes_from_x(xr):
    """The code as the header defines it, computed from the forward output in numpy."""
    n = xr.shape[1]
    code = np.zeros(len(xr), dtype=np.uint64)
    for k in range(n - 1):
        code |= (xr[:, k + 1] != xr[:, k]).astype(np.uint64) << np.uint64(k)
        code |= (xr[:, k + 1] > xr[:, k]).astype(np.uint64) << np.uint64(32 + k)
    return code


def _check(y, lam, lam_div, g, axis, label):
    seg = run_1d(y, lam, lam_div, g, axis=axis, use_seg=True)
    ref = run_1d(y, lam, lam_div, g, axis=axis)
    # same kernels, same arithmetic: nothing may differ from the plain pair, bit for bit
    assert np.array_equal(seg["x"], ref["x"]), label
    assert np.array_equal(seg["gy"], ref["gy"]), label
    assert np.array_equal(seg["gl"], ref["gl"]), label
    assert np.array_equal(seg["seg"], _codes_from_x(rows_view(seg["x"], axis))), label
    yr, gr = rows_view(y, axis), rows_view(g, axis)
    lr = lam_per_row(lam, len(yr), lam_div)
    check_batch(yr, lr, gr, rows_view(seg["x"], axis), rows_view(seg["gy"], axis), gl_gpu=seg["gl"],
                lam_count=np.asarray(lam).size, lam_div=lam_div, label=label)


def test_config3_reduced_rows_and_columns():
    y, lam, g = workloads.config3(B=3, C=128)
    _check(y, lam, 32, g, -1, "cfg3 rows (seg)")
    _check(y, lam, 32, g, -2, "cfg3 columns (seg)")


@pytest.mark.parametrize("n,rows,axis", [(28, 16384 + 77, -1), (32, 16384 + 64, -1), (31, 16384 + 5, 0),
                                         (28, 500, -1), (32, 8192, -1), (17, 300, 0)])
def test_rows_of_17_to_32_samples_small_and_large_batches(n, rows, axis):
    # ragged rows, packed and strided, a few tiles and several hundred
    rng = np.random.default_rng(370 + n + rows)
    y = rng.normal(size=(rows, n)).astype(np.float32)
    g = rng.normal(size=(rows, n)).astype(np.float32)
    lam = (10 ** rng.uniform(-3, 1, size=3)).astype(np.float32)
    if axis == 0:
        y, g = np.ascontiguousarray(y.T), np.ascontiguousarray(g.T)
    _check(y, lam, 5, g, axis, "seg n=%d rows=%d axis=%d" % (n, rows, axis))


def test_config2_reduced_ties():
    y, lam, g = workloads.config2(B=4, C=64)
    _check(y, lam, 32, g, -1, "cfg2 rows (seg)")


@pytest.mark.parametrize("n", [1, 2, 3, 8, 9, 16, 17, 31, 32])
def test_short_lengths_ragged(n):
    rng = np.random.default_rng(700 + n)
    rows = 333
    y = rng.normal(size=(rows, n)).astype(np.float32)
    g = rng.normal(size=(rows, n)).astype(np.float32)
    lam = (10 ** rng.uniform(-3, 1, size=rows)).astype(np.float32)
    _check(y, lam, 1, g, -1, "seg n=%d" % n)


def test_lambda_zero_and_huge():
    rng = np.random.default_rng(43)
    y = rng.normal(size=(130, 32)).astype(np.float32)
    y[:, 5] = y[:, 4]                                    # a tie: no jump although lam = 0
    g = rng.normal(size=y.shape).astype(np.float32)
    out = run_1d(y, np.array([0.0], np.float32), 1, g, use_seg=True)
    assert np.array_equal(out["x"], y)
    assert np.all((out["seg"] >> np.uint64(4)) & np.uint64(1) == 0)
    assert np.array_equal(out["seg"], _codes_from_x(y))
    out = run_1d(y, np.array([1e4], np.float32), 1, g, use_seg=True)
    assert np.all(out["seg"] == 0)
    np.testing.assert_allclose(out["gy"], np.repeat(g.astype(np.float64).mean(1, keepdims=True), 32, 1),
                               atol=1e-5)
    assert abs(out["gl"][0]) == 0.0


def test_zero_rows():
    y = np.zeros((0, 32), np.float32)
    out = run_1d(y, np.array([0.5, 0.25], np.float32), 1, y, use_seg=True)
    assert out["x"].shape == (0, 32) and np.array_equal(out["gl"], np.zeros(2, np.float32))


# ---- tv1d_prox_fwd_ex with its workspace: slots visited in the order of decreasing predicted cost


def _check_ordered(y, lam, lam_div, g, axis, expect_order):
    ref = run_1d(y, lam, lam_div, g, axis=axis, use_seg=True)
    out = run_1d(y, lam, lam_div, g, axis=axis, use_seg=True, use_ws=True, want_info=True)
    # the order only changes which workgroup handles which rows
    assert np.array_equal(out["x"], ref["x"])
    assert np.array_equal(out["seg"], ref["seg"])
    assert np.array_equal(out["gy"], ref["gy"]) and np.array_equal(out["gl"], ref["gl"])
    if expect_order:
        count = np.asarray(lam).size
        assert out["ws_bytes"] >= 4 * count
        assert np.array_equal(np.sort(out["order"]), np.arange(count))     # a permutation of the slots
    else:
        assert out["ws_bytes"] == 0
    return out


def test_ordered_config3_reduced():
    y, lam, g = workloads.config3(B=6, C=128)
    out = _check_ordered(y, lam, 32, g, -1, True)
    # slots whose rows need the most Newton steps come first, the one-step slots last
    steps = (out["info"] & 0xffff).reshape(6, 128, 32).transpose(1, 0, 2).reshape(128, -1).mean(1)
    by_order = steps[out["order"]]
    assert by_order[:16].mean() > 2.0 * by_order[-16:].mean()
    assert by_order[-16:].max() <= 1.5
    _check_ordered(y, lam, 32, g, -2, True)                                # columns: strided rows


def test_ordered_falls_back_where_slots_do_not_group():
    rng = np.random.default_rng(44)
    y = rng.normal(size=(333, 32)).astype(np.float32)
    g = rng.normal(size=y.shape).astype(np.float32)
    _check_ordered(y, (10 ** rng.uniform(-3, 1, size=333)).astype(np.float32), 1, g, -1, False)
    _check_ordered(y, np.array([0.3], np.float32), 1, g, -1, False)         # one slot: nothing to order
    y = rng.normal(size=(3, 6, 16, 16)).astype(np.float32)                  # slots do not fill tiles
    g = rng.normal(size=y.shape).astype(np.float32)
    _check_ordered(y, (10 ** rng.uniform(-2, 0.5, size=6)).astype(np.float32), 16, g, -1, False)
    y = rng.normal(size=(32, 6, 16, 16)).astype(np.float32)                 # now every slot fills tiles
    g = rng.normal(size=y.shape).astype(np.float32)
    _check_ordered(y, (10 ** rng.uniform(-2, 0.5, size=6)).astype(np.float32), 16, g, -1, True)


@pytest.mark.parametrize("shape", [(32, 100, 8, 32), (64, 1000, 2, 16), (32, 40, 16, 32)])
def test_ordered_many_slots_small_groups(shape):
    # slot counts that are no power of two, groups of 8, 2 and 16 rows, up to 1000 slots
    rng = np.random.default_rng(45 + shape[1])
    y = rng.normal(size=shape).astype(np.float32)
    g = rng.normal(size=shape).astype(np.float32)
    lam = (10 ** rng.uniform(-3, 1, size=shape[1])).astype(np.float32)
    _check_ordered(y, lam, shape[2], g, -1, True)
    ref = run_1d(y, lam, shape[2], g, axis=-1)
    yr, gr = rows_view(y, -1), rows_view(g, -1)
    check_batch(yr, lam_per_row(lam, len(yr), shape[2]), gr, rows_view(ref["x"], -1), rows_view(ref["gy"], -1),
                gl_gpu=ref["gl"], lam_count=shape[1], lam_div=shape[2], label="slots %s" % (shape,))


def test_forward_with_a_kept_slot_order():
    """TV_FWD_ORDER_READY: the call uses whatever order its workspace holds.  The order an earlier
    call left there, the reverse of it and a buffer of numbers that are no slots at all (clamped
    by the kernel) all give the same bits: the order only decides who works on what when."""
    import torch

    import paper_2204_03643_amd as tv

    y, lam, g = workloads.config3(B=6, C=128)
    dev = torch.device("cuda:0")
    yt, lt = torch.from_numpy(y).to(dev), torch.from_numpy(lam).to(dev)
    rows, L = tv.rows_along(y.shape, -1), tv.tv_lambda(lt.data_ptr(), lt.numel(), 32)
    wsb = tv.tv1d_fwd_workspace_bytes(rows, L)
    assert wsb >= 4 * 128
    ws = torch.zeros(wsb, dtype=torch.uint8, device=dev)
    n_rows = y.size // 32
    ref, seg_ref = torch.empty_like(yt), torch.zeros(n_rows, dtype=torch.int64, device=dev)
    tv.tv1d_prox_fwd_ex(yt, ref, rows, L, seg=seg_ref, ws=ws, ws_bytes=wsb)
    torch.cuda.synchronize()
    order = ws.view(torch.int32)[:128].clone()
    assert sorted(order.tolist()) == list(range(128))
    for new_order in (order, order.flip(0), torch.arange(128, dtype=torch.int32, device=dev)):
        ws.view(torch.int32)[:128] = new_order
        x, seg = torch.full_like(yt, float("nan")), torch.zeros_like(seg_ref)
        tv.tv1d_prox_fwd_ex(yt, x, rows, L, seg=seg, ws=ws, ws_bytes=wsb, flags=tv.TV_FWD_ORDER_READY)
        torch.cuda.synchronize()
        assert torch.equal(ws.view(torch.int32)[:128], new_order)        # not recomputed
        assert torch.equal(x, ref) and torch.equal(seg, seg_ref)
    # entries beyond the slot count are clamped: the rows of the slots left out stay untouched,
    # the rest is as before, and nothing is read or written out of bounds
    ws.fill_(0xff)
    x = torch.full_like(yt, float("nan"))
    tv.tv1d_prox_fwd_ex(yt, x, rows, L, ws=ws, ws_bytes=wsb, flags=tv.TV_FWD_ORDER_READY)
    torch.cuda.synchronize()
    xs, rs = x.reshape(6, 128, 32, 32), ref.reshape(6, 128, 32, 32)
    assert torch.equal(xs[:, 127], rs[:, 127]) and bool(torch.isnan(xs[:, :127]).all())
