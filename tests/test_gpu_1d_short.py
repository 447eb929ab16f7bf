"""GPU parity: rows of at most 32 samples against the oracle, through the C ABI.  Every test of
this module runs three times: with a lane per row (the row-per-lane kernels, which large batches
get), with the library's own choice, which gives batches of up to 40 960 rows a few threads per
row on the long-row kernels (`thread_per_sample_1d_rows`: sixteen threads with two samples each
up to `thread_per_sample_wide_rows` rows), and with eight threads of four samples per row, which
the library picks for the larger of those batches."""
import numpy as np
import pytest

import oracle
import workloads
from gpuutil import lam_per_row, rows_view, run_1d
from parity import FWD_TOL, check_batch, forward_errors
from refmath import certificate

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["lane per row", "library's choice", "eight threads per row"])
def row_mapping(request):
    import paper_2204_03643_amd as tv
    saved = {k: tv.tv_dispatch_threshold(k) for k in ("thread_per_sample_1d_rows", "thread_per_sample_wide_rows")}
    if request.param == "lane per row":
        tv.tv_dispatch_override("thread_per_sample_1d_rows", 0)
    elif request.param == "eight threads per row":
        tv.tv_dispatch_override("thread_per_sample_wide_rows", 0)
    yield request.param
    for k, v in saved.items():
        tv.tv_dispatch_override(k, v)


def _check(y, lam, lam_div, g, axis, label):
    out = run_1d(y, lam, lam_div, g, axis=axis)
    yr, gr = rows_view(y, axis), rows_view(g, axis)
    lr = lam_per_row(lam, len(yr), lam_div)
    return check_batch(yr, lr, gr, rows_view(out["x"], axis), rows_view(out["gy"], axis),
                       gl_gpu=out["gl"], lam_count=np.asarray(lam).size, lam_div=lam_div, label=label)


def test_config3_reduced_rows_and_columns():
    # same distribution as the 2^20-row workload; several 256-row workgroups + per-channel lam
    y, lam, g = workloads.config3(B=3, C=128)
    st = _check(y, lam, 32, g, -1, "cfg3 rows")
    assert st["near_degenerate"] < 0.02 * st["rows"]
    _check(y, lam, 32, g, -2, "cfg3 columns")


def test_config2_reduced_rows_and_columns():
    # post-ReLU maps: about half the samples are exact zeros, so inputs are full of ties
    y, lam, g = workloads.config2(B=4, C=64)
    _check(y, lam, 32, g, -1, "cfg2 rows")
    _check(y, lam, 32, g, -2, "cfg2 columns")


def test_timing_batch_shape():
    y, lam, g = workloads.timing_batch(rows=1000)        # ragged: not a multiple of 64
    _check(y, lam, 1, g, -1, "timing")


@pytest.mark.parametrize("n", [1, 2, 3, 5, 7, 8, 9, 13, 16, 17, 24, 31, 32])
def test_every_short_length(n):
    rng = np.random.default_rng(300 + n)
    rows = 333                                            # ragged tail inside a workgroup
    y = rng.normal(size=(rows, n)).astype(np.float32)
    g = rng.normal(size=(rows, n)).astype(np.float32)
    lam = (10 ** rng.uniform(-3, 1, size=rows)).astype(np.float32)
    _check(y, lam, 1, g, -1, "n=%d" % n)


@pytest.mark.parametrize("n,axis", [(17, -1), (20, -1), (28, -1), (31, -1), (32, -1), (20, 0), (31, 0), (32, 0)])
def test_many_rows_of_17_to_32_samples(n, axis):
    # several hundred tiles of rows shorter than (or exactly) 32 samples, packed and strided, with
    # a ragged last tile
    rng = np.random.default_rng(350 + n)
    rows = 16384 + 77
    y = rng.normal(size=(rows, n)).astype(np.float32)
    g = rng.normal(size=(rows, n)).astype(np.float32)
    lam = (10 ** rng.uniform(-3, 1, size=3)).astype(np.float32)
    if axis == 0:
        y, g = np.ascontiguousarray(y.T), np.ascontiguousarray(g.T)
    _check(y, lam, 5, g, axis, "n=%d rows=%d axis=%d" % (n, rows, axis))


def test_strided_columns_odd_shape():
    rng = np.random.default_rng(41)
    y = rng.normal(size=(5, 3, 19, 11)).astype(np.float32)
    g = rng.normal(size=y.shape).astype(np.float32)
    lam = np.array([0.05, 0.4, 2.0], dtype=np.float32)
    _check(y, lam, 11, g, -2, "columns 19x11")
    _check(y, lam, 19, g, -1, "rows 19x11")


def test_lambda_extremes_and_identity(row_mapping):
    rng = np.random.default_rng(42)
    y = rng.normal(size=(200, 32)).astype(np.float32)
    g = rng.normal(size=y.shape).astype(np.float32)
    out = run_1d(y, np.array([0.0], np.float32), 1, g)
    assert np.array_equal(out["x"], y)                    # lam = 0 is the identity (paper Sec. 3.1)
    assert np.array_equal(out["gy"], g)
    out = run_1d(y, np.array([1e4], np.float32), 1, g)
    # (the row-per-lane kernel starts such rows at their solution; the long-row kernels start every
    # dual on its bound, with lam cut down to a bound on lam_max, and x = y - D^T u carries the
    # rounding errors of duals of that size)
    np.testing.assert_allclose(out["x"], np.repeat(y.astype(np.float64).mean(1, keepdims=True), 32, 1),
                               atol=1e-5 if row_mapping == "lane per row" else 5e-5)
    assert np.all(out["x"] == out["x"][:, :1])            # one segment, bit-identical
    np.testing.assert_allclose(out["gy"], np.repeat(g.astype(np.float64).mean(1, keepdims=True), 32, 1),
                               atol=1e-5)
    assert abs(out["gl"][0]) == 0.0
    out = run_1d(y, np.array([-3.0], np.float32), 1)      # negative lam acts as 0
    assert np.array_equal(out["x"], y)


def test_in_place_and_sum_preserved():
    y, lam, g = workloads.config3(B=1, C=16)
    a = run_1d(y, lam, 32)
    b = run_1d(y, lam, 32, in_place=True)
    assert np.array_equal(a["x"], b["x"])
    np.testing.assert_allclose(a["x"].astype(np.float64).sum(-1), y.astype(np.float64).sum(-1), atol=2e-4)


def test_constant_and_tied_rows():
    y = np.zeros((130, 32), np.float32)
    y[1] = 3.0
    y[2, 16:] = 1.0                                       # exact unit step
    y[3] = np.tile([0.0, 1.0], 16)                        # alternating
    y[4:] = np.round(np.random.default_rng(43).normal(size=(126, 32)) * 2) / 2   # many exact ties
    g = np.random.default_rng(44).normal(size=y.shape).astype(np.float32)
    lam = np.array([0.25], np.float32)
    out = run_1d(y, lam, 1, g, want_info=True)
    x_ref = oracle.prox1d_batch(y.astype(np.float64), lam.astype(np.float64))
    assert forward_errors(out["x"], x_ref, y).max() <= FWD_TOL
    assert np.array_equal(out["x"][0], y[0]) and np.array_equal(out["x"][1], y[1])
    assert not np.any(out["info"] & (1 << 18))            # nobody hit the iteration cap


def test_nan_row_stays_in_its_row():
    rng = np.random.default_rng(45)
    y = rng.normal(size=(128, 32)).astype(np.float32)
    y[5, 7] = np.nan
    out = run_1d(y, np.array([0.3], np.float32), 1)
    assert np.isnan(out["x"][5, 7])                      # confined to its own row
    ok = np.delete(np.arange(128), 5)
    x_ref = oracle.prox1d_batch(y[ok].astype(np.float64), np.array([0.3]))
    assert forward_errors(out["x"][ok], x_ref, y[ok]).max() <= FWD_TOL


def test_empty_batch():
    out = run_1d(np.zeros((0, 32), np.float32), np.array([0.5], np.float32), 1,
                 np.zeros((0, 32), np.float32))
    assert out["x"].shape == (0, 32) and out["gl"][0] == 0.0


def test_info_word_reports_convergence():
    y, lam, g = workloads.config3(B=2, C=128)
    out = run_1d(y, lam, 32, want_info=True)
    info = out["info"]
    assert np.all((info & (3 << 16)) != 0)                # every row: optimality test or no-change stop
    assert not np.any(info & (1 << 18))
    assert (info & 0xffff).max() <= 16


def test_info_word_of_lambda_zero_rows(row_mapping):
    """lambda = 0 is the identity (Sec. 3.1): the row stops before any Newton step, and its info
    word must not claim that it stopped short of an optimal point (bit 19)."""
    rng = np.random.default_rng(8)
    y = rng.normal(size=(200, 32)).astype(np.float32)
    lam = np.where(np.arange(200) % 3 == 0, 0.0, 0.3).astype(np.float32)
    out = run_1d(y, lam, 1, want_info=True)
    zero = lam == 0
    assert np.array_equal(out["x"][zero], y[zero])
    assert not np.any(out["info"] & (1 << 19)) and not np.any(out["info"] & (1 << 18))
    if row_mapping == "lane per row":
        assert np.all((out["info"][zero] & 0xffff) == 0) and np.all(out["info"][zero] & (1 << 16))
    else:       # the long-row kernels take the one step that changes nothing
        assert np.all((out["info"][zero] & 0xffff) <= 1) and np.all(out["info"][zero] & (3 << 16))
    y17 = rng.normal(size=(70, 17)).astype(np.float32)
    out = run_1d(y17, np.zeros(1, np.float32), 1, want_info=True)
    assert np.array_equal(out["x"], y17) and not np.any(out["info"] & (1 << 19))


def test_full_size_config3_sampled():
    """The 2^20-row workload in the launch configuration the benchmark times: sampled rows
    against the oracle, the certificate on further samples, and global properties."""
    y, lam, g = workloads.config3()
    out = run_1d(y, lam, 32, g, want_info=True)
    x, gy = out["x"], out["gy"]
    assert np.all(np.isfinite(x)) and np.all(np.isfinite(gy))
    assert not np.any(out["info"] & (1 << 18))
    yr, xr, gr, gyr = (a.reshape(-1, 32) for a in (y, x, g, gy))
    lr = lam_per_row(lam, len(yr), 32)
    rng = np.random.default_rng(46)
    idx = np.sort(rng.choice(len(yr), size=20000, replace=False))
    idx = np.concatenate((idx, [0, 1, len(yr) - 2, len(yr) - 1]))
    check_batch(yr[idx], lr[idx], gr[idx], xr[idx], gyr[idx], label="cfg3 full sampled")
    for r in rng.choice(len(yr), size=300, replace=False):
        gap, resid, viol = certificate(xr[r], yr[r], float(lr[r]))
        assert gap < 1e-4 and abs(resid) < 1e-3 and viol < 1e-4
    # properties that hold at any size
    np.testing.assert_allclose(xr.astype(np.float64).sum(1), yr.astype(np.float64).sum(1), atol=3e-4)
    np.testing.assert_allclose(gyr.astype(np.float64).sum(1), gr.astype(np.float64).sum(1), atol=3e-4)
    assert np.all(xr.max(1) <= yr.max(1) + 1e-5) and np.all(xr.min(1) >= yr.min(1) - 1e-5)
    # grad_lam against per-row oracle contributions computed from the GPU's own segments
    xs, gs = xr.astype(np.float64), gr.astype(np.float64)
    _, gl_ref = oracle.prox1d_bwd_batch(gs, xs, lam_count=128, lam_div=32)
    np.testing.assert_allclose(out["gl"], gl_ref, rtol=1e-4, atol=1e-2)


@pytest.mark.parametrize("scale", [1e-4, 1e3, 1e6])
def test_input_scale(scale):
    # prox(c y, c lam) = c prox(y, lam): the stopping rules are relative, so parity must hold at
    # any magnitude (the tolerance 1e-4 (1 + max|y|) is checked on the rescaled problem)
    rng = np.random.default_rng(46)
    y = rng.normal(size=(300, 32)).astype(np.float32)
    g = rng.normal(size=y.shape).astype(np.float32)
    lam = (10 ** rng.uniform(-3, 1, size=300)).astype(np.float32)
    ys, ls = (y * np.float32(scale)).astype(np.float32), (lam * np.float32(scale)).astype(np.float32)
    out = run_1d(ys, ls, 1, g, want_info=True)
    assert not np.any(out["info"] >> 18 & 1)                       # no row ran into the iteration cap
    xr = oracle.prox1d_batch(ys.astype(np.float64), ls.astype(np.float64), lam_div=1)
    err = np.abs(out["x"] - xr).max(1) / np.abs(ys).max(1)
    assert err.max() <= 1e-5, err.max()                            # relative to the row's own scale
    check_batch(y, lam, g, (out["x"] / np.float32(scale)).astype(np.float32), None, label="scale %g" % scale)


@pytest.mark.parametrize("planes,pitch,count", [(5, 1024, 1), (7, 1280, 3), (8, 1024, 4)])
def test_columns_of_32x32_planes(planes, pitch, count):
    """The column pass on contiguous 32 x 32 planes moves whole planes through LDS: an odd number
    of planes (half-empty last wave), planes that are not adjacent in memory, lambda per plane
    group; forward and backward, against the oracle column by column."""
    import torch

    import paper_2204_03643_amd as tv

    rng = np.random.default_rng(planes * 7 + count)
    buf = rng.normal(size=(planes, pitch)).astype(np.float32)
    gbuf = rng.normal(size=(planes, pitch)).astype(np.float32)
    lam = (10 ** rng.uniform(-1.5, 0.5, size=count)).astype(np.float32)
    dev = torch.device("cuda:0")
    yt, gt, lt = (torch.from_numpy(a).to(dev) for a in (buf, gbuf, lam))
    xt, gy = torch.full_like(yt, float("nan")), torch.full_like(yt, float("nan"))
    gl = torch.full((count,), float("nan"), device=dev)
    r = tv.tv_rows(planes, pitch, 32, 1, 32, 32)          # row id = plane * 32 + column
    L = tv.tv_lambda(lt.data_ptr(), count, 32)
    wsb = tv.tv1d_bwd_workspace_bytes(r, L)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
    tv.tv1d_prox_fwd(yt, xt, r, L)
    tv.tv1d_prox_bwd(gt, xt, gy, gl, r, L, ws, wsb)
    torch.cuda.synchronize()
    x, gyn = xt.cpu().numpy(), gy.cpu().numpy()
    assert np.isnan(x[:, 1024:]).all() and np.isnan(gyn[:, 1024:]).all()      # nothing outside the planes
    cols = lambda a: a[:, :1024].reshape(planes, 32, 32).transpose(0, 2, 1).reshape(-1, 32)
    lr = lam[(np.arange(planes * 32) // 32) % count]
    check_batch(cols(buf), lr, cols(gbuf), cols(x), cols(gyn), gl_gpu=gl.cpu().numpy(), lam_count=count,
                lam_div=32, label="plane columns %d/%d/%d" % (planes, pitch, count))


@pytest.mark.parametrize("shape,axis,lam_div", [((6, 128, 32, 32), -1, 32), ((3, 7, 20, 31), -1, 20), ((5, 24, 130), -2, 130),
                                                ((333, 9), -1, 1)])
def test_parallel_step_size_search(shape, axis, lam_div):
    """The forward call with the paper's other step-size rule (Sec. 3.2, search over halving step
    sizes tried side by side): the same minimiser, so the same parity rules; and the output agrees
    with the backtracking call far inside the forward tolerance."""
    import torch

    import paper_2204_03643_amd as tv

    rng = np.random.default_rng(60 + shape[-1])
    y = rng.normal(size=shape).astype(np.float32)
    g = rng.normal(size=shape).astype(np.float32)
    n_slots = shape[1] if len(shape) == 4 else 3
    lam = (10 ** rng.uniform(-3, 1, size=n_slots)).astype(np.float32)
    dev = torch.device("cuda:0")
    yt, lt, gt = (torch.from_numpy(a).to(dev) for a in (y, lam, g))
    rows, L = tv.rows_along(shape, axis), tv.tv_lambda(lt.data_ptr(), lt.numel(), lam_div)
    n_rows = rows.n_outer * rows.n_inner
    x, x_bt = torch.full_like(yt, float("nan")), torch.empty_like(yt)
    info = torch.zeros(n_rows, dtype=torch.int32, device=dev)
    seg = torch.zeros(n_rows, dtype=torch.int64, device=dev)
    tv.tv1d_prox_fwd_ex(yt, x, rows, L, info=info, seg=seg, flags=tv.TV_FWD_PARALLEL_SEARCH)
    tv.tv1d_prox_fwd(yt, x_bt, rows, L)
    gy, gl = torch.empty_like(yt), torch.empty_like(lt)
    wsb = tv.tv1d_bwd_workspace_bytes(rows, L)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
    tv.tv1d_prox_bwd_seg(gt, seg, gy, gl, rows, L, ws, wsb)
    torch.cuda.synchronize()
    assert not bool((info & (1 << 18)).any())
    assert float((x - x_bt).abs().max()) <= 2e-5 * (1 + np.abs(y).max())
    yr, gr = rows_view(y, axis), rows_view(g, axis)
    check_batch(yr, lam_per_row(lam, len(yr), lam_div), gr, rows_view(x.cpu().numpy(), axis),
                rows_view(gy.cpu().numpy(), axis), gl_gpu=gl.cpu().numpy(), lam_count=lam.size, lam_div=lam_div,
                label="parallel search %s" % (shape,))
    # rows longer than the row-per-lane kernels take: not offered
    yl = torch.zeros(4, 40, device=dev)
    with pytest.raises(tv.TVError) as e:
        tv.tv1d_prox_fwd_ex(yl, yl, tv.rows_along((4, 40), -1), tv.tv_lambda(lt.data_ptr(), 1, 1),
                            flags=tv.TV_FWD_PARALLEL_SEARCH)
    assert e.value.status == 6
