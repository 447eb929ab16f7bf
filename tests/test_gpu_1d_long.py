"""GPU parity: rows longer than 32 samples (T threads per row, Thomas + PCR) against the
oracle, through the C ABI."""
import numpy as np
import pytest

import oracle
import workloads
from gpuutil import lam_per_row, rows_view, run_1d
from parity import FWD_TOL, check_batch, forward_errors

pytestmark = pytest.mark.gpu


def _check(y, lam, lam_div, g, axis, label, want_info=True, use_ws=False, in_place=False):
    out = run_1d(y, lam, lam_div, g, axis=axis, want_info=want_info, use_ws=use_ws, in_place=in_place)
    yr, gr = rows_view(y, axis), rows_view(g, axis)
    lr = lam_per_row(lam, len(yr), lam_div)
    st = check_batch(yr, lr, gr, rows_view(out["x"], axis), rows_view(out["gy"], axis),
                     gl_gpu=out["gl"], lam_count=np.asarray(lam).size, lam_div=lam_div, label=label)
    if want_info:
        assert not np.any(out["info"] & (1 << 18)), label       # nobody hit the iteration cap
        st["max_steps"] = int((out["info"] & 0xffff).max())
        st["steps"] = out["info"] & 0xffff
    st["ws_bytes"] = out.get("ws_bytes", 0)
    return st


def _mixed_rows(rng, rows, n):
    """Half random-walk rows with jumps, half white noise around steps."""
    y = np.empty((rows, n), np.float32)
    for r in range(rows):
        if r % 2 == 0:
            steps = rng.normal(0, 0.05, size=n)
            jumps = (rng.random(n) < 5e-3) * rng.uniform(0.5, 2, size=n) * rng.choice([-1, 1], size=n)
            y[r] = np.cumsum(steps + jumps)
        else:
            y[r] = np.repeat(rng.uniform(-1, 1, size=(n + 15) // 16), 16)[:n] + rng.normal(0, 0.1, size=n)
    return y


def test_config1_full():
    y, lam, g = workloads.config1()
    st = _check(y, lam, 1, g, -1, "cfg1")
    assert st["max_steps"] <= 40


@pytest.mark.parametrize("n", [33, 64, 65, 96, 100, 128, 129, 192, 255, 256, 300, 384, 512, 513, 768, 1000, 1024,
                               1025, 1536, 2048, 3000, 4096, 5000, 6144, 8192, 10000, 12288, 16384])
def test_every_long_length(n):
    rng = np.random.default_rng(500 + n)
    rows = 7 if n <= 4096 else 3
    y = _mixed_rows(rng, rows, n)
    g = rng.normal(size=y.shape).astype(np.float32)
    lam = (10 ** rng.uniform(-2.5, 1, size=rows)).astype(np.float32)
    _check(y, lam, 1, g, -1, "n=%d" % n)


@pytest.mark.parametrize("n", [769, 900, 1024, 1025, 1280, 1536, 1537, 2048, 2049, 3000, 4096, 5000, 8192, 10001, 16384])
def test_multilevel_start(n):
    """Long unit-stride rows start from the duals of the averaged rows: with the workspace of
    tv1d_prox_fwd_ex, and without one when x is a buffer of its own (packed rows), whose rows then
    hold the levels until the fine level overwrites them; both give the same bits.  A call in
    place (x = y) has no such room and starts cold.  Same parity bar for all three; rows with a
    large lambda need far fewer steps from the multilevel start."""
    rng = np.random.default_rng(700 + n)
    rows = 12 if n <= 4096 else 6
    y = _mixed_rows(rng, rows, n)
    g = rng.normal(size=y.shape).astype(np.float32)
    lam = (10 ** np.linspace(-2.5, 1, rows)).astype(np.float32)        # small ones start cold
    cold = _check(y, lam, 1, g, -1, "cold (in place) n=%d" % n, in_place=True)
    ml = _check(y, lam, 1, g, -1, "multilevel n=%d" % n, use_ws=True)
    own = _check(y, lam, 1, g, -1, "multilevel inside x n=%d" % n)
    assert ml["ws_bytes"] > 0
    big = lam >= 1.0
    assert ml["steps"][big].max() <= 10, (ml["steps"], cold["steps"])
    assert ml["steps"][big].sum() < cold["steps"][big].sum(), (ml["steps"], cold["steps"])
    assert np.array_equal(own["steps"], ml["steps"])
    a = run_1d(y, lam, 1, use_ws=True)["x"]
    b = run_1d(y, lam, 1)["x"]
    assert np.array_equal(a, b)


@pytest.mark.parametrize("n", [2049, 5000, 16384])
def test_multilevel_start_with_stacked_levels(n):
    """Levels n/4, n/16, ... down to 256 samples instead of the one level that the library takes
    by default: every level but the coarsest starts from the level below it."""
    import paper_2204_03643_amd as tv
    rng = np.random.default_rng(1700 + n)
    y = _mixed_rows(rng, 6, n)
    g = rng.normal(size=y.shape).astype(np.float32)
    lam = (10 ** np.linspace(-2, 1, 6)).astype(np.float32)
    default = tv.tv_dispatch_threshold("ml_coarsest")
    tv.tv_dispatch_override("ml_coarsest", 256)
    try:
        ml = _check(y, lam, 1, g, -1, "stacked levels n=%d" % n, use_ws=True)
        own = _check(y, lam, 1, g, -1, "stacked levels inside x n=%d" % n)
        a = run_1d(y, lam, 1, use_ws=True)["x"]
        b = run_1d(y, lam, 1)["x"]
    finally:
        tv.tv_dispatch_override("ml_coarsest", default)
    assert np.array_equal(own["steps"], ml["steps"]) and np.array_equal(a, b)
    assert ml["steps"][lam >= 1.0].max() <= 10


@pytest.mark.parametrize("n", [40, 90, 160, 300, 700, 3000])
@pytest.mark.parametrize("lam", [1e3, 1e5])
def test_lambda_far_beyond_lam_max(n, lam):
    """Every lambda from lam_max on gives the row mean.  A dual box far larger than the data must
    not cost accuracy (12 samples per thread: the separator system's diagonal is formed without
    cancellation; lambda is capped at a bound on lam_max).  Random-walk rows of thousands of
    samples have a lam_max above 1e3: those are ordinary parity cases."""
    rng = np.random.default_rng(900 + n)
    y = _mixed_rows(rng, 6, n)
    g = rng.normal(size=y.shape).astype(np.float32)
    _check(y, np.array([lam], np.float32), 1, g, -1, "n=%d lam=%g" % (n, lam))


@pytest.mark.parametrize("n,lam", [(3000, 1e3), (5000, 1e3), (8192, 3e3)])
def test_multilevel_start_with_lambda_of_the_order_of_lam_max(n, lam):
    """Random-walk rows whose lam_max is in the thousands, with a lambda of that order: a few long
    segments, duals a thousand times the data.  From the multilevel start such a row is done in
    two or three Newton steps, and a large last step leaves more rounding error in the free duals
    than the output may carry: the solve then takes one more, small step.  With the workspace and
    with the levels inside x."""
    rng = np.random.default_rng(900 + n)
    y = _mixed_rows(rng, 6, n)
    g = rng.normal(size=y.shape).astype(np.float32)
    a = _check(y, np.array([lam], np.float32), 1, g, -1, "ws n=%d lam=%g" % (n, lam), use_ws=True)
    b = _check(y, np.array([lam], np.float32), 1, g, -1, "plain n=%d lam=%g" % (n, lam))
    assert a["max_steps"] <= 8 and np.array_equal(a["steps"], b["steps"])
    assert a["fwd_max_err"] <= 0.5 * FWD_TOL


@pytest.mark.parametrize("n,fac", [(5000, 0.3), (5000, 1.0), (12000, 1.0), (12000, 3.0), (16384, 3.0)])
@pytest.mark.parametrize("layout", ["in place", "strided"])
def test_cold_long_rows_with_lambda_of_the_order_of_lam_max(n, fac, layout):
    """Long rows that cannot take the multilevel start (a call in place, strided rows) start cold
    with two candidates: every dual on the bound its local difference points to, or the clipped
    dual of the constant row, which is the solution from lam_max on.  Random-walk rows with
    lambda = 0.3-3 lam_max ran into the step cap from the first candidate alone."""
    rng = np.random.default_rng(4000 + n)
    rows = 4
    y = np.cumsum(0.05 * rng.normal(size=(rows, n)), axis=-1).astype(np.float32)
    lmax = np.abs(np.cumsum(y.mean(1, keepdims=True) - y.astype(np.float64), axis=1)).max(1)
    lam = (fac * lmax).astype(np.float32)
    g = rng.normal(size=y.shape).astype(np.float32)
    if layout == "in place":
        st = _check(y, lam, 1, g, -1, "in place n=%d fac=%g" % (n, fac), in_place=True)
    else:
        st = _check(np.ascontiguousarray(y.T), lam, 1, np.ascontiguousarray(g.T), 0, "strided n=%d fac=%g" % (n, fac))
    assert st["max_steps"] <= (100 if fac < 1 else 20)


def test_noise_rows_with_lambda_near_lam_max():
    """Noise-like long rows with lambda a third of their lam_max are the worst case of the cold
    start (every dual on the bound its local difference points to): dozens of Newton steps.
    Strided, so that no multilevel start helps; they must still converge below the cap."""
    rng = np.random.default_rng(2561)
    n, rows = 2561, 12
    y = (0.3 * rng.normal(size=(n, rows))).astype(np.float32)
    g = rng.normal(size=y.shape).astype(np.float32)
    pre = np.cumsum(y.mean(0, keepdims=True) - y, axis=0)
    lam = (np.abs(pre).max(0) / 3.2).astype(np.float32)
    st = _check(y, lam, 1, g, 0, "noise rows, lam near lam_max")
    assert st["max_steps"] <= 128


def test_multilevel_degenerate_rows():
    """Constant rows, a row of exactly the minimum length, a single row, lambda = 0 and a lambda so
    large that the whole row is one segment, all through the workspace path."""
    rng = np.random.default_rng(3)
    n = 2048
    y = np.stack([np.full(n, 1.5, np.float32), rng.normal(size=n).astype(np.float32),
                  np.cumsum(rng.normal(scale=0.1, size=n)).astype(np.float32),
                  np.repeat(rng.normal(size=n // 64), 64).astype(np.float32)])
    g = rng.normal(size=y.shape).astype(np.float32)
    _check(y, np.array([0.7, 0.0, 1e4, 0.25], np.float32), 1, g, -1, "ml degenerate", use_ws=True)
    _check(y[2:3], np.array([2.0], np.float32), 1, g[2:3], -1, "ml single row", use_ws=True)


def test_multilevel_per_channel_lambda_and_strided_rows():
    """Rows inside a larger buffer (row stride > length), lambda shared by groups of rows."""
    rng = np.random.default_rng(77)
    n, rows = 2500, 10
    buf = np.zeros((rows, 2600), np.float32)
    buf[:, :n] = _mixed_rows(rng, rows, n)
    import torch
    import paper_2204_03643_amd as tv
    dev = torch.device("cuda:0")
    lam = np.array([3.0, 0.02, 0.8], np.float32)
    yt, lt = torch.from_numpy(buf).to(dev), torch.from_numpy(lam).to(dev)
    xt = torch.full_like(yt, float("nan"))
    r = tv.tv_rows(1, 0, rows, 2600, n, 1)
    L = tv.tv_lambda(lt.data_ptr(), 3, 2)
    wsb = tv.tv1d_fwd_workspace_bytes(r, L)
    assert wsb > 0
    ws = torch.full((wsb,), 0xff, dtype=torch.uint8, device=dev)
    tv.tv1d_prox_fwd_ex(yt, xt, r, L, ws=ws, ws_bytes=wsb)
    torch.cuda.synchronize()
    x = xt.cpu().numpy()
    assert np.isnan(x[:, n:]).all()
    lr = lam[(np.arange(rows) // 2) % 3]
    x_ref = oracle.prox1d_batch(buf[:, :n].astype(np.float64), lr.astype(np.float64))
    err = forward_errors(x[:, :n], x_ref, buf[:, :n])
    assert err.max() <= FWD_TOL, err


@pytest.mark.parametrize("n,width", [(40, 37), (64, 16), (90, 33), (130, 17), (200, 20), (300, 18), (512, 48), (700, 17),
                                          (1000, 20), (1024, 16), (1500, 9), (2000, 9), (2600, 5), (4096, 6), (9000, 3),
                                          (12000, 2)])
def test_long_columns(n, width):
    rng = np.random.default_rng(600 + n)
    y = np.stack([_mixed_rows(rng, width, n).T for _ in range(2)])        # [2, n, width]
    g = rng.normal(size=y.shape).astype(np.float32)
    lam = np.array([0.08, 1.3], np.float32)
    _check(y, lam, width, g, -2, "cols n=%d" % n)


def test_config5_reduced():
    y, lam, g = workloads.config5(rows=24, n=16384)
    st = _check(y, lam, 1, g, -1, "cfg5 reduced")
    assert st["max_steps"] <= 48


def test_config4_single_passes():
    y, lam, g = workloads.config4(B=1, C=2, H=512, W=512, n_poly=6)
    _check(y, lam, 1, g, -1, "cfg4 rows")
    _check(y, lam, 1, g, -2, "cfg4 columns")


def test_long_lambda_extremes_and_in_place():
    rng = np.random.default_rng(47)
    y = _mixed_rows(rng, 6, 700)
    g = rng.normal(size=y.shape).astype(np.float32)
    out = run_1d(y, np.array([0.0], np.float32), 1, g)
    assert np.array_equal(out["x"], y) and np.array_equal(out["gy"], g)
    out = run_1d(y, np.array([1e5], np.float32), 1, g)
    np.testing.assert_allclose(out["x"], np.repeat(y.astype(np.float64).mean(1, keepdims=True), 700, 1),
                               atol=1e-4 * (1 + np.abs(y).max()))
    assert np.all(out["x"] == out["x"][:, :1])
    assert out["gl"][0] == 0.0
    lam = np.array([0.3], np.float32)
    a = run_1d(y, lam, 1)
    b = run_1d(y, lam, 1, in_place=True)
    assert np.array_equal(a["x"], b["x"])


def test_long_constant_and_tied_rows():
    n = 400
    y = np.zeros((5, n), np.float32)
    y[1] = -2.5
    y[2, n // 2:] = 1.0
    y[3] = np.tile([0.0, 1.0], n // 2)
    y[4] = np.round(np.random.default_rng(48).normal(size=n) * 2) / 2
    g = np.random.default_rng(49).normal(size=y.shape).astype(np.float32)
    lam = np.array([0.25], np.float32)
    out = run_1d(y, lam, 1, g, want_info=True)
    x_ref = oracle.prox1d_batch(y.astype(np.float64), lam.astype(np.float64))
    assert forward_errors(out["x"], x_ref, y).max() <= FWD_TOL
    assert not np.any(out["info"] & (1 << 18))


@pytest.mark.parametrize("n,axis", [(100, -1), (100, 0), (700, -1), (700, 0), (5000, -1)])
def test_nan_row_stays_in_its_row(n, axis):
    """A row with a non-finite sample gets unspecified values; its neighbours (several rows share
    a wave or a workgroup) are solved as usual and the call terminates."""
    rng = np.random.default_rng(45 + n)
    rows = 21
    y = _mixed_rows(rng, rows, n)
    y[5, n // 3] = np.nan
    y[17, n - 1] = np.inf
    ya = y if axis == -1 else np.ascontiguousarray(y.T)
    out = run_1d(ya, np.array([0.3], np.float32), 1, axis=axis)
    x = out["x"] if axis == -1 else out["x"].T
    assert np.isnan(x[5, n // 3]) and not np.isfinite(x[17, n - 1])
    ok = np.delete(np.arange(rows), [5, 17])
    x_ref = oracle.prox1d_batch(y[ok].astype(np.float64), np.array([0.3]))
    assert forward_errors(x[ok], x_ref, y[ok]).max() <= FWD_TOL

