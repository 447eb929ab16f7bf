"""GPU parity at the full sizes of the benchmark workloads (the launch configurations the
benchmark times).  Forward results are compared with the oracle on every element (the C
oracle is fast enough); gradients on sampled rows under the parity rules of parity.py."""
import numpy as np
import pytest

import oracle
import workloads
from gpuutil import lam_per_row, rows_view, run_1d, run_2d
from parity import FWD_TOL, check_batch, forward_errors

pytestmark = pytest.mark.gpu


def _full_1d(y, lam, lam_div, g, axis, label, n_sample):
    out = run_1d(y, lam, lam_div, g, axis=axis, want_info=True)
    assert not np.any(out["info"] & (1 << 18)), label               # nobody hit the iteration cap
    assert np.count_nonzero(out["info"] & (1 << 19)) <= 1e-4 * out["info"].size, label
    yr, gr = rows_view(y, axis), rows_view(g, axis)
    xr, gyr = rows_view(out["x"], axis), rows_view(out["gy"], axis)
    lr = lam_per_row(lam, len(yr), lam_div)
    x_ref = oracle.prox1d_batch(yr.astype(np.float64), lr.astype(np.float64), axis=-1, lam_div=1)
    ferr = forward_errors(xr, x_ref, yr)
    assert ferr.max() <= FWD_TOL, (label, float(ferr.max()))
    rng = np.random.default_rng(len(yr))
    idx = np.sort(rng.choice(len(yr), size=min(n_sample, len(yr)), replace=False))
    st = check_batch(yr[idx], lr[idx], gr[idx], xr[idx], gyr[idx], label=label)
    # grad_lam against the oracle's per-row contributions on the GPU's own segments
    _, gl_ref = oracle.prox1d_bwd_batch(gr.astype(np.float64), xr.astype(np.float64),
                                        lam_count=np.asarray(lam).size, axis=-1, lam_div=lam_div)
    np.testing.assert_allclose(out["gl"], gl_ref, rtol=2e-4, atol=2e-2)
    return st


def test_config2_full():
    y, lam, g = workloads.config2()
    _full_1d(y, lam, 32, g, -1, "cfg2 rows", 5000)
    _full_1d(y, lam, 32, g, -2, "cfg2 columns", 5000)


def test_config3_full_columns():
    y, lam, g = workloads.config3()
    _full_1d(y, lam, 32, g, -2, "cfg3 columns", 5000)


def test_config4_full_forward_and_reduced_backward():
    y, lam, g = workloads.config4()
    out = run_2d(y, lam, 10)
    x_ref, _ = oracle.prox2d_fwd(y.astype(np.float64), lam.astype(np.float64), 10)
    err = np.abs(out["x"] - x_ref).max() / (1.0 + np.abs(y).max())
    assert err <= FWD_TOL, err
    # reverse sweep at full image size on two of the eight images
    y2, g2 = y[:2], g[:2]
    out = run_2d(y2, lam, 10, g2)
    gy_rep, gl_rep = oracle.prox2d_bwd(g2.astype(np.float64), out["saved"].astype(np.float64), 1, 10)
    assert np.abs(out["gy"] - gy_rep).max() <= 1e-4 * np.abs(gy_rep).max()
    assert abs(out["gl"][0] - gl_rep[0]) <= 1e-4 * (abs(gl_rep[0]) + np.sqrt(y2.size))


def test_config5_full():
    y, lam, g = workloads.config5()
    _full_1d(y, lam, 1, g, -1, "cfg5", 48)
