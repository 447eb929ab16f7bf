"""Pins for the CPU oracle's 1D forward and backward (no GPU needed).

The oracle has no implementation to compare against, so it is pinned by what the
paper's Eq. 1 / Eq. 3 / Eq. 5-6 and the mathematics fix: hand-worked cases,
brute force over sign patterns, closed forms, invariances, a duality-gap
certificate, a bound-constrained solve of the dual by a library optimiser, the
dense form of the backward formula, and finite differences.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy.optimize import minimize

import oracle
import workloads
from refmath import (brute_force_prox1d, certificate, dense_backward, lam_max,
                     tv1d_objective)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tv1d_hand_cases.txt")


def _golden_cases():
    out = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            lam, y, x = [p.strip() for p in line.split("|")]
            out.append((float(Fraction(lam)),
                        np.array([float(Fraction(t)) for t in y.split()]),
                        np.array([float(Fraction(t)) for t in x.split()])))
    return out


@pytest.mark.parametrize("lam,y,x", _golden_cases())
def test_hand_worked_cases(lam, y, x):
    np.testing.assert_allclose(oracle.prox1d(y, lam), x, rtol=0, atol=1e-14)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6, 7, 8])
def test_brute_force_small(n):
    rng = np.random.default_rng(100 + n)
    worst = 0.0
    for trial in range(60):
        y = rng.normal(size=n) * rng.choice([0.1, 1.0, 5.0])
        if trial % 5 == 0:
            y = np.round(y)              # ties and exact zeros in the input
        lam = float(rng.choice([0.0, 1e-3, 0.05, 0.3, 1.0, 3.0]) * rng.uniform(0.5, 1.5))
        x = oracle.prox1d(y, lam)
        xb = brute_force_prox1d(y, lam)
        worst = max(worst, float(np.max(np.abs(x - xb))))
    assert worst < 1e-12


def test_brute_force_n10_few():
    rng = np.random.default_rng(7)
    for _ in range(3):
        y = rng.normal(size=10)
        lam = float(rng.uniform(0.1, 1.0))
        assert np.max(np.abs(oracle.prox1d(y, lam) - brute_force_prox1d(y, lam))) < 1e-12


def test_closed_form_n2_soft_threshold():
    rng = np.random.default_rng(1)
    for _ in range(200):
        y = rng.normal(size=2) * 3
        lam = float(rng.uniform(0, 3))
        d = y[1] - y[0]
        ds = np.sign(d) * max(abs(d) - 2 * lam, 0.0)
        m = y.mean()
        np.testing.assert_allclose(oracle.prox1d(y, lam), [m - ds / 2, m + ds / 2], atol=1e-14)


def test_lambda_zero_is_identity():
    # paper Sec. 3.1: with lam = 0 the layer is the identity
    rng = np.random.default_rng(2)
    for n in (1, 2, 5, 33, 1000):
        y = rng.normal(size=n)
        assert np.array_equal(oracle.prox1d(y, 0.0), y)


def test_lambda_max_threshold():
    rng = np.random.default_rng(3)
    for n in (2, 3, 17, 64, 500):
        y = rng.normal(size=n)
        lm = lam_max(y)
        x = oracle.prox1d(y, lm * (1 + 1e-12) + 1e-15)
        np.testing.assert_allclose(x, np.full(n, y.mean()), atol=1e-12)
        x2 = oracle.prox1d(y, 0.999 * lm)
        assert np.ptp(x2) > 0
        x3 = oracle.prox1d(y, 50.0 * lm + 1.0)
        np.testing.assert_allclose(x3, np.full(n, y.mean()), atol=1e-12)


def test_invalid_arguments():
    with pytest.raises(ValueError):
        oracle.prox1d(np.zeros(4), -1.0)
    with pytest.raises(ValueError):
        oracle.prox1d(np.zeros(4), float("nan"))
    with pytest.raises(ValueError):
        oracle.prox1d(np.zeros(4), float("inf"))


def _rows_for_certificate():
    y1, l1, _ = workloads.config1(rows=6, n=256)
    y2, l2, _ = workloads.config2(B=1, C=4, H=8, W=32)
    y3, l3, _ = workloads.config3(B=1, C=8, H=4, W=32)
    y4, l4, _ = workloads.config4(B=1, C=1, H=64, W=512, n_poly=4)
    y5, l5, _ = workloads.config5(rows=6, n=16384)
    rows = [(r, float(l1[0])) for r in y1]
    rows += [(y2[0, c, h], float(l2[c])) for c in range(4) for h in range(8)]
    rows += [(y3[0, c, h], float(l3[c])) for c in range(8) for h in range(4)]
    rows += [(y4[0, 0, h], float(l4[0])) for h in range(0, 64, 8)]
    rows += [(y5[r], float(l5[r])) for r in range(6)]
    rows += [(y4[0, 0, :, w].copy(), float(l4[0])) for w in (0, 100)]
    return rows


def test_certificate_on_workload_rows():
    """Duality gap ~ rounding on rows from every workload distribution."""
    for y, lam in _rows_for_certificate():
        y = y.astype(np.float64)
        x = oracle.prox1d(y, lam)
        gap, resid, viol = certificate(x, y, lam)
        scale = 1.0 + tv1d_objective(x, y, lam)
        assert abs(resid) < 1e-9 * (1 + np.abs(y).sum())       # sum(x) = sum(y)
        assert viol < 1e-9 * (1 + lam)
        assert gap < 1e-10 * scale, (gap, scale, y.size, lam)


def test_sum_preserved_and_range():
    rng = np.random.default_rng(5)
    for _ in range(50):
        n = int(rng.integers(2, 200))
        y = rng.normal(size=n)
        lam = float(10 ** rng.uniform(-3, 1))
        x = oracle.prox1d(y, lam)
        assert abs(x.sum() - y.sum()) < 1e-10 * n
        assert x.min() >= y.min() - 1e-12 and x.max() <= y.max() + 1e-12


def test_invariances():
    rng = np.random.default_rng(6)
    for _ in range(30):
        n = int(rng.integers(2, 120))
        y = rng.normal(size=n)
        lam = float(10 ** rng.uniform(-2, 0.5))
        x = oracle.prox1d(y, lam)
        c, a = 3.7, 2.5
        np.testing.assert_allclose(oracle.prox1d(y + c, lam), x + c, atol=1e-11)
        np.testing.assert_allclose(oracle.prox1d(a * y, a * lam), a * x, atol=1e-11)
        np.testing.assert_allclose(oracle.prox1d(-y, lam), -x, atol=1e-11)
        np.testing.assert_allclose(oracle.prox1d(y[::-1].copy(), lam), x[::-1], atol=1e-11)
        y2 = y + 0.1 * rng.normal(size=n)
        x2 = oracle.prox1d(y2, lam)
        assert np.linalg.norm(x - x2) <= np.linalg.norm(y - y2) + 1e-12     # non-expansive


def test_segment_count_monotone_in_lambda():
    rng = np.random.default_rng(8)
    y = rng.normal(size=300)
    prev = None
    for lam in np.geomspace(1e-3, 30, 25):
        nseg = 1 + int(np.count_nonzero(np.diff(oracle.prox1d(y, float(lam)))))
        if prev is not None:
            assert nseg <= prev
        prev = nseg


def test_dual_qp_by_library_optimiser():
    """Second opinion: solve paper Eq. 3 (the box-constrained dual) with L-BFGS-B and
    recover x = y - D^T u."""
    rng = np.random.default_rng(9)
    for n, lam in ((12, 0.4), (25, 1.0), (40, 0.15)):
        y = rng.normal(size=n)
        D = np.diff(np.eye(n), axis=0)

        def negphi(u):
            r = D.T @ u
            return 0.5 * r @ r - u @ (D @ y), D @ r - D @ y

        res = minimize(negphi, np.zeros(n - 1), jac=True, method="L-BFGS-B",
                       bounds=[(-lam, lam)] * (n - 1),
                       options={"maxiter": 20000, "ftol": 1e-16, "gtol": 1e-12})
        x_qp = y - D.T @ res.x
        assert np.max(np.abs(oracle.prox1d(y, lam) - x_qp)) < 1e-5


# ------------------------------------------------------------------ backward


def _nondegenerate(y, lam, margin=1e-3):
    x = oracle.prox1d(y, lam)
    u = np.cumsum(x - y)[:-1]
    dx = np.diff(x)
    jumps = dx != 0
    ok = True
    if np.any(jumps):
        ok &= np.min(np.abs(dx[jumps])) > margin
    if np.any(~jumps):
        ok &= np.min(lam - np.abs(u[~jumps])) > margin
    return ok


def test_backward_matches_dense_formula():
    """Eq. 5-6 with explicit L matrices equals the segment form, n <= 12."""
    rng = np.random.default_rng(11)
    for _ in range(60):
        n = int(rng.integers(1, 13))
        y = rng.normal(size=n)
        lam = float(10 ** rng.uniform(-2, 0.7))
        g = rng.normal(size=n)
        x = oracle.prox1d(y, lam)
        gy, gl = oracle.prox1d_bwd(g, x)
        gy_d, gl_d = dense_backward(x, g)
        np.testing.assert_allclose(gy, gy_d, atol=1e-12)
        assert abs(gl - gl_d) < 1e-12


def test_backward_matches_finite_differences():
    rng = np.random.default_rng(12)
    checked = 0
    for _ in range(200):
        n = int(rng.integers(2, 40))
        y = rng.normal(size=n)
        lam = float(10 ** rng.uniform(-1.5, 0.5))
        if not _nondegenerate(y, lam):
            continue
        g = rng.normal(size=n)
        x = oracle.prox1d(y, lam)
        gy, gl = oracle.prox1d_bwd(g, x)
        h = 1e-6
        fd = np.empty(n)
        for i in range(n):
            e = np.zeros(n)
            e[i] = h
            fd[i] = g @ (oracle.prox1d(y + e, lam) - oracle.prox1d(y - e, lam)) / (2 * h)
        fdl = g @ (oracle.prox1d(y, lam + h) - oracle.prox1d(y, lam - h)) / (2 * h)
        np.testing.assert_allclose(gy, fd, atol=1e-7)
        assert abs(gl - fdl) < 1e-7
        checked += 1
    assert checked > 100


def test_backward_special_cases():
    rng = np.random.default_rng(13)
    y = rng.normal(size=50)
    g = rng.normal(size=50)
    gy, gl = oracle.prox1d_bwd(g, oracle.prox1d(y, 0.0))
    # lam = 0: every sample is its own segment (continuous input) -> identity Jacobian
    np.testing.assert_allclose(gy, g, atol=0)
    gy, gl = oracle.prox1d_bwd(g, oracle.prox1d(y, 2 * lam_max(y)))
    np.testing.assert_allclose(gy, np.full(50, g.mean()), atol=1e-14)
    assert gl == 0.0


def test_backward_is_an_orthogonal_projector():
    rng = np.random.default_rng(14)
    y = rng.normal(size=80)
    x = oracle.prox1d(y, 0.3)
    a, b = rng.normal(size=80), rng.normal(size=80)
    pa, _ = oracle.prox1d_bwd(a, x)
    pb, _ = oracle.prox1d_bwd(b, x)
    ppa, _ = oracle.prox1d_bwd(pa, x)
    np.testing.assert_allclose(ppa, pa, atol=1e-13)
    assert abs(pa.sum() - a.sum()) < 1e-12
    assert abs(pa @ b - a @ pb) < 1e-12


# ------------------------------------------------------------------ batched layouts


def test_batch_layouts_and_lambda_slots():
    rng = np.random.default_rng(15)
    y = rng.normal(size=(3, 4, 6, 5))
    lam = np.array([0.1, 0.5, 1.0, 2.0])
    g = rng.normal(size=y.shape)
    # rows along W, per-channel lam: row id = ((b*4 + c)*6 + h), slot = (id // 6) % 4
    xr = oracle.prox1d_batch(y, lam, axis=-1, lam_div=6)
    gyr, glr = oracle.prox1d_bwd_batch(g, xr, lam_count=4, axis=-1, lam_div=6)
    # columns along H: row id = ((b*4 + c)*5 + w), slot = (id // 5) % 4
    xc = oracle.prox1d_batch(y, lam, axis=-2, lam_div=5)
    gyc, glc = oracle.prox1d_bwd_batch(g, xc, lam_count=4, axis=-2, lam_div=5)
    glr_ref = np.zeros(4)
    glc_ref = np.zeros(4)
    for b in range(3):
        for c in range(4):
            for h in range(6):
                np.testing.assert_array_equal(xr[b, c, h], oracle.prox1d(y[b, c, h], lam[c]))
                gy1, gl1 = oracle.prox1d_bwd(g[b, c, h], xr[b, c, h])
                np.testing.assert_array_equal(gyr[b, c, h], gy1)
                glr_ref[c] += gl1
            for w in range(5):
                np.testing.assert_array_equal(xc[b, c, :, w], oracle.prox1d(y[b, c, :, w], lam[c]))
                gy1, gl1 = oracle.prox1d_bwd(g[b, c, :, w], xc[b, c, :, w])
                np.testing.assert_array_equal(gyc[b, c, :, w], gy1)
                glc_ref[c] += gl1
    np.testing.assert_allclose(glr, glr_ref, atol=1e-12)
    np.testing.assert_allclose(glc, glc_ref, atol=1e-12)
    # per-row lam
    lam_rows = rng.uniform(0.01, 1, size=3 * 4 * 6)
    xp = oracle.prox1d_batch(y, lam_rows, axis=-1, lam_div=1)
    np.testing.assert_array_equal(xp[1, 2, 3], oracle.prox1d(y[1, 2, 3], lam_rows[(1 * 4 + 2) * 6 + 3]))
