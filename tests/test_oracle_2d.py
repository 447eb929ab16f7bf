"""Pins for the oracle's 2D path: K sweeps of paper Alg. 1 and the reverse sweep.

The 2D result is a composition of pinned 1D pieces; what is checked here is the
composition itself: K=1 is rows-then-columns, mass is conserved, lam=0 is the
identity, the Eq. 2 objective decreases towards the optimum of Eq. 2 (computed by
a library optimiser on the dual) as K grows, and the reverse sweep agrees with
finite differences of the forward sweep.
"""
import numpy as np
from scipy.optimize import minimize

import oracle
from refmath import tv2d_objective


def test_k1_is_rows_then_columns():
    rng = np.random.default_rng(21)
    y = rng.normal(size=(2, 3, 7, 9))
    lam = np.array([0.2, 0.7, 1.5])
    x, saved = oracle.prox2d_fwd(y, lam, sweeps=1)
    z = oracle.prox1d_batch(y, lam, axis=-1, lam_div=7)
    x_ref = oracle.prox1d_batch(z, lam, axis=-2, lam_div=9)
    np.testing.assert_array_equal(x, x_ref)
    np.testing.assert_array_equal(saved[0], z)
    np.testing.assert_array_equal(saved[1], x_ref)


def test_mass_and_identity():
    rng = np.random.default_rng(22)
    y = rng.normal(size=(4, 6, 5))
    lam = np.array([0.3])
    for K in (1, 3, 6):
        x, _ = oracle.prox2d_fwd(y, lam, sweeps=K)
        np.testing.assert_allclose(x.sum(axis=(-1, -2)), y.sum(axis=(-1, -2)), atol=1e-11)
    x0, _ = oracle.prox2d_fwd(y, np.array([0.0]), sweeps=4)
    np.testing.assert_array_equal(x0, y)


def _solve_eq2_dual(Y, lam):
    """Library solve of the dual of paper Eq. 2 on a tiny grid."""
    H, W = Y.shape
    n = H * W
    eye = np.eye(n).reshape(n, H, W)
    Dr = np.diff(eye, axis=2).reshape(n, -1).T        # row differences
    Dc = np.diff(eye, axis=1).reshape(n, -1).T        # column differences
    D = np.vstack([Dr, Dc])
    yv = Y.ravel()

    def negphi(u):
        r = D.T @ u
        return 0.5 * r @ r - u @ (D @ yv), D @ r - D @ yv

    res = minimize(negphi, np.zeros(D.shape[0]), jac=True, method="L-BFGS-B",
                   bounds=[(-lam, lam)] * D.shape[0],
                   options={"maxiter": 50000, "ftol": 1e-16, "gtol": 1e-12})
    return (yv - D.T @ res.x).reshape(H, W)


def test_objective_decreases_to_the_eq2_optimum():
    rng = np.random.default_rng(23)
    Y = rng.normal(size=(5, 6))
    lam = 0.4
    x_star = _solve_eq2_dual(Y, lam)
    f_star = tv2d_objective(x_star, Y, lam)
    prev = np.inf
    for K in (1, 2, 4, 10, 50, 400):
        x, _ = oracle.prox2d_fwd(Y, np.array([lam]), sweeps=K)
        f = tv2d_objective(x, Y, lam)
        assert f <= prev + 1e-12
        assert f >= f_star - 1e-6      # the library solve is itself only ~1e-7 accurate
        prev = f
    assert prev - f_star < 1e-6
    assert np.max(np.abs(x - x_star)) < 1e-3


def test_reverse_sweep_matches_finite_differences():
    rng = np.random.default_rng(24)
    planes, H, W, K = 2, 6, 7, 4
    y = rng.normal(size=(planes, H, W))
    lam = np.array([0.25, 0.6])
    g = rng.normal(size=y.shape)
    x, saved = oracle.prox2d_fwd(y, lam, sweeps=K)
    gy, gl = oracle.prox2d_bwd(g, saved, lam_count=2, sweeps=K)
    h = 1e-6

    def loss(yy, ll):
        return float(np.sum(g * oracle.prox2d_fwd(yy, ll, sweeps=K)[0]))

    idx = [(p, i, j) for p in range(planes) for i in range(H) for j in range(W)]
    for t in rng.choice(len(idx), size=30, replace=False):
        e = np.zeros_like(y)
        e[idx[t]] = h
        fd = (loss(y + e, lam) - loss(y - e, lam)) / (2 * h)
        assert abs(fd - gy[idx[t]]) < 2e-6, (idx[t], fd, gy[idx[t]])
    for s in range(2):
        e = np.zeros(2)
        e[s] = h
        fd = (loss(y, lam + e) - loss(y, lam - e)) / (2 * h)
        assert abs(fd - gl[s]) < 2e-6 * (1 + abs(gl[s]))


def test_reverse_sweep_k1_composition():
    rng = np.random.default_rng(25)
    y = rng.normal(size=(3, 5, 4))
    lam = np.array([0.3])
    g = rng.normal(size=y.shape)
    x, saved = oracle.prox2d_fwd(y, lam, sweeps=1)
    gy, gl = oracle.prox2d_bwd(g, saved, lam_count=1, sweeps=1)
    gb, gl_c = oracle.prox1d_bwd_batch(g, saved[1], lam_count=1, axis=-2, lam_div=4)
    ga, gl_r = oracle.prox1d_bwd_batch(gb, saved[0], lam_count=1, axis=-1, lam_div=5)
    np.testing.assert_allclose(gy, ga, atol=1e-14)
    np.testing.assert_allclose(gl, gl_c + gl_r, atol=1e-12)
