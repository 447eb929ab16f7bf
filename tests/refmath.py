"""Independent mathematical checks used to pin the oracle (and, in the GPU tests, to
certify outputs at sizes where running the oracle everywhere is too slow).

Nothing here is shared with oracle/ or with the HIP path: brute force over sign
patterns, the duality-gap certificate, the dense form of paper Eq. 5-6, and the
objective functions of paper Eq. 1 and Eq. 2, written out directly in numpy.
"""
from __future__ import annotations

import itertools

import numpy as np


def tv1d_objective(x, y, lam):
    """Paper Eq. 1 objective."""
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    return 0.5 * np.sum((x - y) ** 2) + lam * np.sum(np.abs(np.diff(x)))


def tv2d_objective(X, Y, lam):
    """Paper Eq. 2 objective (anisotropic: row differences + column differences)."""
    X = np.asarray(X, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    return (0.5 * np.sum((X - Y) ** 2)
            + lam * (np.sum(np.abs(np.diff(X, axis=-1))) + np.sum(np.abs(np.diff(X, axis=-2)))))


def brute_force_prox1d(y, lam):
    """Exact minimiser of Eq. 1 for tiny n by enumeration.

    For a fixed pattern s in {-1,0,+1}^(n-1) of jump signs the stationarity
    conditions give x in closed form: on each maximal run [a..b] without a jump,
    x = mean(y[a..b]) + lam*(s_b - s_{a-1})/(b-a+1) with s outside the row = 0.
    Every candidate is a feasible primal point and the true minimiser is one of
    them, so the candidate with the smallest objective is the answer."""
    y = np.asarray(y, dtype=np.float64)
    n = y.size
    if n == 1:
        return y.copy()
    best, best_x = np.inf, None
    for s in itertools.product((-1.0, 0.0, 1.0), repeat=n - 1):
        x = np.empty(n)
        a = 0
        while a < n:
            b = a
            while b < n - 1 and s[b] == 0.0:
                b += 1
            s_left = s[a - 1] if a > 0 else 0.0
            s_right = s[b] if b < n - 1 else 0.0
            x[a:b + 1] = y[a:b + 1].mean() + lam * (s_right - s_left) / (b - a + 1)
            a = b + 1
        f = tv1d_objective(x, y, lam)
        if f < best:
            best, best_x = f, x
    return best_x


def certificate(x, y, lam):
    """Duality-gap certificate for a candidate x of Eq. 1 (any n).

    With u = cumsum(x - y) (the dual that reproduces x through x = y - D^T u),
    clipped into the box |u| <= lam, the dual value of paper Eq. 3 is a lower
    bound of the optimum; strong convexity gives ||x - x*||^2 <= 2*gap.
    Returns (gap, sum_residual, max_box_violation)."""
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    u_full = np.cumsum(x - y)
    u = u_full[:-1]
    viol = max(0.0, float(np.max(np.abs(u)) - lam)) if u.size else 0.0
    uc = np.clip(u, -lam, lam)
    # D^T u: (D^T u)_j = u_{j-1} - u_j with zero padding at both ends
    dtu = np.concatenate(([0.0], uc)) - np.concatenate((uc, [0.0]))
    dual = -0.5 * np.sum(dtu ** 2) + np.sum(uc * np.diff(y))
    primal = tv1d_objective(x, y, lam)
    return float(primal - dual), float(u_full[-1]), viol


def dense_backward(x, g_up):
    """Paper Eq. 5-6 with explicit matrices (small n only).

    L = lower-triangular all-ones; the selected columns are column 0 (constant)
    plus column k+1 for every jump between k and k+1; M = L_S (L_S^T L_S)^-1;
    dx/dy = M L_S^T, dx/dlam = -M sign(Dx)_S (the constant column's sign is 0)."""
    x = np.asarray(x, dtype=np.float64)
    g = np.asarray(g_up, dtype=np.float64)
    n = x.size
    L = np.tril(np.ones((n, n)))
    dx = np.diff(x)
    cols = [0] + [k + 1 for k in range(n - 1) if dx[k] != 0.0]
    sg = np.array([0.0] + [np.sign(dx[k]) for k in range(n - 1) if dx[k] != 0.0])
    Ls = L[:, cols]
    M = Ls @ np.linalg.inv(Ls.T @ Ls)
    J = M @ Ls.T
    dlam = -M @ sg
    return J.T @ g, float(dlam @ g)


def lam_max(y):
    """Smallest lam for which the minimiser of Eq. 1 is the constant mean(y)."""
    y = np.asarray(y, dtype=np.float64)
    return float(np.max(np.abs(np.cumsum(y - y.mean())[:-1]))) if y.size > 1 else 0.0
