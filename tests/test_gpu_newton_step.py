"""One projected-Newton step and the descent of the dual objective, checked from outside the
kernels (paper Eq. 3-4) through the step records of tv1d_prox_fwd_steps.

For each recorded row the test rebuilds, in float64 numpy, the gradient at the recorded starting
dual, and compares the recorded Newton direction d with (a) a dense solve of tridiag(-1, 2, -1)
restricted to the recorded free set and (b) the closed form on every free run: with s_j the running
sums of the run's gradient entries and C_j the running sums of s (C_0 = 0),
d_j = j C_m / (m + 1) - C_{j-1}.  Then: the recorded objective values never increase (up to the
Armijo slack of fp32), the duality gap of the returned x is at rounding level, and the bound set
is made of duals that sit exactly on +-lambda.  Row lengths cover the row-per-lane kernel (Thomas
recurrences with table pivots), a wavefront per row, and a workgroup per row with 256 and 1024
threads (chunk Thomas + parallel cyclic reduction over the chunk separators)."""
import numpy as np
import pytest

from refmath import certificate

pytestmark = pytest.mark.gpu


def _run(y, lam, lam_div=1):
    import torch

    import paper_2204_03643_amd as tv

    dev = torch.device("cuda:0")
    R, n = y.shape
    yt = torch.from_numpy(y).to(dev)
    lt = torch.from_numpy(np.ascontiguousarray(lam, dtype=np.float32)).to(dev)
    rows, L = tv.rows_along(y.shape, -1), tv.tv_lambda(lt.data_ptr(), lt.numel(), lam_div)
    per = tv.tv1d_fwd_steps_floats_per_row(n)
    assert per == 48 + 3 * n
    rec = torch.full((R, per), float("nan"), device=dev)
    info = torch.zeros(R, dtype=torch.int32, device=dev)
    x, x_ref = torch.empty_like(yt), torch.empty_like(yt)
    tv.tv1d_prox_fwd_steps(yt, x, info, rec, R, rows, L)
    tv.tv1d_prox_fwd(yt, x_ref, rows, L)
    torch.cuda.synchronize()
    return x.cpu().numpy(), x_ref.cpu().numpy(), rec.cpu().numpy(), info.cpu().numpy()


def _closed_form_direction(g, bound):
    """Newton direction run by run from the closed form; 0 on bound duals."""
    d = np.zeros_like(g)
    k, M = 0, g.size
    while k < M:
        if bound[k]:
            k += 1
            continue
        e = k
        while e < M and not bound[e]:
            e += 1
        s = np.cumsum(g[k:e])
        C = np.concatenate(([0.0], np.cumsum(s)))          # C_0 .. C_m
        m = e - k
        j = np.arange(1, m + 1)
        d[k:e] = j * C[m] / (m + 1) - C[j - 1]
        k = e
    return d


def _dense_direction(g, bound):
    free = np.flatnonzero(~bound)
    d = np.zeros_like(g)
    if free.size:
        M = g.size
        H = 2 * np.eye(M) - np.eye(M, k=1) - np.eye(M, k=-1)
        d[free] = np.linalg.solve(H[np.ix_(free, free)], g[free])
    return d


def _longest_free_run(bound):
    best = cur = 0
    for b in bound:
        cur = 0 if b else cur + 1
        best = max(best, cur)
    return best


@pytest.mark.parametrize("n,rows,noise", [(32, 96, 1.0), (20, 70, 1.0), (200, 12, 1.0), (512, 8, 1.0),
                                          (1500, 4, 1.0), (4096, 3, 1.0), (6000, 2, 1.0)])
def test_newton_direction_objective_descent_and_gap(n, rows, noise):
    rng = np.random.default_rng(1000 + n)
    y = rng.normal(scale=noise, size=(rows, n)).astype(np.float32)
    # lambdas around the sample-to-sample variation: a mix of bound and free duals with free
    # runs of a few to a few dozen duals
    lam = (10 ** rng.uniform(-1.0, 0.2, size=rows)).astype(np.float32)
    x, x_plain, rec, info = _run(y, lam)
    assert np.allclose(x, x_plain, atol=2e-6 * (1 + np.abs(y).max()))
    checked = 0
    for r in range(rows):
        q = rec[r]
        steps, l = int(q[0]), float(q[1])
        assert steps <= (info[r] & 0xffff), (n, r, steps, info[r])
        assert abs(l - lam[r]) <= 1e-6 * lam[r]
        u0 = q[48:48 + n - 1].astype(np.float64)
        bound = q[48 + 2 * n:48 + 3 * n - 1] != 0
        assert not np.any(np.isnan(q[48:48 + n - 1]))
        # a row whose start already passes the optimality test takes no step and records no direction
        took_step = (info[r] & 0xffff) >= 1
        assert took_step or steps == 0
        d_gpu = q[48 + n:48 + 2 * n - 1].astype(np.float64) if took_step else np.zeros(n - 1)
        assert not np.any(np.isnan(d_gpu))
        # bound duals sit exactly on the box, and the direction vanishes there
        assert np.all(np.abs(q[48:48 + n - 1][bound]) == np.float32(l))
        assert np.all(d_gpu[bound] == 0.0)
        # gradient of the dual objective at u0:  x = y - D^T u,  g_k = x_k - x_{k+1}
        y64 = y[r].astype(np.float64)
        ue = np.concatenate(([0.0], u0, [0.0]))
        x0 = y64 + ue[1:] - ue[:-1]
        g = x0[:-1] - x0[1:]
        # Bertsekas' bound set: on the bound and pushed outwards (wherever the sign is beyond rounding)
        tol = 16 * np.finfo(np.float32).eps * (np.abs(y64).max() + l)
        on_bound = np.abs(u0) == np.float64(np.float32(l))
        outward = np.sign(u0) * g < -tol
        inward = np.sign(u0) * g > tol
        assert np.all(bound[on_bound & outward]) and not np.any(bound[on_bound & inward])
        assert not np.any(bound & ~on_bound)
        # f at the start
        assert abs(q[8] - 0.5 * np.sum(x0 ** 2)) <= 1e-5 * (1 + 0.5 * np.sum(x0 ** 2))
        # the Newton direction
        run = _longest_free_run(bound)
        if run <= 64 and took_step:
            d_cf = _closed_form_direction(g, bound)
            d_dn = _dense_direction(g, bound)
            # (floor: the fp32 gradient carries rounding noise of x = y - D^T u, which a run of m
            # free duals amplifies by up to m + 1)
            floor = 16 * np.finfo(np.float32).eps * (np.abs(y64).max() + l) * (run + 1)
            scale = max(np.abs(d_dn).max(), 1e-30)
            assert np.abs(d_cf - d_dn).max() <= 1e-9 * scale + 1e-14         # the closed form itself
            assert np.abs(d_gpu - d_dn).max() <= 2e-4 * scale + floor, (n, r, run, np.abs(d_gpu - d_dn).max() / scale)
            checked += 1
        # the dual objective never increases (fp32: up to the Armijo slack of 4 eps |f|)
        f = q[8:8 + steps + 1].astype(np.float64)
        assert np.all(np.diff(f) <= 8 * np.finfo(np.float32).eps * np.abs(f[:-1]) + 1e-12), (n, r, f)
        # the returned x: duality gap at rounding level
        gap, resid, viol = certificate(x[r], y[r], float(lam[r]))
        fscale = 1.0 + 0.5 * np.sum(y64 ** 2)
        assert gap <= 2e-6 * fscale and abs(resid) <= 1e-4 * n ** 0.5 and viol <= 1e-5 * (1 + l), (n, r, gap, resid, viol)
    assert checked >= max(1, rows // 2), (n, checked)


def test_records_only_the_rows_asked_for_and_rejects_strided_long_rows():
    import torch

    import paper_2204_03643_amd as tv

    dev = torch.device("cuda:0")
    rng = np.random.default_rng(5)
    y = torch.from_numpy(rng.normal(size=(10, 40)).astype(np.float32)).to(dev)
    lt = torch.tensor([0.4], device=dev)
    rows, L = tv.rows_along((10, 40), -1), tv.tv_lambda(lt.data_ptr(), 1, 1)
    per = tv.tv1d_fwd_steps_floats_per_row(40)
    rec = torch.full((10, per), -7.0, device=dev)
    x = torch.empty_like(y)
    tv.tv1d_prox_fwd_steps(y, x, None, rec, 3, rows, L)
    torch.cuda.synchronize()
    assert bool((rec[3:] == -7.0).all()) and bool((rec[:3, 0] >= 1).all())
    with pytest.raises(tv.TVError) as e:
        tv.tv1d_prox_fwd_steps(y, x, None, rec, 3, tv.rows_along((40, 10), 0), L)    # columns of 40 samples
    assert e.value.status == 6
