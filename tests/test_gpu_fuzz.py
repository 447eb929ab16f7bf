"""Bounded, seeded random testing of the HIP path against the oracle: a few hundred 1D and 2D
shapes, lambda layouts, strides and entry-point flags drawn from a fixed seed, each under the
parity rules of parity.py.  Stops at the first failure and names the case."""
import numpy as np
import pytest

from gpuutil import lam_per_row, rows_view, run_1d, run_2d
from parity import check_2d, check_batch

pytestmark = pytest.mark.gpu


def _gen(rng, shape):
    kind = rng.integers(3)
    if kind == 0:                       # white noise
        return rng.normal(size=shape).astype(np.float32)
    if kind == 1:                       # random walk + noise: long segments
        return (np.cumsum(rng.normal(scale=0.1, size=shape), axis=-1)
                + rng.normal(scale=0.05, size=shape)).astype(np.float32)
    return np.maximum(rng.normal(size=shape), 0).astype(np.float32)      # half exact zeros: ties


def _case_1d(rng):
    nd = int(rng.integers(2, 4))
    n = int(rng.choice([rng.integers(1, 40), rng.integers(33, 700), rng.integers(769, 1600), rng.integers(2048, 2600)]))
    pos = int(rng.integers(0, nd))
    shape = [int(rng.integers(1, 7)) for _ in range(nd)]
    if rng.random() < 0.5:
        shape[0] = int(rng.integers(1, 40))
    if n <= 32 and rng.random() < 0.3:                  # several tiles of the row-per-lane kernels
        shape[0 if pos != 0 else nd - 1] = int(rng.integers(100, 400))
    shape[pos] = n
    shape, axis = tuple(shape), pos - nd
    y, g = _gen(rng, shape), rng.normal(size=shape).astype(np.float32)
    n_rows = y.size // n
    mode = rng.integers(3)
    if mode == 0:
        lam, div = np.array([10 ** rng.uniform(-3, 1)], np.float32), 1
    elif mode == 1:
        lam, div = (10 ** rng.uniform(-3, 1, size=n_rows)).astype(np.float32), 1
    else:
        div = int(rng.choice([1, 2, 3, 4, 8]))
        lam = (10 ** rng.uniform(-2, 0.5, size=int(rng.integers(1, 5)))).astype(np.float32)
    use_seg = bool(n <= 32 and rng.random() < 0.5)
    use_ws = bool(rng.random() < 0.5)
    label = "1d shape %s axis %d lam %d/%d seg %d ws %d" % (shape, axis, lam.size, div, use_seg, use_ws)
    return label, (y, lam, div, g, axis, use_seg, use_ws)


def _case_2d(rng):
    P, H, W = int(rng.integers(1, 6)), int(rng.integers(1, 90)), int(rng.integers(1, 90))
    if rng.random() < 0.4:
        H, W = int(rng.integers(1, 33)), int(rng.integers(1, 33))
    if rng.random() < 0.08:
        P, H, W = int(rng.integers(1000, 1100)), int(rng.integers(1, 33)), int(rng.integers(1, 33))
    if rng.random() < 0.03:
        P, H, W = int(rng.integers(4090, 4200)), int(rng.integers(1, 17)), int(rng.integers(1, 17))
    K = int(rng.integers(1, 5))
    y, g = _gen(rng, (P, H, W)), rng.normal(size=(P, H, W)).astype(np.float32)
    lam = (10 ** rng.uniform(-2, 0.3, size=int(rng.integers(1, min(P, 7) + 1)))).astype(np.float32)
    return "2d %dx%dx%d K=%d lam %d" % (P, H, W, K, lam.size), (y, lam, K, g)


# (seed 106 holds a plane whose x is one constant and whose mean upstream gradient cancels to 2.5e-6:
# the case behind the rounding floor of check_2d's grad_y rule)
@pytest.mark.parametrize("seed,cases", [(20220403, 120), (3643, 120), (106, 100)])
def test_seeded_random_cases(seed, cases):
    rng = np.random.default_rng(seed)
    n1 = n2 = 0
    for c in range(cases):
        if rng.random() < 0.6:
            label, (y, lam, div, g, axis, use_seg, use_ws) = _case_1d(rng)
            print("case %d: %s" % (c, label), flush=True)
            out = run_1d(y, lam, div, g, axis=axis, use_seg=use_seg, use_ws=use_ws)
            yr, gr = rows_view(y, axis), rows_view(g, axis)
            check_batch(yr, lam_per_row(lam, len(yr), div), gr, rows_view(out["x"], axis),
                        rows_view(out["gy"], axis), gl_gpu=out["gl"], lam_count=lam.size, lam_div=div,
                        label="seed %d case %d: %s" % (seed, c, label))
            n1 += 1
        else:
            label, (y, lam, K, g) = _case_2d(rng)
            print("case %d: %s" % (c, label), flush=True)
            check_2d(y, lam, K, g, run_2d(y, lam, K, g), "seed %d case %d: %s" % (seed, c, label))
            n2 += 1
    assert n1 > 0 and n2 > 0
