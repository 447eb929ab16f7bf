"""GPU parity on rows with one sample far larger than the rest.  The rounding floor of the solve
follows the row's largest sample, so the small segments elsewhere in the row carry noise that is
large next to their own values; the outputs must still be bit-constant on the oracle's segments
(the parity rules of every other test), in every mapping of rows to threads."""
import numpy as np
import pytest

from gpuutil import lam_per_row, run_1d
from parity import check_batch

pytestmark = pytest.mark.gpu


def _rows(n, rows, amp, seed):
    rng = np.random.default_rng(seed)
    y = rng.normal(scale=0.05, size=(rows, n)) + np.cumsum(rng.normal(scale=0.02, size=(rows, n)), axis=-1)
    k = rng.integers(0, n, size=rows)
    y[np.arange(rows), k] += amp * rng.choice([-1.0, 1.0], size=rows)
    return y.astype(np.float32), rng.normal(size=(rows, n)).astype(np.float32)


@pytest.mark.parametrize("amp", [10.0, 100.0, 1000.0])
@pytest.mark.parametrize("n,rows,mapping", [(32, 4096, "lane per row"), (32, 4096, "library's choice"),
                                            (24, 3000, "lane per row"), (24, 3000, "library's choice"),
                                            (32, 3000, "eight threads per row"), (200, 2048, None), (512, 1024, None),
                                            (1500, 300, None), (3000, 256, None)])
def test_rows_with_one_large_sample(n, rows, mapping, amp):
    import paper_2204_03643_amd as tv
    y, g = _rows(n, rows, amp, 5 + n)
    saved = tv.tv_dispatch_thresholds()
    try:
        if mapping == "lane per row":
            tv.tv_dispatch_override("thread_per_sample_1d_rows", 0)
        elif mapping == "eight threads per row":
            tv.tv_dispatch_override("thread_per_sample_wide_rows", 0)
        for lam in (0.02, 0.3):
            lamv = np.array([lam], np.float32)
            out = run_1d(y, lamv, 1, g)
            check_batch(y, lam_per_row(lamv, rows, 1), g, out["x"], out["gy"], gl_gpu=out["gl"], lam_count=1,
                        lam_div=1, label="one sample of %g among samples of 0.1, n=%d, lam=%g" % (amp, n, lam))
    finally:
        for k, v in saved.items():
            tv.tv_dispatch_override(k, v)


@pytest.mark.parametrize("shape,K", [((40, 32, 32), 2), ((9, 64, 64), 2), ((6, 40, 56), 3), ((3, 200, 300), 2)])
def test_planes_with_a_few_large_samples(shape, K):
    """The 2D operator on planes that hold a few samples 100 times larger than the rest (small
    batches: a plane per workgroup; the last shape: pass by pass on the long-row kernels)."""
    from gpuutil import run_2d
    from parity import check_2d
    rng = np.random.default_rng(17 + shape[1])
    y = rng.normal(scale=0.05, size=shape) + np.cumsum(rng.normal(scale=0.02, size=shape), axis=-1)
    hot = rng.random(size=shape) < 0.002
    y = (y + hot * 10.0 * rng.choice([-1.0, 1.0], size=shape)).astype(np.float32)
    g = rng.normal(size=shape).astype(np.float32)
    lam = np.array([0.02, 0.3], np.float32)
    out = run_2d(y, lam, K, g)
    check_2d(y, lam, K, g, out, "hot samples %s K=%d" % (shape, K))
