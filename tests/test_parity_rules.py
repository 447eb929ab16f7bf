"""The parity rules themselves, on the CPU: with the oracle's own results (rounded to fp32)
standing in for the HIP path they pass, and a mistake planted in that stand-in fails them."""
import numpy as np
import pytest

import oracle
from parity import check_2d, check_batch, dykstra_pass_inputs, near_degenerate


def _standin_2d(y, lam, K, g):
    x, saved = oracle.prox2d_fwd(y.astype(np.float64), lam.astype(np.float64), K)
    gy, gl = oracle.prox2d_bwd(g.astype(np.float64), saved, lam.size, K)
    return {"x": x.astype(np.float32), "saved": saved.astype(np.float32), "gy": gy.astype(np.float32),
            "gl": gl.astype(np.float32)}


def _case(seed=3, shape=(5, 12, 9), K=3):
    rng = np.random.default_rng(seed)
    y = rng.normal(size=shape).astype(np.float32)
    g = rng.normal(size=shape).astype(np.float32)
    lam = np.array([0.15, 0.6], np.float32)
    return y, lam, K, g


def test_pass_inputs_reproduce_alg1():
    y, lam, K, g = _case()
    y64 = y.astype(np.float64)
    _, saved = oracle.prox2d_fwd(y64, lam.astype(np.float64), K)
    ins = dykstra_pass_inputs(y64, saved)
    assert len(ins) == 2 * K and np.array_equal(ins[0], y64)
    # every pass output is the 1D prox of the rebuilt input along its axis
    lam_rows = np.repeat(lam.astype(np.float64)[np.arange(y.shape[0]) % 2], y.shape[1])
    z = oracle.prox1d_batch(ins[2].reshape(-1, y.shape[2]), lam_rows)
    np.testing.assert_allclose(z.reshape(y.shape), saved[2], atol=1e-12)


def test_check_2d_accepts_the_oracle_and_counts():
    y, lam, K, g = _case()
    st = check_2d(y, lam, K, g, _standin_2d(y, lam, K, g), "stand-in")
    assert st["pass_rows_checked"] + st["pass_rows_near_degenerate"] == 5 * (12 + 9) * K
    assert st["planes_without_near_degenerate_rows"] >= 1
    assert st["grad_max_rel"] < 1e-5 and st["grad_lam_slots_needing_floor"] == 0


def test_check_2d_rejects_a_spurious_micro_jump():
    """One sample of a constant run moved by one ulp in one saved pass (an output that is not
    bit-constant inside a segment): far below the forward tolerance, so only the segment rule
    can see it -- and it must, on any row that is not near-degenerate."""
    y, lam, K, g = _case()
    y64 = y.astype(np.float64)
    _, saved = oracle.prox2d_fwd(y64, lam.astype(np.float64), K)
    ins = dykstra_pass_inputs(y64, saved)
    i, p = 2, 1                                   # second sweep's row pass, plane 1
    deg = near_degenerate(saved[i][p], ins[i][p], np.full(y.shape[1], float(lam[p % 2])))
    out = _standin_2d(y, lam, K, g)
    row = out["saved"][i][p]
    for r in np.flatnonzero(~deg):
        runs = np.flatnonzero(np.diff(row[r]) == 0)
        if runs.size:
            k = runs[0]
            row[r, k + 1] = np.nextafter(row[r, k + 1], np.float32(np.inf))
            break
    else:
        pytest.skip("no ordinary row with a constant run in this pass")
    with pytest.raises(AssertionError, match="segments differ at an ordinary dual"):
        check_2d(y, lam, K, g, out, "planted")


def test_check_2d_rejects_wrong_gradients():
    y, lam, K, g = _case()
    out = _standin_2d(y, lam, K, g)
    bad = dict(out, gy=out["gy"].copy())
    bad["gy"][2, 3, 4] += 5e-3 * np.abs(out["gy"][2]).max()
    with pytest.raises(AssertionError, match="grad_y"):
        check_2d(y, lam, K, g, bad, "planted")
    bad = dict(out, gl=out["gl"] * np.float32(1.02))
    with pytest.raises(AssertionError, match="grad_lam"):
        check_2d(y, lam, K, g, bad, "planted")
    # a reverse sweep that forgets the correction terms (plain composition of the passes)
    g64 = g.astype(np.float64)
    _, saved = oracle.prox2d_fwd(y.astype(np.float64), lam.astype(np.float64), K)
    t = g64
    for i in range(2 * K - 1, -1, -1):
        t, _ = oracle.prox1d_bwd_batch(t, saved[i], axis=(-1 if i % 2 == 0 else -2))
    with pytest.raises(AssertionError, match="grad_y"):
        check_2d(y, lam, K, g, dict(out, gy=t.astype(np.float32)), "planted")


def test_check_batch_counts_floor_use():
    rng = np.random.default_rng(9)
    y = rng.normal(size=(400, 32)).astype(np.float32)
    g = rng.normal(size=y.shape).astype(np.float32)
    lam = (10 ** rng.uniform(-2, 0.5, size=400))
    x = oracle.prox1d_batch(y.astype(np.float64), lam)
    gy, gl = oracle.prox1d_bwd_batch(g.astype(np.float64), x, lam_count=4, lam_div=100)
    st = check_batch(y, lam, g, x.astype(np.float32), gy.astype(np.float32), gl_gpu=gl.astype(np.float32),
                     lam_count=4, lam_div=100)
    assert st["rows"] == 400 and st["grad_y_rows_needing_floor"] == 0 and st["grad_lam_slots_needing_floor"] == 0
    with pytest.raises(AssertionError, match="grad_y"):
        bad = gy.astype(np.float32)
        bad[7] *= 1.01
        check_batch(y, lam, g, x.astype(np.float32), bad)
