"""GPU parity for the 2D operator (paper Alg. 1) and its reverse sweep, under the rules of
parity.check_2d: forward and every saved pass element-wise against the oracle's K-sweep run;
in every pass the oracle's exact jump set and jump directions on every row that is not
near-degenerate; grad_y and grad_lam against the oracle's reverse sweep (its own segments,
except on near-degenerate rows)."""
import numpy as np
import pytest

import oracle
import workloads
from gpuutil import run_2d
from parity import check_2d

pytestmark = pytest.mark.gpu


def _check_2d(y, lam, K, g, label):
    out = run_2d(y, lam, K, g)
    st = check_2d(y, lam, K, g, out, label)
    # (kept from before: the reverse-sweep arithmetic alone, replayed by the oracle on the HIP
    # path's own pass outputs, to ten times the gradient bar)
    g64 = g.astype(np.float64)
    gy_rep, gl_rep = oracle.prox2d_bwd(g64, out["saved"].astype(np.float64), lam.size, K)
    assert np.abs(out["gy"] - gy_rep).max() <= 1e-4 * np.abs(gy_rep).max(), (label, "grad_y replay")
    assert np.all(np.abs(out["gl"] - gl_rep) <= 1e-4 * (np.abs(gl_rep) + np.sqrt(y.size))), (label, "grad_lam replay")
    print("%s: %s" % (label, st))
    return st


def test_small_maps_k1_and_k3():
    y, lam, g = workloads.config2(B=2, C=8)
    _check_2d(y, lam, 1, g, "cfg2 K=1")
    _check_2d(y, lam, 3, g, "cfg2 K=3")


def test_config3_planes_k1():
    y, lam, g = workloads.config3(B=2, C=128)
    _check_2d(y, lam, 1, g, "cfg3 K=1")


@pytest.mark.parametrize("shape,K", [((5, 64, 64), 3), ((3, 40, 64), 2), ((4, 64, 33), 2), ((7, 50, 47), 4),
                                     ((2, 33, 1), 2), ((2, 20, 60), 3), ((1, 64, 64), 12)])
def test_mid_planes(shape, K):
    # planes of 33-64 samples a side: pass-by-pass forward; 64 x 64: reverse sweep in one launch
    # with the segments read off the saved pass outputs
    rng = np.random.default_rng(87 + shape[1] * 64 + shape[2])
    y = rng.normal(size=shape).astype(np.float32)
    g = rng.normal(size=shape).astype(np.float32)
    lam = (10 ** rng.uniform(-2, 0.3, size=min(shape[0], 3))).astype(np.float32)
    _check_2d(y, lam, K, g, "mid %s K=%d" % (shape, K))


def test_wide_planes_whose_first_row_pass_takes_the_multilevel_start():
    """Planes 2304 samples wide: the first row pass of the 2D call is a cold call on packed
    unit-stride rows of 769 samples or more, which keeps the levels of its multilevel start in the
    rows of its output (the first saved pass output); the later row passes start from their own
    dual, and the column passes are strided rows of 6 samples."""
    rng = np.random.default_rng(2304)
    y = (np.cumsum(rng.normal(scale=0.05, size=(2, 6, 2304)), axis=-1) + 0.05 * rng.normal(size=(2, 6, 2304))).astype(np.float32)
    g = rng.normal(size=y.shape).astype(np.float32)
    lam = np.array([0.3, 2.0], np.float32)
    _check_2d(y, lam, 2, g, "2x6x2304 K=2")


def test_odd_sizes_mixed_paths():
    rng = np.random.default_rng(71)
    y = rng.normal(size=(3, 19, 45)).astype(np.float32)         # rows of 45 (long path), columns of 19
    g = rng.normal(size=y.shape).astype(np.float32)
    lam = np.array([0.1, 0.5, 2.0], np.float32)
    _check_2d(y, lam, 4, g, "19x45 K=4")
    y = rng.normal(size=(2, 70, 33)).astype(np.float32)
    g = rng.normal(size=y.shape).astype(np.float32)
    _check_2d(y, lam[:2], 2, g, "70x33 K=2")


@pytest.mark.parametrize("shape,K", [((5, 19, 11), 3), ((3, 32, 16), 2), ((7, 8, 32), 2), ((2, 1, 17), 2),
                                     ((3, 32, 32), 5), ((1, 2, 2), 1), ((1, 32, 32), 20), ((2, 32, 1), 3),
                                     ((1, 1, 32), 3), ((9, 31, 32), 4),
                                     # planes of at most 16 x 16 and 8 x 8: four and eight to a wave
                                     ((37, 16, 16), 3), ((11, 13, 16), 2), ((3, 16, 9), 4), ((70, 8, 8), 2),
                                     ((9, 5, 7), 3), ((13, 8, 3), 2), ((5, 1, 8), 2), ((6, 12, 1), 2),
                                     ((4099, 8, 8), 1), ((2050, 16, 16), 2),
                                     # more than 768 planes of 17-32 samples a side: the one-launch forward
                                     ((1600, 32, 32), 2), ((1540, 19, 27), 3), ((1537, 32, 20), 1)])
def test_small_planes(shape, K):
    # planes of at most 32 x 32, ragged in both directions: up to 768 planes of 17-32 samples a side
    # pass by pass on the long-row kernels (reverse sweep from the saved outputs), otherwise the
    # one-launch kernels
    rng = np.random.default_rng(73 + shape[1] * 64 + shape[2])
    y = rng.normal(size=shape).astype(np.float32)
    g = rng.normal(size=shape).astype(np.float32)
    lam = (10 ** rng.uniform(-2, 0.3, size=min(shape[0], 3))).astype(np.float32)
    _check_2d(y, lam, K, g, "small %s K=%d" % (shape, K))


@pytest.mark.parametrize("shape,K", [((6200, 20, 9), 1), ((4099, 20, 9), 2), ((4097, 32, 32), 2), ((16390, 16, 16), 1)])
def test_many_small_planes(shape, K):
    # many small planes: beyond 4096 planes padded to 32 x 32 with a single sweep the forward goes
    # pass by pass (plane columns, warm rows) and leaves segment codes for the fused reverse sweep;
    # the others are one-launch cases with many workgroups (every mapping is also forced on small
    # batches in test_every_forward_mapping_of_small_planes)
    rng = np.random.default_rng(79 + shape[2])
    y = rng.normal(size=shape).astype(np.float32)
    g = rng.normal(size=shape).astype(np.float32)
    lam = (10 ** rng.uniform(-2, 0.3, size=5)).astype(np.float32)
    _check_2d(y, lam, K, g, "many small %s K=%d" % (shape, K))


@pytest.mark.parametrize("shape", [(1, 1100, 2100), (2, 40, 9000), (1, 1800, 70), (1, 900, 40), (1, 3000, 33)])
def test_long_rows_and_columns_k2(shape):
    """Rows and columns beyond 1024 samples (a workgroup per row; interleaved columns), two
    sweeps, so that the second sweep's passes start from the first sweep's duals; the last three
    shapes put the warm-started variants of the strided kernels with 16 samples per thread (the
    ones that spill registers) under the parity rules: columns of 1800, 900 and 3000 samples."""
    rng = np.random.default_rng(91 + shape[1])
    y = (np.cumsum(rng.normal(scale=0.05, size=shape), axis=-1) + rng.normal(scale=0.2, size=shape)).astype(np.float32)
    g = rng.normal(size=shape).astype(np.float32)
    lam = np.array([0.3, 0.05][:shape[0]], np.float32)
    _check_2d(y, lam, 2, g, "long %s K=2" % (shape,))


def test_config4_reduced():
    y, lam, g = workloads.config4(B=1, C=3, H=512, W=512, n_poly=8)
    _check_2d(y, lam, 3, g, "cfg4 reduced K=3")


def test_lambda_zero_identity_and_mass():
    rng = np.random.default_rng(72)
    y = rng.normal(size=(4, 32, 32)).astype(np.float32)
    g = rng.normal(size=y.shape).astype(np.float32)
    out = run_2d(y, np.array([0.0], np.float32), 3, g)
    assert np.array_equal(out["x"], y) and np.array_equal(out["gy"], g)
    out = run_2d(y, np.array([0.4], np.float32), 4)
    np.testing.assert_allclose(out["x"].astype(np.float64).sum((-1, -2)), y.astype(np.float64).sum((-1, -2)), atol=2e-3)


@pytest.mark.parametrize("shape,value", [((5, 32, 32), np.nan), ((9, 16, 16), np.nan), ((3, 40, 70), np.nan),
                                         ((4, 48, 64), np.nan), ((5, 32, 32), np.inf), ((3, 64, 40), -np.inf)])
def test_nan_plane_stays_in_its_plane(shape, value):
    """A non-finite sample spoils its own plane at most (the row-per-lane kernels hold several
    planes per wave, the others a plane per workgroup or a row per wave or workgroup); the other
    planes match the oracle and the call terminates."""
    rng = np.random.default_rng(83 + shape[1])
    y = rng.normal(size=shape).astype(np.float32)
    bad = 1
    y[bad, shape[1] // 2, shape[2] // 3] = value
    lam = np.array([0.2, 0.7], np.float32)
    out = run_2d(y, lam, 3)
    assert not np.all(np.isfinite(out["x"][bad]))
    ok = np.delete(np.arange(shape[0]), bad)
    lam_ok = lam[ok % 2].astype(np.float64)
    for p, l in zip(ok, lam_ok):
        x_ref, _ = oracle.prox2d_fwd(y[p:p + 1].astype(np.float64), np.array([l]), 3)
        err = np.abs(out["x"][p] - x_ref[0]).max() / (1 + np.abs(y[p]).max())
        assert err <= 1e-4, (shape, p, err)



@pytest.fixture
def dispatch_defaults():
    import paper_2204_03643_amd as tv
    saved = tv.tv_dispatch_thresholds()
    yield saved
    for k, v in saved.items():
        tv.tv_dispatch_override(k, v)


@pytest.mark.parametrize("shape,K", [((70, 32, 32), 2), ((37, 28, 30), 3), ((90, 16, 16), 1), ((33, 13, 16), 2)])
def test_every_forward_mapping_of_small_planes(shape, K, dispatch_defaults):
    """The same call through each mapping the dispatch can choose for planes of at most 32 x 32
    (a plane per workgroup, all passes in one launch of the row-per-lane kernel, pass by pass on
    the row-per-lane kernels with plane columns and segment codes), forced through the thresholds:
    the choice is a matter of speed only, so each one must meet the parity rules."""
    import paper_2204_03643_amd as tv
    rng = np.random.default_rng(97 + shape[1])
    y = rng.normal(size=shape).astype(np.float32)
    g = rng.normal(size=shape).astype(np.float32)
    lam = (10 ** rng.uniform(-2, 0.3, size=3)).astype(np.float32)
    names = ("fused32_full_planes", "fused32_full_planes_k2", "fused32_full_planes_k3", "fused32_ragged_planes",
             "fused16_one_sweep_planes")
    big = 1 << 40
    outs = []
    for per_plane, fused in ((big, big), (0, big), (0, 0)):
        tv.tv_dispatch_override("plane_per_group_planes", per_plane)
        for nme in names:
            tv.tv_dispatch_override(nme, fused)
        out = run_2d(y, lam, K, g)
        check_2d(y, lam, K, g, out, "forced (%d, %d) %s K=%d" % (per_plane > 0, fused > 0, shape, K))
        outs.append(out)
    # every mapping solves the same problems to rounding: outputs agree far inside the parity bar
    for o in outs[1:]:
        assert np.abs(o["x"] - outs[0]["x"]).max() <= 2e-5 * (1 + np.abs(y).max())


@pytest.mark.parametrize("shape,K", [((70, 16, 16), 1), ((70, 16, 16), 3), ((33, 12, 14), 2), ((9, 9, 16), 4)])
def test_one_launch_forward_of_16_side_planes_in_its_large_batch_variant(shape, K, dispatch_defaults):
    """Planes of 9-16 a side: from `fused16_dense_planes` planes on the one-launch forward kernel is
    the variant built for four waves per SIMD.  Same source, other register allocation: forced
    onto a small batch, it must give the bits of the ordinary variant and pass the parity rules."""
    import paper_2204_03643_amd as tv
    rng = np.random.default_rng(160 + shape[1] * 16 + shape[2] + K)
    y = rng.normal(size=shape).astype(np.float32)
    g = rng.normal(size=shape).astype(np.float32)
    lam = (10 ** rng.uniform(-2, 0.3, size=3)).astype(np.float32)
    tv.tv_dispatch_override("fused16_one_sweep_planes", 1 << 40)
    tv.tv_dispatch_override("fused16_dense_planes", 1 << 40)
    ref = run_2d(y, lam, K, g)
    tv.tv_dispatch_override("fused16_dense_planes", 0)
    out = run_2d(y, lam, K, g)
    check_2d(y, lam, K, g, out, "dense 16-side variant %s K=%d" % (shape, K))
    assert np.array_equal(out["x"], ref["x"]) and np.array_equal(out["gy"], ref["gy"])


@pytest.mark.parametrize("shape,K", [((70, 32, 32), 2), ((37, 28, 30), 3), ((9, 17, 32), 4), ((5, 32, 3), 2), ((3, 1, 20), 2),
                                     ((4, 31, 1), 1), ((260, 32, 32), 1), ((5, 64, 64), 3), ((3, 40, 56), 2), ((4, 33, 64), 2),
                                     ((2, 64, 35), 1), ((70, 48, 48), 4), ((1, 33, 33), 1), ((3, 2, 64), 2), ((300, 64, 64), 1)])
def test_plane_per_workgroup_forward_and_reverse_sweep(shape, K, dispatch_defaults):
    """All 2K passes in one launch with a plane per workgroup (16 threads x 2 samples per row for
    sides of 17-32, 8 x 8 for sides of 33-64), forced through its thresholds for plane counts on
    both sides of what the dispatch would pick: the parity rules of every other mapping, reverse
    sweep included (from the segment codes up to 32 x 32, from the saved pass outputs beyond),
    and agreement with the default mapping far inside the parity bar."""
    import paper_2204_03643_amd as tv
    rng = np.random.default_rng(211 + shape[1] + 3 * shape[2])
    y = rng.normal(size=shape).astype(np.float32)
    g = rng.normal(size=shape).astype(np.float32)
    lam = (10 ** rng.uniform(-2, 0.3, size=3)).astype(np.float32)
    fwd_knobs = ("plane_per_group_planes", "plane_per_group64_planes", "plane_per_group64_planes_k2",
                 "plane_per_group64_full_planes_k2", "plane_per_group64_full_planes_k3",
                 "plane_per_group64_full_planes_k5")
    bwd_knobs = ("plane_per_group_bwd_planes", "plane_per_group64_bwd_planes", "plane_per_group64_bwd_ragged_planes",
                 "plane_per_group64_bwd_ragged_planes_k2")
    for k in fwd_knobs + bwd_knobs:
        tv.tv_dispatch_override(k, 0)
    ref = run_2d(y, lam, K, g)
    for k in fwd_knobs + bwd_knobs:
        tv.tv_dispatch_override(k, 1 << 40)
    out = run_2d(y, lam, K, g)
    check_2d(y, lam, K, g, out, "plane per workgroup %s K=%d" % (shape, K))
    assert np.abs(out["x"] - ref["x"]).max() <= 2e-5 * (1 + np.abs(y).max())
    # the plane-per-workgroup reverse sweep behind the other forward mappings (their codes, or
    # their saved pass outputs): the same segments as the reference run, so the same gradient
    # up to the order of the sums
    for k in fwd_knobs:
        tv.tv_dispatch_override(k, 0)
    mixed = run_2d(y, lam, K, g)
    check_2d(y, lam, K, g, mixed, "plane per workgroup, reverse sweep only, %s K=%d" % (shape, K))
    assert np.array_equal(mixed["x"], ref["x"])
    assert np.abs(mixed["gy"] - ref["gy"]).max() <= 1e-5 * max(np.abs(ref["gy"]).max(), 1e-30)


@pytest.mark.parametrize("shape,K", [((900, 32, 32), 3), ((1000, 20, 27), 2), ((300, 16, 16), 2)])
def test_one_launch_forward_without_the_pass_outputs(shape, K, dispatch_defaults):
    """By default the one-launch forward of planes of at most 32 x 32 writes the codes and x only
    (its reverse sweep reads nothing else): the part of the workspace that would hold the pass
    outputs stays as the caller left it, and x, grad_y and grad_lam are bit for bit what the call
    gives when it is asked to write the pass outputs too (which is how every other test runs it)."""
    import paper_2204_03643_amd as tv
    rng = np.random.default_rng(131 + shape[1])
    y = np.maximum(rng.normal(size=shape), 0).astype(np.float32)
    g = rng.normal(size=shape).astype(np.float32)
    lam = (10 ** rng.uniform(-2, 0.3, size=4)).astype(np.float32)
    tv.tv_dispatch_override("plane_per_group_planes", 0)      # onto the row-per-lane one-launch kernel whatever the count
    for nme in ("fused32_full_planes", "fused32_full_planes_k2", "fused32_full_planes_k3", "fused32_ragged_planes",
                "fused16_one_sweep_planes"):
        tv.tv_dispatch_override(nme, 1 << 40)
    assert tv.tv_dispatch_threshold("fused_keeps_passes") == 0
    kept = run_2d(y, lam, K, g, keep_passes=True)
    check_2d(y, lam, K, g, kept, "kept passes %s K=%d" % (shape, K))
    lean = run_2d(y, lam, K, g, keep_passes=False)
    for k in ("x", "gy", "gl"):
        assert np.array_equal(kept[k], lean[k]), k
    assert np.all(np.isnan(lean["saved"]))                     # run_2d hands over a workspace of NaN bytes


@pytest.mark.parametrize("H,W", [(60, 90), (120, 180), (250, 380), (380, 250), (500, 760), (760, 500), (1000, 1500),
                                 (2000, 3000), (4000, 6000), (40, 8000), (16000, 40), (12000, 36), (36, 12000)])
def test_every_thread_mapping_of_long_rows_cold_and_warm(H, W):
    """One plane, two sweeps, with H and W walking through the row lengths at which the long-row
    kernels change their threads-per-row x samples-per-thread mapping (8 x 8 up to 1024 x 16),
    unit-stride rows and strided columns alike (columns of 193-768 samples: eight to a workgroup
    in the forward kernels, sixteen in the backward ones): the first sweep starts cold, the second from the
    duals of the first, so every mapping runs in both variants under the parity rules."""
    rng = np.random.default_rng(3 * H + W)
    y = (np.cumsum(rng.normal(scale=0.05, size=(1, H, W)), axis=-1)
         + np.cumsum(rng.normal(scale=0.05, size=(1, H, W)), axis=-2) + rng.normal(scale=0.2, size=(1, H, W))).astype(np.float32)
    g = rng.normal(size=y.shape).astype(np.float32)
    _check_2d(y, np.array([0.3], np.float32), 2, g, "mappings %dx%d K=2" % (H, W))
