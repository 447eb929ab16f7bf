"""Parity rules shared by the GPU tests: how a HIP result is compared with the oracle.

Forward: per row, max|x - x_ref| <= 1e-4 * (1 + max|y|)   (fp32 tolerance of the build).
Backward: per row, max|grad_y - ref| <= 1e-3 * max|ref| on rows that are not
near-degenerate.  The Jacobian of the prox is discontinuous where a dual sits exactly on
its bound without a jump, or where a jump has zero height: there one differently
classified boundary changes the whole row's gradient by O(1) and any segment partition
consistent with the KKT conditions is a valid generalised Jacobian.  A row is called
near-degenerate when, in the oracle's solution, min over non-jumps of (lam - |u_k|) or min
over jumps of |x_{k+1} - x_k| is below tau = 1e-4 * (1 + max|y|).  On those rows the GPU
gradient must equal the oracle's segment averaging applied to the GPU's own output.
grad_lam: |delta| <= 1e-3 * (|ref| + l2 norm of the per-row contributions) per slot, plus
two rounding floors of fp32 arithmetic: 32 * eps32 * (sum of the magnitudes of the jump terms
that enter the slot) -- the terms are O(1) with both signs, and where they cancel the result
cannot be resolved below that in the kernel's precision -- and, because each term is itself
a difference of two segment means that can cancel (a single jump between two segments of
about 1000 samples whose means differ by 2e-6 turned up in random testing), the floor the
grad_y rule grants each mean, 8 * eps32 * max|g| of the row, twice per jump, added up
within a row and in quadrature over the rows of a slot (rounding errors of different rows
are independent).
"""
from __future__ import annotations

import numpy as np

import oracle

FWD_TOL = 1e-4
GRAD_TOL = 1e-3


def forward_errors(x_gpu, x_ref, y):
    """Per-row error normalised by (1 + max|y|); rows along the last axis."""
    err = np.max(np.abs(x_gpu.astype(np.float64) - x_ref), axis=-1)
    return err / (1.0 + np.max(np.abs(y.astype(np.float64)), axis=-1))


def ordinary_duals(x_ref, y, lam_rows, tau_scale=FWD_TOL):
    """Boolean per dual (rows along the last axis of 2D arrays): True where the oracle's solution
    decides the dual's status with a margin of at least tau = tau_scale (1 + max|y| of the row):
    a jump at least tau high, or a dual at least tau inside its box where there is no jump."""
    y = y.astype(np.float64)
    u = np.cumsum(x_ref - y, axis=-1)[..., :-1]
    dx = np.diff(x_ref, axis=-1)
    jump = dx != 0
    lam_rows = np.asarray(lam_rows, dtype=np.float64).reshape(-1, 1)
    tau = (tau_scale * (1.0 + np.max(np.abs(y), axis=-1))).reshape(-1, 1)
    margin = np.where(jump, np.abs(dx), lam_rows - np.abs(u))
    return margin >= tau


def near_degenerate(x_ref, y, lam_rows, tau_scale=FWD_TOL):
    """Boolean per row: some dual of the row is not ordinary (see ordinary_duals)."""
    return ~np.all(ordinary_duals(x_ref, y, lam_rows, tau_scale), axis=-1)


def check_batch(y, lam_rows, g, x_gpu, gy_gpu, part_slots=None, gl_gpu=None, lam_count=1,
                lam_div=1, label=""):
    """y, g, x_gpu, gy_gpu: [R, N] (rows along the last axis, row ids in order).
    lam_rows: [R].  gl_gpu: [lam_count] summed per slot (slot = (r // lam_div) % lam_count).
    Returns a dict of statistics; raises AssertionError on a parity failure."""
    R, N = y.shape
    y64 = y.astype(np.float64)
    lam_rows = np.asarray(lam_rows, dtype=np.float64)
    x_ref = oracle.prox1d_batch(y64, lam_rows, axis=-1, lam_div=1)
    ferr = forward_errors(x_gpu, x_ref, y)
    assert np.all(np.isfinite(x_gpu)), label
    assert ferr.max() <= FWD_TOL, (label, "forward", float(ferr.max()), int(ferr.argmax()))
    stats = {"fwd_max_err": float(ferr.max())}
    if gy_gpu is None:
        return stats
    g64 = g.astype(np.float64)
    ordinary = ordinary_duals(x_ref, y, lam_rows)
    deg = ~np.all(ordinary, axis=-1)
    # segments, dual by dual: wherever the oracle decides a dual's status with a margin, the HIP
    # path's output jumps there in the same direction, or is bit-constant there, as the oracle's is
    bad = (np.sign(np.diff(x_ref, axis=-1)) != np.sign(np.diff(x_gpu.astype(np.float64), axis=-1))) & ordinary
    assert not bad.any(), (label, "segments differ at an ordinary dual", int(bad.sum()), np.argwhere(bad)[:4].tolist())
    stats.update(duals_checked=int(ordinary.sum()), duals_near_degenerate=int(ordinary.size - ordinary.sum()))
    # segments: the oracle's own on ordinary rows, the GPU's on near-degenerate ones; one batch
    # call with a slot per row returns every row's dL/dlam contribution
    src = np.where(deg[:, None], x_gpu.astype(np.float64), x_ref)
    gy_ref, part_ref = oracle.prox1d_bwd_batch(g64, src, lam_count=R, axis=-1, lam_div=1)
    n_jumps = np.count_nonzero(np.diff(src, axis=-1), axis=-1).astype(np.float64)
    term_mag = np.abs(np.diff(gy_ref, axis=-1)).sum(axis=-1)       # sum over jumps |mean_l - mean_r|
    gerr = np.max(np.abs(gy_gpu.astype(np.float64) - gy_ref), axis=-1)
    gscale = np.maximum(np.max(np.abs(gy_ref), axis=-1), 1e-30)
    # grad_y is a segment mean, a signed sum that can cancel to far below its terms (a row of 15
    # N(0,1) gradients with mean 8e-7 turned up in random testing): like grad_lam below, the
    # relative bar is read against the scale of what is summed, with the rounding floor of an
    # fp32 sum, 8 eps max|g|, beside it
    floor = 8 * np.finfo(np.float32).eps * np.max(np.abs(g64), axis=-1)
    rel = np.maximum(gerr - floor, 0.0) / gscale
    assert rel.max() <= GRAD_TOL, (label, "grad_y", float(rel.max()), int(rel.argmax()),
                                   bool(deg[rel.argmax()]))
    # rows that meet the 1e-3 bar only thanks to the rounding floor
    stats.update(grad_max_rel=float(rel.max()), near_degenerate=int(deg.sum()), rows=R,
                 grad_y_rows_needing_floor=int(np.count_nonzero(gerr / gscale > GRAD_TOL)))
    if gl_gpu is not None:
        slots = (np.arange(R) // lam_div) % lam_count
        ref = np.zeros(lam_count)
        nrm = np.zeros(lam_count)
        np.add.at(ref, slots, part_ref)
        np.add.at(nrm, slots, part_ref ** 2)
        nrm = np.sqrt(nrm)
        mag = np.zeros(lam_count)
        np.add.at(mag, slots, term_mag)
        means_floor = np.zeros(lam_count)
        np.add.at(means_floor, slots, (2 * floor * n_jumps) ** 2)
        d = np.abs(gl_gpu.astype(np.float64) - ref)
        bound = (GRAD_TOL * (np.abs(ref) + nrm) + 32 * np.finfo(np.float32).eps * mag
                 + np.sqrt(means_floor) + 1e-12)
        assert np.all(d <= bound), (label, "grad_lam", float((d / bound).max()))
        stats["grad_lam_max_ratio"] = float((d / bound).max())
        stats["slots"] = int(lam_count)
        stats["grad_lam_slots_needing_floor"] = int(np.count_nonzero(d > GRAD_TOL * (np.abs(ref) + nrm) + 1e-12))
    return stats


# ---- 2D (paper Alg. 1): every one of the 2K passes is a batch of 1D problems ----------------


def dykstra_pass_inputs(y64, saved):
    """Inputs of the 2K prox passes of Alg. 1, rebuilt from the pass outputs `saved` (Z^1, Y^2,
    Z^2, ...): A^k = Y^k + P^k, B^k = Z^k + Q^k with P^{k+1} = A^k - Z^k, Q^{k+1} = B^k - Y^{k+1}."""
    ins = []
    Y, P, Q = y64, 0.0, 0.0
    for k in range(saved.shape[0] // 2):
        A = Y + P
        Z = saved[2 * k]
        P = A - Z
        B = Z + Q
        Yn = saved[2 * k + 1]
        Q = B - Yn
        ins += [A, B]
        Y = Yn
    return ins


def check_2d(y, lam, K, g, out, label=""):
    """2D parity: y, g [planes, H, W] (or [..., H, W]); lam per plane slot (plane p uses
    lam[p % len(lam)]); out: the HIP path's x, saved (2K pass outputs), gy, gl.

    Forward: x and every saved pass within 1e-4 (1 + max|y|) of the oracle's.
    Segments: in each of the 2K passes, at every dual whose status the oracle's run decides with
    a margin (ordinary_duals(), applied to that pass's own input and lambda) the HIP path's pass
    output must jump exactly where the oracle's does, in the same direction, and be bit-constant
    where the oracle's is; rows all of whose duals are ordinary thus have exactly the oracle's
    segments.
    Backward: grad_y within 1e-3 of the plane's largest reference gradient on every entry (plus
    the rounding floor of an fp32 sum, 8 eps max|g_up| of the plane; the planes that need it are
    counted), grad_lam per slot within 1e-3 (|ref| + l2 norm of the per-plane contributions) plus the
    rounding floor of the fp32 sums.  The reference is the oracle's reverse sweep over the
    oracle's own pass outputs, except that near-degenerate rows of a pass take the HIP path's
    segments (any KKT-consistent partition is a valid generalised Jacobian there).  Planes
    without any near-degenerate row are therefore compared with the oracle's own gradient,
    and their number is returned."""
    shape = y.shape
    H, W = shape[-2:]
    y3, g3 = y.reshape(-1, H, W), g.reshape(-1, H, W)
    planes = y3.shape[0]
    lam = np.asarray(lam, dtype=np.float64).ravel()
    y64, g64 = y3.astype(np.float64), g3.astype(np.float64)
    x_ref, saved_ref = oracle.prox2d_fwd(y64, lam, K)
    x_gpu = out["x"].reshape(-1, H, W)
    saved_gpu = out["saved"].reshape(2 * K, -1, H, W)
    scale = 1.0 + np.abs(y64).max()
    assert np.all(np.isfinite(x_gpu)), label
    err = np.abs(x_gpu - x_ref).max() / scale
    assert err <= FWD_TOL, (label, "forward", err)
    perr = np.abs(saved_gpu - saved_ref).max() / scale
    assert perr <= FWD_TOL, (label, "saved passes", perr)
    assert np.array_equal(saved_gpu[-1], x_gpu), label
    stats = {"fwd_max_err": float(err), "planes": planes}
    if "gy" not in out:
        return stats

    lam_plane = lam[np.arange(planes) % lam.size]
    ins = dykstra_pass_inputs(y64, saved_ref)
    hybrid = np.array(saved_ref)
    dirty = np.zeros(planes, dtype=bool)
    rows_checked = rows_deg = duals_checked = duals_deg = 0
    for i in range(2 * K):
        ax = 2 if i % 2 == 0 else 1                     # row pass: along W; column pass: along H
        ref_r = np.moveaxis(saved_ref[i], ax, -1)       # [planes, rows of the plane, samples]
        in_r = np.moveaxis(ins[i], ax, -1)
        gpu_r = np.moveaxis(saved_gpu[i].astype(np.float64), ax, -1)
        rpp = ref_r.shape[1]
        ordinary = ordinary_duals(ref_r.reshape(planes * rpp, -1), in_r.reshape(planes * rpp, -1),
                                  np.repeat(lam_plane, rpp)).reshape(planes, rpp, -1)
        deg = ~np.all(ordinary, axis=-1)
        d_ref, d_gpu = np.diff(ref_r, axis=-1), np.diff(gpu_r, axis=-1)
        bad = (np.sign(d_ref) != np.sign(d_gpu)) & ordinary
        assert not bad.any(), (label, "pass %d: segments differ at an ordinary dual" % i,
                               int(bad.sum()), np.argwhere(bad)[:4].tolist())
        rows_checked += int((~deg).sum())
        rows_deg += int(deg.sum())
        duals_checked += int(ordinary.sum())
        duals_deg += int(ordinary.size - ordinary.sum())
        dirty |= deg.any(axis=1)
        hy = np.moveaxis(hybrid[i], ax, -1)             # a view: writes go through to `hybrid`
        hy[deg] = gpu_r[deg]
    stats.update(pass_duals_checked=duals_checked, pass_duals_near_degenerate=duals_deg,
                 pass_rows_checked=rows_checked, pass_rows_near_degenerate=rows_deg,
                 planes_without_near_degenerate_rows=int((~dirty).sum()))

    gy_gpu = out["gy"].reshape(-1, H, W).astype(np.float64)
    gy_ref, gl_plane = oracle.prox2d_bwd(g64, hybrid, planes, K)       # a slot per plane
    gerr = np.abs(gy_gpu - gy_ref).max(axis=(1, 2))
    gscale = np.maximum(np.abs(gy_ref).max(axis=(1, 2)), 1e-30)
    # rounding floor, as in check_batch: every entry of grad_y is a chain of segment means, signed
    # fp32 sums of entries of the size of g_up, and a plane whose x is one constant gets
    # mean(g_up) everywhere, which can cancel to 1e-6 of max|g_up| (random testing: 232 samples,
    # mean 2.5e-6, fp32 error 6e-9)
    gfloor = 8 * np.finfo(np.float32).eps * np.abs(g64).max(axis=(1, 2))
    ratio = gerr / (GRAD_TOL * gscale + gfloor)
    assert ratio.max() <= 1.0, (label, "grad_y", float((gerr / gscale).max()), int(ratio.argmax()))
    stats["grad_max_rel"] = float((gerr / gscale).max())
    stats["grad_y_planes_needing_floor"] = int(np.count_nonzero(gerr > GRAD_TOL * gscale))
    if (~dirty).any():
        # the oracle's own gradient, nothing of the HIP path in the reference
        gy_own, _ = oracle.prox2d_bwd(g64, saved_ref, planes, K)
        c = ~dirty
        assert np.array_equal(gy_own[c], gy_ref[c])
        own = np.abs(gy_gpu[c] - gy_own[c]).max(axis=(1, 2)) / (GRAD_TOL * gscale[c] + gfloor[c])
        assert own.max() <= 1.0, (label, "grad_y against the oracle's own gradient", float(own.max()))
    if out.get("gl") is not None:
        slots = np.arange(planes) % lam.size
        ref = np.zeros(lam.size)
        nrm = np.zeros(lam.size)
        np.add.at(ref, slots, gl_plane)
        np.add.at(nrm, slots, gl_plane ** 2)
        nrm = np.sqrt(nrm)
        # rounding floor: every jump of every pass contributes a difference of two fp32 means
        # of the adjoint tensor, each good to 8 eps of its largest term; errors of different
        # jumps are independent
        jumps = np.zeros(lam.size)
        np.add.at(jumps, slots, sum(np.count_nonzero(np.diff(hybrid[i], axis=(2 if i % 2 == 0 else 1)),
                                                     axis=(1, 2)) for i in range(2 * K)))
        amax = max(np.abs(g64).max(), np.abs(gy_ref).max())
        floor = 2 * 8 * np.finfo(np.float32).eps * amax * np.sqrt(jumps)
        d = np.abs(out["gl"].astype(np.float64) - ref)
        bound = GRAD_TOL * (np.abs(ref) + nrm) + floor + 1e-12
        assert np.all(d <= bound), (label, "grad_lam", float((d / bound).max()))
        stats["grad_lam_max_ratio"] = float((d / bound).max())
        stats["grad_lam_slots_needing_floor"] = int(np.count_nonzero(d > GRAD_TOL * (np.abs(ref) + nrm) + 1e-12))
    return stats
