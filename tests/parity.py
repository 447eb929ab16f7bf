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


def near_degenerate(x_ref, y, lam_rows, tau_scale=FWD_TOL):
    """Boolean per row (rows along the last axis of 2D arrays)."""
    y = y.astype(np.float64)
    u = np.cumsum(x_ref - y, axis=-1)[..., :-1]
    dx = np.diff(x_ref, axis=-1)
    jump = dx != 0
    lam_rows = np.asarray(lam_rows, dtype=np.float64).reshape(-1, 1)
    tau = tau_scale * (1.0 + np.max(np.abs(y), axis=-1))
    slack = np.where(jump, np.inf, lam_rows - np.abs(u))
    height = np.where(jump, np.abs(dx), np.inf)
    m = np.minimum(slack.min(axis=-1, initial=np.inf), height.min(axis=-1, initial=np.inf))
    return m < tau


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
    deg = near_degenerate(x_ref, y, lam_rows)
    gy_ref = np.empty_like(y64)
    part_ref = np.empty(R)
    n_jumps = np.empty(R)
    x_gpu64 = x_gpu.astype(np.float64)
    for r in range(R):
        src = x_gpu64[r] if deg[r] else x_ref[r]
        gy_ref[r], part_ref[r] = oracle.prox1d_bwd(g64[r], src)
        n_jumps[r] = np.count_nonzero(np.diff(src))
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
    stats.update(grad_max_rel=float(rel.max()), near_degenerate=int(deg.sum()), rows=R)
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
    return stats
