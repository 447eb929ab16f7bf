"""Seeded synthetic inputs for the five benchmark / parity workloads.

This module only draws random arrays; it contains none of the method's
arithmetic and is the one piece shared by the oracle-side and HIP-side tests.
Every generator takes size overrides so that parity tests can run reduced
versions with the same value distribution and structure.

The workloads stand in for the paper's own (its Sec. 4.1 timing batch of
32x32 maps; CIFAR-scale feature maps; sigma=25 denoising images), none of
which ship with this build.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 220403643


def _rng(index: int, salt: int = 0) -> np.random.Generator:
    return np.random.default_rng(BASE_SEED + index + 1000003 * salt)


def config1(rows: int = 64, n: int = 256, salt: int = 0):
    """Piecewise-constant rows (8 segments, levels U(-1,1)) + N(0, 0.1^2); scalar lam 0.5."""
    rng = _rng(1, salt)
    y = np.empty((rows, n), dtype=np.float64)
    nseg = min(8, n)
    for r in range(rows):
        cuts = np.sort(rng.choice(np.arange(1, n), size=nseg - 1, replace=False)) if nseg > 1 else []
        edges = np.concatenate(([0], cuts, [n])).astype(int)
        levels = rng.uniform(-1.0, 1.0, size=nseg)
        for s in range(nseg):
            y[r, edges[s]:edges[s + 1]] = levels[s]
    y += rng.normal(0.0, 0.1, size=y.shape)
    g = rng.normal(size=y.shape)
    return y.astype(np.float32), np.array([0.5], dtype=np.float32), g.astype(np.float32)


def config2(B: int = 64, C: int = 64, H: int = 32, W: int = 32, salt: int = 0):
    """Post-ReLU feature maps max(0, N(0,1)); per-channel lam ~ U(0.01, 1)."""
    rng = _rng(2, salt)
    y = np.maximum(rng.standard_normal((B, C, H, W), dtype=np.float32), 0.0)
    lam = rng.uniform(0.01, 1.0, size=C).astype(np.float32)
    g = rng.standard_normal((B, C, H, W), dtype=np.float32)
    return y, lam, g


def config3(B: int = 256, C: int = 128, H: int = 32, W: int = 32, salt: int = 0):
    """N(0,1) maps; per-channel lam log-uniform in [1e-3, 10]."""
    rng = _rng(3, salt)
    y = rng.standard_normal((B, C, H, W), dtype=np.float32)
    lam = (10.0 ** rng.uniform(-3.0, 1.0, size=C)).astype(np.float32)
    g = rng.standard_normal((B, C, H, W), dtype=np.float32)
    return y, lam, g


def _polygon_mask(H: int, W: int, verts: np.ndarray) -> np.ndarray:
    """Even-odd rule point-in-polygon test on the pixel-centre grid."""
    yy, xx = np.mgrid[0:H, 0:W]
    px = (xx + 0.5) / W
    py = (yy + 0.5) / H
    inside = np.zeros((H, W), dtype=bool)
    nv = len(verts)
    for i in range(nv):
        x0, y0 = verts[i]
        x1, y1 = verts[(i + 1) % nv]
        if y0 == y1:
            continue
        crosses = ((y0 <= py) & (py < y1)) | ((y1 <= py) & (py < y0))
        xint = x0 + (py - y0) * (x1 - x0) / (y1 - y0)
        inside ^= crosses & (px < xint)
    return inside


def config4(B: int = 8, C: int = 3, H: int = 512, W: int = 512, n_poly: int = 12, salt: int = 0):
    """Piecewise-smooth images: a background ramp plus random polygons, each filled with
    its own linear ramp (per-channel coefficients), clipped to [0,1]; + N(0,(25/255)^2)
    (not clipped afterwards); scalar lam 0.1."""
    rng = _rng(4, salt)
    yy, xx = np.mgrid[0:H, 0:W]
    px = (xx + 0.5) / W
    py = (yy + 0.5) / H
    img = np.empty((B, C, H, W), dtype=np.float64)
    for b in range(B):
        coef = rng.uniform(-0.5, 0.5, size=(C, 2))
        off = rng.uniform(0.2, 0.8, size=C)
        for c in range(C):
            img[b, c] = off[c] + coef[c, 0] * (px - 0.5) + coef[c, 1] * (py - 0.5)
        for _ in range(n_poly):
            nv = int(rng.integers(3, 8))
            centre = rng.uniform(0.1, 0.9, size=2)
            radius = rng.uniform(0.05, 0.35)
            ang = np.sort(rng.uniform(0.0, 2 * np.pi, size=nv))
            rad = radius * rng.uniform(0.5, 1.0, size=nv)
            verts = np.stack([centre[0] + rad * np.cos(ang), centre[1] + rad * np.sin(ang)], axis=1)
            m = _polygon_mask(H, W, verts)
            coef = rng.uniform(-0.5, 0.5, size=(C, 2))
            off = rng.uniform(0.0, 1.0, size=C)
            for c in range(C):
                ramp = off[c] + coef[c, 0] * (px - centre[0]) + coef[c, 1] * (py - centre[1])
                img[b, c][m] = ramp[m]
    np.clip(img, 0.0, 1.0, out=img)
    img += rng.normal(0.0, 25.0 / 255.0, size=img.shape)
    g = rng.standard_normal((B, C, H, W), dtype=np.float32)
    return img.astype(np.float32), np.array([0.1], dtype=np.float32), g


def config5(rows: int = 4096, n: int = 16384, salt: int = 0):
    """Random walk (steps N(0, 0.05^2)) + sparse jumps (p=1e-3, magnitude U(0.5,2), random
    sign); per-row lam log-uniform in [1e-3, 10]."""
    rng = _rng(5, salt)
    y = np.empty((rows, n), dtype=np.float32)
    chunk = max(1, (1 << 22) // max(n, 1))
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        steps = rng.normal(0.0, 0.05, size=(r1 - r0, n))
        jump = rng.random((r1 - r0, n)) < 1e-3
        mag = rng.uniform(0.5, 2.0, size=(r1 - r0, n)) * rng.choice([-1.0, 1.0], size=(r1 - r0, n))
        steps += np.where(jump, mag, 0.0)
        y[r0:r1] = np.cumsum(steps, axis=1).astype(np.float32)
    lam = (10.0 ** rng.uniform(-3.0, 1.0, size=rows)).astype(np.float32)
    g = np.empty((rows, n), dtype=np.float32)
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        g[r0:r1] = rng.standard_normal((r1 - r0, n), dtype=np.float32)
    return y, lam, g


def timing_batch(rows: int = 8192, n: int = 32, sigma: float = 0.5, salt: int = 0):
    """The paper's Sec. 4.1 timing workload read as 8192 rows of length 32: a unit step
    plus Gaussian noise (sigma is not given there; 0.5 here), lam = 1."""
    rng = _rng(6, salt)
    y = np.zeros((rows, n), dtype=np.float64)
    y[:, n // 2:] = 1.0
    y += rng.normal(0.0, sigma, size=y.shape)
    g = rng.standard_normal((rows, n), dtype=np.float32)
    return y.astype(np.float32), np.array([1.0], dtype=np.float32), g
