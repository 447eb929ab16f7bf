"""Helpers for the GPU tests: run the HIP path (through the C ABI) on numpy inputs."""
from __future__ import annotations

import numpy as np


def run_1d(y, lam, lam_div, g=None, axis=-1, want_info=False, in_place=False, use_seg=False,
           use_ws=False):
    """Forward (+ backward when g is given) along `axis` of a contiguous array.
    use_seg: the pair tv1d_prox_fwd_seg / tv1d_prox_bwd_seg instead of the plain one.
    use_ws: forward through tv1d_prox_fwd_ex with its workspace (cost-ordered slots).
    Returns dict with x, gy, gl, info, seg (numpy)."""
    import torch

    import paper_2204_03643_amd as tv

    dev = torch.device("cuda:0")
    yt = torch.from_numpy(np.ascontiguousarray(y, dtype=np.float32)).to(dev)
    lt = torch.from_numpy(np.ascontiguousarray(lam, dtype=np.float32).ravel()).to(dev)
    rows = tv.rows_along(y.shape, axis)
    L = tv.tv_lambda(lt.data_ptr(), lt.numel(), lam_div)
    n_rows = rows.n_outer * rows.n_inner
    xt = yt if in_place else torch.full_like(yt, float("nan"))
    out = {}
    if use_ws:
        wsb = tv.tv1d_fwd_workspace_bytes(rows, L)
        ws = torch.full((max(wsb, 16),), 0xff, dtype=torch.uint8, device=dev)
        info = torch.zeros(max(n_rows, 1), dtype=torch.int32, device=dev) if want_info else None
        seg = torch.full((max(n_rows, 1),), -1, dtype=torch.int64, device=dev) if use_seg else None
        tv.tv1d_prox_fwd_ex(yt, xt, rows, L, info=info, seg=seg, ws=ws, ws_bytes=wsb)
        out["ws_bytes"] = wsb
        if want_info:
            out["info"] = info.cpu().numpy()[:n_rows]
        if use_seg:
            out["seg"] = seg.cpu().numpy()[:n_rows].view(np.uint64)
        if wsb:
            out["order"] = ws.cpu().numpy().view(np.uint32)[:lt.numel()]
    elif want_info:
        info = torch.zeros(max(n_rows, 1), dtype=torch.int32, device=dev)
        tv.tv1d_prox_fwd_info(yt, xt, info, rows, L)
        out["info"] = info.cpu().numpy()[:n_rows]
    elif use_seg:
        seg = torch.full((max(n_rows, 1),), -1, dtype=torch.int64, device=dev)
        tv.tv1d_prox_fwd_seg(yt, xt, seg, rows, L)
        out["seg"] = seg.cpu().numpy()[:n_rows].view(np.uint64)
    else:
        tv.tv1d_prox_fwd(yt, xt, rows, L)
    torch.cuda.synchronize()
    out["x"] = xt.cpu().numpy()
    if g is not None:
        gt = torch.from_numpy(np.ascontiguousarray(g, dtype=np.float32)).to(dev)
        gy = torch.full_like(gt, float("nan"))
        gl = torch.full((lt.numel(),), float("nan"), device=dev)
        wsb = tv.tv1d_bwd_workspace_bytes(rows, L)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
        if use_seg:
            xt.fill_(float("nan"))             # the backward call must not depend on x
            tv.tv1d_prox_bwd_seg(gt, seg, gy, gl, rows, L, ws, wsb)
        else:
            tv.tv1d_prox_bwd(gt, xt, gy, gl, rows, L, ws, wsb)
        torch.cuda.synchronize()
        out["gy"] = gy.cpu().numpy()
        out["gl"] = gl.cpu().numpy()
    return out


def rows_view(a, axis):
    """[R, N] view-copy of `a` with rows taken along `axis`, in the library's row-id order."""
    a = np.moveaxis(a, axis, -1)
    return np.ascontiguousarray(a).reshape(-1, a.shape[-1])


def lam_per_row(lam, n_rows, lam_div):
    lam = np.asarray(lam).ravel()
    return lam[(np.arange(n_rows) // lam_div) % lam.size]


def run_2d(y, lam, sweeps, g=None, keep_passes=True):
    """2D prox on y[..., H, W] with per-plane lam (plane p uses lam[p % len(lam)])."""
    import torch

    import paper_2204_03643_amd as tv

    dev = torch.device("cuda:0")
    H, W = y.shape[-2:]
    planes = int(np.prod(y.shape[:-2], dtype=np.int64))
    yt = torch.from_numpy(np.ascontiguousarray(y, dtype=np.float32)).to(dev)
    lt = torch.from_numpy(np.ascontiguousarray(lam, dtype=np.float32).ravel()).to(dev)
    L = tv.tv_lambda(lt.data_ptr(), lt.numel(), 1)
    wsb = tv.tv2d_workspace_bytes(planes, H, W, sweeps)
    ws = torch.full((max(wsb, 16),), 0xff, dtype=torch.uint8, device=dev)       # floats of all-ones bits are NaN
    xt = torch.full_like(yt, float("nan"))
    # the tests compare every pass's output with the oracle's: the one-launch forward writes them
    # on request only (its reverse sweep reads the codes)
    keeps = tv.tv_dispatch_threshold("fused_keeps_passes")
    tv.tv_dispatch_override("fused_keeps_passes", 1 if keep_passes else 0)
    try:
        tv.tv2d_prox_fwd(yt, xt, planes, H, W, L, sweeps, ws, wsb)
    finally:
        tv.tv_dispatch_override("fused_keeps_passes", keeps)
    torch.cuda.synchronize()
    out = {"x": xt.cpu().numpy()}
    if g is not None:
        gt = torch.from_numpy(np.ascontiguousarray(g, dtype=np.float32)).to(dev)
        gy = torch.full_like(gt, float("nan"))
        gl = torch.full((lt.numel(),), float("nan"), device=dev)
        tv.tv2d_prox_bwd(gt, gy, gl, planes, H, W, L, sweeps, ws, wsb)
        torch.cuda.synchronize()
        out["gy"] = gy.cpu().numpy()
        out["gl"] = gl.cpu().numpy()
        nt = planes * H * W
        saved = ws[: 2 * sweeps * ((nt * 4 + 15) // 16 * 16)].view(torch.float32)
        out["saved"] = saved.cpu().numpy().reshape(2 * sweeps, -1)[:, :nt].reshape((2 * sweeps,) + y.shape)
    return out
