"""The differentiable TV layer of the paper (Sec. 3.1) on top of the C-ABI library.

``TVLayer`` applies the TV proximity operator to every channel of a ``[B, C, H, W]`` feature
map: 2D (paper Eq. 2, by the sweeps of Alg. 1), or 1D per row / per column (the two
sub-problems below Alg. 1).  Its trainable parameter passes through a SoftPlus so that the
lambda handed to the operator is positive (Sec. 3.1); ``sharpen=True`` returns ``2 x - prox(x)``
(the sharpening mode of Sec. 3.1).  Forward and backward are the library's kernels
(``tv1d_prox_fwd_ex`` / ``tv1d_prox_bwd[_seg]`` and ``tv2d_prox_fwd`` / ``tv2d_prox_bwd``); torch
only carries the tensors, the stream and the chain rule around them.  CUDA tensors only: there
is no CPU path.  fp32 everywhere; bf16 feature maps (lambda stays fp32) where the library has
bf16 storage: 2D on planes of at most 32 x 32 and 1D along the last axis of rows of 32 samples
(fp32 arithmetic inside, see ``include/tvprox.h``).
"""
from __future__ import annotations

import math

import torch

from . import binding as _b

_SEG_MAX = 32          # TV_SEG_MAX_LENGTH


def _check_input(x: torch.Tensor, what: str, bf16_ok: bool = False) -> torch.Tensor:
    if not x.is_cuda:
        raise RuntimeError("%s: the TV layer runs on the GPU only (got a %s tensor)" % (what, x.device))
    if x.dtype != torch.float32 and not (bf16_ok and x.dtype == torch.bfloat16):
        raise TypeError("%s: float32%s expected, got %s" % (what, " or bfloat16" if bf16_ok else "", x.dtype))
    return x.contiguous()


class _Prox1d(torch.autograd.Function):
    """x = prox along `axis` of a contiguous tensor; lam[(row // lam_div) % lam.numel()] per row."""

    @staticmethod
    def forward(ctx, y, lam, axis, lam_div):
        y = _check_input(y, "tv prox 1d", bf16_ok=True)
        ctx.lam_shape = lam.shape                  # the gradient goes back in the caller's shape
        lam = _check_input(lam, "tv prox 1d (lambda)").reshape(-1)
        rows = _b.rows_along(tuple(y.shape), axis)
        ctx.bf16 = y.dtype == torch.bfloat16
        if ctx.bf16 and not (rows.length == 32 and rows.elem_stride == 1):
            raise TypeError("tv prox 1d: bfloat16 only for rows of 32 samples along the last axis")
        L = _b.tv_lambda(lam.data_ptr(), lam.numel(), int(lam_div))
        n_rows = rows.n_outer * rows.n_inner
        x = torch.empty_like(y)
        wsb = _b.tv1d_fwd_workspace_bytes(rows, L)
        if rows.length <= _SEG_MAX and n_rows < _b.tv_dispatch_threshold("order_min_rows"):
            wsb = 0        # the slot order costs a 5 us kernel and gains about 1 us (see tv_dispatch.hpp)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=y.device)
        seg = None
        if rows.length <= _SEG_MAX:
            seg = torch.empty(max(n_rows, 1), dtype=torch.int64, device=y.device)
        if ctx.bf16:
            _b.tv1d_prox_fwd_seg_bf16(y, x, seg, rows, L, ws if wsb else None, wsb)
        else:
            _b.tv1d_prox_fwd_ex(y, x, rows, L, seg=seg, ws=ws if wsb else None, ws_bytes=wsb)
        ctx.rows, ctx.lam_count, ctx.lam_div = rows, lam.numel(), int(lam_div)
        if seg is not None:
            ctx.save_for_backward(seg, lam)
            ctx.has_seg = True
        else:
            ctx.save_for_backward(x, lam)
            ctx.has_seg = False
        return x

    @staticmethod
    def backward(ctx, g):
        saved, lam = ctx.saved_tensors
        g = _check_input(g, "tv prox 1d (gradient)", bf16_ok=ctx.bf16)
        if ctx.bf16 and g.dtype != torch.bfloat16:
            g = g.to(torch.bfloat16)
        rows = ctx.rows
        L = _b.tv_lambda(lam.data_ptr(), ctx.lam_count, ctx.lam_div)
        gy = torch.empty_like(g)
        want_lam = ctx.needs_input_grad[1]
        gl = torch.empty(ctx.lam_count, dtype=torch.float32, device=g.device) if want_lam else None
        wsb = _b.tv1d_bwd_workspace_bytes(rows, L) if want_lam else 0
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=g.device) if want_lam else None
        if ctx.bf16:
            _b.tv1d_prox_bwd_seg_bf16(g, saved, gy, gl, rows, L, ws, wsb)
        elif ctx.has_seg:
            _b.tv1d_prox_bwd_seg(g, saved, gy, gl, rows, L, ws, wsb)
        else:
            _b.tv1d_prox_bwd(g, saved, gy, gl, rows, L, ws, wsb)
        return gy, (gl.reshape(ctx.lam_shape) if want_lam else None), None, None


class _Prox2d(torch.autograd.Function):
    """x = 2D prox of the trailing two axes; plane p uses lam[p % lam.numel()]."""

    @staticmethod
    def forward(ctx, y, lam, sweeps):
        y = _check_input(y, "tv prox 2d", bf16_ok=True)
        ctx.lam_shape = lam.shape                  # the gradient goes back in the caller's shape
        lam = _check_input(lam, "tv prox 2d (lambda)").reshape(-1)
        H, W = int(y.shape[-2]), int(y.shape[-1])
        ctx.bf16 = y.dtype == torch.bfloat16
        if ctx.bf16 and (H > _SEG_MAX or W > _SEG_MAX):
            raise TypeError("tv prox 2d: bfloat16 only for planes of at most 32 x 32")
        planes = y.numel() // (H * W) if H * W else 0
        L = _b.tv_lambda(lam.data_ptr(), lam.numel(), 1)
        wsb = _b.tv2d_workspace_bytes(planes, H, W, int(sweeps))
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=y.device)
        x = torch.empty_like(y)
        (_b.tv2d_prox_fwd_bf16 if ctx.bf16 else _b.tv2d_prox_fwd)(y, x, planes, H, W, L, int(sweeps), ws, wsb)
        ctx.dims = (planes, H, W, int(sweeps), wsb)
        ctx.save_for_backward(ws, lam)
        return x

    @staticmethod
    def backward(ctx, g):
        ws, lam = ctx.saved_tensors
        planes, H, W, sweeps, wsb = ctx.dims
        g = _check_input(g, "tv prox 2d (gradient)", bf16_ok=ctx.bf16)
        if ctx.bf16 and g.dtype != torch.bfloat16:
            g = g.to(torch.bfloat16)
        L = _b.tv_lambda(lam.data_ptr(), lam.numel(), 1)
        gy = torch.empty_like(g)
        want_lam = ctx.needs_input_grad[1]
        gl = torch.empty(lam.numel(), dtype=torch.float32, device=g.device) if want_lam else None
        # (the reverse sweep restarts from g and only reads the saved pass outputs; the two
        # correction tensors of the workspace are its scratch, so it may run again on the same graph)
        (_b.tv2d_prox_bwd_bf16 if ctx.bf16 else _b.tv2d_prox_bwd)(g, gy, gl, planes, H, W, L, sweeps, ws, wsb)
        return gy, (gl.reshape(ctx.lam_shape) if want_lam else None), None


def tv_prox_1d(x: torch.Tensor, lam: torch.Tensor, axis: int = -1, lam_div: int = 1) -> torch.Tensor:
    """Differentiable batched 1D TV prox along `axis` (paper Eq. 1); see ``tv_lambda`` in
    ``include/tvprox.h`` for how `lam` and `lam_div` map rows to lambdas."""
    return _Prox1d.apply(x, lam, axis, lam_div)


def tv_prox_2d(x: torch.Tensor, lam: torch.Tensor, sweeps: int = 4) -> torch.Tensor:
    """Differentiable 2D anisotropic TV prox of the trailing two axes (paper Eq. 2, Alg. 1)."""
    return _Prox2d.apply(x, lam, sweeps)


class TVLayer(torch.nn.Module):
    """TV layer over ``[B, C, H, W]`` (or ``[C, H, W]``) feature maps.

    mode: "2d" (paper Eq. 2), "rows" (1D along W) or "cols" (1D along H).
    shared_lambda: one lambda for all channels instead of one per channel.
    sharpen: return ``2 x - prox(x)``.
    sweeps: iterations of Alg. 1 in 2D mode (the paper found three or four enough).
    init_lambda: initial value of lambda = SoftPlus(parameter).
    """

    def __init__(self, num_channels: int, mode: str = "2d", sharpen: bool = False,
                 shared_lambda: bool = False, sweeps: int = 4, init_lambda: float = math.log(2.0)):
        super().__init__()
        if mode not in ("2d", "rows", "cols"):
            raise ValueError("mode must be '2d', 'rows' or 'cols'")
        if init_lambda <= 0:
            raise ValueError("init_lambda must be positive")
        self.num_channels, self.mode, self.sharpen, self.sweeps = int(num_channels), mode, bool(sharpen), int(sweeps)
        raw = math.log(math.expm1(init_lambda))                  # SoftPlus^-1
        n = 1 if shared_lambda else self.num_channels
        self.raw_lambda = torch.nn.Parameter(torch.full((n,), raw, dtype=torch.float32))

    def lambdas(self) -> torch.Tensor:
        return torch.nn.functional.softplus(self.raw_lambda)

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        if x.dim() not in (3, 4) or x.shape[-3] != self.num_channels:
            raise ValueError("expected [B, %d, H, W] or [%d, H, W]" % (self.num_channels, self.num_channels))
        lam = self.lambdas()
        H, W = x.shape[-2], x.shape[-1]
        if self.mode == "2d":
            y = tv_prox_2d(x, lam, self.sweeps)                  # plane p = b * C + c uses lam[p % C]
        elif self.mode == "rows":
            y = tv_prox_1d(x, lam, axis=-1, lam_div=H)           # row id = (b * C + c) * H + h
        else:
            y = tv_prox_1d(x, lam, axis=-2, lam_div=W)           # row id = (b * C + c) * W + w
        return 2.0 * x - y if self.sharpen else y
