"""MI355X-native batched TV proximal operators (paper 2204.03643, Eq. 1-6, Alg. 1).

A thin ctypes binding over the C-ABI library ``libtvprox.so`` (see ``include/tvprox.h``).
PyTorch is used only for device memory and streams; every step of the path runs in the
library's HIP kernels.  There is no CPU fallback: if the library is missing it is built
with hipcc, and if that fails the import raises.
"""
from .binding import (TVError, lib, status_str, tv_dispatch_thresholds, tv_dispatch_threshold, tv_dispatch_override, tv1d_bwd_workspace_bytes, tv1d_fwd_workspace_bytes,
                      tv1d_prox_fwd_ex, tv_fwd_extra, TV_FWD_ORDER_READY, TV_FWD_PARALLEL_SEARCH, tv1d_prox_fwd_steps,
                      tv1d_fwd_steps_floats_per_row, tv1d_prox_bwd, tv1d_prox_bwd_noalloc,
                      tv1d_prox_bwd_seg, tv1d_prox_fwd, tv1d_prox_fwd_info, tv1d_prox_fwd_seg, tv1d_prox_fwd_seg_bf16,
                      tv1d_prox_bwd_seg_bf16, tv2d_prox_bwd, tv2d_prox_fwd, tv2d_prox_fwd_bf16, tv2d_prox_bwd_bf16,
                      tv2d_workspace_bytes, tv_lambda, tv_rows, rows_along)

__all__ = ["TVError", "lib", "status_str", "tv_dispatch_thresholds", "tv_dispatch_threshold", "tv_dispatch_override", "tv_rows", "tv_lambda", "rows_along", "tv1d_prox_fwd",
           "tv1d_prox_fwd_info", "tv1d_prox_bwd", "tv1d_prox_bwd_noalloc", "tv1d_prox_fwd_seg", "tv1d_prox_bwd_seg", "tv1d_prox_fwd_ex",
           "tv1d_prox_fwd_seg_bf16", "tv1d_prox_bwd_seg_bf16",
           "tv1d_fwd_workspace_bytes", "tv_fwd_extra", "TV_FWD_ORDER_READY", "TV_FWD_PARALLEL_SEARCH", "tv1d_prox_fwd_steps",
           "tv1d_fwd_steps_floats_per_row", "tv1d_bwd_workspace_bytes", "tv2d_prox_fwd",
           "tv2d_prox_bwd", "tv2d_workspace_bytes", "tv2d_prox_fwd_bf16", "tv2d_prox_bwd_bf16"]
