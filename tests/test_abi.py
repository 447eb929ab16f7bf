"""The C-ABI library loads, exports every symbol include/tvprox.h declares, and rejects
invalid arguments before touching the device (so these run without a GPU)."""
import os
import re

import pytest

import paper_2204_03643_amd as tv

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "tvprox.h")


def _declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b(tv[0-9a-z_]+)\s*\(", src)
    return sorted(set(names))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert {"tv1d_prox_fwd", "tv1d_prox_bwd", "tv2d_prox_fwd", "tv2d_prox_bwd",
            "tv1d_bwd_workspace_bytes", "tv2d_workspace_bytes", "tv_status_str",
            "tv1d_prox_fwd_info", "tv1d_prox_fwd_seg", "tv1d_prox_bwd_seg"} <= set(names)
    L = tv.lib()
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    assert tv.status_str(0) == "ok"
    for s in range(1, 9):
        assert tv.status_str(s) not in ("ok", "unknown status")
    assert tv.status_str(99) == "unknown status"


FAKE = 0x1000  # non-null, 16-byte aligned, never dereferenced: validation fails first


def _fwd(y, x, rows, lam):
    return tv.lib().tv1d_prox_fwd(y, x, rows, lam, None)


def test_forward_validation():
    ok_rows = tv.tv_rows(4, 32, 1, 1, 32, 1)
    lam = tv.tv_lambda(FAKE, 1, 1)
    assert _fwd(None, FAKE, ok_rows, lam) == 1          # TV_ERR_NULL
    assert _fwd(FAKE, None, ok_rows, lam) == 1
    assert _fwd(FAKE, FAKE, ok_rows, tv.tv_lambda(None, 1, 1)) == 1
    assert _fwd(FAKE, FAKE, tv.tv_rows(4, 32, 1, 1, 0, 1), lam) == 2     # length < 1
    assert _fwd(FAKE, FAKE, tv.tv_rows(-1, 32, 1, 1, 32, 1), lam) == 2   # negative count
    assert _fwd(FAKE, FAKE, tv.tv_rows(1 << 20, 32, 1 << 20, 1, 32, 1), lam) == 2  # too many rows
    assert _fwd(FAKE, FAKE, tv.tv_rows(4, 32, 1, 1, 32, 0), lam) == 3    # zero element stride
    assert _fwd(FAKE, FAKE, tv.tv_rows(4, 16, 1, 1, 32, 1), lam) == 3    # rows overlap
    assert _fwd(FAKE, FAKE, tv.tv_rows(4, 1024, 8, 16, 32, 1), lam) == 3  # inner rows overlap
    assert _fwd(FAKE, FAKE, tv.tv_rows(2, 64, 8, 1, 8, 4), lam) == 3     # columns: stride < extent
    assert _fwd(FAKE, FAKE, ok_rows, tv.tv_lambda(FAKE, 0, 1)) == 4      # TV_ERR_LAMBDA
    assert _fwd(FAKE, FAKE, ok_rows, tv.tv_lambda(FAKE, 1, 0)) == 4
    assert _fwd(FAKE, FAKE, tv.tv_rows(1, 1 << 20, 1, 1, 16385, 1), lam) == 6  # TV_ERR_UNSUPPORTED
    # zero rows: nothing to do, no device access
    assert _fwd(None, None, tv.tv_rows(0, 32, 1, 1, 32, 1), lam) == 0
    assert _fwd(None, None, tv.tv_rows(4, 32, 0, 1, 32, 1), lam) == 0


def test_backward_validation():
    L = tv.lib()
    rows = tv.tv_rows(4, 32, 1, 1, 32, 1)
    lam = tv.tv_lambda(FAKE, 1, 1)
    assert tv.tv1d_bwd_workspace_bytes(rows, lam) == 16
    assert tv.tv1d_bwd_workspace_bytes(tv.tv_rows(100, 32, 1, 1, 32, 1), lam) == 400
    assert L.tv1d_prox_bwd(None, FAKE, FAKE, FAKE, rows, lam, FAKE, 64, None) == 1
    assert L.tv1d_prox_bwd(FAKE, None, FAKE, FAKE, rows, lam, FAKE, 64, None) == 1
    assert L.tv1d_prox_bwd(FAKE, FAKE, None, FAKE, rows, lam, FAKE, 64, None) == 1
    assert L.tv1d_prox_bwd(FAKE, FAKE, FAKE, FAKE, rows, lam, None, 64, None) == 5   # no workspace
    assert L.tv1d_prox_bwd(FAKE, FAKE, FAKE, FAKE, rows, lam, FAKE, 8, None) == 5    # too small
    assert L.tv1d_prox_bwd(FAKE, FAKE, FAKE, FAKE, rows, lam, FAKE + 4, 64, None) == 5  # misaligned
    assert L.tv1d_prox_bwd(FAKE, FAKE, FAKE, FAKE, tv.tv_rows(4, 32, 1, 1, 0, 1), lam, FAKE, 64, None) == 2


def test_noalloc_backward_validation():
    """Same checks as tv1d_prox_bwd, and the row limit of the static scratch, all before any HIP call."""
    L = tv.lib()
    rows = tv.tv_rows(4, 32, 1, 1, 32, 1)
    lam = tv.tv_lambda(FAKE, 1, 1)
    assert L.tv1d_prox_bwd_noalloc(None, FAKE, FAKE, FAKE, rows, lam, None) == 1
    assert L.tv1d_prox_bwd_noalloc(FAKE, None, FAKE, FAKE, rows, lam, None) == 1
    assert L.tv1d_prox_bwd_noalloc(FAKE, FAKE, FAKE, FAKE, tv.tv_rows(4, 32, 1, 1, 0, 1), lam, None) == 2
    assert L.tv1d_prox_bwd_noalloc(FAKE, FAKE, FAKE, FAKE, rows, tv.tv_lambda(FAKE, 0, 1), None) == 4
    too_many = tv.tv_rows((1 << 20) + 1, 32, 1, 1, 32, 1)
    assert L.tv1d_prox_bwd_noalloc(FAKE, FAKE, FAKE, FAKE, too_many, lam, None) == 8     # TV_ERR_SCRATCH
    assert L.tv1d_prox_bwd_noalloc(FAKE, FAKE, FAKE, None, too_many, lam, None) == 8
    assert "scratch" in tv.status_str(8)


def test_step_record_validation():
    L = tv.lib()
    lam = tv.tv_lambda(FAKE, 1, 1)
    assert tv.tv1d_fwd_steps_floats_per_row(32) == 48 + 96
    assert tv.tv1d_fwd_steps_floats_per_row(0) == 0 and tv.tv1d_fwd_steps_floats_per_row(16385) == 0
    rows = tv.tv_rows(4, 64, 1, 1, 64, 1)
    assert L.tv1d_prox_fwd_steps(FAKE, FAKE, None, None, 2, rows, lam, None) == 1        # no record buffer
    assert L.tv1d_prox_fwd_steps(FAKE, FAKE, None, FAKE, -1, rows, lam, None) == 2
    assert L.tv1d_prox_fwd_steps(FAKE, FAKE, None, FAKE, 2, tv.rows_along((64, 4), 0), lam, None) == 6   # strided long rows
    assert L.tv1d_prox_fwd_steps(None, None, None, None, 0, tv.tv_rows(0, 64, 1, 1, 64, 1), lam, None) == 0


def test_dispatch_thresholds_are_listed_and_overridable():
    th = tv.tv_dispatch_thresholds()
    assert {"stream_bytes", "plane_per_group_planes", "fused32_full_planes", "ml_min_length"} <= set(th)
    assert th["ml_min_length"] == 769 and tv.tv_dispatch_threshold("no_such_name") == -1
    tv.tv_dispatch_override("ml_min_length", 4096)
    assert tv.tv_dispatch_threshold("ml_min_length") == 4096
    assert tv.tv1d_fwd_workspace_bytes(tv.rows_along((10, 2048), -1), tv.tv_lambda(FAKE, 1, 1)) == 0
    tv.tv_dispatch_override("ml_min_length", th["ml_min_length"])
    assert tv.tv1d_fwd_workspace_bytes(tv.rows_along((10, 2048), -1), tv.tv_lambda(FAKE, 1, 1)) > 0
    L = tv.lib()
    assert L.tv_dispatch_override(b"no_such_name", 1) == 6 and L.tv_dispatch_override(b"ml_min_length", -1) == 2


def test_seg_pair_validation():
    L = tv.lib()
    rows = tv.tv_rows(4, 32, 1, 1, 32, 1)
    lam = tv.tv_lambda(FAKE, 1, 1)
    long_rows = tv.tv_rows(4, 33, 1, 1, 33, 1)
    assert L.tv1d_prox_fwd_seg(FAKE, FAKE, None, rows, lam, None) == 1
    assert L.tv1d_prox_fwd_seg(FAKE, FAKE, FAKE + 4, rows, lam, None) == 3       # code misaligned
    assert L.tv1d_prox_fwd_seg(FAKE, FAKE, FAKE, long_rows, lam, None) == 6      # rows too long
    assert L.tv1d_prox_bwd_seg(FAKE, None, FAKE, FAKE, rows, lam, FAKE, 64, None) == 1
    assert L.tv1d_prox_bwd_seg(FAKE, FAKE, FAKE, FAKE, long_rows, lam, FAKE, 64, None) == 6
    assert L.tv1d_prox_bwd_seg(FAKE, FAKE, FAKE, FAKE, rows, lam, None, 64, None) == 5
    assert L.tv1d_prox_bwd_seg(None, None, None, None, tv.tv_rows(0, 32, 1, 1, 32, 1), lam, None, 0, None) == 0


def test_forward_ex_workspace_validation():
    L = tv.lib()
    lam = tv.tv_lambda(FAKE, 128, 32)
    rows = tv.rows_along((256, 128, 32, 32), -1)
    need = tv.tv1d_fwd_workspace_bytes(rows, lam)
    assert need == 512                                    # a slot number per slot
    assert tv.tv1d_fwd_workspace_bytes(rows, tv.tv_lambda(FAKE, 1, 1)) == 0
    assert tv.tv1d_fwd_workspace_bytes(tv.rows_along((256, 128, 32, 64), -1), tv.tv_lambda(FAKE, 128, 32)) == 0
    ex = lambda ws, n: L.tv1d_prox_fwd_ex(FAKE, FAKE, rows, lam, tv.tv_fwd_extra(None, None, ws, n), None)
    assert ex(FAKE, need - 1) == 5
    assert ex(FAKE + 8, need) == 5                        # misaligned
    assert L.tv1d_prox_fwd_ex(None, FAKE, rows, lam, tv.tv_fwd_extra(None, None, FAKE, need), None) == 1


def test_2d_validation():
    L = tv.lib()
    lam = tv.tv_lambda(FAKE, 3, 1)
    need = tv.tv2d_workspace_bytes(6, 32, 32, 2)
    # 2K + 2 tensors, 2K sets of dL/dlam partials, (planes of at most 32 x 32) 2K sets of segment
    # codes, and 32 KiB for the split dL/dlam reduction
    assert need == 6 * 32 * 32 * 4 * (2 * 2 + 2) + 2 * 2 * 6 * 32 * 4 + 2 * 2 * 6 * 32 * 8 + 32768
    assert tv.tv2d_workspace_bytes(6, 32, 64, 2) == 6 * 32 * 64 * 4 * (2 * 2 + 2) + 2 * 2 * 6 * 64 * 4 + 32768
    assert tv.tv2d_workspace_bytes(6, 0, 32, 2) == 0
    assert L.tv2d_prox_fwd(None, FAKE, 6, 32, 32, lam, 2, FAKE, need, None) == 1
    assert L.tv2d_prox_fwd(FAKE, FAKE, 6, 32, 32, lam, 0, FAKE, need, None) == 2
    assert L.tv2d_prox_fwd(FAKE, FAKE, 6, 32, 0, lam, 2, FAKE, need, None) == 2
    assert L.tv2d_prox_fwd(FAKE, FAKE, 6, 32, 32, tv.tv_lambda(FAKE, 0, 1), 2, FAKE, need, None) == 4
    assert L.tv2d_prox_fwd(FAKE, FAKE, 6, 32, 32, lam, 2, FAKE, need - 1, None) == 5
    assert L.tv2d_prox_fwd(FAKE, FAKE, 6, 32, 32, lam, 2, None, need, None) == 5
    assert L.tv2d_prox_fwd(FAKE, FAKE, 1, 32, 20000, lam, 1, FAKE, 1 << 40, None) == 6
    assert L.tv2d_prox_fwd(None, None, 0, 32, 32, lam, 2, None, 0, None) == 0
    assert L.tv2d_prox_bwd(None, FAKE, FAKE, 6, 32, 32, lam, 2, FAKE, need, None) == 1
    assert L.tv2d_prox_bwd(FAKE, FAKE, FAKE, 6, 32, 32, lam, 2, FAKE, need - 1, None) == 5


def test_binding_raises():
    with pytest.raises(tv.TVError) as e:
        tv.tv1d_prox_fwd(FAKE, FAKE, tv.tv_rows(4, 32, 1, 1, 0, 1), tv.tv_lambda(FAKE, 1, 1), stream=0)
    assert e.value.status == 2


def test_rows_along():
    r = tv.rows_along((2, 3, 5, 7), -1)
    assert (r.n_outer, r.outer_stride, r.n_inner, r.inner_stride, r.length, r.elem_stride) == (30, 7, 1, 1, 7, 1)
    r = tv.rows_along((2, 3, 5, 7), -2)
    assert (r.n_outer, r.outer_stride, r.n_inner, r.inner_stride, r.length, r.elem_stride) == (6, 35, 7, 1, 5, 7)


def test_forward_workspace_of_long_rows():
    lam = tv.tv_lambda(FAKE, 1, 1)
    # unit-stride rows of 769 samples or more: one coarse level of n/4 samples (further ones
    # only beyond ml_coarsest = 4096 samples), two arrays, plus a flag per row
    r = tv.rows_along((10, 16384), -1)
    assert tv.tv1d_fwd_workspace_bytes(r, lam) == 2 * 10 * 4096 * 4 + 48
    tv.tv_dispatch_override("ml_coarsest", 256)
    assert tv.tv1d_fwd_workspace_bytes(r, lam) == 2 * 10 * (4096 + 1024 + 256) * 4 + 48
    tv.tv_dispatch_override("ml_coarsest", 4096)
    assert tv.tv1d_fwd_workspace_bytes(tv.rows_along((10, 768), -1), lam) == 0
    assert tv.tv1d_fwd_workspace_bytes(tv.rows_along((4096, 8), 0), lam) == 0          # strided rows
    L = tv.lib()
    need = tv.tv1d_fwd_workspace_bytes(r, lam)
    extra = tv.tv_fwd_extra(None, None, FAKE, need - 1)
    assert L.tv1d_prox_fwd_ex(FAKE, FAKE, r, lam, extra, None) == 5
