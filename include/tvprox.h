/*
 * tvprox -- batched total-variation proximal operators for AMD MI355X (gfx950).
 *
 * C ABI.  Every data pointer is a DEVICE pointer to fp32 data (bf16 bit patterns in the
 * two *_bf16 entry points) owned by the caller; the library allocates nothing, keeps no state
 * between calls (tv1d_prox_bwd_noalloc alone remembers, per device, where its static scratch
 * array lies), and only enqueues kernels on the stream it is given (asynchronous, no implicit sync).
 * Every function returns a tv_status; argument validation happens before any
 * HIP call, so invalid calls fail the same way on a machine without a GPU.
 *
 * Letters: y = input, x = output, lam = lambda.  (The paper's Eq. 1 writes the
 * input as x and the output as y.)
 *
 *   1D operator (paper Eq. 1):  x* = argmin_x 1/2||x - y||^2 + lam * sum_k |x[k+1] - x[k]|
 *   solved per row by projected Newton on the box-constrained dual (paper Eq. 3-4);
 *   backward by implicit differentiation (paper Eq. 5-6);
 *   2D anisotropic operator (paper Eq. 2) by K sweeps of proximal Dykstra (paper Alg. 1).
 */
#ifndef TVPROX_H
#define TVPROX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Same declaration as HIP's own; repeated so that plain C callers need no HIP header. */
struct ihipStream_t;
typedef struct ihipStream_t *hipStream_t;

typedef enum {
    TV_OK = 0,
    TV_ERR_NULL = 1,        /* a required pointer is NULL                              */
    TV_ERR_SHAPE = 2,       /* negative count, length < 1, sweeps < 1, size overflow   */
    TV_ERR_STRIDE = 3,      /* rows would overlap; segment-code buffer not 8-byte aligned */
    TV_ERR_LAMBDA = 4,      /* lam.count < 1 or lam.div < 1                            */
    TV_ERR_WORKSPACE = 5,   /* workspace NULL, misaligned or too small                 */
    TV_ERR_UNSUPPORTED = 6, /* row longer than TV_MAX_LENGTH (TV_SEG_MAX_LENGTH with codes);
                               bf16 storage on anything but packed rows of 32 samples       */
    TV_ERR_HIP = 7,         /* a HIP runtime call (kernel launch) failed               */
    TV_ERR_SCRATCH = 8      /* tv1d_prox_bwd_noalloc: more than TV_NOALLOC_MAX_ROWS rows */
} tv_status;

/* Longest row any entry point accepts. */
#define TV_MAX_LENGTH 16384

/*
 * A batch of rows inside a dense fp32 buffer; all strides in ELEMENTS.
 * Row id r = outer * n_inner + inner starts at
 *     base + outer * outer_stride + inner * inner_stride
 * and its k-th sample is elem_stride * k further on (k = 0 .. length-1).
 * Examples for a [P, H, W] tensor:
 *   rows    (along W): { P, H*W, H, W, W, 1 }
 *   columns (along H): { P, H*W, W, 1, H, W }
 * Rows must not overlap each other.
 */
typedef struct {
    int64_t n_outer, outer_stride;
    int64_t n_inner, inner_stride;
    int64_t length, elem_stride;
} tv_rows;

/*
 * lam: device pointer to `count` floats.  Row r uses lam[(r / div) % count].
 *   scalar: count = 1.   per-row: count = number of rows, div = 1.
 *   per-channel over [B, C, H, W]: count = C, div = H for the row pass (W for columns).
 * A negative or NaN lam read on the device is treated as 0 (the identity, paper Sec. 3.1).
 */
typedef struct {
    const float *lam;
    int64_t count;
    int64_t div;
} tv_lambda;

/*
 * Forward 1D prox over a batch of rows (paper Eq. 1, solved through Eq. 3-4).
 * x may alias y exactly (same pointer, same layout); any other overlap is undefined.
 * While the call runs the rows of x may hold intermediate data (see tv1d_prox_fwd_ex, ws).
 * length == 1 copies the row.  Zero rows: TV_OK without a launch.
 * A row whose input holds NaN/Inf gets unspecified values in that row (NaN at least at
 * the non-finite samples); other rows are unaffected and the call still terminates.
 * Within a maximal constant run of the result all samples are bit-identical, which
 * is what tv1d_prox_bwd relies on to recover the segments.
 */
int tv1d_prox_fwd(const float *y, float *x, tv_rows rows, tv_lambda lam, hipStream_t stream);

/*
 * As tv1d_prox_fwd, and additionally writes one int32 per row to `info` (device
 * pointer, n_outer*n_inner entries, may be NULL): bits 0..15 = Newton steps taken,
 * bit 16 = stopped on the optimality test, bit 17 = stopped because a step left
 * the dual unchanged, bit 18 = iteration cap reached, bit 19 = the row stopped short of an
 * optimal point (cap, or line search run dry) and its output is the plain y - D^T u, whose
 * segments are constant only up to rounding.
 */
int tv1d_prox_fwd_info(const float *y, float *x, int32_t *info, tv_rows rows, tv_lambda lam,
                       hipStream_t stream);

/*
 * The general forward call: tv1d_prox_fwd plus optional outputs and scratch, each of which
 * may be NULL.
 *   info: as in tv1d_prox_fwd_info.
 *   seg:  as in tv1d_prox_fwd_seg (below).
 *   ws:   device scratch of at least tv1d_fwd_workspace_bytes() bytes, 16-byte aligned
 *         (TV_ERR_WORKSPACE otherwise), contents undefined afterwards.  Two uses:
 *         - rows of up to 32 samples whose lambda slots form whole groups of 64 rows are
 *           processed slot by slot in the order of decreasing predicted cost, which shortens
 *           the drain of the launch when the slots' costs differ widely (the order costs a
 *           5 us kernel, which it has not earned back on any batch measured since single rows
 *           stopped needing many more steps than their neighbours); with it the call always
 *           runs the row-per-lane kernels, and its results are bit-identical to those of
 *           the same kernels without it;
 *         - unit-stride rows of 769 samples or more get a multilevel start: the row averaged
 *           in groups of 4 samples, with lambda / 4, is solved first, from the cold start, and
 *           its dual, prolonged, is where the Newton iteration of the row itself starts.  The
 *           paper does not fix the starting point (Sec. 3.2); the minimiser is the same, and
 *           rows whose lambda is large against their sample-to-sample variation take 4 steps
 *           instead of 10-30.  Scratch: half of the input's size.  Without ws (and in tv1d_prox_fwd) the same start is taken
 *           with the levels of a row kept in that row of x until the fine level overwrites it,
 *           whenever the rows are packed (no gap between them) and x does not overlap y; the
 *           results are bit-identical to those with ws.  A call in place (x == y) and rows
 *           with gaps between them start cold without ws; strided rows always do.
 *         tv1d_fwd_workspace_bytes() returns 0 where neither applies (ws is then unused).
 *   flags: 0 or a combination of
 *         TV_FWD_ORDER_READY: ws still holds the slot order that an earlier call with
 *         the same rows and lam descriptors left there, and it is used as it stands (the order
 *         depends on lambda and on the scale of the rows, which drift slowly from one training
 *         step to the next; recomputing it costs a 5 us kernel).  Any order gives the same
 *         results; entries that are no slot numbers are clamped, so a stale or foreign buffer
 *         costs time, not correctness of the addressing.  Ignored where no slot order applies.
 *         TV_FWD_PARALLEL_SEARCH (rows of at most TV_SEG_MAX_LENGTH samples; TV_ERR_UNSUPPORTED
 *         beyond): the step size of every Newton iteration comes from the paper's other rule
 *         (Sec. 3.2), a search over four halving step sizes tried side by side, instead of
 *         backtracking with quadratic interpolation.  Same minimiser, x agrees to rounding; the
 *         paper found backtracking faster, and so it is here (the benchmark prints both).
 */
#define TV_FWD_ORDER_READY 1u
#define TV_FWD_PARALLEL_SEARCH 2u
typedef struct {
    int32_t *info;
    uint64_t *seg;
    void *ws;
    size_t ws_bytes;
    uint32_t flags;
} tv_fwd_extra;
int tv1d_prox_fwd_ex(const float *y, float *x, tv_rows rows, tv_lambda lam, tv_fwd_extra extra,
                     hipStream_t stream);
size_t tv1d_fwd_workspace_bytes(tv_rows rows, tv_lambda lam);

/*
 * A test instrument: tv1d_prox_fwd_info from the cold start that, for the first record_rows
 * rows, also writes a record of the projected-Newton iteration itself (paper Eq. 3-4), so that a
 * single Newton step and the descent of the dual objective can be checked from outside:
 * tv1d_fwd_steps_floats_per_row(length) floats per row, record r at record + r * that many,
 *   [0] Newton steps recorded, [1] lambda as used, [2] the info word,
 *   [8 + i], i = 0 .. [0] (at most 40 entries): the dual objective f(u) = 1/2 ||y - D^T u||^2 at
 *        the starting point and after every accepted step,
 *   [48 + k], k < length - 1: the dual u the first iteration starts from,
 *   [48 + length + k]: the Newton direction d of the first iteration (the solution of
 *        H_SS d_S = grad_S on the free set S, 0 on the bound duals; the step is clip(u - alpha d)),
 *        left untouched for a row of up to 32 samples whose start already passes the optimality
 *        test (info reports 0 steps),
 *   [48 + 2 length + k]: 1 where the first iteration holds dual k on its bound, else 0.
 * Rows of up to 32 samples run the general row-per-lane kernel; longer rows (unit element stride
 * only: TV_ERR_UNSUPPORTED otherwise) one of three mappings: a wavefront per row up to 512
 * samples, a workgroup of 256 threads up to 4096, of 1024 threads beyond.  Slower than
 * tv1d_prox_fwd; x and info are what that call returns up to rounding order.
 */
size_t tv1d_fwd_steps_floats_per_row(int64_t length);
int tv1d_prox_fwd_steps(const float *y, float *x, int32_t *info, float *record, int64_t record_rows,
                        tv_rows rows, tv_lambda lam, hipStream_t stream);

/*
 * Backward of tv1d_prox_fwd (paper Eq. 5-6, evaluated as segment averaging).
 *   g_up:     upstream gradient dL/dx, laid out like x.
 *   x:        the OUTPUT of tv1d_prox_fwd for the same rows and lam.
 *   grad_y:   receives dL/dy (may alias g_up exactly).
 *   grad_lam: lam.count floats, OVERWRITTEN with dL/dlam summed over the rows of each
 *             slot; may be NULL (then ws may be NULL too).
 *   ws:       scratch of at least tv1d_bwd_workspace_bytes() bytes, 16-byte aligned;
 *             contents undefined afterwards.  lam.lam itself is not read.
 */
int tv1d_prox_bwd(const float *g_up, const float *x, float *grad_y, float *grad_lam,
                  tv_rows rows, tv_lambda lam, void *ws, size_t ws_bytes, hipStream_t stream);
size_t tv1d_bwd_workspace_bytes(tv_rows rows, tv_lambda lam);

/*
 * tv1d_prox_bwd for callers that cannot allocate device memory and have no workspace to hand
 * over (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * same arguments without ws / ws_bytes, same kernels, same results bit for bit.  The scratch
 * that tv1d_prox_bwd takes from its caller (one float per row for the dL/dlam terms) lies in
 * a static device array of the library instead: TV_NOALLOC_MAX_ROWS floats (4 MiB), which
 * every GPU the library runs on holds until the process ends.  More rows than that:
 * TV_ERR_SCRATCH, nothing is launched.  The call allocates and frees nothing.  Its first call
 * on a device looks the array's address up (with that device current; make that call outside
 * a graph capture); the stream must belong to the current device.  All calls on one GPU share
 * the one array: two calls that may overlap there (different streams, no dependency) race on
 * it.  Nothing has to be cleared between calls: a call overwrites every entry it reads.
 */
#define TV_NOALLOC_MAX_ROWS (1 << 20)
int tv1d_prox_bwd_noalloc(const float *g_up, const float *x, float *grad_y, float *grad_lam,
                          tv_rows rows, tv_lambda lam, hipStream_t stream);

/*
 * Forward/backward pair for rows of at most TV_SEG_MAX_LENGTH samples in which the
 * backward pass does not read x again.  All that paper Eq. 5-6 need from the solution is
 * its partition into constant segments and the direction of every jump; the forward call
 * writes that as one 64-bit code per row and the backward call reads the code (8 bytes per
 * row) instead of x (4 * length bytes per row).  Results are bit-identical to
 * tv1d_prox_fwd / tv1d_prox_bwd on the same batch.  (Which kernels a forward call runs
 * depends on the batch: up to tv_dispatch_threshold("thread_per_sample_1d_rows") rows of at
 * most 32 samples get sixteen threads per row, larger batches a lane per row; the two agree
 * to rounding, not bit for bit.)
 *   seg: device pointer, 8-byte aligned, one uint64 per row in row order
 *        (entry o * n_inner + i for the row at o * outer_stride + i * inner_stride);
 *        bit k (k < 31) is set when x[k+1] != x[k], bit 32 + k when x[k+1] > x[k].
 * Longer rows: TV_ERR_UNSUPPORTED.  Everything else as in the plain pair.
 */
#define TV_SEG_MAX_LENGTH 32
int tv1d_prox_fwd_seg(const float *y, float *x, uint64_t *seg, tv_rows rows, tv_lambda lam,
                      hipStream_t stream);
int tv1d_prox_bwd_seg(const float *g_up, const uint64_t *seg, float *grad_y, float *grad_lam,
                      tv_rows rows, tv_lambda lam, void *ws, size_t ws_bytes, hipStream_t stream);

/*
 * The same pair with bf16 storage and fp32 arithmetic (the inputs are widened exactly, the
 * solve and the segment averaging run as in the fp32 kernels, the outputs are rounded to
 * nearest even): y, x, g_up and grad_y are arrays of bf16 bit patterns (uint16_t), 16-byte
 * aligned.  The paper computes in fp32; this halves the bytes the pair moves.  x is bit for bit
 * the rounded output of tv1d_prox_fwd_seg (its row-per-lane kernel) on the widened input, the codes are identical, and
 * the backward pass uses the codes (segments of the unrounded x), so rounding never merges or
 * splits a segment.  Only packed rows of exactly 32 samples (unit element stride, rows back
 * to back): TV_ERR_UNSUPPORTED otherwise.  ws / ws_bytes of the forward call: as in
 * tv1d_prox_fwd_ex (may be NULL / 0); grad_lam stays fp32.
 */
int tv1d_prox_fwd_seg_bf16(const uint16_t *y, uint16_t *x, uint64_t *seg, tv_rows rows,
                           tv_lambda lam, void *ws, size_t ws_bytes, hipStream_t stream);
int tv1d_prox_bwd_seg_bf16(const uint16_t *g_up, const uint64_t *seg, uint16_t *grad_y,
                           float *grad_lam, tv_rows rows, tv_lambda lam, void *ws, size_t ws_bytes,
                           hipStream_t stream);

/*
 * 2D anisotropic TV prox on `planes` images of H x W (row-major, contiguous) by
 * `sweeps` iterations of paper Alg. 1; plane p uses lam[p % count] (lam.div is
 * ignored).  ws has room for every pass's output (2*sweeps tensors) plus two scratch
 * tensors, for every backward pass's dL/dlam terms (one float per row and pass) and,
 * for planes of at most 32 x 32, every pass's segment codes, which is what the backward
 * call then reads; it must be handed unchanged to tv2d_prox_bwd.  The forward call leaves
 * there what the backward call will read: the pass outputs, or, where planes of at most
 * 32 x 32 run all their passes in one launch, the codes alone (the pass outputs as well
 * after tv_dispatch_override("fused_keeps_passes", 1)).  x must not alias y.
 * From the second sweep on, the correction term a pass adds to its input is D^T u of the
 * same pass one sweep earlier (x = y - D^T u), and the pass starts its Newton iteration
 * from that dual.  Planes of at most 64 x 64 run all their passes in one launch where that is
 * faster (small batches with a plane per workgroup, larger ones of planes of at most 32 x 32
 * with a row per lane; the plane counts: csrc/tv_dispatch.hpp).
 */
size_t tv2d_workspace_bytes(int64_t planes, int64_t H, int64_t W, int sweeps);
int tv2d_prox_fwd(const float *y, float *x, int64_t planes, int64_t H, int64_t W,
                  tv_lambda lam, int sweeps, void *ws, size_t ws_bytes, hipStream_t stream);

/*
 * Reverse sweep through paper Alg. 1 (replaces autograd through the loop, paper
 * Sec. 3.2).  ws is the buffer tv2d_prox_fwd filled; its two scratch tensors are
 * overwritten, the saved pass outputs are only read.  Planes of at most 64 x 64 run the
 * whole sweep in one launch (small batches with a plane per workgroup, planes of at most
 * 32 x 32 and of 64 x 64 otherwise with a row per lane); which mapping the forward call used
 * does not matter.  grad_lam (lam.count floats,
 * overwritten) may be NULL; it is one fp64 sum, in a fixed order, over the terms of all
 * passes.  grad_y must not alias g_up.
 */
int tv2d_prox_bwd(const float *g_up, float *grad_y, float *grad_lam, int64_t planes, int64_t H,
                  int64_t W, tv_lambda lam, int sweeps, void *ws, size_t ws_bytes,
                  hipStream_t stream);

/*
 * The 2D pair with bf16 storage and fp32 arithmetic, for planes of at most 32 x 32 (the paper's
 * usual feature-map size; TV_ERR_UNSUPPORTED beyond): y, x, g_up and grad_y are arrays of bf16 bit
 * patterns (2-byte aligned; 16-byte aligned plane blocks move with 16-byte accesses), widened
 * exactly on the way in and rounded to nearest even on the way out; everything between is an
 * fp32 one-launch kernel (all 2K passes with the planes resident in LDS; a plane per workgroup
 * for small batches of planes of 17-32 samples a side, a row per lane otherwise, as for fp32),
 * so x is bit for bit the rounded output of that kernel on the widened input, and the reverse
 * sweep uses the segment codes of the unrounded passes.  ws: as for tv2d_prox_fwd / tv2d_prox_bwd (same size, fp32
 * contents); grad_lam stays fp32.
 */
int tv2d_prox_fwd_bf16(const uint16_t *y, uint16_t *x, int64_t planes, int64_t H, int64_t W,
                       tv_lambda lam, int sweeps, void *ws, size_t ws_bytes, hipStream_t stream);
int tv2d_prox_bwd_bf16(const uint16_t *g_up, uint16_t *grad_y, float *grad_lam, int64_t planes,
                       int64_t H, int64_t W, tv_lambda lam, int sweeps, void *ws, size_t ws_bytes,
                       hipStream_t stream);

const char *tv_status_str(int status);

/*
 * The sizes at which the library switches between kernel mappings (csrc/tv_dispatch.hpp lists
 * them with the measurements behind them).  tv_dispatch_name(i) is the name of the i-th one
 * (NULL past the end), tv_dispatch_threshold(name) its current value (-1: no such name).
 * tv_dispatch_override sets one, for benchmarks that time both sides of a threshold at the
 * threshold; results never depend on these values.  Not thread-safe against concurrent calls
 * of the library; TV_ERR_UNSUPPORTED for an unknown name, TV_ERR_SHAPE for a negative value.
 */
const char *tv_dispatch_name(int index);
int64_t tv_dispatch_threshold(const char *name);
int tv_dispatch_override(const char *name, int64_t value);

#ifdef __cplusplus
}
#endif
#endif /* TVPROX_H */
