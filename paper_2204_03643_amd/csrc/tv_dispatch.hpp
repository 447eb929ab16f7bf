// Every size at which the library switches from one kernel mapping to another, in one place,
// each with the measurement that set it (one MI355X; times in microseconds, forward unless
// noted).  They are crossover points of two ways to compute the same bits, never a matter of
// results.  The values are variables so that the benchmark can time both sides of a threshold
// at the threshold (tv_dispatch_override); nothing else writes them.
#pragma once
#include <stdint.h>

namespace tvd {

struct Threshold {
    const char *name;
    int64_t     value;
    const char *what;
};

// Index constants of `table` below.
enum {
    kStreamBytes = 0,
    kOrderMinRows,
    kTinyBatchPlanes,
    kFused32FullPlanes,
    kFused32FullPlanesK2,
    kFused32FullPlanesK3,
    kFused32RaggedPlanes,
    kFused16OneSweepPlanes,
    kFused64Planes,
    kThreadPerSampleWideRows,
    kMlMinLength,
    kMlCoarsest,
    kCount
};

inline Threshold table[kCount] = {
    // A tensor of this many bytes or more is touched once per call and does not survive in the
    // 256 MB last-level cache until the next call; its 16-byte accesses are marked non-temporal.
    // 128 MiB tensors, forward + backward: 147 -> 136 with the hint; 64 MiB: 104 with it against 100
    // without; 32 MiB: 74 against 72; 16 MiB tensors (the 2D workloads, re-read by the next pass):
    // 3-9 % slower with it.
    {"stream_bytes", (int64_t)96 << 20, "non-temporal accesses from this tensor size on"},
    // The slot order of the row-per-lane forward kernel costs a 5 us kernel of one workgroup and
    // shortens the drain of the main kernel: 2^20 rows 97 -> 80 + 5; 2^17 rows 45 -> 44 + 5.  The
    // library computes the order whenever it is handed the workspace; this is where the layer
    // (layer.py) starts to hand it over.
    {"order_min_rows", (int64_t)1 << 18, "the layer passes the slot-order workspace from this many rows on"},
    // 2D, planes of 17-32 samples a side: up to this many planes the 2K forward passes run one by
    // one on the thread-per-few-samples kernels (a lone row-per-lane wave per SIMD issues an
    // instruction every 9 cycles): 256 planes, K = 10: 507 -> 180; 1536 planes: 526 -> 347
    // (feature-map-like data), 437 -> 361 (white noise); around 2000 planes the one-launch kernel
    // catches up (2048 planes, K = 3: 123-151 against 135-140).
    {"tiny_batch_planes", 1536, "2D planes of 17-32 a side: pass by pass on the long-row kernels up to this many planes"},
    // 2D, planes of exactly 32 x 32: the one-launch forward kernel holds two waves per SIMD (17 KB
    // of LDS per wave) where the pass-by-pass kernels hold three, but pays no launches and no
    // memory round trips between the passes, which weighs more the more sweeps there are.
    // One launch against pass by pass, feature-map-like data (white noise within 10 %):
    //   K = 1:  4096 planes  74 /  90,  6144: 109 /  93,  8192: 123 / 121, 16 384: 218 / 177;
    //   K = 2:  4096 planes 123 / 182,  8192: 219 / 250, 12 288: 305 / 323 (noise 285 / 274), 16 384: 388 / 373;
    //   K = 4:  4096 planes 204 / 359,  8192: 369 / 498, 16 384: 676 / 699, 32 768: 1244 / 1207.
    // (4097 planes still take 72 / 84, 219 / 261 with K = 2, 16 385 planes 676 / 757 with K = 4: the
    // one launch loses its lead gradually over its second round of waves.)
    {"fused32_full_planes", 4608, "2D planes of 32 x 32, one sweep: all passes in one launch up to this many planes"},
    {"fused32_full_planes_k2", 10240, "... two sweeps"},
    {"fused32_full_planes_k3", 24576, "... three sweeps or more"},
    // 2D, planes of 17-32 samples a side that do not fill 32 x 32, single sweep (with two sweeps
    // or more the one launch always wins: 28 x 28, 32 768 planes, K = 4: 1.46 ms against 1.94).
    // 28 x 28, K = 1, one launch against pass by pass: 4096 planes 96 / 122, 5120: 134 / 125,
    // 6144: 136 / 131, 8192: 148 / 155.
    {"fused32_ragged_planes", 4352, "2D ragged planes padded to 32 x 32, one sweep: one launch up to this many planes"},
    // 2D, planes of 9-16 samples a side, single sweep: 16 384 planes 47 in one launch against 47
    // pass by pass, 20 480: 49 / 55, 32 768: 69 / 58 (K = 3: 166 against 206, so several sweeps
    // always take the one launch).
    {"fused16_one_sweep_planes", 24576, "2D planes of at most 16 x 16, one sweep: one launch up to this many planes"},
    // 2D, planes of 33-64 samples a side: all passes in one launch, a plane per wave and a row or
    // column per lane (the solver then fills the register file: 256 VGPRs + 256 AGPRs, one wave per
    // SIMD), against pass by pass with eight threads per row.  The one launch never wins: 64 x 64,
    // K = 4: 64 planes 541 / 168, 1024 planes 616 / 324, 8192 planes 3390 / 1577; 48 x 48, K = 1:
    // 256 planes 153 / 54.  It is kept (and tested) as the stated variant for planes of up to
    // 64 x 64; the default of 0 planes means "never".
    {"fused64_planes", 0, "2D planes of 33-64 samples a side: one launch up to this many planes"},
    // Rows of at most 32 samples on the long-row kernels (only the 2D operator on small batches
    // of planes asks for that): 16 threads x 2 samples up to this many rows, 8 x 4 beyond
    // (256 planes of 32 x 32, K = 10: 204 -> 180 with 16 x 2).
    {"thread_per_sample_wide_rows", 16384, "short rows on the long-row kernels: 16 threads per row up to this many rows"},
    // Multilevel start of unit-stride rows (workspace of tv1d_prox_fwd_ex): from this length on.
    // 4096 rows x 16384: 1410 -> 880; below 2048 samples the coarse levels cost what they save.
    {"ml_min_length", 2048, "multilevel start for unit-stride rows of this many samples or more"},
    // ... and levels are stacked until a row has at most this many samples.
    {"ml_coarsest", 256, "coarsest level of the multilevel start"},
};

inline int64_t get(int which) { return table[which].value; }

}  // namespace tvd
