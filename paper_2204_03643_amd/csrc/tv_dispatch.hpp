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
    kFused32FullPlanes,
    kFused32FullPlanesK2,
    kFused32FullPlanesK3,
    kFused32RaggedPlanes,
    kFused16OneSweepPlanes,
    kFused16DensePlanes,
    kPlanePerGroupPlanes,
    kPlanePerGroup64Planes,
    kPlanePerGroup64PlanesK2,
    kPlanePerGroup64FullPlanesK2,
    kPlanePerGroup64FullPlanesK3,
    kPlanePerGroup64FullPlanesK5,
    kPlanePerGroupBwdPlanes,
    kPlanePerGroup64BwdPlanes,
    kPlanePerGroup64BwdRaggedPlanes,
    kPlanePerGroup64BwdRaggedPlanesK2,
    kFusedKeepsPasses,
    kThreadPerSampleWideRows,
    kThreadPerSample1dRows,
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
    // shortens the drain of the main kernel.  It paid while single rows of a wave could take 16
    // Newton iterations; since clipped trial points are polished and rows stop on their Newton
    // decrement, the slowest wave of a slot is no longer far from the others, and the order gains
    // about 1 us: 2^20 rows x 32, forward + backward alternating, 124 natural order / 128 with
    // the slot order; with the lambdas sorted along the slots 121 / 126 (ascending), 119 / 130
    // (descending); with the expensive slots last 125 / 129.  The library still computes the
    // order whenever it is handed the workspace; the layer (layer.py) would hand it over from
    // this many rows on, and the value means "never".
    {"order_min_rows", (int64_t)1 << 40, "the layer passes the slot-order workspace from this many rows on"},
    // 2D, planes of exactly 32 x 32: the one-launch forward kernel holds two waves per SIMD (17 KB
    // of LDS per wave) where the pass-by-pass kernels hold three, but pays no launches and no
    // memory round trips between the passes, which weighs more the more sweeps there are.
    // One launch against pass by pass, forward + backward, feature-map-like data:
    //   K = 1:  4096 planes  69 /  76,  4352:  91 /  82,  6144: 115 /  95, 16 384: 235 / 188;
    //   K = 2:  4096 planes 108 / 146, 20 480: 442 / 465, 32 768: 700 / 704, 49 152: 1000 / 975;
    //   K = 4:  4096 planes 183 / 290, 32 768: 1162 / 1257, 65 536: 2206 / 2305, 81 920: 2767 / 2881
    //   (with three sweeps or more the one launch wins at every count: the value means "always").
    // (The one launch holds 4096 planes at once: with a single sweep it loses over its second
    // round of waves what the saved launches gained.)
    {"fused32_full_planes", 4096, "2D planes of 32 x 32, one sweep: all passes in one launch up to this many planes"},
    {"fused32_full_planes_k2", 32768, "... two sweeps"},
    {"fused32_full_planes_k3", (int64_t)1 << 40, "... three sweeps or more"},
    // 2D, planes of 17-32 samples a side that do not fill 32 x 32, single sweep (with two sweeps
    // or more the one launch always wins: 28 x 28, 32 768 planes, K = 4: 1.46 ms against 1.94).
    // 28 x 28, K = 1, one launch against pass by pass, forward + backward: 2048 planes 91 / 98,
    // 4096: 96 / 101, 4352: 127 / 105, 5120: 140 / 120, 6144: 154 / 122.
    {"fused32_ragged_planes", 4096, "2D ragged planes padded to 32 x 32, one sweep: one launch up to this many planes"},
    // 2D, planes of 9-16 samples a side, single sweep, forward + backward: 16 384 planes 58 in one
    // launch against 58 pass by pass, 24 576: 70 / 75, 32 768: 88 / 86 (K = 3: 166 against 206
    // forward, so several sweeps always take the one launch).  With the four-waves variant of
    // the one-launch kernel (fused16_dense_planes below): 49 152 planes 110 / 113, 61 440: 132 / 134.
    {"fused16_one_sweep_planes", 49152, "2D planes of at most 16 x 16, one sweep: one launch up to this many planes"},
    // ... and from this many planes on the one-launch kernel for planes of 9-16 a side is the
    // variant held to 128 VGPRs (four waves per SIMD, 16-54 registers spilled): 8192 planes do not
    // fill the three waves that the other variant allows (K = 2: 43 us against 45), 65 536 do
    // (K = 4: 334 against 302).  The crossover is where the waves outnumber three per SIMD: 4
    // planes per wave x 3 x 1024 SIMDs.
    {"fused16_dense_planes", 24576, "2D planes of 9-16 a side in one launch: the four-waves-per-SIMD variant from this many planes on"},
    // 2D, small batches: one plane per workgroup of 512 threads, resident in LDS for all passes,
    // 16 threads x 2 samples per row (sides of 17-32) or 8 x 8 (sides of 33-64); tv_plane2d.hpp.
    // A lone row-per-lane wave per SIMD issues an instruction every 9 cycles, and pass by pass a
    // small batch pays a launch and a trip through memory per pass; this mapping has 8x the waves,
    // short chains and one launch.  Its time is set by the slowest row of each pass (a barrier
    // between passes), so it stops paying once the other kernels fill the chip.  Forward, this
    // kernel / the library's choice without it, feature-map-like data:
    //   32 x 32, K = 1:  512 planes 22 /  42,  1024: 33 /  45,  1536:  44 /  46,  1792:  50 /  45;
    //            K = 2:  512 planes 32 /  68,  1024: 51 /  75,  1536:  69 /  80,  2048:  88 /  77;
    //            K = 4:  512 planes 51 / 119,  1024: 81 / 130,  1536: 110 / 129,  2048: 143 / 133;
    //   28 x 30, K = 1: 1280 planes 37 /  59,  2048: 52 /  68;  K = 3: 2048 planes 108 / 153;
    //   20 x 32, K = 1: 2048 planes 47 /  59,  4096: 80 /  67;  K = 4: 2048 planes 120 / 177.
    {"plane_per_group_planes", 1536, "2D planes of 17-32 a side: one launch, a plane per workgroup, up to this many planes"},
    //   64 x 64, K = 1:  128 planes  34 /  49, 1024:  85 / 104, 1536: 121 / 129, 2048: 158 / 159, 2560: 193 / 172;
    //            K = 2:  128 planes  53 /  91, 1024: 134 / 181, 2048: 248 / 276, 4096: 472 / 474;
    //            K = 4:  128 planes  83 / 157, 1024: 219 / 314, 2048: 415 / 484, 4096: 790 / 827;
    //   48 x 48, K = 1: 1536 planes  98 /  97, 2048: 128 / 116;
    //            K = 2: 1536 planes 162 / 177, 2048: 207 / 203, 3072: 295 / 273;
    //            K = 4: 1536 planes 266 / 313, 2048: 350 / 360, 3072: 509 / 483.
    {"plane_per_group64_planes", 1536, "2D planes of 33-64 a side, one sweep: one launch, a plane per workgroup, up to this many planes"},
    {"plane_per_group64_planes_k2", 1536, "... two sweeps or more, planes smaller than 64 x 64"},
    //   64 x 64 again, to larger batches (full planes keep every lane of the 8 x 8 mapping busy):
    //            K = 2: 2560 planes 321 / 339, 3072: 386 / 401, 3584: 443 / 446, 4096: 503 / 488;
    //            K = 3: 3072 planes 513 / 540, 4096: 661 / 694, 5120: 819 / 807;
    //            K = 4: 4096 planes 820 / 876, 5120: 1011 / 1020;  K = 6: 4096: 1107 / 1218, 5120: 1364 / 1416.
    //   (48 x 48 once more, forward + reverse sweep: K = 2, 2048 planes 291 / 275;  K = 4: 486 / 473)
    {"plane_per_group64_full_planes_k2", 3584, "... planes of 64 x 64, two sweeps"},
    //            K = 4: 8192 planes 1587 / 1637, 16384: 3030 / 3034, 32768: 6064 / 5790;
    //            K = 6: 8192 planes 2121 / 2300, 16384: 4172 / 4185, 32768: 8403 / 8207;
    //            K = 10: 8192 planes 3237 / 3479, 16384: 6377 / 6548, 32768: 12837 / 12927.
    {"plane_per_group64_full_planes_k3", 8192, "... planes of 64 x 64, three or four sweeps"},
    {"plane_per_group64_full_planes_k5", 12288, "... planes of 64 x 64, five sweeps or more"},
    // 2D reverse sweep of small batches with a plane per workgroup (tv_plane2d.hpp): both adjoint
    // state tensors of the plane in LDS, 16 x 2 or 8 x 8 threads x samples per row, the segment
    // sums across a row's threads by row shifts.  Against the row-per-lane one-launch kernel (a
    // chain of 32 or 64 samples per lane and pass, one or two waves per CU on such batches),
    // backward call with its lambda reduction, this kernel / that one:
    //   32 x 32, K = 4:  64 planes 14 / 19,  256: 14 / 20,  512: 18 / 22,  768: 23 / 24,  896: 27 / 25;
    //            K = 10: 256 planes 23 / 38;  K = 1: 15 / 15 at every count up to 768 (launches);
    //   28 x 30, K = 2: 512 planes 14 / 21, 1024: 21 / 26;
    //   64 x 64, K = 4:  64 planes 31 / 54,  256: 35 / 58,  512: 43 / 62,  640: 65 / 64;
    //            K = 1: 256 planes 15 / 21,  512: 21 / 23,  640: 29 / 27.
    {"plane_per_group_bwd_planes", 768, "2D reverse sweep, planes of 17-32 a side: a plane per workgroup up to this many planes"},
    {"plane_per_group64_bwd_planes", 512, "2D reverse sweep, planes of 64 x 64: a plane per workgroup up to this many planes"},
    // ... and against the pass-by-pass reverse sweep (2K launches), which is what other planes of
    // 33-64 samples a side get otherwise: 40 x 48, K = 1: 256 planes 14 / 20, 512: 18 / 22,
    // 1024: 29 / 28, 2048: 53 / 40; K = 3: 256 planes 22 / 44, 1024: 52 / 74, 2048: 95 / 108.
    // K = 4: 1024 planes 63 / 97, 4096: 219 / 245, 8192: 424 / 429; K = 2: 4096 planes 112 / 121,
    // 8192: 242 / 211; 56 x 60, K = 2: 2048 planes 80 / 114, 8192: 293 / 401; 33 x 33, K = 2: 4096
    // planes 103 / 111, 16 384: 418 / 381;  40 x 48, K = 3 again: 5120 planes 216 / 228, 8192: 336 / 323.
    {"plane_per_group64_bwd_ragged_planes", 768, "2D reverse sweep, other planes of 33-64 a side, one sweep: a plane per workgroup up to this many planes"},
    {"plane_per_group64_bwd_ragged_planes_k2", 6144, "... two sweeps or more"},
    // 2D, planes of at most 32 x 32 in one launch: the reverse sweep reads the segment codes of the
    // passes, not their outputs, so the forward kernel writes only the codes and x.  1 = it also
    // writes every pass's output into the workspace, where the pass-by-pass forward leaves them (the
    // tests set it to compare each pass with the oracle's).  Not writing them: 4096 planes of
    // 32 x 32, K = 1 / 4 / 10: 56 -> 52, 156 -> 149, 403 -> 385; 16 384 planes, K = 4: 560 -> 512.
    {"fused_keeps_passes", 0, "2D one-launch forward of planes of at most 32 x 32: 1 = also write every pass's output"},
    // Rows of at most 32 samples on the long-row kernels (small 1D batches, see
    // thread_per_sample_1d_rows): 16 threads x 2 samples up to this many rows, 8 x 4 beyond
    // (8192 rows of 32 samples as 256 planes, ten passes each way: 204 -> 180 with 16 x 2).
    {"thread_per_sample_wide_rows", 16384, "short rows on the long-row kernels: 16 threads per row up to this many rows"},
    // 1D calls on rows of 2-32 samples (without segment codes): up to this many rows sixteen
    // threads per row on the long-row kernels instead of a lane per row, whose few waves are bound
    // by their dependency chains.  Forward, lane per row / threads per row: 8192 rows x 32 (the
    // paper's timing batch) 23.6 / 11.7, 32 768 rows 25.0 / 18.0, 65 536 rows 26.6 / 26.6, 131 072
    // rows 34.7 / 43.7; rows of 20 samples: 8192 rows 30.2 / 11.3, 65 536 rows 32.8 / 24.0; rows of
    // 12 samples: 8192 rows 12.8 / 11.9, 32 768 rows 14.0 / 13.7, 65 536 rows 14.4 / 20.0; N(0,1) rows
    // of 32 samples in 128 lambda slots, forward + backward: 40 960 rows 39.6 / 38.2, 49 152 rows
    // 38.2 / 39.6.
    {"thread_per_sample_1d_rows", 40960, "1D rows of at most 32 samples: a few threads per row up to this many rows"},
    // Multilevel start of unit-stride rows: from this length on.  4096 rows x 16384: 1410 -> 880.
    // 8M samples in rows of n, lambda 10^U(-3, 1) per row, cold / multilevel, for random walks,
    // white noise and noisy steps of 64 samples: n = 768: 106 / 101, 113 / 116, 88 / 103; 1024:
    // 115 / 95, 127 / 118, 96 / 105 (these two with rows taking the start from lambda >= 2 x their
    // mean |y[k+1] - y[k]| on; the others from 0.5 x); 1280: 200 / 153, 233 / 187, 163 / 156;
    // 2048: 140 / 122, 187 / 151, 125 / 128; 4096: 150 / 124, 185 / 167, 125 / 123.  With the
    // one coarse level of ml_coarsest below: n = 520: 135 / 123, 136 / 151, 113 / 121; 600:
    // 123 / 114, 123 / 131, 105 / 113; 768: 105 / 100, 114 / 117, 88 / 98; 900: 136 / 105,
    // 158 / 133, 114 / 104; 1024: 118 / 96, 127 / 115, 98 / 104; 1100: 229 / 142, 248 / 183,
    // 195 / 152.  From 769 samples on (16 samples per thread and more) it wins on two kinds of
    // rows out of three and is within 6 % on the third.
    {"ml_min_length", 769, "multilevel start for unit-stride rows of this many samples or more"},
    // ... and levels are stacked (one at least) until a row has at most this many samples.  One
    // level, solved from the cold start, is what pays: every further level is two more launches,
    // and the cold start of a row of a few thousand samples is cheap next to the fine level.
    // Rows as above, coarsest level at most 256 / 1024 / 4096 samples: n = 2048: 125 / 102 / -,
    // 153 / 120 / -, 131 / 107 / -; 8192 (32M samples): - / 344 / 317, - / 343 / 316, - / 347 / 323;
    // 16 384: 460 / 430 / 398 (8M samples), - / 445 / 412, - / 443 / 413 (32M).
    {"ml_coarsest", 4096, "coarsest level of the multilevel start"},
};

inline int64_t get(int which) { return table[which].value; }

}  // namespace tvd
