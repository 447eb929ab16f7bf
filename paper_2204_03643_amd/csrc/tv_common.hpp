// Shared device-side types for the TV-prox kernels (gfx950 / CDNA4, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tvk {

// Solver constants.  The paper fixes none of them (Sec. 3.2 only names the Armijo
// rule with quadratic-interpolation backtracking); these are the values chosen here.
constexpr int   kMaxNewtonSteps  = 128;     // iteration cap per row
constexpr int   kMaxBacktracks   = 24;      // line-search rounds per Newton step
constexpr float kArmijoSigma     = 1e-4f;   // sufficient-decrease fraction
constexpr float kArmijoSlackEps  = 4.0f * 1.1920929e-7f;  // slack = this * |f|
// A gradient entry below kGradNoise * (max|y| + lam) is rounding noise of x = y - D^T u: a
// dual that sits on its bound with such a gradient satisfies the KKT conditions (zero
// multiplier) and must not keep the optimality test from firing.
constexpr float kGradNoise       = 16.0f * 1.1920929e-7f;
// The Newton decrement g^T H_S^-1 g is twice the distance of the dual objective from its minimum
// over the free subspace, and that distance bounds 1/2 ||x - x*||^2 there.  Below
// kDecNoise * f (the square of the same 16 ulp) no step can lower f by an amount that fp32
// resolves: a row with such a decrement and no dual held against an inward gradient is at
// its solution (||x - x*|| <= 16 ulp * sqrt(2 f)).
constexpr float kDecNoise        = kGradNoise * kGradNoise;

// info word written per row by the *_info entry point
constexpr int kInfoConverged = 1 << 16;
constexpr int kInfoStalled   = 1 << 17;
constexpr int kInfoCapped    = 1 << 18;
constexpr int kInfoPlain     = 1 << 19;   // output is y - D^T u, segments not bit-constant

// Row addressing, mirrored from tv_rows / tv_lambda (host guarantees the 32-bit fields fit).
struct Layout {
    uint32_t n_rows;
    uint32_t n_inner;
    int64_t  outer_stride;
    int64_t  inner_stride;
    int64_t  elem_stride;
    int32_t  n;            // row length
    uint32_t lam_count;
    uint32_t lam_div;
    uint32_t stream;       // tensors too large to stay in cache: use non-temporal accesses
};

// Which 64 rows a wave of the row-per-lane forward kernel works on.  Row t of a tile is
//     first + (t >> lg) * hop + (t & ((1 << lg) - 1)).
// Identity: lg = 6, tile w starts at row 64 w, the grid is one-dimensional.  Grouped by
// lambda slot (lam.div = 2^lg < 64 and every slot owning a whole number of tiles): tile
// (qb, slot) takes the 64 >> lg consecutive row groups qb * (64 >> lg) ... of ONE slot,
// which lie hop = lam.count << lg rows apart, so that all 64 rows share their lambda and tend
// to need the same number of Newton steps.  The grid is then (tiles per slot, slots) with qb
// as the fast index: the cost of a tile depends mostly on its lambda, and workgroups go to
// the 8 XCDs round-robin in linear order, so with the slot as the fast index an XCD would
// keep getting the same few slots and the XCDs with the expensive ones would finish late.
struct TileMap {
    uint32_t lg;
    uint32_t hop;
    uint32_t grouped;     // 0: identity
    uint32_t count;       // lam.count (grouped only)
    // first row of tile (qb, slot)
    __device__ __forceinline__ uint32_t first(uint32_t qb, uint32_t slot) const
    {
        if (!grouped) return qb * 64u;
        return ((qb * (64u >> lg)) * count + slot) << lg;
    }
    __device__ __forceinline__ uint32_t row(uint32_t first_row, uint32_t t) const
    {
        return first_row + (t >> lg) * hop + (t & ((1u << lg) - 1u));
    }
};

__device__ __forceinline__ int64_t row_offset(const Layout &L, uint32_t r)
{
    uint32_t o = r / L.n_inner;
    uint32_t i = r - o * L.n_inner;
    return (int64_t)o * L.outer_stride + (int64_t)i * L.inner_stride;
}

__device__ __forceinline__ uint32_t lam_slot(const Layout &L, uint32_t r)
{
    if (L.lam_count == 1) return 0;
    return (r / L.lam_div) % L.lam_count;
}

// Negative and NaN lambdas act as 0 (fmaxf returns the non-NaN operand).
__device__ __forceinline__ float load_lambda(const float *lam, const Layout &L, uint32_t r)
{
    return fmaxf(lam[lam_slot(L, r)], 0.0f);
}

// A dual that the warm start finds within this relative distance of its bound is put on the
// bound (the prefix sums that recover it carry rounding errors, and a dual that sits a hair
// inside the box would cost a clipped step to get back).
constexpr float kWarmSnap = 1.0f + 1.0f / 4096.0f;

// Multilevel start of long rows: a level averages groups of this many samples of the level below.
constexpr int kMlFactor = 4;

// Step record of one row, written by the DEBUG variants of the forward kernels for the first
// debug_rows rows of a call (a test instrument: it lets a test check one Newton step, paper
// Eq. 4, and the descent of the dual objective, paper Eq. 3, from outside).  Floats:
//   [0] Newton steps recorded, [1] lambda as used, [2] the info word;
//   [kRecF + i], i = 0 .. [0]: the dual objective f = 1/2 ||x(u)||^2 at the start and after
//        every accepted step (at most kRecMaxF entries; later ones are dropped);
//   [kRecU + k], k < n - 1: the dual the first iteration starts from;
//   [kRecU + n + k]: the Newton direction d of the first iteration (u <- clip(u - alpha d)); not
//        written for a row whose start already passes the optimality test (it takes no step);
//   [kRecU + 2n + k]: 1 where the first iteration holds dual k on its bound, else 0.
constexpr int kRecF = 8, kRecMaxF = 40, kRecU = 48;
__host__ __device__ constexpr int64_t step_record_floats(int64_t n) { return kRecU + 3 * n; }

// Segment code of a row of n <= 32 samples: .x bit k is set when x[k+1] != x[k] (a jump after
// sample k), .y bit k when x[k+1] > x[k].  It carries everything the backward pass reads from x.
struct FwdParams {
    const float *y;        // input rows
    const float *addend;   // optional: the prox input is y + addend (Dykstra correction term)
    float       *x;        // output rows
    float       *x2;       // optional second copy of the output (same layout)
    float       *resid;    // optional: receives (y + addend) - x  (next correction term)
    const float *lam;
    int32_t     *info;     // optional per-row info word
    uint2       *seg;      // optional per-row segment code (rows of up to 32 samples only)
    const uint32_t *order; // optional: grid row j of the grouped grid works on slot order[j]
    uint32_t     io16;     // y and x are bf16 arrays (row-per-lane kernel, packed rows of 32 only)
    uint32_t     psearch;  // row-per-lane kernel, rows of up to 32 samples: parallel step-size search
    uint32_t     warm;     // 1: addend is D^T u of an earlier solve of nearly the same rows: start from that u
                           // 2: start from the dual of the row averaged in groups of kMlFactor (coarse_u)
    // long-row kernels only (multilevel start; the three pitches sit where the pointers' alignment
    // left holes, so that they cost no kernel argument space):
    int32_t      dual_pitch;   // floats between the rows of dual_out
    const float *coarse_u; // warm == 2: duals of the averaged rows, coarse_n per row, coarse_pitch floats apart
    int32_t      coarse_n;
    int32_t      coarse_pitch;
    float       *dual_out; // optional: receives the final dual, L.n per row (entry n - 1 is 0)
    const uint32_t *ml_flag; // optional, per row (flag_pitch words apart): 0 = this row takes no part in the multilevel start
    uint32_t     ml_skip;  // rows with ml_flag == 0 are not solved at all (the launch is a coarse level)
    float        lam_scale; // lambda of this launch = lam[slot] * lam_scale (1 / kMlFactor per level)
    // step record (kernel variants with DEBUG only; see StepRecord):
    float       *debug;     // debug_rows records of step_record_floats(L.n) floats
    uint32_t     debug_rows;
    uint32_t     flag_pitch;
    Layout       L;
    TileMap      tm;       // row-per-lane kernels only
};

struct BwdParams {
    const float *g;        // upstream gradient
    const float *sub;      // optional: the averaged quantity is g - sub, and sub is added back
    const float *x;        // forward output (defines the segments) ...
    const uint2 *seg;      // ... or the segment code the forward pass wrote (row-per-lane kernels)
    float       *gy;       // output
    float       *partial;  // optional: dL/dlam contributions, one per group of 1 << part_lg rows
    uint32_t     part_lg;  // row-per-lane kernels only; a group never spans two lambda slots
    uint32_t     io16;     // g and gy are bf16 arrays (row-per-lane kernel with codes, packed rows of 32 only)
    Layout       L;
};

}  // namespace tvk
