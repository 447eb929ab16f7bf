// Row-per-lane kernels for short rows (length <= 32).
//
// Each lane owns one whole row: the row, its dual and the Newton direction stay in
// VGPRs for the entire solve, there is no cross-lane traffic, and a 64-lane wave
// works on 64 independent rows.  With one sample per register index the masked
// tridiagonal system of paper Eq. 4 is solved by the Thomas recurrences, fully
// unrolled; its pivots depend only on the position inside a run of free duals, so
// they come from a small table in LDS instead of divisions.
//
// Contiguous rows are brought in through an LDS transpose (coalesced 16-byte global
// accesses, conflict-free pitch NMAX+1); strided rows (the column pass of the 2D
// operator) are read directly, where consecutive lanes touch consecutive addresses.
#pragma once
#include "tv_common.hpp"

namespace tvk {

constexpr int kShortBlock = 64;    // one wave per workgroup: waves never wait for each other

template <int NMAX>
struct ShortSmem {
    static constexpr int kPitch      = NMAX + 1;
    static constexpr int kTileFloats = 64 * kPitch;
    static constexpr int kTabFloats  = NMAX + 2;
    static constexpr int kFloats     = kTileFloats + 2 * kTabFloats;
};

// gtab[j] = j/(j+1): reciprocal Thomas pivot at position j of a free run (gtab[0] = 0
// cuts the recurrence at a bound dual).  rtab[j] = 1/j.
template <int NMAX>
__device__ __forceinline__ void fill_tables(float *gtab, float *rtab)
{
    for (int t = threadIdx.x; t <= NMAX; t += kShortBlock) {
        gtab[t] = (float)t / (float)(t + 1);
        rtab[t] = t > 0 ? 1.0f / (float)t : 0.0f;
    }
}

// ---------------------------------------------------------------------------------
// Tile movers.  A wave's 64 packed rows form one contiguous block of 64*NMAX floats; it
// is moved with coalesced 16-byte accesses and transposed through a wave-private LDS
// tile, so no workgroup barrier is involved and a wave that finishes early is not held
// back by its neighbours.
// ---------------------------------------------------------------------------------

// Orders this wave's LDS writes before its later LDS reads (all lanes run in lockstep).
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// 16-byte global accesses of the tile movers.  Tensors far larger than the last-level cache
// are touched once per call: marking those accesses non-temporal keeps them from evicting
// each other and raised the measured bandwidth of forward + backward by 7 % on 128 MiB
// tensors; tensors that fit (the next pass or the backward call re-reads them) are better off
// with ordinary accesses.
typedef float tv_v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float4 load16(const float *p, bool stream)
{
    if (stream) {
        const tv_v4f q = __builtin_nontemporal_load(reinterpret_cast<const tv_v4f *>(p));
        return make_float4(q.x, q.y, q.z, q.w);
    }
    return *reinterpret_cast<const float4 *>(p);
}

__device__ __forceinline__ void store16(float *p, const float4 &v, bool stream)
{
    if (stream) {
        tv_v4f q;
        q.x = v.x; q.y = v.y; q.z = v.z; q.w = v.w;
        __builtin_nontemporal_store(q, reinterpret_cast<tv_v4f *>(p));
    } else {
        *reinterpret_cast<float4 *>(p) = v;
    }
}

template <int NMAX>
struct TileRegs {
    float4 q[NMAX / 4];
};

// Global -> registers, in tile order (coalesced).  Rows past the end of the batch read as 0.
// One 64-lane float4 access covers 256 / NMAX whole rows; when that divides the row-group
// size and the tile is full, every access is "wave-uniform base + lane * 16 bytes".
template <int NMAX>
__device__ __forceinline__ bool tile_is_simple(const TileMap &tm, uint32_t first_row, uint32_t n_rows)
{
    constexpr uint32_t R = 256 / NMAX;
    return ((1u << tm.lg) % R) == 0 && tm.row(first_row, 63) < n_rows;
}

template <int NMAX>
__device__ __forceinline__ void tile_fetch(const float *__restrict__ src, const TileMap &tm,
                                           uint32_t first_row, uint32_t n_rows, int lane,
                                           TileRegs<NMAX> &t, bool stream = false)
{
    constexpr uint32_t R = 256 / NMAX;
    if (tile_is_simple<NMAX>(tm, first_row, n_rows)) {
        const float *ls = src + lane * 4;
#pragma unroll
        for (int i = 0; i < NMAX / 4; ++i) {
            const uint32_t g0 = __builtin_amdgcn_readfirstlane(tm.row(first_row, i * R));
            t.q[i] = load16(ls + (size_t)g0 * NMAX, stream);
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < NMAX / 4; ++i) {
        const int e4 = i * 64 + lane;
        const uint32_t g = tm.row(first_row, (uint32_t)(e4 * 4) / NMAX);
        t.q[i] = g < n_rows
                     ? *reinterpret_cast<const float4 *>(src + (size_t)g * NMAX + (e4 * 4) % NMAX)
                     : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

// ---- bf16 storage (fp32 arithmetic).  A wave's 64 packed rows of 32 bf16 are one contiguous
//      4 KB block: four 16-byte accesses per lane, eight samples each, straight into or out of
//      the wave's tile (fp32, pitch NMAX + 1).
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// two floats -> two bf16 in one word (lo in the low half), round to nearest even: the
// conversion instruction of gfx950
typedef float tv_f2 __attribute__((ext_vector_type(2)));
typedef __bf16 tv_bf2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi)
{
    tv_f2 v;
    v.x = lo; v.y = hi;
    const tv_bf2 r = __builtin_convertvector(v, tv_bf2);
    uint32_t w;
    __builtin_memcpy(&w, &r, sizeof(w));
    return w;
}

__device__ __forceinline__ void tile16_fetch(const uint16_t *__restrict__ src, const TileMap &tm,
                                             uint32_t first_row, uint32_t n_rows, int lane, float *tile,
                                             bool stream)
{
    const bool simple = ((1u << tm.lg) % 16u) == 0 && tm.row(first_row, 63) < n_rows;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = (i * 64 + lane) * 8;                 // sample index inside the tile
        const int rt = e >> 5, c = e & 31;
        float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
        if (simple) {
            const uint32_t g0 = __builtin_amdgcn_readfirstlane(tm.row(first_row, i * 16));
            q = load16(reinterpret_cast<const float *>(src + (size_t)g0 * 32) + lane * 4, stream);
        } else {
            const uint32_t g = tm.row(first_row, rt);
            if (g < n_rows) q = *reinterpret_cast<const float4 *>(src + (size_t)g * 32 + c);
        }
        const uint32_t w[4] = {__float_as_uint(q.x), __float_as_uint(q.y), __float_as_uint(q.z),
                               __float_as_uint(q.w)};
        float *d = tile + rt * 33 + c;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            d[2 * j] = __uint_as_float(w[j] << 16);
            d[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
        }
    }
}

__device__ __forceinline__ void tile16_put(uint16_t *__restrict__ dst, const TileMap &tm,
                                           uint32_t first_row, uint32_t n_rows, int lane,
                                           const float *tile, bool stream)
{
    const bool simple = ((1u << tm.lg) % 16u) == 0 && tm.row(first_row, 63) < n_rows;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = (i * 64 + lane) * 8;
        const int rt = e >> 5, c = e & 31;
        const float *sp = tile + rt * 33 + c;
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = f32x2_to_bf16x2(sp[2 * j], sp[2 * j + 1]);
        const float4 q = make_float4(__uint_as_float(w[0]), __uint_as_float(w[1]), __uint_as_float(w[2]),
                                     __uint_as_float(w[3]));
        if (simple) {
            const uint32_t g0 = __builtin_amdgcn_readfirstlane(tm.row(first_row, i * 16));
            store16(reinterpret_cast<float *>(dst + (size_t)g0 * 32) + lane * 4, q, stream);
        } else {
            const uint32_t g = tm.row(first_row, rt);
            if (g < n_rows) *reinterpret_cast<float4 *>(dst + (size_t)g * 32 + c) = q;
        }
    }
}

// Registers in tile order -> one row per lane.
template <int NMAX>
__device__ __forceinline__ void tile_to_rows(const TileRegs<NMAX> &t, float *tile, int lane,
                                             float (&v)[NMAX])
{
    constexpr int P = NMAX + 1;
    wave_lds_sync();                       // earlier readers of the tile are done
#pragma unroll
    for (int i = 0; i < NMAX / 4; ++i) {
        const int e4 = i * 64 + lane;
        float *d = tile + ((e4 * 4) / NMAX) * P + (e4 * 4) % NMAX;
        d[0] = t.q[i].x; d[1] = t.q[i].y; d[2] = t.q[i].z; d[3] = t.q[i].w;
    }
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < NMAX; ++k) v[k] = tile[lane * P + k];
}

// Registers in tile order -> per lane the negated running sums of its row: u[k] = -(a_0 + .. + a_k).
template <int NMAX, int MA>
__device__ __forceinline__ void tile_to_neg_prefix(const TileRegs<NMAX> &t, float *tile, int lane,
                                                   float (&u)[MA])
{
    constexpr int P = NMAX + 1;
    wave_lds_sync();
#pragma unroll
    for (int i = 0; i < NMAX / 4; ++i) {
        const int e4 = i * 64 + lane;
        float *d = tile + ((e4 * 4) / NMAX) * P + (e4 * 4) % NMAX;
        d[0] = t.q[i].x; d[1] = t.q[i].y; d[2] = t.q[i].z; d[3] = t.q[i].w;
    }
    wave_lds_sync();
    float run = 0.f;
#pragma unroll
    for (int k = 0; k < NMAX - 1; ++k) {
        run -= tile[lane * P + k];
        u[k] = run;
    }
}

// One row per lane -> registers in tile order.
template <int NMAX>
__device__ __forceinline__ void rows_to_tile(const float (&v)[NMAX], float *tile, int lane,
                                             TileRegs<NMAX> &t)
{
    constexpr int P = NMAX + 1;
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < NMAX; ++k) tile[lane * P + k] = v[k];
    wave_lds_sync();
#pragma unroll
    for (int i = 0; i < NMAX / 4; ++i) {
        const int e4 = i * 64 + lane;
        const float *s = tile + ((e4 * 4) / NMAX) * P + (e4 * 4) % NMAX;
        t.q[i] = make_float4(s[0], s[1], s[2], s[3]);
    }
}

template <int NMAX>
__device__ __forceinline__ void tile_put(float *__restrict__ dst, const TileMap &tm,
                                         uint32_t first_row, uint32_t n_rows, int lane,
                                         const TileRegs<NMAX> &t, bool stream = false)
{
    constexpr uint32_t R = 256 / NMAX;
    if (tile_is_simple<NMAX>(tm, first_row, n_rows)) {
        float *ld = dst + lane * 4;
#pragma unroll
        for (int i = 0; i < NMAX / 4; ++i) {
            const uint32_t g0 = __builtin_amdgcn_readfirstlane(tm.row(first_row, i * R));
            store16(ld + (size_t)g0 * NMAX, t.q[i], stream);
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < NMAX / 4; ++i) {
        const int e4 = i * 64 + lane;
        const uint32_t g = tm.row(first_row, (uint32_t)(e4 * 4) / NMAX);
        if (g < n_rows)
            *reinterpret_cast<float4 *>(dst + (size_t)g * NMAX + (e4 * 4) % NMAX) = t.q[i];
    }
}

template <int NMAX>
__device__ __forceinline__ void tile_add(TileRegs<NMAX> &a, const TileRegs<NMAX> &b, float sign)
{
#pragma unroll
    for (int i = 0; i < NMAX / 4; ++i) {
        a.q[i].x = fmaf(sign, b.q[i].x, a.q[i].x); a.q[i].y = fmaf(sign, b.q[i].y, a.q[i].y);
        a.q[i].z = fmaf(sign, b.q[i].z, a.q[i].z); a.q[i].w = fmaf(sign, b.q[i].w, a.q[i].w);
    }
}

// ---- packed rows shorter than NMAX (row r starts r * n floats after the base, rows in natural
//      order): a wave's 64 rows are one contiguous block of 64 n floats.  It moves with coalesced
//      4-byte accesses (element e = i * 64 + lane of the block in step i) through the wave's tile;
//      a lane's (row, column) advances by 64 = dq * n + dr per step, so there is one division.
template <int NMAX>
__device__ __forceinline__ void ragged_fetch(const float *__restrict__ src, uint32_t first_row,
                                             uint32_t n_rows, int n, int lane, float *tile,
                                             float (&v)[NMAX])
{
    constexpr int P = NMAX + 1;
    const int rows_here = first_row < n_rows ? (int)min(64u, n_rows - first_row) : 0;
    const int total = rows_here * n;
    const float *blk = src + (size_t)first_row * n;
    const int dq = 64 / n, dr = 64 - dq * n;
    int row = lane / n, col = lane - row * n;
    wave_lds_sync();                       // earlier readers of the tile are done
    for (int e = lane; e < total; e += 64) {
        tile[row * P + col] = blk[e];
        row += dq; col += dr;
        if (col >= n) { col -= n; row += 1; }
    }
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < NMAX; ++k) v[k] = (k < n && lane < rows_here) ? tile[lane * P + k] : 0.f;
}

template <int NMAX>
__device__ __forceinline__ void ragged_put(float *__restrict__ dst, uint32_t first_row, uint32_t n_rows,
                                           int n, int lane, float *tile, const float (&v)[NMAX])
{
    constexpr int P = NMAX + 1;
    const int rows_here = first_row < n_rows ? (int)min(64u, n_rows - first_row) : 0;
    const int total = rows_here * n;
    float *blk = dst + (size_t)first_row * n;
    const int dq = 64 / n, dr = 64 - dq * n;
    int row = lane / n, col = lane - row * n;
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < NMAX; ++k) tile[lane * P + k] = v[k];
    wave_lds_sync();
    for (int e = lane; e < total; e += 64) {
        blk[e] = tile[row * P + col];
        row += dq; col += dr;
        if (col >= n) { col -= n; row += 1; }
    }
}

// ---- the rows are the columns of contiguous 32 x 32 planes (the column pass of the 2D operator
//      on such planes): a wave's 64 rows are the columns of two planes, each plane a contiguous
//      4 KB block.  The planes move with coalesced 16-byte accesses through the wave's tile
//      (memory rows at pitch 33), and a lane reads or writes its column there, conflict-free.
struct PlanePair {
    uint32_t row[2];       // row id of column 0 of each plane; offsets are recomputed where they
                           // are used, so that only two scalars stay live across the solve
    __device__ __forceinline__ bool there(const Layout &L, int hh) const { return row[hh] < L.n_rows; }
    // 32 x 32 planes: row / 32 is the plane
    __device__ __forceinline__ int64_t base(const Layout &L, int hh) const
    {
        return (int64_t)(row[hh] >> 5) * L.outer_stride;
    }
};

// global -> registers, in plane order (coalesced)
__device__ __forceinline__ void planes_fetch(const float *__restrict__ src, const PlanePair &pp,
                                             const Layout &L, int lane, TileRegs<32> &t)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int hh = i >> 2, e = ((i & 3) * 64 + lane) * 4;
        t.q[i] = pp.there(L, hh) ? load16(src + pp.base(L, hh) + e, L.stream)
                                 : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

// registers in plane order -> the tile (memory rows at pitch 33)
__device__ __forceinline__ void planes_into_tile(const TileRegs<32> &t, float *tile, int lane)
{
    wave_lds_sync();                       // earlier readers of the tile are done
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int hh = i >> 2, e = ((i & 3) * 64 + lane) * 4;
        float *d = tile + (hh * 32 + (e >> 5)) * 33 + (e & 31);
        d[0] = t.q[i].x; d[1] = t.q[i].y; d[2] = t.q[i].z; d[3] = t.q[i].w;
    }
    wave_lds_sync();
}

__device__ __forceinline__ const float *plane_column(const float *tile, int lane)
{
    return tile + ((lane >> 5) * 32) * 33 + (lane & 31);
}

__device__ __forceinline__ void planes_to_columns(const float *__restrict__ src, const PlanePair &pp,
                                                  const Layout &L, float *tile, int lane, float (&v)[32])
{
    TileRegs<32> t;
    planes_fetch(src, pp, L, lane, t);
    planes_into_tile(t, tile, lane);
    const float *col = plane_column(tile, lane);
#pragma unroll
    for (int k = 0; k < 32; ++k) v[k] = col[k * 33];
}

__device__ __forceinline__ void columns_to_planes(const float (&v)[32], float *tile, int lane,
                                                  float *__restrict__ dst, float *__restrict__ dst2,
                                                  const PlanePair &pp, const Layout &L)
{
    wave_lds_sync();
    float *col = tile + ((lane >> 5) * 32) * 33 + (lane & 31);
#pragma unroll
    for (int k = 0; k < 32; ++k) col[k * 33] = v[k];
    wave_lds_sync();
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int hh = i >> 2, e = ((i & 3) * 64 + lane) * 4;
        const float *sp = tile + (hh * 32 + (e >> 5)) * 33 + (e & 31);
        const float4 q = make_float4(sp[0], sp[1], sp[2], sp[3]);
        if (pp.there(L, hh)) {
            store16(dst + pp.base(L, hh) + e, q, L.stream);
            if (dst2) store16(dst2 + pp.base(L, hh) + e, q, L.stream);
        }
    }
}

template <int NMAX, bool FULL>
__device__ __forceinline__ void row_load_strided(const float *__restrict__ src,
                                                 const float *__restrict__ add, int64_t off,
                                                 int64_t es, int n, bool valid, float (&v)[NMAX])
{
#pragma unroll
    for (int k = 0; k < NMAX; ++k) {
        float t = 0.f;
        if (valid && (FULL || k < n)) {
            t = src[off + k * es];
            if (add) t += add[off + k * es];
        }
        v[k] = t;
    }
}

// The same with the negated running sums of the addend: u[k] = -(add_0 + .. + add_k).
template <int NMAX, bool FULL, int MA>
__device__ __forceinline__ void row_load_strided_warm(const float *__restrict__ src,
                                                      const float *__restrict__ add, int64_t off,
                                                      int64_t es, int n, bool valid, float (&v)[NMAX],
                                                      float (&u)[MA])
{
    float run = 0.f;
#pragma unroll
    for (int k = 0; k < NMAX; ++k) {
        float t = 0.f, a = 0.f;
        if (valid && (FULL || k < n)) {
            t = src[off + k * es];
            a = add[off + k * es];
        }
        v[k] = t + a;
        run -= a;
        if (k < NMAX - 1) u[k] = run;
    }
}

template <int NMAX, bool FULL>
__device__ __forceinline__ void row_store_strided(float *__restrict__ dst, int64_t off, int64_t es,
                                                  int n, bool valid, const float (&v)[NMAX])
{
#pragma unroll
    for (int k = 0; k < NMAX; ++k)
        if (valid && (FULL || k < n)) dst[off + k * es] = v[k];
}

// ---------------------------------------------------------------------------------
// Projected Newton on the dual of one row (paper Eq. 3-4), one row per lane.
//
//   dual (minimisation form): f(u) = 1/2 ||x(u)||^2 - 1/2 ||y||^2,  x(u) = y - D^T u,
//   |u_k| <= lam; gradient g_k = x_k - x_{k+1}; Hessian tridiag(-1, 2, -1).
//
// Registers hold the dual, x(u), the Newton direction and the pivots.  The input row is read-only
// after the start and is parked in LDS, sample-major: yl[k * 64] is sample k of this lane's
// row (consecutive lanes -> consecutive banks).  Samples k >= n must be 0.
// ---------------------------------------------------------------------------------
template <int NMAX, bool FULL, bool DEBUG = false>
struct RowSolver {
    float *rec = nullptr;                   // DEBUG: this row's step record, or null
    static constexpr int M = NMAX - 1;
    static constexpr int MA = M > 0 ? M : 1;

    float X[NMAX];      // x(u) for the current dual, carried between passes
    float u[MA];        // the dual
    float D[MA];        // g, then gamma*w, then the Newton direction d
    float G[MA];        // pivots gamma (0 exactly at bound duals), then the previous dual
    const float *yl, *gtab;
    float lam, fcur, alpha_try, gtol;
    int m, steps, flags, nfail;
    bool active, prev_unclipped;

    // (rows shorter than 32 samples in the 32-sample variant: the comparison is redone at every
    // use; as a loop invariant the compiler keeps all 31 selected values in registers for the
    // whole solve, which costs a wave of occupancy.  The shorter variants have the registers to
    // spare and are faster with the invariant.)
    __device__ __forceinline__ float lk(int k) const
    {
        if (FULL) return lam;
        int mm = m;
        if (NMAX >= 32) asm volatile("" : "+s"(mm));
        return k < mm ? lam : 0.0f;
    }
    __device__ __forceinline__ float yk(int k) const { return yl[k * 64]; }
    __device__ __forceinline__ float tab(const float *t, int off4) const
    {
        return *reinterpret_cast<const float *>(reinterpret_cast<const char *>(t) + off4);
    }
    // The parked row must be re-read where it is used; without this the compiler hoists the
    // loop-invariant LDS loads into registers for the whole solve and occupancy drops.
    static __device__ __forceinline__ void reread() { asm volatile("" ::: "memory"); }

    // ---- starting point, one of two feasible candidates:
    //      A = one full Newton step from u = 0 with every dual free, clipped into the box
    //          (exact whenever lam >= lam_max = max_k |prefix_k(mean(y) - y)|);
    //      B = every dual at the bound its local difference points to (exact for small lam).
    //      A is taken when lam >= lam_max / 4, which picks the candidate with the lower dual
    //      objective in all but a few percent of rows (measured on the five workloads).
    //      Two Gauss-Seidel sweeps then polish the chosen candidate.
    __device__ __forceinline__ void start(const float (&y)[NMAX], float inv_n)
    {
        float sum = 0.f, ymax = 0.f;
#pragma unroll
        for (int k = 0; k < NMAX; ++k) { sum += y[k]; ymax = fmaxf(ymax, fabsf(y[k])); }
        // rounding floor of a difference of two x values (lambda = 0: the box is a point, every dual
        // sits on both of its bounds, and no gradient entry may count as pointing inwards)
        gtol = lam > 0.f ? kGradNoise * (ymax + lam) : __builtin_inff();
        const float ybar = sum * inv_n;
        float run = 0.f, rmax = 0.f;
#pragma unroll
        for (int k = 0; k < M; ++k) {
            run += ybar - y[k];
            if (FULL || k < m) rmax = fmaxf(rmax, fabsf(run));
            D[k] = run;
        }
        const bool pickA = lam >= 0.25f * rmax;
        // X[k] temporarily holds half the local difference of y
#pragma unroll
        for (int k = 0; k < M; ++k) {
            const float l = lk(k);
            const float hd = 0.5f * (y[k + 1] - y[k]);
            const float v = pickA ? D[k] : hd * 1e30f;
            u[k] = __builtin_amdgcn_fmed3f(v, -l, l);
            X[k] = hd;
        }
        // two Gauss-Seidel sweeps on the dual (exact coordinate minimisation, u_k <-
        // clip((u_{k-1} + u_{k+1} + y_{k+1} - y_k) / 2)), one in each direction: cheap, and
        // they repair the local structure of the start so that Newton needs fewer steps
        {
            float up = 0.f;
#pragma unroll
            for (int k = 0; k < M; ++k) {
                const float l = lk(k);
                const float un = (k + 1 < M) ? u[k + 1] : 0.f;
                up = __builtin_amdgcn_fmed3f(fmaf(0.5f, up + un, X[k]), -l, l);
                u[k] = up;
            }
            float un = 0.f;
#pragma unroll
            for (int k = M - 1; k >= 0; --k) {
                const float l = lk(k);
                const float ul = (k > 0) ? u[k - 1] : 0.f;
                un = __builtin_amdgcn_fmed3f(fmaf(0.5f, ul + un, X[k]), -l, l);
                u[k] = un;
            }
        }
        primal_of_start(y);
    }

    // x(u) and the dual objective of the starting dual
    __device__ __forceinline__ void primal_of_start(const float (&y)[NMAX])
    {
        float acc = 0.f, prev = 0.f;
#pragma unroll
        for (int k = 0; k < M; ++k) {
            const float c = u[k];
            const float xc = y[k] + c - prev;
            acc = fmaf(xc, xc, acc);
            X[k] = xc; prev = c;
        }
        {
            const float xc = y[M] - prev;
            acc = fmaf(xc, xc, acc);
            X[M] = xc;
        }
        fcur = 0.5f * acc;
    }

    // ---- warm start: u already holds the dual of an earlier solve of nearly the same row (in
    //      Alg. 1 the correction term that is added to a pass's input is D^T u of the same pass
    //      one sweep earlier, so that dual is the negated running sum of the correction term).
    //      It is brought into the box, duals within rounding distance of a bound onto it.
    __device__ __forceinline__ void start_warm(const float (&y)[NMAX])
    {
        float ymax = 0.f;
#pragma unroll
        for (int k = 0; k < NMAX; ++k) ymax = fmaxf(ymax, fabsf(y[k]));
        gtol = lam > 0.f ? kGradNoise * (ymax + lam) : __builtin_inff();
#pragma unroll
        for (int k = 0; k < M; ++k) {
            const float l = lk(k);
            u[k] = __builtin_amdgcn_fmed3f(u[k] * kWarmSnap, -l, l);
        }
        primal_of_start(y);
    }

    // One projected-Newton iteration.  Returns true when every row of the wave has stopped;
    // G[k] == 0 then flags the bound duals of each row's final dual and X is its x.
    __device__ __forceinline__ bool iterate(int it)
    {
        // ---- gradient, bound set (Bertsekas' sign test with exact comparisons: a clipped
        //      dual is bit-equal to +-lam) and optimality test.  The pivot of every dual is
        //      fetched from the table as soon as its position in the free run is known.
        bool vio = false;
        {
            int pos4 = 0;                           // 4 * position inside the free run
#pragma unroll
            for (int k = 0; k < M; ++k) {
                const float g = X[k] - X[k + 1];
                const float s = copysignf(lk(k), g);
                const bool bnd = (u[k] == -s);      // at a bound and pushed outwards
                if (FULL || k < m) vio |= (u[k] == s) && (fabsf(g) > gtol);  // at a bound, pushed inwards
                pos4 = bnd ? 0 : pos4 + 4;
                D[k] = g;
                G[k] = tab(gtab, pos4);
            }
        }
        // ---- Thomas forward elimination w_k = g_k + gamma_{k-1} w_{k-1}, kept as t_k = gamma_k w_k
        float dec = 0.f;
        {
            float tprev = 0.f;
#pragma unroll
            for (int k = 0; k < M; ++k) {
                const float w = D[k] + tprev;
                const float t = G[k] * w;
                dec = fmaf(t, w, dec);              // accumulates g^T H_S^-1 g
                D[k] = t;
                tprev = t;
            }
        }
        asm volatile("" : "+v"(dec));               // summed here, not later from kept products
        if constexpr (DEBUG) {
            // (a row that stops right here has taken no step: its record then holds the start, the
            // bound set and no direction)
            if (rec && it == 0) {
                rec[kRecF] = fcur;
#pragma unroll
                for (int k = 0; k < M; ++k)
                    if (FULL || k < m) {
                        rec[kRecU + k] = u[k];
                        rec[kRecU + 2 * (m + 1) + k] = G[k] == 0.f ? 1.f : 0.f;
                    }
            }
        }
        // A full, unclipped Newton step zeroes the gradient on the free set, and so does any
        // point whose Newton decrement is below what fp32 resolves (see kDecNoise; a start that
        // is already the solution is caught here before any step is taken); if no dual sits on
        // a bound with the gradient pointing inwards, the KKT conditions hold.
        if (active && !vio && (prev_unclipped || dec <= fmaxf(kDecNoise * fcur, gtol * gtol))) {
            active = false; flags = kInfoConverged;
        }
        if (active && it >= kMaxNewtonSteps) { active = false; flags = kInfoCapped; }
        if (!__any(active)) return true;
        steps += active ? 1 : 0;

        // ---- the old x is spent (its differences are in D): fetch the row into the same
        //      registers while the back substitution runs
        reread();
#pragma unroll
        for (int k = 0; k < NMAX; ++k) X[k] = yk(k);
        // ---- back substitution d_k = gamma_k (w_k + d_{k+1}) = t_k + gamma_k d_{k+1}
        {
            float dn = 0.f;
#pragma unroll
            for (int k = M - 1; k >= 0; --k) {
                dn = fmaf(G[k], dn, D[k]);
                D[k] = dn;
            }
        }
        if constexpr (DEBUG) {
            if (rec && it == 0) {
#pragma unroll
                for (int k = 0; k < M; ++k)
                    if (FULL || k < m) rec[kRecU + (m + 1) + k] = D[k];
            }
        }
        // ---- projected step u(alpha) = clip(u - alpha d); alpha = 1 is taken outright when
        //      nothing clips (it is the exact minimiser over the free subspace), otherwise it
        //      must pass the Armijo test (paper Sec. 3.2).  The trial moves the previous dual
        //      into G (the pivots are spent once d is known) and writes the new dual and its x
        //      in place.  A row that fails takes its dual back and retries in the next
        //      iteration with a step length from quadratic interpolation; that is rare (under
        //      one row in a hundred), so the direction is simply recomputed there.
        const float alpha = active ? alpha_try : 0.f;
        float tmax = 0.f;
#pragma unroll
        for (int k = 0; k < M; ++k) {
            const float l = lk(k);
            const float uo = u[k];
            const float t = fmaf(-alpha, D[k], uo);
            tmax = fmaxf(tmax, fabsf(t));
            G[k] = uo;
            u[k] = __builtin_amdgcn_fmed3f(t, -l, l);
        }
        const bool clipped = tmax > lam;
        // ---- A clipped trial point is polished by two sweeps of projected coordinate descent on
        //      the dual (u_k <- clip((u_{k-1} + u_{k+1} + y_{k+1} - y_k) / 2), the exact minimiser of
        //      Eq. 3 over one dual), one in each direction.  The direction was computed as if the
        //      duals that the projection stops were free to move, so the free duals next to them
        //      overshoot: the sweeps repair that locally, only ever lower the dual objective, and
        //      the polished point then has to pass the same Armijo test.  Measured on the
        //      workloads, rejected trials all but vanish (0.17 -> 0.005 per row on post-ReLU maps)
        //      and the slowest row of a wave needs 6 iterations where it needed 16.  The wave does
        //      it for all its unfinished rows whenever one of them clipped.  A row that took the
        //      full step unclipped is still accepted outright (the sweeps lower its objective by
        //      less than the rounding error of the Armijo test), but no longer counts as sitting
        //      on the minimiser of its free subspace: that costs it one more iteration, which the
        //      wave runs anyway for the row that clipped.
        const bool polish = __any(clipped && active);
        if (polish) {
            // (the constant is made opaque so that these differences are formed here, after the
            // direction in D is spent, and not ahead of the branch, where they would need registers
            // of their own)
            float half = 0.5f;
            asm volatile("" : "+v"(half));
#pragma unroll
            for (int k = 0; k < M; ++k) D[k] = half * (X[k + 1] - X[k]);     // X holds y here
            float up = 0.f;
#pragma unroll
            for (int k = 0; k < M; ++k) {
                const float l = lk(k);
                const float un = (k + 1 < M) ? u[k + 1] : 0.f;
                up = __builtin_amdgcn_fmed3f(fmaf(0.5f, up + un, D[k]), -l, l);
                u[k] = up;
            }
            float un = 0.f;
#pragma unroll
            for (int k = M - 1; k >= 0; --k) {
                const float l = lk(k);
                const float ul = (k > 0) ? u[k - 1] : 0.f;
                un = __builtin_amdgcn_fmed3f(fmaf(0.5f, ul + un, D[k]), -l, l);
                u[k] = active ? un : G[k];          // a finished row keeps its dual
                un = u[k];
            }
        }
        bool changed = false;
        float acc = 0.f, prev = 0.f;
#pragma unroll
        for (int k = 0; k < M; ++k) {
            const float c = u[k];
            changed |= (c != G[k]);
            const float xc = X[k] + c - prev;       // X[k] holds y_k here
            acc = fmaf(xc, xc, acc);
            X[k] = xc; prev = c;
        }
        {
            const float xc = X[M] - prev;
            acc = fmaf(xc, xc, acc);
            X[M] = xc;
        }
        const float fc = 0.5f * acc;
        // a row with NaN in it stops here and leaves x = y - D^T u as it stands (NaN at the samples
        // that were NaN at least; the clipping of the sweeps above would otherwise wash the NaN
        // out of the dual and the row would go on as if it were sound)
        if (active && fc != fc) { active = false; flags = kInfoStalled | kInfoPlain; }
        const bool ok = !active || (alpha == 1.f && !clipped) ||
                        (fc <= fcur - kArmijoSigma * alpha * dec + kArmijoSlackEps * fabsf(fcur));
        if (__any(!ok)) {
            reread();
            float pv = 0.f;
#pragma unroll
            for (int k = 0; k < M; ++k) {
                const float c = ok ? u[k] : G[k];
                u[k] = c;
                X[k] = yk(k) + c - pv;
                pv = c;
            }
            X[M] = yk(M) - pv;
            if (!ok) {
                const float den = 2.f * (fc - fcur + dec * alpha);
                const float an = den > 0.f ? dec * alpha * alpha / den : 0.5f * alpha;
                alpha_try = fminf(fmaxf(an, 0.1f * alpha), 0.5f * alpha);
                prev_unclipped = false;
                if (++nfail > kMaxBacktracks) { active = false; flags = kInfoStalled | kInfoPlain; }
            }
        }
        if constexpr (DEBUG) {
            if (rec && ok && active) {
                const int c = (int)rec[0] + 1;
                if (c < kRecMaxF) { rec[kRecF + c] = fc; rec[0] = (float)c; }
            }
        }
        if (ok && active) {
            fcur = fc;
            prev_unclipped = (alpha == 1.f) && !clipped && !polish;
            alpha_try = 1.f;
            nfail = 0;
            if (!changed) {
                // a step that moves nothing: a KKT point if it was a full step with no dual
                // held against an inward gradient, or a full step that the sweeps took back (a
                // point no single dual can improve is the minimiser of a convex function over a
                // box; the inward gradient was rounding noise above the floor); otherwise the line
                // search has run dry
                active = false;
                flags = kInfoStalled | ((alpha == 1.f && (!vio || polish)) ? 0 : kInfoPlain);
            }
        }
        if (!__any(active)) {
            // G holds the previous dual now: rebuild the bound flags of the final one
#pragma unroll
            for (int k = 0; k < M; ++k) {
                const float g = X[k] - X[k + 1];
                G[k] = (u[k] == -copysignf(lk(k), g)) ? 0.f : 1.f;
            }
            return true;
        }
        return false;
    }

    // The same iteration with the paper's other step-size rule (Sec. 3.2): instead of backtracking
    // from alpha = 1 with quadratic interpolation, the kPar step sizes alpha_0 2^-j, j = 0 .. kPar-1,
    // are tried side by side -- one sweep over the duals carries all their trial points and
    // objective values -- and the largest that passes the Armijo test is taken (alpha = 1 outright
    // when nothing clips).  If none passes, the next iteration goes on from alpha_0 2^-kPar.  A
    // second sweep then writes the chosen step, so no previous dual has to be kept.
    static constexpr int kPar = 4;
    __device__ __forceinline__ bool iterate_psearch(int it)
    {
        bool vio = false;
        {
            int pos4 = 0;
#pragma unroll
            for (int k = 0; k < M; ++k) {
                const float g = X[k] - X[k + 1];
                const float s = copysignf(lk(k), g);
                const bool bnd = (u[k] == -s);
                if (FULL || k < m) vio |= (u[k] == s) && (fabsf(g) > gtol);
                pos4 = bnd ? 0 : pos4 + 4;
                D[k] = g;
                G[k] = tab(gtab, pos4);
            }
        }
        float dec = 0.f;
        {
            float tprev = 0.f;
#pragma unroll
            for (int k = 0; k < M; ++k) {
                const float w = D[k] + tprev;
                const float t = G[k] * w;
                dec = fmaf(t, w, dec);
                D[k] = t;
                tprev = t;
            }
        }
        if (active && !vio && (prev_unclipped || dec <= fmaxf(kDecNoise * fcur, gtol * gtol))) {
            active = false; flags = kInfoConverged;
        }
        if (active && it >= kMaxNewtonSteps) { active = false; flags = kInfoCapped; }
        if (!__any(active)) return true;
        steps += active ? 1 : 0;
        reread();
#pragma unroll
        for (int k = 0; k < NMAX; ++k) X[k] = yk(k);
        {
            float dn = 0.f;
#pragma unroll
            for (int k = M - 1; k >= 0; --k) {
                dn = fmaf(G[k], dn, D[k]);
                D[k] = dn;
            }
        }
        // ---- all kPar trial points in one sweep
        const float a0 = active ? alpha_try : 0.f;
        float al[kPar], acc[kPar], pv[kPar];
#pragma unroll
        for (int j = 0; j < kPar; ++j) { al[j] = a0 * (1.0f / (float)(1 << j)); acc[j] = 0.f; pv[j] = 0.f; }
        float tmax = 0.f;
#pragma unroll
        for (int k = 0; k < M; ++k) {
            const float l = lk(k);
#pragma unroll
            for (int j = 0; j < kPar; ++j) {
                const float t = fmaf(-al[j], D[k], u[k]);
                const float c = __builtin_amdgcn_fmed3f(t, -l, l);
                if (j == 0) tmax = fmaxf(tmax, fabsf(t));
                const float xc = X[k] + c - pv[j];          // X[k] holds y_k here
                acc[j] = fmaf(xc, xc, acc[j]);
                pv[j] = c;
            }
        }
#pragma unroll
        for (int j = 0; j < kPar; ++j) {
            const float xc = X[M] - pv[j];
            acc[j] = fmaf(xc, xc, acc[j]);
        }
        const bool clipped = tmax > lam;
        // the largest step that passes
        float alpha = 0.f, fc = fcur;
        bool found = false;
#pragma unroll
        for (int j = kPar - 1; j >= 0; --j) {
            const float fj = 0.5f * acc[j];
            const bool okj = (j == 0 && a0 == 1.f && !clipped) ||
                             (fj <= fcur - kArmijoSigma * al[j] * dec + kArmijoSlackEps * fabsf(fcur));
            if (okj) { alpha = al[j]; fc = fj; found = true; }
        }
        if (!active) { alpha = 0.f; found = true; }
        // ---- the chosen step (alpha = 0: the dual stays, X becomes x(u) again)
        bool changed = false;
        {
            float prev = 0.f;
#pragma unroll
            for (int k = 0; k < M; ++k) {
                const float l = lk(k);
                const float uo = u[k];
                const float c = __builtin_amdgcn_fmed3f(fmaf(-alpha, D[k], uo), -l, l);
                changed |= (c != uo);
                X[k] = X[k] + c - prev;
                u[k] = c; prev = c;
            }
            X[M] = X[M] - prev;
        }
        if (active && !found) {
            alpha_try = al[kPar - 1] * 0.5f;
            prev_unclipped = false;
            nfail += kPar;
            if (nfail > kMaxBacktracks) { active = false; flags = kInfoStalled | kInfoPlain; }
        } else if (active) {
            fcur = fc;
            prev_unclipped = (alpha == 1.f) && !clipped;
            alpha_try = 1.f;
            nfail = 0;
            if (!changed) {
                active = false;
                flags = kInfoStalled | ((alpha == 1.f && !vio) ? 0 : kInfoPlain);
            }
        }
        if (!__any(active)) {
#pragma unroll
            for (int k = 0; k < M; ++k) {
                const float g = X[k] - X[k + 1];
                G[k] = (u[k] == -copysignf(lk(k), g)) ? 0.f : 1.f;
            }
            return true;
        }
        return false;
    }

    // ---- primal recovery.  X is x = y - D^T u at the final dual, bound duals are known; at
    //      its bound duals (flagged by G[k] == 0).  Between two bound duals x is constant up to rounding; every
    //      sample takes the value of the first sample of its block, so that constant runs are
    //      bit-identical, which is what the backward pass keys on.  Rows that stopped without
    //      reaching a KKT point (iteration cap, line search run dry) keep the plain x.
    __device__ __forceinline__ void recover(float (&xs)[NMAX])
    {
        float val = X[0];
        xs[0] = val;
#pragma unroll
        for (int k = 1; k < NMAX; ++k) {
            val = (G[k - 1] == 0.f) ? X[k] : val;
            xs[k] = val;
        }
        const bool plain = (flags & (kInfoCapped | kInfoPlain)) != 0;
        if (__any(plain)) {
#pragma unroll
            for (int k = 0; k < NMAX; ++k) xs[k] = plain ? X[k] : xs[k];
        }
    }
};

// ---------------------------------------------------------------------------------
// Forward kernel: one row per lane.  Grid: see TileMap; waves of a workgroup never wait
// for each other.  With a grouped grid the slots may be visited in a given order (p.order).
// ---------------------------------------------------------------------------------
// WARM: p.addend is given and the solve starts from the dual it encodes (see start_warm).
// PLANE (NMAX = 32, FULL, not PACKED, not WARM): the rows are the columns of contiguous 32 x 32 planes.
// IO16 (NMAX = 32, FULL, PACKED, no addend / second output / residual): y and x are bf16.
// DEBUG: the first p.debug_rows rows leave a step record in p.debug (see step_record_floats).
// PSEARCH: the step size comes from the parallel search over halving step sizes (iterate_psearch).
// (The variants for rows of exactly NMAX samples are asked to leave room for 3 waves per SIMD
// : the 32-sample one fits 150 registers when told so and takes
// some 200 when left alone.  The others are left alone; held to that budget they spill.)
template <int NMAX, bool FULL, bool PACKED, bool WARM = false, bool PLANE = false, bool IO16 = false,
          bool DEBUG = false, bool PSEARCH = false>
__global__ __launch_bounds__(kShortBlock) __attribute__((amdgpu_waves_per_eu((FULL && !DEBUG && !PSEARCH) ? 3 : 1)))
void tv1d_fwd_short_kernel(FwdParams p)
{
    using S = ShortSmem<NMAX>;
    __shared__ float smem[S::kFloats];
    const int lane = threadIdx.x & 63;
    float *tile = smem;
    float *gtab = smem + S::kTileFloats;
    float *rtab = gtab + S::kTabFloats;
    fill_tables<NMAX>(gtab, rtab);

    // (clamped: an order buffer that the caller declared ready may hold anything)
    const uint32_t slot = p.order ? min(p.order[blockIdx.y], gridDim.y - 1u) : blockIdx.y;
    const uint32_t r0 = p.tm.first(__builtin_amdgcn_readfirstlane(blockIdx.x), slot);
    const uint32_t row = p.tm.row(r0, lane);
    const bool valid = row < p.L.n_rows;
    const int n = FULL ? NMAX : p.L.n;
    float lam = 0.f;
    if (p.tm.grouped) lam = fmaxf(p.lam[slot], 0.f);            // one slot per tile
    else if (valid) lam = load_lambda(p.lam, p.L, row);
    const int64_t off = (!PACKED && valid) ? row_offset(p.L, row) : 0;
    static_assert(!PLANE || (NMAX == 32 && FULL && !PACKED), "plane columns: 32 x 32 planes only");
    PlanePair pp = {{0u, 0u}};
    if constexpr (PLANE) {
        pp.row[0] = __builtin_amdgcn_readfirstlane(p.tm.row(r0, 0));
        pp.row[1] = __builtin_amdgcn_readfirstlane(p.tm.row(r0, 32));
    }

    float y[NMAX], xs[NMAX];
    RowSolver<NMAX, FULL, DEBUG> sv;
    if constexpr (DEBUG) {
        if (valid && row < p.debug_rows) {
            sv.rec = p.debug + (size_t)row * step_record_floats(n);
            sv.rec[0] = 0.f; sv.rec[1] = lam;
        }
    }
    if constexpr (PLANE) {
        // (no warm-start variant: the solver's bound masks already fill the scalar registers, the
        // extra pointers of a warm pass spill them, and the spill costs a wave of occupancy)
        static_assert(!(PLANE && WARM), "plane columns: cold start only");
        TileRegs<32> t;
        planes_fetch(p.y, pp, p.L, lane, t);
        if (p.addend) {
            TileRegs<32> a;
            planes_fetch(p.addend, pp, p.L, lane, a);
            tile_add<32>(t, a, 1.f);
        }
        planes_into_tile(t, tile, lane);
        const float *col = plane_column(tile, lane);
#pragma unroll
        for (int k = 0; k < NMAX; ++k) y[k] = col[k * 33];
    } else if constexpr (IO16) {
        static_assert(!IO16 || (NMAX == 32 && FULL && PACKED && !WARM), "bf16 storage: packed rows of 32");
        wave_lds_sync();
        tile16_fetch(reinterpret_cast<const uint16_t *>(p.y), p.tm, r0, p.L.n_rows, lane, tile, p.L.stream);
        wave_lds_sync();
#pragma unroll
        for (int k = 0; k < NMAX; ++k) y[k] = tile[lane * (NMAX + 1) + k];
    } else if constexpr (PACKED && !FULL) {
        // (rows in natural order: the host asks for this variant with the identity tile map only)
        if (WARM || p.addend) {
            float a[NMAX];
            ragged_fetch<NMAX>(p.addend, r0, p.L.n_rows, n, lane, tile, a);
            ragged_fetch<NMAX>(p.y, r0, p.L.n_rows, n, lane, tile, y);
            float run = 0.f;
#pragma unroll
            for (int k = 0; k < NMAX; ++k) {
                y[k] += a[k];
                if constexpr (WARM) {
                    run -= a[k];
                    if (k < NMAX - 1) sv.u[k] = run;
                }
            }
        } else {
            ragged_fetch<NMAX>(p.y, r0, p.L.n_rows, n, lane, tile, y);
        }
    } else if constexpr (PACKED) {
        TileRegs<NMAX> t;
        tile_fetch<NMAX>(p.y, p.tm, r0, p.L.n_rows, lane, t, p.L.stream);
        if (WARM || p.addend) {
            TileRegs<NMAX> a;
            tile_fetch<NMAX>(p.addend, p.tm, r0, p.L.n_rows, lane, a, p.L.stream);
            tile_add<NMAX>(t, a, 1.f);
            if constexpr (WARM) tile_to_neg_prefix<NMAX>(a, tile, lane, sv.u);
        }
        tile_to_rows<NMAX>(t, tile, lane, y);
    } else if constexpr (WARM) {
        row_load_strided_warm<NMAX, FULL>(p.y, p.addend, off, p.L.elem_stride, n, valid, y, sv.u);
    } else {
        row_load_strided<NMAX, FULL>(p.y, p.addend, off, p.L.elem_stride, n, valid, y);
    }
    // park the row in LDS, sample-major
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < NMAX; ++k) tile[k * 64 + lane] = y[k];
    wave_lds_sync();

    sv.yl = tile + lane; sv.gtab = gtab; sv.lam = lam; sv.m = n - 1;
    sv.alpha_try = 1.f; sv.steps = 0; sv.flags = 0; sv.nfail = 0;
    sv.active = valid; sv.prev_unclipped = false;
    if constexpr (WARM) sv.start_warm(y);
    else sv.start(y, rtab[n]);
    if constexpr (PSEARCH) { for (int it = 0; !sv.iterate_psearch(it); ++it) {} }
    else { for (int it = 0; !sv.iterate(it); ++it) {} }
    sv.recover(xs);

    const bool want_resid = p.resid != nullptr;
    float rs[NMAX];
    if (want_resid) {
#pragma unroll
        for (int k = 0; k < NMAX; ++k) rs[k] = tile[k * 64 + lane] - xs[k];
    }
    if constexpr (PLANE) {
        columns_to_planes(xs, tile, lane, p.x, p.x2, pp, p.L);
        if (want_resid) columns_to_planes(rs, tile, lane, p.resid, nullptr, pp, p.L);
    } else if constexpr (IO16) {
        wave_lds_sync();
#pragma unroll
        for (int k = 0; k < NMAX; ++k) tile[lane * (NMAX + 1) + k] = xs[k];
        wave_lds_sync();
        tile16_put(reinterpret_cast<uint16_t *>(p.x), p.tm, r0, p.L.n_rows, lane, tile, p.L.stream);
    } else if constexpr (PACKED && !FULL) {
        ragged_put<NMAX>(p.x, r0, p.L.n_rows, n, lane, tile, xs);
        if (p.x2) ragged_put<NMAX>(p.x2, r0, p.L.n_rows, n, lane, tile, xs);
        if (want_resid) ragged_put<NMAX>(p.resid, r0, p.L.n_rows, n, lane, tile, rs);
    } else if constexpr (PACKED) {
        TileRegs<NMAX> t;
        rows_to_tile<NMAX>(xs, tile, lane, t);
        tile_put<NMAX>(p.x, p.tm, r0, p.L.n_rows, lane, t, p.L.stream);
        if (p.x2) tile_put<NMAX>(p.x2, p.tm, r0, p.L.n_rows, lane, t, p.L.stream);
        if (want_resid) {
            rows_to_tile<NMAX>(rs, tile, lane, t);
            tile_put<NMAX>(p.resid, p.tm, r0, p.L.n_rows, lane, t, p.L.stream);
        }
    } else {
        row_store_strided<NMAX, FULL>(p.x, off, p.L.elem_stride, n, valid, xs);
        if (p.x2) row_store_strided<NMAX, FULL>(p.x2, off, p.L.elem_stride, n, valid, xs);
        if (want_resid) row_store_strided<NMAX, FULL>(p.resid, off, p.L.elem_stride, n, valid, rs);
    }
    if (p.info && valid) p.info[row] = sv.steps | sv.flags;
    if constexpr (DEBUG) {
        if (sv.rec) sv.rec[2] = (float)(sv.steps | sv.flags);
    }
    if (p.seg) {
        // built from the highest dual down, one shift-in per dual, so that bit k ends up at
        // position k.  d = x[k] - x[k+1] is +0 exactly inside a segment (its samples are
        // bit-identical) and carries the sign bit iff x rises; 0 - |d| carries it iff d != 0.
        uint32_t jm = 0, up = 0;
#pragma unroll
        for (int k = NMAX - 2; k >= 0; --k) {
            const float d = xs[k] - xs[k + 1];
            up = __builtin_amdgcn_alignbit(up, __float_as_uint(d), 31);
            jm = __builtin_amdgcn_alignbit(jm, __float_as_uint(0.0f - fabsf(d)), 31);
        }
        if (!FULL) {
            const uint32_t in = n > 1 ? (0xffffffffu >> (33 - n)) : 0u;   // duals 0 .. n-2
            jm &= in; up &= in;
        }
        if (valid) p.seg[row] = make_uint2(jm, up);
    }
}

// ---------------------------------------------------------------------------------
// Backward kernel (paper Eq. 5-6 as segment averaging): one row per lane.
//   segments = maximal runs of bit-equal neighbours in the forward output x, read either
//              from x itself or (SEG) from the code the forward pass wrote for the row;
//   grad_y   = per-segment mean of (g - sub), plus sub;
//   dL/dlam  = sum over jumps k of sign(x[k+1]-x[k]) * (mean_left - mean_right).
// ---------------------------------------------------------------------------------
// PLANE: as in the forward kernel.
// IO16 (NMAX = 32, FULL, PACKED, SEG, no sub): g and gy are bf16.
template <int NMAX, bool FULL, bool PACKED, bool HAS_SUB, bool SEG, bool PLANE = false, bool IO16 = false>
__global__ __launch_bounds__(kShortBlock) void tv1d_bwd_short_kernel(BwdParams p)
{
    using S = ShortSmem<NMAX>;
    __shared__ float smem[S::kFloats];
    const int lane = threadIdx.x & 63;
    float *tile = smem;
    float *gtab = smem + S::kTileFloats;
    float *rtab = gtab + S::kTabFloats;
    fill_tables<NMAX>(gtab, rtab);

    const TileMap tm = {6u, 0u, 0u, 1u};
    const uint32_t r0 = blockIdx.x * 64u;
    const uint32_t row = r0 + lane;
    const bool valid = row < p.L.n_rows;
    const int n = FULL ? NMAX : p.L.n;
    const int64_t off = (!PACKED && valid) ? row_offset(p.L, row) : 0;

    float g[NMAX], x[NMAX];
    uint2 code = make_uint2(0u, 0u);
    if constexpr (SEG) { if (valid) code = p.seg[row]; }
    float sb[NMAX];                   // sub per row (strided path)
    TileRegs<NMAX> st;                // sub in tile order, kept until the store (packed path)
    static_assert(!PLANE || (NMAX == 32 && FULL && !PACKED), "plane columns: 32 x 32 planes only");
    PlanePair pp = {{0u, 0u}};
    if constexpr (PLANE) {
        pp.row[0] = __builtin_amdgcn_readfirstlane(r0);
        pp.row[1] = __builtin_amdgcn_readfirstlane(r0 + 32);
        planes_to_columns(p.g, pp, p.L, tile, lane, g);
        if constexpr (!SEG) planes_to_columns(p.x, pp, p.L, tile, lane, x);
        if constexpr (HAS_SUB) {
            planes_to_columns(p.sub, pp, p.L, tile, lane, sb);
#pragma unroll
            for (int k = 0; k < NMAX; ++k) g[k] -= sb[k];
        }
        wave_lds_sync();
    } else if constexpr (IO16) {
        static_assert(!IO16 || (NMAX == 32 && FULL && PACKED && SEG && !HAS_SUB), "bf16 storage: packed rows of 32");
        wave_lds_sync();                  // the tables are ready
        tile16_fetch(reinterpret_cast<const uint16_t *>(p.g), tm, r0, p.L.n_rows, lane, tile, p.L.stream);
        wave_lds_sync();
#pragma unroll
        for (int k = 0; k < NMAX; ++k) g[k] = tile[lane * (NMAX + 1) + k];
    } else if constexpr (PACKED && !FULL) {
        ragged_fetch<NMAX>(p.g, r0, p.L.n_rows, n, lane, tile, g);
        if constexpr (!SEG) ragged_fetch<NMAX>(p.x, r0, p.L.n_rows, n, lane, tile, x);
        if constexpr (HAS_SUB) {
            ragged_fetch<NMAX>(p.sub, r0, p.L.n_rows, n, lane, tile, sb);
#pragma unroll
            for (int k = 0; k < NMAX; ++k) g[k] -= sb[k];
        }
    } else if constexpr (PACKED) {
        TileRegs<NMAX> tg, tx;
        tile_fetch<NMAX>(p.g, tm, r0, p.L.n_rows, lane, tg, p.L.stream);
        if constexpr (!SEG) tile_fetch<NMAX>(p.x, tm, r0, p.L.n_rows, lane, tx, p.L.stream);
        if constexpr (HAS_SUB) {
            tile_fetch<NMAX>(p.sub, tm, r0, p.L.n_rows, lane, st, p.L.stream);
            tile_add<NMAX>(tg, st, -1.f);
        }
        tile_to_rows<NMAX>(tg, tile, lane, g);
        if constexpr (!SEG) tile_to_rows<NMAX>(tx, tile, lane, x);
    } else {
        row_load_strided<NMAX, FULL>(p.g, nullptr, off, p.L.elem_stride, n, valid, g);
        if constexpr (!SEG) row_load_strided<NMAX, FULL>(p.x, nullptr, off, p.L.elem_stride, n, valid, x);
        if constexpr (HAS_SUB) {
            row_load_strided<NMAX, FULL>(p.sub, nullptr, off, p.L.elem_stride, n, valid, sb);
#pragma unroll
            for (int k = 0; k < NMAX; ++k) g[k] -= sb[k];
        }
        wave_lds_sync();                  // the tables are ready
    }

    // jump after sample k / its direction
    auto jump = [&](int k) -> bool {
        if constexpr (SEG) return (code.x & (1u << k)) != 0u;
        else return x[k + 1] != x[k];
    };
    auto signed_by_jump = [&](int k, float v) -> float {
        if constexpr (SEG) return (code.y & (1u << k)) != 0u ? v : -v;
        else return copysignf(1.f, x[k + 1] - x[k]) * v;
    };
    // forward sweep: segment sums; a segment ends at k when x jumps after k (or the row ends);
    // g[k] is overwritten by the mean of the segment that ends at k
    {
        float s = 0.f;
        int c4 = 0;
#pragma unroll
        for (int k = 0; k < NMAX; ++k) {
            s += g[k];
            c4 += 4;
            const bool last = FULL ? (k == NMAX - 1) : (k >= n - 1);
            const bool end = last || (k + 1 < NMAX && jump(k));
            g[k] = s * *reinterpret_cast<const float *>(reinterpret_cast<const char *>(rtab) + c4);
            if (end) { s = 0.f; c4 = 0; }
        }
    }
    // backward sweep: broadcast each segment's mean; accumulate dL/dlam at the jumps (where
    // there is no jump the two means coincide and the term vanishes by itself)
    float glam = 0.f;
    {
        float carry = 0.f;
#pragma unroll
        for (int k = NMAX - 1; k >= 0; --k) {
            const float right = carry;
            const bool last = FULL ? (k == NMAX - 1) : (k >= n - 1);
            const bool end = last || (k + 1 < NMAX && jump(k));
            carry = end ? g[k] : carry;
            g[k] = carry;
            if (k + 1 < NMAX && (FULL || k < n - 1)) glam += signed_by_jump(k, carry - right);
        }
    }
    if constexpr (PLANE) {
        if constexpr (HAS_SUB) {
#pragma unroll
            for (int k = 0; k < NMAX; ++k) g[k] += sb[k];
        }
        columns_to_planes(g, tile, lane, p.gy, nullptr, pp, p.L);
    } else if constexpr (IO16) {
        wave_lds_sync();
#pragma unroll
        for (int k = 0; k < NMAX; ++k) tile[lane * (NMAX + 1) + k] = g[k];
        wave_lds_sync();
        tile16_put(reinterpret_cast<uint16_t *>(p.gy), tm, r0, p.L.n_rows, lane, tile, p.L.stream);
    } else if constexpr (PACKED && !FULL) {
        if constexpr (HAS_SUB) {
#pragma unroll
            for (int k = 0; k < NMAX; ++k) g[k] += sb[k];
        }
        ragged_put<NMAX>(p.gy, r0, p.L.n_rows, n, lane, tile, g);
    } else if constexpr (PACKED) {
        TileRegs<NMAX> t;
        rows_to_tile<NMAX>(g, tile, lane, t);
        if constexpr (HAS_SUB) tile_add<NMAX>(t, st, 1.f);
        tile_put<NMAX>(p.gy, tm, r0, p.L.n_rows, lane, t, p.L.stream);
    } else {
        if constexpr (HAS_SUB) {
#pragma unroll
            for (int k = 0; k < NMAX; ++k) g[k] += sb[k];
        }
        row_store_strided<NMAX, FULL>(p.gy, off, p.L.elem_stride, n, valid, g);
    }
    if (p.partial) {
        // one value per aligned group of 1 << part_lg rows (lanes), summed in a fixed order
        float v = valid ? glam : 0.f;
        const uint32_t gs = 1u << p.part_lg;
        for (uint32_t d = 1; d < gs; d <<= 1) v += __shfl_xor(v, (int)d);
        if (valid && (lane & (gs - 1u)) == 0u) p.partial[row >> p.part_lg] = v;
    }
}

}  // namespace tvk
