// Kernels for rows longer than 32 samples: T threads share one row, C contiguous samples
// (and duals) per thread, G rows per workgroup.
//
// T = 32 and T = 64 keep a row inside one wavefront (G rows per workgroup, two per wave at
// T = 32); T = 256, 512 and 1024 put one row on a whole workgroup.  The row, its dual and the
// Newton direction stay in registers for the entire solve; only chunk edges, the interface
// system and row-wide reductions go through LDS.
//
// The masked tridiagonal system of paper Eq. 4 is solved by substructuring:
//   1. every thread eliminates the interior of its chunk with the Thomas recurrences
//      (pivots from a table: they depend only on the position inside a free run);
//   2. the last dual of every chunk is a separator; the T separators obey a tridiagonal
//      Schur-complement system whose entries follow from step 1 and from the closed-form
//      corner entries of the inverse of tridiag(-1,2,-1): (A^-1)_11 = m/(m+1),
//      (A^-1)_1m = 1/(m+1); it is solved by parallel cyclic reduction in LDS, stopping as
//      soon as every equation has decoupled;
//   3. every thread back-substitutes its interior with the separator values as boundary
//      terms (a second Thomas pass).
//
// Thread mapping: ROWS (unit element stride): tid = row_in_group * T + t, so a wave reads
// one row's consecutive chunks; COLS (strided samples, e.g. image columns): tid = t * G +
// row_in_group, so adjacent lanes read adjacent columns and global accesses coalesce.
#pragma once
#include "tv_common.hpp"
#include "tv_dispatch.hpp"

namespace tvk {

template <int T, int G, bool COLS>
struct LongMap {
    static constexpr int NT = T * G;
    static constexpr int NW = NT / 64;
    static constexpr int RG = COLS ? G : 1;            // rows interleaved inside a wave
    static constexpr int WPR = COLS ? NW : (T + 63) / 64;   // waves holding parts of one row
    static constexpr int LANES = T < 64 ? T : 64;      // ROWS mapping: lanes of a wave on one row
    // A row that lives in exactly one wave (which holds nothing else) never has to wait for
    // the other waves of its workgroup: its LDS slices are its own, every barrier becomes a
    // wave-level fence and every workgroup vote a wave vote, and the wave leaves when its
    // row is done.
    static constexpr bool PRIVATE = !COLS && T <= 64;
    // One row per workgroup: row-wide flags are workgroup-uniform.
    static constexpr bool SOLO = G == 1;
    __device__ static __forceinline__ int row_of(int tid) { return G == 1 ? 0 : (COLS ? tid % G : tid / T); }
    __device__ static __forceinline__ int t_of(int tid) { return G == 1 ? tid : (COLS ? tid / G : tid % T); }
    // orders LDS writes before later LDS reads among the threads that share rows
    __device__ static __forceinline__ void sync()
    {
        if (PRIVATE) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        } else {
            __syncthreads();
        }
    }
    // sync() plus: does any thread that shares rows with this one pass `pred`?  Across a workgroup
    // the vote rides on the one barrier that the exchange of data needs anyway: every wave leaves
    // its own vote in LDS ahead of the barrier and reads all of them behind it.  `vote` holds two
    // sets of NW flags and `vp` says which one this call uses (it flips with every call, the same
    // in all threads): the set written now was last read two calls ago, a barrier back.
    __device__ static __forceinline__ bool sync_any(bool pred, int *vote, int &vp)
    {
        if (PRIVATE) { sync(); return __any(pred ? 1 : 0) != 0; }
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        const bool mine = __any(pred ? 1 : 0) != 0;
        if (lane == 0) vote[vp * NW + wave] = mine ? 1 : 0;
        __syncthreads();
        const int seen = lane < NW ? vote[vp * NW + lane] : 0;
        vp ^= 1;
        return __any(seen) != 0;
    }
};

// A thread's C contiguous samples k0 .. k0 + C - 1 of a row (zero past the end).  With unit
// stride and 16-byte alignment they move as float4: a wave then touches every cache line of
// its 64 * C samples C / 4 times instead of C times.
// Which group of G rows a workgroup of a strided launch works on.  Workgroups go to the 8 XCDs
// round-robin in launch order, and each XCD has its own L2.  The G adjacent columns of a
// workgroup are 4 G bytes of every image row, a part of a 128-byte line (half of it for G = 16);
// with the identity mapping the other parts belong to the next workgroups, which run on other
// XCDs, so several L2s fetch the whole line (measured with G = 16: twice the algorithmic bytes on
// the read side).  Here the SH = 32 / G workgroups b, b + 8, ..., which the same XCD starts one
// after the other, take the SH neighbouring groups that share a line.
template <int G>
__device__ __forceinline__ uint32_t xcd_grouped(uint32_t b, uint32_t n_groups)
{
    constexpr uint32_t SH = G >= 32 ? 1u : 32u / (uint32_t)G;     // groups per 128-byte line
    if (SH == 1u) return b;
    const uint32_t base = b - b % (8u * SH);
    if (base + 8u * SH > n_groups) return b;        // the ragged end keeps the launch order
    const uint32_t x = b & 7u, s = (b >> 3) % SH;
    return base + SH * x + s;
}

template <int C>
__device__ __forceinline__ bool chunk_vec_ok(const void *base, int64_t off, int64_t es, int k0)
{
    return C % 4 == 0 && es == 1 && (((uintptr_t)base >> 2) + (uint64_t)(off + k0)) % 4 == 0 &&
           ((uintptr_t)base & 3u) == 0;
}

typedef float tv_long_v4f __attribute__((ext_vector_type(4)));

// stream: the tensor is far larger than the last-level cache and touched once per call;
// non-temporal accesses keep such streams from evicting each other.
template <int C>
__device__ __forceinline__ void chunk_load(const float *__restrict__ base, int64_t off, int64_t es,
                                           int k0, int n, bool rvalid, float (&v)[C], bool stream = false)
{
    if (rvalid && chunk_vec_ok<C>(base, off, es, k0)) {
#pragma unroll
        for (int i = 0; i < C; i += 4) {
            if (k0 + i + 3 < n) {
                tv_long_v4f q;
                if (stream) q = __builtin_nontemporal_load(reinterpret_cast<const tv_long_v4f *>(base + off + k0 + i));
                else q = *reinterpret_cast<const tv_long_v4f *>(base + off + k0 + i);
                v[i] = q.x; v[i + 1] = q.y; v[i + 2] = q.z; v[i + 3] = q.w;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[i + e] = (k0 + i + e < n) ? base[off + k0 + i + e] : 0.f;
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < C; ++i) v[i] = (rvalid && k0 + i < n) ? base[off + (int64_t)(k0 + i) * es] : 0.f;
}

template <int C>
__device__ __forceinline__ void chunk_store(float *__restrict__ base, int64_t off, int64_t es, int k0,
                                            int n, bool rvalid, const float (&v)[C], bool stream = false)
{
    if (!rvalid) return;
    if (chunk_vec_ok<C>(base, off, es, k0)) {
#pragma unroll
        for (int i = 0; i < C; i += 4) {
            if (k0 + i + 3 < n) {
                tv_long_v4f q;
                q.x = v[i]; q.y = v[i + 1]; q.z = v[i + 2]; q.w = v[i + 3];
                if (stream) __builtin_nontemporal_store(q, reinterpret_cast<tv_long_v4f *>(base + off + k0 + i));
                else *reinterpret_cast<tv_long_v4f *>(base + off + k0 + i) = q;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (k0 + i + e < n) base[off + k0 + i + e] = v[i + e];
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < C; ++i)
        if (k0 + i < n) base[off + (int64_t)(k0 + i) * es] = v[i];
}

// v of the lane that a row-local DPP pattern names (0xB1 / 0x4E: quad_perm [1,0,3,2] / [2,3,0,1];
// 0x141 / 0x140: mirror within 8 / 16 lanes).
template <int CTRL>
__device__ __forceinline__ float long_dpp(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// Rows of at most 16 threads lie inside one 16-lane DPP row (ROWS mapping: consecutive lanes are
// consecutive threads of a row; two rows share a DPP row when T = 8): a thread then gets the
// value of thread t - S / t + S of its own row from a row shift that rides on the reading
// instruction, instead of a write to LDS, a fence and a read.  Beyond the ends of the row: 0.
// Every lane of the wave must take part: a shift reads 0 from a lane that a branch has switched off.
template <int T, int S>
__device__ __forceinline__ float from_left(float v, int t)
{
    static_assert(T <= 16 && S >= 1 && S < 16, "row shifts stay inside a 16-lane row");
    const float r = long_dpp<0x110 + S>(v);                    // row_shr:S
    return (T < 16 && t < S) ? 0.f : r;
}
template <int T, int S>
__device__ __forceinline__ float from_right(float v, int t)
{
    static_assert(T <= 16 && S >= 1 && S < 16, "row shifts stay inside a 16-lane row");
    const float r = long_dpp<0x100 + S>(v);                    // row_shl:S
    return (T < 16 && t + S >= T) ? 0.f : r;
}
// (Rows of 32 and 64 threads could fetch their direct neighbours by a shift of the whole wave
// (wave_shr:1); measured, that changes nothing for them: their time goes into the PCR steps at
// distances that no single shift covers.)

// Sum over the 64 lanes of a wave, the same total in every lane, in a fixed order: four
// exchanges inside the 16-lane rows ride on the adds themselves (DPP), two cross the rows.
template <int LANES = 64>
__device__ __forceinline__ float wave_sum_all(float v)
{
    v += long_dpp<0xB1>(v);
    v += long_dpp<0x4E>(v);
    v += long_dpp<0x141>(v);
    if (LANES > 8) v += long_dpp<0x140>(v);
    if (LANES > 16) v += __shfl_xor(v, 16);           // LANES = 16: four rows per wave, kept apart
    if (LANES > 32) v += __shfl_xor(v, 32);           // LANES = 32: two rows per wave
    return v;
}

// Sums NV values over the T threads of each row; every thread of the row gets the totals.
// Deterministic: fixed shuffle tree inside a wave, then a fixed-order sum over waves.
template <int T, int G, bool COLS, int NV>
__device__ __forceinline__ void row_sum(float (&v)[NV], float *red, int j, int tid)
{
    using Mp = LongMap<T, G, COLS>;
    if constexpr (Mp::RG == 1) {
#pragma unroll
        for (int q = 0; q < NV; ++q) v[q] = wave_sum_all<Mp::LANES>(v[q]);
    } else {
#pragma unroll
        for (int off = 32; off >= Mp::RG; off >>= 1) {
#pragma unroll
            for (int q = 0; q < NV; ++q) v[q] += __shfl_xor(v[q], off);
        }
    }
    if (Mp::WPR == 1) return;
    const int wave = tid >> 6, lane = tid & 63;
    __syncthreads();
    if (lane < Mp::RG) {
#pragma unroll
        for (int q = 0; q < NV; ++q) red[(q * Mp::NW + wave) * Mp::RG + (COLS ? j : 0)] = v[q];
    }
    __syncthreads();
    const int w0 = COLS ? 0 : j * Mp::WPR;
#pragma unroll
    for (int q = 0; q < NV; ++q) {
        float s = 0.f;
        for (int w = 0; w < Mp::WPR; ++w) s += red[(q * Mp::NW + w0 + w) * Mp::RG + (COLS ? j : 0)];
        v[q] = s;
    }
}

// The same with ONE barrier: consecutive calls alternate between two halves of `red`
// (par = 0, 1, 0, ...), so the writes of a call cannot overtake the reads of the one before.
template <int T, int G, bool COLS, int NV>
__device__ __forceinline__ void row_sum_alt(float (&v)[NV], float *red, int j, int tid, int par)
{
    using Mp = LongMap<T, G, COLS>;
    if constexpr (Mp::RG == 1) {
#pragma unroll
        for (int q = 0; q < NV; ++q) v[q] = wave_sum_all<Mp::LANES>(v[q]);
    } else {
#pragma unroll
        for (int off = 32; off >= Mp::RG; off >>= 1) {
#pragma unroll
            for (int q = 0; q < NV; ++q) v[q] += __shfl_xor(v[q], off);
        }
    }
    if (Mp::WPR == 1) return;
    float *r = red + par * (4 * Mp::NW * Mp::RG);
    const int wave = tid >> 6, lane = tid & 63;
    if (lane < Mp::RG) {
#pragma unroll
        for (int q = 0; q < NV; ++q) r[(q * Mp::NW + wave) * Mp::RG + (COLS ? j : 0)] = v[q];
    }
    __syncthreads();
    const int w0 = COLS ? 0 : j * Mp::WPR;
#pragma unroll
    for (int q = 0; q < NV; ++q) {
        float s = 0.f;
        for (int w = 0; w < Mp::WPR; ++w) s += r[(q * Mp::NW + w0 + w) * Mp::RG + (COLS ? j : 0)];
        v[q] = s;
    }
}

// Maximum of one non-negative value over the T threads of each row.
template <int T, int G, bool COLS>
__device__ __forceinline__ void row_max(float (&v)[1], float *red, int j, int tid)
{
    using Mp = LongMap<T, G, COLS>;
#pragma unroll
    for (int off = (COLS ? 32 : Mp::LANES / 2); off >= Mp::RG; off >>= 1) v[0] = fmaxf(v[0], __shfl_xor(v[0], off));
    if (Mp::WPR == 1) return;
    const int wave = tid >> 6, lane = tid & 63;
    __syncthreads();
    if (lane < Mp::RG) red[wave * Mp::RG + (COLS ? j : 0)] = v[0];
    __syncthreads();
    const int w0 = COLS ? 0 : j * Mp::WPR;
    float s = 0.f;
    for (int w = 0; w < Mp::WPR; ++w) s = fmaxf(s, red[(w0 + w) * Mp::RG + (COLS ? j : 0)]);
    v[0] = s;
}

// Segmented exclusive scan over the T threads of a row, from t = 0 upwards (DIR = +1) or
// from t = T-1 downwards (DIR = -1).  Each thread contributes (closed, s, n): `closed`
// says its chunk holds a segment boundary, and (s, n) describe the part of the chunk
// beyond its last boundary in scan direction (the whole chunk if there is none).
// ADD: open parts accumulate (sums and counts).  !ADD: the value of the nearest closed
// chunk is copied forward.  Returns what arrives at this thread from the scan's origin
// side; zero at the origin.  buf: [2][3][G][T] floats.
template <int T, int G, bool COLS, int DIR, bool ADD>
__device__ __forceinline__ void seg_scan(bool closed, float s, float n, float *buf, int j, int t,
                                         float &cs, float &cn)
{
    using Mp = LongMap<T, G, COLS>;
    if constexpr (!COLS) {
        // A wave holds 64 consecutive threads of one row: scan inside the wave with lane
        // shuffles (no LDS, no barrier), then combine the waves' totals, which takes one
        // barrier.  combine(A earlier, B later) = B if B is closed, else A with B's open part
        // added (ADD) or A unchanged (copy).
        constexpr int LN = Mp::LANES;                     // lanes of the wave that hold this row
        const int lane = t & (LN - 1);
        float f = closed ? 1.f : 0.f;
#pragma unroll
        for (int d = 1; d < LN; d <<= 1) {
            const float of = DIR > 0 ? __shfl_up(f, d, LN) : __shfl_down(f, d, LN);
            const float os = DIR > 0 ? __shfl_up(s, d, LN) : __shfl_down(s, d, LN);
            const float on = DIR > 0 ? __shfl_up(n, d, LN) : __shfl_down(n, d, LN);
            const bool has = DIR > 0 ? (lane >= d) : (lane + d < LN);
            if (has && f == 0.f) {
                if (ADD) { s += os; n += on; } else { s = os; n = on; }
                f = of;
            }
        }
        // what arrives at this lane from inside its wave: the inclusive value of the lane before
        float ef = DIR > 0 ? __shfl_up(f, 1, LN) : __shfl_down(f, 1, LN);
        float es = DIR > 0 ? __shfl_up(s, 1, LN) : __shfl_down(s, 1, LN);
        float en = DIR > 0 ? __shfl_up(n, 1, LN) : __shfl_down(n, 1, LN);
        const bool edge = DIR > 0 ? (lane == 0) : (lane == LN - 1);
        if (edge) { ef = 0.f; es = 0.f; en = 0.f; }
        if constexpr (T > 64) {
            constexpr int NWR = T / 64;                       // waves per row
            float *tot = buf + (DIR > 0 ? 0 : 3 * G * NWR);   // the two directions never share
            const int w = t >> 6;
            const bool lastlane = DIR > 0 ? (lane == LN - 1) : (lane == 0);
            if (lastlane) {
                tot[(0 * G + j) * NWR + w] = f; tot[(1 * G + j) * NWR + w] = s; tot[(2 * G + j) * NWR + w] = n;
            }
            __syncthreads();
            // Exclusive scan over the waves' totals, done by every wave for itself: lane q (< NWR)
            // takes the totals of the q-th wave in scan order, a segmented inclusive scan runs
            // over those lanes (row-shift DPP: NWR <= 16 lanes lie in one DPP row), and the wave
            // picks the lane before its own position (a uniform index).
            static_assert(NWR <= 16, "the waves' totals must fit one 16-lane DPP row");
            const int wl = t & 63;
            float bf = 0.f, bs = 0.f, bn = 0.f;
            if (wl < NWR) {
                const int ww = DIR > 0 ? wl : NWR - 1 - wl;
                bf = tot[(0 * G + j) * NWR + ww]; bs = tot[(1 * G + j) * NWR + ww]; bn = tot[(2 * G + j) * NWR + ww];
            }
#define TV_SHR(v, D) __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x110 + (D), 0xf, 0xf, true))
#define TV_STEP(D)                                                                         \
            if constexpr ((D) < NWR) {                                                     \
                const float of = TV_SHR(bf, D), os = TV_SHR(bs, D), on = TV_SHR(bn, D);    \
                if (wl >= (D) && bf == 0.f) {                                              \
                    if (ADD) { bs += os; bn += on; } else { bs = os; bn = on; }            \
                    bf = of;                                                               \
                }                                                                          \
            }
            TV_STEP(1) TV_STEP(2) TV_STEP(4) TV_STEP(8)
#undef TV_STEP
#undef TV_SHR
            const int qme = DIR > 0 ? w : NWR - 1 - w;                 // this wave's position in scan order
            const int src = __builtin_amdgcn_readfirstlane(qme > 0 ? qme - 1 : 0);
            float af = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(bf), src));
            float as = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(bs), src));
            float an = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(bn), src));
            if (qme == 0 || (!ADD && af == 0.f)) { as = 0.f; an = 0.f; }
            // combine(waves before, lanes before)
            if (ef == 0.f) {
                if (ADD) { es += as; en += an; } else { es = as; en = an; }
            }
        }
        cs = es; cn = en;
        return;
    } else {
#define TV_B(c, q, tt) buf[(((c) * 3 + (q)) * G + j) * T + (tt)]
    float f = closed ? 1.f : 0.f;
    int cur = 0;
    for (int d = 1; d < T; d <<= 1) {
        TV_B(cur, 0, t) = f; TV_B(cur, 1, t) = s; TV_B(cur, 2, t) = n;
        Mp::sync();
        const int o = t - DIR * d;
        if (o >= 0 && o < T && f == 0.f) {
            const float of = TV_B(cur, 0, o), os = TV_B(cur, 1, o), on = TV_B(cur, 2, o);
            if (ADD) { s += os; n += on; } else { s = os; n = on; }
            f = of;
        }
        cur ^= 1;
    }
    TV_B(cur, 1, t) = s; TV_B(cur, 2, t) = n;
    Mp::sync();
    const int o = t - DIR;
    cs = 0.f; cn = 0.f;
    if (o >= 0 && o < T) { cs = TV_B(cur, 1, o); cn = TV_B(cur, 2, o); }
    Mp::sync();
#undef TV_B
    }
}

// Pitch of the tile through which the transposing kernels turn G strided rows: T chunks of C
// samples with a pad word each (a wave's chunk accesses t * (C + 1) + i then hit 32 different
// banks per half wave with any pitch), rounded up so that consecutive rows start 32 / G banks
// apart: the transposing accesses of half a wave are G rows x 32 / G neighbouring samples, which
// then cover the 32 banks exactly once.  (With an odd pitch, which serves only G = 32, 9 % of
// the LDS cycles of the sixteen-row forward kernels were bank conflicts, 31 % of the backward
// kernels' and 49 % of the eight-row forward kernels'.)
template <int T, int C, int G>
constexpr int xpose_tile_pitch()
{
    constexpr int base = T * (C + 1);
    constexpr int want = G >= 32 ? 1 : 32 / G;
    return base + ((want - base % 32) + 32) % 32;
}

template <int T, int C, int G, bool COLS>
struct LongSmem {
    using Mp = LongMap<T, G, COLS>;
    static constexpr int TP = T + 2;                   // one zero sentinel on either side
    float gtab[C + 2];
    float rtab[C + 2];                                 // rtab[m] = 1 / (m + 1) = 1 - gtab[m]
    float ex[5][G][TP];
    float buf[2 * 3 * G * T];
    float red[2 * 4 * Mp::NW * Mp::RG];
    int   vote[2 * Mp::NW];                            // workgroup votes (LongMap::sync_any)
};

// The backward kernel exchanges two values per thread and scans through LDS only where a row
// spans several waves: a smaller footprint lets more workgroups share a CU.
template <int T, int C, int G, bool COLS>
struct LongSmemBwd {
    using Mp = LongMap<T, G, COLS>;
    static constexpr int TP = T + 2;
    float ex[2][G][TP];
    float buf[COLS ? 2 * 3 * G * T : (T > 64 ? 2 * 3 * G * (T / 64) : 1)];
    float red[2 * 4 * Mp::NW * Mp::RG];
};

// ---------------------------------------------------------------------------------
// Forward: projected Newton on the dual (paper Eq. 3-4), one row per T threads.
// ---------------------------------------------------------------------------------
//
// XPOSE (strided samples, T <= 64): global memory is accessed as in the COLS mapping (adjacent
// lanes <-> adjacent rows, so that the accesses coalesce), but the G rows of the workgroup
// are transposed through an LDS tile on the way in and out, and the solve itself runs in the
// ROWS mapping with one row per wave, i.e. without any workgroup barrier.
// WARM = 1: p.addend is given and the solve starts from the dual it encodes.
// WARM = 3: the cold start picks between two candidates (see there); for long rows that cannot
// take the multilevel start.
// WARM = 2 (unit-stride rows, C a multiple of kMlFactor): rows flagged in p.ml_flag start from
// the dual of the same row averaged in groups of kMlFactor samples (p.coarse_u), which a launch
// on the averaged rows with lambda / kMlFactor left behind (p.dual_out of that launch).
// DEBUG: the first p.debug_rows rows leave a step record in p.debug (see step_record_floats).

// Waves per SIMD that the forward kernel asks the register allocator for (the second argument
// of __launch_bounds__; 1 = no request).  Left alone, the kernels with 8 samples per thread take
// 85-96 VGPRs and those with 12 take 100-108: a few registers above the step to one more
// resident wave (80 for six, 96 for five).  These kernels wait 40-50 % of their time (barriers,
// LDS exchanges, the drain of a launch in partly filled rounds), so where the allocator can
// get below the step with at most a handful of spilled registers the extra wave pays:
// 12 288 columns of 512 samples 57 -> 52 us (three 512-thread workgroups per CU, two rounds
// instead of three), warm row passes of the same 2-3 %, 3000 rows of 3000 samples 910 -> 730 us.
// Not requested where it costs 10-18 spilled registers (128 threads x 12 samples, and the
// transposing kernel with 32 x 12): those ran 2-3 % slower with it.
template <int T, int C, int G, bool COLS, bool XPOSE>
constexpr int fwd_waves_per_simd()
{
    if (T * G == 512 && !COLS) return 4;        // at most 128 VGPRs: a CU holds two such workgroups
    if (XPOSE && C <= 4) return 8;
    if (C == 8 && (T * G <= 256 || (XPOSE && T * G == 512))) return 6;
    if (C == 12 && T * G <= 256 && T != 128 && !(XPOSE && T == 32)) return 5;
    // (64 threads x 16 samples from an addend's dual: 130 VGPRs left alone, 128 and a fourth wave
    // on request; six images of 1024 x 1024, K = 3: 434 -> 418 us)
    if (C == 16 && T * G <= 256) return 4;
    return 1;
}
template <int T, int C, int G, bool COLS, bool XPOSE = false, int WARM = 0, bool DEBUG = false>
__global__ __launch_bounds__(T *G, (fwd_waves_per_simd<T, C, G, COLS, XPOSE>())) void tv1d_fwd_long_kernel(FwdParams p)
{
    static_assert(!XPOSE || (COLS && T <= 64), "the transposing variant is for strided rows inside one wave");
    constexpr bool MCOLS = COLS && !XPOSE;             // mapping used by the solve
    using Mp = LongMap<T, G, MCOLS>;
    // a row inside one 16-lane DPP row: neighbours' values by row shifts, not through LDS (from_left)
    constexpr bool DPPX = !MCOLS && T <= 16;
    __shared__ LongSmem<T, C, G, MCOLS> sm;
    // tile[row][k + k / C]: the pad after every chunk makes a wave's chunk reads conflict-free,
    // the pitch does the same for the transposing accesses (xpose_tile_pitch)
    constexpr int TILE_PITCH = xpose_tile_pitch<T, C, G>();
    // The tile is in use before the solve and after it, the exchange and PCR buffers during it:
    // where it fits it lies on top of them (two barriers more), which is what lets a second
    // workgroup share the CU's LDS.
    constexpr bool TILE_ALIAS = XPOSE && (size_t)G * TILE_PITCH * sizeof(float) <= sizeof(sm.ex) + sizeof(sm.buf);
    using Smem = LongSmem<T, C, G, MCOLS>;
    static_assert(__builtin_offsetof(Smem, buf) == __builtin_offsetof(Smem, ex) + sizeof(sm.ex),
                  "ex and buf must be adjacent");
    __shared__ float tile_own[(XPOSE && !TILE_ALIAS) ? G * TILE_PITCH : 1];
    float *tile = TILE_ALIAS ? &sm.ex[0][0][0] : tile_own;
    const int tid = threadIdx.x;
    const int j = Mp::row_of(tid), t = Mp::t_of(tid);
#define TV_EX(q, tt) sm.ex[q][j][(tt) + 1]
#define TV_PB(c, q, tt) sm.buf[(((c) * 3 + (q)) * G + j) * T + (tt)]

    const uint32_t group = COLS ? xcd_grouped<G>(blockIdx.x, gridDim.x) : blockIdx.x;
    const uint32_t row = group * G + j;
    bool rvalid = row < p.L.n_rows;
    bool from_coarse = false;
    if (p.ml_flag && rvalid) {
        const bool flagged = p.ml_flag[(size_t)row * p.flag_pitch] != 0;
        if (p.ml_skip) rvalid = flagged;            // a coarse level: only rows that asked for it
        else from_coarse = WARM == 2 && flagged;
    }
    const int n = p.L.n, M = n - 1;
    const int k0 = t * C;

    if (tid <= C) {
        sm.gtab[tid] = (float)tid / (float)(tid + 1);
        sm.rtab[tid] = 1.0f / (float)(tid + 1);
    }
    if (!TILE_ALIAS && t == 0) {
#pragma unroll
        for (int q = 0; q < 5; ++q) { sm.ex[q][j][0] = 0.f; sm.ex[q][j][T + 1] = 0.f; }
    }
    if (Mp::PRIVATE) __syncthreads();       // the pivot table is the one thing the waves share

    const int64_t off = rvalid ? row_offset(p.L, row) : 0;
    const int64_t es = p.L.elem_stride;
    float lam = rvalid ? load_lambda(p.lam, p.L, row) * p.lam_scale : 0.f;
    float y[C];
    // transposing variant: thread tid moves samples k = tid / G, tid / G + T, ... of row tid % G
    const int xj = tid % G, xk0 = tid / G;
    const uint32_t xrow = group * G + xj;
    const int64_t xoff = (XPOSE && xrow < p.L.n_rows) ? row_offset(p.L, xrow) : 0;
    // Warm start: the addend is D^T u of an earlier solve of nearly the same rows, so
    // u_k = -(addend_0 + .. + addend_k).  u first takes the negated running sums inside the
    // chunk; the chunks before this one are added further down.
    constexpr bool warm = WARM == 1;
    float u[C];
    float wsum = 0.f;                                  // negated sum of the chunk's addend
    if constexpr (XPOSE) {
        // every global load is issued before the first trip through the tile
        const bool xvalid = xrow < p.L.n_rows;
        float ry[C], ra[C];
#pragma unroll
        for (int i = 0; i < C; ++i) {
            const int k = xk0 + i * T;
            ry[i] = (xvalid && k < n) ? p.y[xoff + (int64_t)k * es] : 0.f;
        }
        if (warm || p.addend) {
#pragma unroll
            for (int i = 0; i < C; ++i) {
                const int k = xk0 + i * T;
                ra[i] = (xvalid && k < n) ? p.addend[xoff + (int64_t)k * es] : 0.f;
            }
            if constexpr (warm) {
                // the addend alone goes through the tile first
#pragma unroll
                for (int i = 0; i < C; ++i) {
                    const int k = xk0 + i * T;
                    tile[xj * TILE_PITCH + k + k / C] = ra[i];
                }
                __syncthreads();
#pragma unroll
                for (int i = 0; i < C; ++i) {
                    wsum -= tile[j * TILE_PITCH + t * (C + 1) + i];
                    u[i] = wsum;
                }
                __syncthreads();
            }
#pragma unroll
            for (int i = 0; i < C; ++i) ry[i] += ra[i];
        }
#pragma unroll
        for (int i = 0; i < C; ++i) {
            const int k = xk0 + i * T;
            tile[xj * TILE_PITCH + k + k / C] = ry[i];
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < C; ++i) y[i] = tile[j * TILE_PITCH + t * (C + 1) + i];
        if constexpr (TILE_ALIAS) {
            __syncthreads();                // everyone has left the tile: its memory turns into ex / buf
            if (t == 0) {
#pragma unroll
                for (int q = 0; q < 5; ++q) { sm.ex[q][j][0] = 0.f; sm.ex[q][j][T + 1] = 0.f; }
            }
        }
    } else {
        chunk_load<C>(p.y, off, es, k0, n, rvalid, y);
        if (warm || p.addend) {
            float ad[C];
            chunk_load<C>(p.addend, off, es, k0, n, rvalid, ad);
#pragma unroll
            for (int i = 0; i < C; ++i) {
                y[i] += ad[i];
                if (warm) { wsum -= ad[i]; u[i] = wsum; }
            }
        }
    }
    // rounding floor of a difference of two x values (|x| <= max|y|, |u| <= lam)
    float gtol;
    {
        float ym[1] = {0.f};
#pragma unroll
        for (int i = 0; i < C; ++i) ym[0] = fmaxf(ym[0], fabsf(y[i]));
        row_max<T, G, MCOLS>(ym, sm.red, j, tid);
        // lam_max = max_k |sum_{i<=k} (mean(y) - y_i)| = max_k |(k / n) sum_{i>k} y_i -
        // ((n - k) / n) sum_{i<=k} y_i| <= 2 k (n - k) / n max|y| <= n / 2 max|y|, and every lambda from
        // lam_max on gives the same minimiser (the row's mean): a lambda beyond that bound is
        // replaced by it, which keeps the dual box, and with it the rounding errors of
        // x = y - D^T u, at the scale of the data.  The cold start needs it (it puts the duals on
        // the bounds), and so does a start from a coarser level's dual, whose stopping tolerance
        // scales with lambda; a pass that starts from the dual an addend encodes is left alone,
        // where the extra dependency cost 3 % of the 2D operator's time.
        if constexpr (WARM != 1) lam = fminf(lam, 0.51f * (float)n * ym[0]);
        gtol = kGradNoise * (ym[0] + lam);
        Mp::sync();
    }

    // duals past the end of the row get an empty box and never move
    const int nvd = min(max(M - k0, 0), C);            // duals of this chunk inside the row
    // (where a row spans several waves the comparison is redone from an opaque copy of nvd in
    // every phase: as a loop invariant the compiler keeps all C results in scalar register pairs
    // for the whole solve, and those kernels then spill scalar registers by the hundred; the
    // wave-per-row kernels have the registers to spare and are 3-5 % faster with the invariant)
    int nv = nvd;
#define TV_NV_REFRESH() do { if constexpr (!Mp::PRIVATE) { nv = nvd; asm volatile("" : "+v"(nv)); } } while (0)
#define TV_LK(i) (((i) < nv) ? lam : 0.0f)
    TV_NV_REFRESH();

    float ynext0;
    if constexpr (DPPX) {
        ynext0 = from_right<T, 1>(y[0], t);
    } else {
        TV_EX(0, t) = y[0];
        Mp::sync();
        ynext0 = TV_EX(0, t + 1);
        Mp::sync();
    }
    // ---- starting point: every dual at the bound its local difference points to, or the
    //      dual the addend encodes, brought into the box (duals within rounding distance of a
    //      bound onto it)
    float fcur;
    float edge_l, edge_r;     // the neighbours' duals next to this chunk, carried between steps
    {
        if (warm) {
            float before, unused;
            seg_scan<T, G, MCOLS, +1, true>(false, wsum, 0.f, sm.buf, j, t, before, unused);
#pragma unroll
            for (int i = 0; i < C; ++i) {
                const float l = TV_LK(i);
                u[i] = __builtin_amdgcn_fmed3f((u[i] + before) * kWarmSnap, -l, l);
            }
        } else {
#pragma unroll
            for (int i = 0; i < C; ++i) {
                const float l = TV_LK(i);
                const float dy = ((i + 1 < C) ? y[i + 1] : ynext0) - y[i];
                u[i] = __builtin_amdgcn_fmed3f(dy * 1e30f, -l, l);
            }
            if constexpr (WARM == 3) {
                // The other candidate: the dual of the constant row, u_k = sum_{i <= k} (mean(y) -
                // y_i), clipped into the box.  It is the solution whenever lam >= lam_max =
                // max_k |u_k|, and from lam_max / 4 on it is the better start by far (few segments:
                // from the bounds every Newton step frees only a few more duals, and random-walk
                // rows of 5000-16 384 samples with lambda from 0.3 lam_max on were still moving
                // after 128 steps; from here they take a handful).  Below lam_max / 4 the bounds
                // win.  Three more row-wide reductions: only the long rows that cannot take the
                // multilevel start pay for it (5-15 % of a cold call).
                int ns = min(max(n - k0, 0), C);               // samples of this chunk inside the row
                asm volatile("" : "+v"(ns));
                float tot[1] = {0.f};
#pragma unroll
                for (int i = 0; i < C; ++i) tot[0] += (i < ns) ? y[i] : 0.f;
                row_sum<T, G, MCOLS, 1>(tot, sm.red, j, tid);
                const float mean = tot[0] / (float)n;
                float mine = 0.f;
#pragma unroll
                for (int i = 0; i < C; ++i) mine += (i < ns) ? mean - y[i] : 0.f;
                float before, unused;
                seg_scan<T, G, MCOLS, +1, true>(false, mine, 0.f, sm.buf, j, t, before, unused);
                float run = before;
                float am[1] = {0.f};
#pragma unroll
                for (int i = 0; i < C; ++i) {
                    run += mean - y[i];
                    if (i < nv) am[0] = fmaxf(am[0], fabsf(run));
                }
                row_max<T, G, MCOLS>(am, sm.red, j, tid);
                if (lam >= 0.25f * am[0]) {                    // (never with a NaN or Inf in the row)
                    run = before;
#pragma unroll
                    for (int i = 0; i < C; ++i) {
                        const float l = TV_LK(i);
                        run += mean - y[i];
                        u[i] = __builtin_amdgcn_fmed3f(run, -l, l);
                    }
                }
                Mp::sync();
            }
        }
        if constexpr (WARM == 2) {
            // Prolongation of the coarse dual.  The coarse row is this row with every group of
            // kMlFactor samples replaced by its mean, and its dual uc solves the same problem
            // restricted to rows that are constant on the groups (lambda / kMlFactor there).
            // At the knot behind a group the fine dual is kMlFactor * uc (exact for a power of
            // two, so bound coarse duals give bound fine duals); inside a group it follows
            // u_k = u_{k-1} + (x_group - y_k) with the group's coarse x, clipped into the box.
            static_assert(WARM != 2 || C % kMlFactor == 0, "groups must not straddle chunks");
            if (from_coarse) {
                constexpr int F = kMlFactor;
                const float *cu = p.coarse_u + (size_t)row * p.coarse_pitch;
                const int j0 = k0 / F;
                float ucl = (j0 > 0 && j0 - 1 < p.coarse_n) ? cu[j0 - 1] : 0.f;
#pragma unroll
                for (int c = 0; c < C / F; ++c) {
                    const float ucr = (j0 + c < p.coarse_n) ? cu[j0 + c] : 0.f;
                    float sum = 0.f, cnt = 0.f;
#pragma unroll
                    for (int r = 0; r < F; ++r)
                        if (k0 + c * F + r < n) { sum += y[c * F + r]; cnt += 1.f; }
                    const float xg = (cnt > 0.f ? sum / cnt : 0.f) + ucr - ucl;
                    float run = (float)F * ucl;
#pragma unroll
                    for (int r = 0; r < F - 1; ++r) {
                        const float l = TV_LK(c * F + r);
                        run += xg - y[c * F + r];
                        u[c * F + r] = __builtin_amdgcn_fmed3f(run, -l, l);
                    }
                    const float l = TV_LK(c * F + F - 1);
                    u[c * F + F - 1] = __builtin_amdgcn_fmed3f((float)F * ucr, -l, l);
                    ucl = ucr;
                }
            }
        }
        float uleft;
        if constexpr (DPPX) {
            uleft = from_left<T, 1>(u[C - 1], t);
            edge_r = from_right<T, 1>(u[0], t);
        } else {
            TV_EX(0, t) = u[C - 1];
            TV_EX(1, t) = u[0];
            Mp::sync();
            uleft = TV_EX(0, t - 1);
            edge_r = TV_EX(1, t + 1);
        }
        edge_l = uleft;
        float acc[1] = {0.f};
#pragma unroll
        for (int i = 0; i < C; ++i) {
            const float xi = y[i] + u[i] - (i > 0 ? u[i - 1] : uleft);
            acc[0] = fmaf(xi, xi, acc[0]);
        }
        row_sum<T, G, MCOLS, 1>(acc, sm.red, j, tid);
        fcur = 0.5f * acc[0];
        Mp::sync();
    }

    bool active = rvalid;
    bool prev_unclipped = false;
    bool prev_tiny = false;          // WARM = 3: the step before moved x by less than the rounding floor
    int steps = 0, flags = 0;
    int par = 0, vp = 0;
    float *rec = nullptr;
    if constexpr (DEBUG) {
        if (rvalid && row < p.debug_rows) {
            rec = p.debug + (size_t)row * step_record_floats(n);
            if (t == 0) { rec[0] = 0.f; rec[1] = lam; rec[kRecF] = fcur; }
        }
    }

    for (int it = 0;; ++it) {
        TV_NV_REFRESH();
        // ---- chunk edges of the dual: exchanged by the accepted trial of the step before
        const float uleft = edge_l;
        const float unext0 = edge_r;

        // ---- gradient, bound set, optimality test, interior elimination (Thomas, pass 1)
        float g[C], gam[C], w[C];
        bool bsep;
        int pos = 0, a = 0;
        bool seen_bound = false;
        float viof[1] = {0.f};
        {
            float wprev = 0.f, gprev = 0.f;
            float xi = y[0] + u[0] - uleft;
#pragma unroll
            for (int i = 0; i < C; ++i) {
                const float xn = (i + 1 < C) ? (y[i + 1] + u[i + 1] - u[i])
                                             : (ynext0 + unext0 - u[C - 1]);
                const float gi = xi - xn;
                g[i] = gi;
                const float s = copysignf(TV_LK(i), gi);
                const bool bnd = (u[i] == -s);
                if (i < nv && u[i] == s && fabsf(gi) > gtol) viof[0] += 1.f;
                if (i < C - 1) {
                    pos = bnd ? 0 : pos + 1;
                    const float gm = sm.gtab[pos];
                    const float wi = fmaf(gprev, wprev, gi);
                    gam[i] = gm; w[i] = wi;
                    wprev = wi; gprev = gm;
                    if (!seen_bound) { if (bnd) seen_bound = true; else a += 1; }
                } else {
                    bsep = bnd;
                }
                xi = xn;
            }
        }
        float p0, pl;
        {
            float pn = 0.f;
            pl = 0.f;
#pragma unroll
            for (int i = C - 2; i >= 0; --i) {
                pn = gam[i] * (w[i] + pn);
                if (i == C - 2) pl = pn;
            }
            p0 = pn;
        }
        // The separator's diagonal is 2 - (A^-1)_{last,last} of this chunk's interior block -
        // (A^-1)_{first,first} of the next one's, with (A^-1)_{first,first} = a / (a + 1) for a
        // leading free duals (likewise at the other end).  Inside a long free run that is
        // 2 - 2 (C - 1) / C: formed from the rounded fractions it loses all but a few bits
        // unless C is a power of two, so the exchange carries 1 - a / (a + 1) = 1 / (a + 1).
        const float c_alpha = sm.rtab[a];                       // 1 - (A^-1)_{first,first}
        const float c_delta = sm.rtab[pos];                     // 1 - (A^-1)_{last,last}
        const float c_beta = (a == C - 1) ? (1.0f / (float)C) : 0.f;  // (A^-1)_{first,last}
        if constexpr (!DPPX) {
            TV_EX(2, t) = p0;
            TV_EX(3, t) = c_alpha;
            TV_EX(4, t) = c_beta;
        }
        bool vio;
        if (Mp::SOLO) {
            vio = Mp::sync_any(viof[0] != 0.f, sm.vote, vp);             // one row: the vote is the row's
        } else {
            row_sum<T, G, MCOLS, 1>(viof, sm.red, j, tid);
            vio = viof[0] != 0.f;
            Mp::sync();
        }
        float p0n, alphan, betan;
        if constexpr (DPPX) {
            p0n = from_right<T, 1>(p0, t); alphan = from_right<T, 1>(c_alpha, t); betan = from_right<T, 1>(c_beta, t);
        } else {
            p0n = TV_EX(2, t + 1); alphan = TV_EX(3, t + 1); betan = TV_EX(4, t + 1);
        }

        if (active && prev_unclipped && !vio) { active = false; flags = kInfoConverged; }
        // (the constant row's dual can leave a dual exactly on its bound with a gradient that is
        // rounding noise, lambda = lam_max being the extreme case: such a dual changes sides with
        // every step and no step is ever clipped-free; a step whose decrement, the squared move of
        // x, is below the floor of a difference of two x values ends the solve there)
        if constexpr (WARM == 3) {
            if (active && prev_tiny && !vio) { active = false; flags = kInfoConverged; }
        }
        if (active && it >= kMaxNewtonSteps) { active = false; flags = kInfoCapped; }
        if (Mp::SOLO) { if (!active) break; }               // row-wide flags are uniform here
        else if (!Mp::sync_any(active, sm.vote, vp)) break;
        steps += active ? 1 : 0;

        // ---- separator system (normalised to unit diagonal) and PCR
        float ea = 0.f, ec = 0.f, er = 0.f;
        if (!bsep) {
            const float inv = __builtin_amdgcn_rcpf(c_delta + alphan);
            ea = -c_beta * inv;
            ec = -betan * inv;
            er = (g[C - 1] + pl + p0n) * inv;
        }
        float sleft;
        if constexpr (DPPX) {
            // the same reduction with the neighbours' equations fetched by row shifts
#define TV_PCR_STEP(S)                                                                              \
            if constexpr ((S) < T) {                                                                \
                if (going && (going = __any((ea != 0.f || ec != 0.f) ? 1 : 0) != 0)) {             \
                    const float la = from_left<T, (S) < T ? (S) : 1>(ea, t), lc = from_left<T, (S) < T ? (S) : 1>(ec, t),      \
                                lr = from_left<T, (S) < T ? (S) : 1>(er, t);                        \
                    const float ra = from_right<T, (S) < T ? (S) : 1>(ea, t), rc = from_right<T, (S) < T ? (S) : 1>(ec, t),    \
                                rr = from_right<T, (S) < T ? (S) : 1>(er, t);                       \
                    const float inv = __builtin_amdgcn_rcpf(1.0f - ea * lc - ec * ra);              \
                    er = (er - ea * lr - ec * rr) * inv;                                            \
                    const float na = -ea * la * inv, nc = -ec * rc * inv;                           \
                    ea = na; ec = nc;                                                               \
                }                                                                                   \
            }
            bool going = true;
            TV_PCR_STEP(1) TV_PCR_STEP(2) TV_PCR_STEP(4) TV_PCR_STEP(8)
#undef TV_PCR_STEP
            sleft = from_left<T, 1>(er, t);
        } else {
            int cur = 0;
            bool published = false;
            for (int s = 1; s < T; s <<= 1) {
                TV_PB(cur, 0, t) = ea; TV_PB(cur, 1, t) = ec; TV_PB(cur, 2, t) = er;
                // every equation decoupled: the right-hand sides just published are the solution
                if (!Mp::sync_any(ea != 0.f || ec != 0.f, sm.vote, vp)) { published = true; break; }
                float la = 0.f, lc = 0.f, lr = 0.f, ra = 0.f, rc = 0.f, rr = 0.f;
                if (t - s >= 0) { la = TV_PB(cur, 0, t - s); lc = TV_PB(cur, 1, t - s); lr = TV_PB(cur, 2, t - s); }
                if (t + s < T) { ra = TV_PB(cur, 0, t + s); rc = TV_PB(cur, 1, t + s); rr = TV_PB(cur, 2, t + s); }
                const float inv = __builtin_amdgcn_rcpf(1.0f - ea * lc - ec * ra);
                er = (er - ea * lr - ec * rr) * inv;
                const float na = -ea * la * inv, nc = -ec * rc * inv;
                ea = na; ec = nc;
                cur ^= 1;
            }
            if (!published) {
                TV_PB(cur, 2, t) = er;
                Mp::sync();
            }
            sleft = t > 0 ? TV_PB(cur, 2, t - 1) : 0.f;
        }
        const float sigma = er;

        // ---- interior back-substitution with the separators as boundary terms (pass 2);
        //      w becomes the Newton direction d
        float decp = 0.f;
        {
            float wprev = 0.f, gprev = 0.f;
#pragma unroll
            for (int i = 0; i < C - 1; ++i) {
                float rhs = g[i];
                if (i == 0) rhs += sleft;
                if (i == C - 2) rhs += sigma;
                const float wi = fmaf(gprev, wprev, rhs);
                w[i] = wi; wprev = wi; gprev = gam[i];
            }
            float dn = 0.f;
#pragma unroll
            for (int i = C - 2; i >= 0; --i) {
                dn = gam[i] * (w[i] + dn);
                w[i] = dn;
                decp = fmaf(g[i], dn, decp);
            }
            w[C - 1] = sigma;
            decp = fmaf(g[C - 1], sigma, decp);
        }

        if constexpr (DEBUG) {
            if (rec && it == 0) {
#pragma unroll
                for (int i = 0; i < C; ++i)
                    if (i < nvd) {
                        rec[kRecU + k0 + i] = u[i];
                        rec[kRecU + n + k0 + i] = w[i];
                        rec[kRecU + 2 * n + k0 + i] = ((i < C - 1) ? (gam[i] == 0.f) : bsep) ? 1.f : 0.f;
                    }
            }
        }
        // ---- projected step with Armijo backtracking (quadratic interpolation)
        float alpha = active ? 1.f : 0.f;
        float uc[C];
        float fc = 0.f, dec = 0.f;
        bool clipped = false, changed = false;
        for (int ls = 0;; ++ls) {
            float v[4] = {0.f, decp, 0.f, 0.f};
            bool cl = false, ch = false;
#pragma unroll
            for (int i = 0; i < C; ++i) {
                const float l = TV_LK(i);
                const float tt = fmaf(-alpha, w[i], u[i]);
                const float cc = __builtin_amdgcn_fmed3f(tt, -l, l);
                cl |= (cc != tt);
                ch |= (cc != u[i]);
                uc[i] = cc;
            }
            float ucleft;
            if constexpr (DPPX) {
                ucleft = from_left<T, 1>(uc[C - 1], t);
                edge_r = from_right<T, 1>(uc[0], t);
            } else {
                TV_EX(0, t) = uc[C - 1];
                TV_EX(1, t) = uc[0];
                Mp::sync();
                ucleft = TV_EX(0, t - 1);
                edge_r = TV_EX(1, t + 1);
            }
            edge_l = ucleft;
#pragma unroll
            for (int i = 0; i < C; ++i) {
                const float xc = y[i] + uc[i] - (i > 0 ? uc[i - 1] : ucleft);
                v[0] = fmaf(xc, xc, v[0]);
            }
            v[2] = cl ? 1.f : 0.f;
            v[3] = ch ? 1.f : 0.f;
            row_sum_alt<T, G, MCOLS, 4>(v, sm.red, j, tid, par);
            par ^= 1;
            fc = 0.5f * v[0]; dec = v[1]; clipped = v[2] > 0.f; changed = v[3] > 0.f;
            const bool ok = !active || alpha == 0.f || (alpha == 1.f && !clipped) ||
                            (fc <= fcur - kArmijoSigma * alpha * dec + kArmijoSlackEps * fabsf(fcur));
            if (Mp::SOLO) { if (ok) break; }                // uniform: every thread sees the row's sums
            else if (!Mp::sync_any(!ok, sm.vote, vp)) break;
            if (!ok) {
                if (ls >= kMaxBacktracks) {
                    alpha = 0.f;
                } else {
                    const float den = 2.f * (fc - fcur + dec * alpha);
                    const float an = den > 0.f ? dec * alpha * alpha / den : 0.5f * alpha;
                    alpha = fminf(fmaxf(an, 0.1f * alpha), 0.5f * alpha);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < C; ++i) u[i] = uc[i];
        prev_unclipped = (alpha == 1.f) && !clipped;
        if constexpr (WARM == 3) prev_tiny = dec <= gtol * gtol;
        // A full Newton step lands on the minimiser of its free set only up to the rounding of
        // the solve, which grows with the step (|d| <= 2 lam).  A cold start ends in small steps;
        // a start from a coarser level's dual can end in its first or second step, and where
        // lambda is large against the data the error of such a step can exceed what the output
        // may be off by.  There a step that moved x by more than 2 % of the data's scale (in the
        // 2-norm; the decrement is that move squared) does not end the solve: the next, small
        // step refines it.  (The scale, 1 + max|y|, is taken back out of gtol.)
        if constexpr (WARM == 2) {
            const float scale = 1.f + fmaxf(gtol * (1.0f / kGradNoise) - lam, 0.f);
            if (lam > 0.25f * scale && !(dec <= fmaxf(gtol * gtol, 4e-4f * scale * scale))) prev_unclipped = false;
        }
        if (active) fcur = fc;
        if constexpr (DEBUG) {
            if (rec && t == 0 && active && alpha > 0.f) {
                const int c = (int)rec[0] + 1;
                if (c < kRecMaxF) { rec[kRecF + c] = fc; rec[0] = (float)c; }
            }
        }
        if (active && !changed) { active = false; flags = kInfoStalled; }
        if (Mp::SOLO) { if (!active) break; }
        else if (!Mp::sync_any(active, sm.vote, vp)) break;
    }

    if (p.dual_out) chunk_store<C>(p.dual_out, (int64_t)row * p.dual_pitch, 1, k0, n, rvalid, u);

    // ---- primal recovery x = y - D^T u, then every block between two bound duals takes
    //      the value of its first sample, so that constant runs are bit-identical
    float xs[C];
    {
        TV_NV_REFRESH();
        float uleft, unext0;
        if constexpr (DPPX) {
            uleft = from_left<T, 1>(u[C - 1], t);
            unext0 = from_right<T, 1>(u[0], t);
        } else {
            TV_EX(0, t) = u[C - 1];
            TV_EX(1, t) = u[0];
            Mp::sync();
            uleft = TV_EX(0, t - 1);
            unext0 = TV_EX(1, t + 1);
        }
        bool bnd[C];
        float xi = y[0] + u[0] - uleft;
#pragma unroll
        for (int i = 0; i < C; ++i) {
            const float xn = (i + 1 < C) ? (y[i + 1] + u[i + 1] - u[i]) : (ynext0 + unext0 - u[C - 1]);
            const float gi = xi - xn;
            bnd[i] = (u[i] == -copysignf(TV_LK(i), gi));
            xs[i] = xi;
            xi = xn;
        }
        // a sample starts a block when the dual on its left is bound; chunk-local pass first
        bool start0;
        if constexpr (DPPX) {
            // (fetched by all lanes before any of them branches: a row shift reads 0 from a lane that is switched off)
            const float left_bound = from_left<T, 1>(bnd[C - 1] ? 1.f : 0.f, t);
            start0 = (t == 0) || (left_bound != 0.f);
        } else {
            TV_EX(2, t) = bnd[C - 1] ? 1.f : 0.f;
            Mp::sync();
            start0 = (t == 0) || (TV_EX(2, t - 1) != 0.f);
        }
        bool closed = start0;
        float last = xs[0];
#pragma unroll
        for (int i = 1; i < C; ++i)
            if (bnd[i - 1]) { closed = true; last = xs[i]; }
        // `last` = first sample of the chunk's last block (valid when closed)
        float cv, cdummy;
        seg_scan<T, G, MCOLS, +1, false>(closed, last, 0.f, sm.buf, j, t, cv, cdummy);
        float val = start0 ? xs[0] : cv;
        float dev[1] = {0.f};
#pragma unroll
        for (int i = 0; i < C; ++i) {
            if (i > 0 && bnd[i - 1]) val = xs[i];
            // (not below four rounding floors of a difference of two x values: the floor follows
            // the row's largest sample, and next to one large sample a converged row's small
            // segments still carry that much noise)
            if (fabsf(val - xs[i]) > fmaxf(2e-5f * (1.f + fabsf(y[i]) + lam), 4.f * gtol)) dev[0] += 1.f;
            u[i] = val;       // u is dead from here on: reuse it for the block values
        }
        row_sum<T, G, MCOLS, 1>(dev, sm.red, j, tid);
        // (an infinite sample makes the floor infinite: such a row keeps its plain output, which shows it)
        const bool use_blocks = !(flags & kInfoCapped) && dev[0] == 0.f && gtol <= 3.0e38f;
        if (use_blocks) {
#pragma unroll
            for (int i = 0; i < C; ++i) xs[i] = u[i];
        } else {
            flags |= 1 << 19;
        }
    }

    if constexpr (XPOSE) {
        // a wave writes only its own row of the tile; the barrier then hands the tile over
        if constexpr (TILE_ALIAS) __syncthreads();      // every wave is done with ex / buf
#pragma unroll
        for (int i = 0; i < C; ++i) tile[j * TILE_PITCH + t * (C + 1) + i] = xs[i];
        __syncthreads();
        for (int k = xk0; k < T * C; k += T)
            if (xrow < p.L.n_rows && k < n) {
                const float v = tile[xj * TILE_PITCH + k + k / C];
                p.x[xoff + (int64_t)k * es] = v;
                if (p.x2) p.x2[xoff + (int64_t)k * es] = v;
            }
        if (p.resid) {
            __syncthreads();
#pragma unroll
            for (int i = 0; i < C; ++i) tile[j * TILE_PITCH + t * (C + 1) + i] = y[i] - xs[i];
            __syncthreads();
            for (int k = xk0; k < T * C; k += T)
                if (xrow < p.L.n_rows && k < n)
                    p.resid[xoff + (int64_t)k * es] = tile[xj * TILE_PITCH + k + k / C];
        }
    } else {
        if (p.x) chunk_store<C>(p.x, off, es, k0, n, rvalid, xs);
        if (p.x2) chunk_store<C>(p.x2, off, es, k0, n, rvalid, xs);
        if (p.resid) {
#pragma unroll
            for (int i = 0; i < C; ++i) y[i] -= xs[i];
            chunk_store<C>(p.resid, off, es, k0, n, rvalid, y);
        }
    }
    if (p.info && rvalid && t == 0) p.info[row] = steps | flags;
    if constexpr (DEBUG) {
        if (rec && t == 0) rec[2] = (float)(steps | flags);
    }
#undef TV_EX
#undef TV_PB
#undef TV_LK
#undef TV_NV_REFRESH
}

// ---------------------------------------------------------------------------------
// Backward (paper Eq. 5-6 as segment averaging), one row per T threads.
// ---------------------------------------------------------------------------------
// XPOSE: as in the forward kernel (strided rows through an LDS tile, one row per wave).
// HAS_SUB: p.sub is given (the reverse sweep of the 2D operator).
// Workgroups of 1024 threads ask for 8 waves per SIMD (at most 64 VGPRs), so that a CU holds two of
// them and one's loads overlap the other's scans.
template <int T, int C, int G, bool COLS, bool XPOSE = false, bool HAS_SUB = false>
__global__ __launch_bounds__(T *G, (T * G == 1024 && !COLS && !HAS_SUB) ? 8 : 1) void tv1d_bwd_long_kernel(BwdParams p)
{
    static_assert(!XPOSE || (COLS && T <= 64), "the transposing variant is for strided rows inside one wave");
    constexpr bool MCOLS = COLS && !XPOSE;
    using Mp = LongMap<T, G, MCOLS>;
    __shared__ LongSmemBwd<T, C, G, MCOLS> sm;
    constexpr int TILE_PITCH = xpose_tile_pitch<T, C, G>();
    __shared__ float tile[XPOSE ? G * TILE_PITCH : 1];
    const int tid = threadIdx.x;
    const int j = Mp::row_of(tid), t = Mp::t_of(tid);
#define TV_EX(q, tt) sm.ex[q][j][(tt) + 1]
    const uint32_t group = COLS ? xcd_grouped<G>(blockIdx.x, gridDim.x) : blockIdx.x;
    const uint32_t row = group * G + j;
    const bool rvalid = row < p.L.n_rows;
    const int n = p.L.n;
    const int k0 = t * C;
    if (t == 0) {
#pragma unroll
        for (int q = 0; q < 2; ++q) { sm.ex[q][j][0] = 0.f; sm.ex[q][j][T + 1] = 0.f; }
    }
    const int64_t off = rvalid ? row_offset(p.L, row) : 0;
    const int64_t es = p.L.elem_stride;

    // transposing variant: thread tid moves samples k = tid / G, tid / G + T, ... of row tid % G
    const int xj = tid % G, xk0 = tid / G;
    const uint32_t xrow = group * G + xj;
    const bool xvalid = XPOSE && xrow < p.L.n_rows;
    const int64_t xoff = xvalid ? row_offset(p.L, xrow) : 0;
    // every global load is issued before the first trip through the tile
    auto fetch = [&](const float *__restrict__ src, float (&raw)[C]) {
#pragma unroll
        for (int i = 0; i < C; ++i) {
            const int k = xk0 + i * T;
            raw[i] = (xvalid && k < n) ? src[xoff + (int64_t)k * es] : 0.f;
        }
    };
    auto turn = [&](const float (&raw)[C], float (&dst)[C]) {
#pragma unroll
        for (int i = 0; i < C; ++i) {
            const int k = xk0 + i * T;
            tile[xj * TILE_PITCH + k + k / C] = raw[i];
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < C; ++i) dst[i] = tile[j * TILE_PITCH + t * (C + 1) + i];
        __syncthreads();
    };

    // g becomes the averaged quantity, then the segment means, then the output; of x only two
    // bits per sample are kept (is there a jump behind it, and does x rise there)
    float g[C], sb[HAS_SUB ? C : 1];
    uint32_t jmask = 0, upmask = 0;
    // duals of this chunk that lie inside the row (dual i sits behind sample k0 + i)
    const int nv = min(max(n - 1 - k0, 0), C);
    const uint32_t inrow = (1u << nv) - 1u;
    {
        float x[C];
        if constexpr (XPOSE) {
            float rg[C], rx[C], rs[HAS_SUB ? C : 1];
            fetch(p.g, rg);
            fetch(p.x, rx);
            if constexpr (HAS_SUB) fetch(p.sub, rs);
            turn(rg, g);
            turn(rx, x);
            if constexpr (HAS_SUB) turn(rs, sb);
        } else {
            chunk_load<C>(p.x, off, es, k0, n, rvalid, x, p.L.stream);
            chunk_load<C>(p.g, off, es, k0, n, rvalid, g, p.L.stream);
            if constexpr (HAS_SUB) chunk_load<C>(p.sub, off, es, k0, n, rvalid, sb, p.L.stream);
        }
        TV_EX(0, t) = x[0];
        Mp::sync();
        const float xnext0 = TV_EX(0, t + 1);
        // jump after sample i (always at the end of the row; samples past the end are their
        // own segments and contribute nothing)
#pragma unroll
        for (int i = 0; i < C; ++i) {
            const float xn = (i + 1 < C) ? x[i + 1] : xnext0;
            if (xn != x[i]) jmask |= 1u << i;
            if (xn > x[i]) upmask |= 1u << i;
        }
    }
    const uint32_t gmask = jmask & inrow;      // jumps that count for dL/dlam
    jmask |= ~inrow;
    if constexpr (HAS_SUB) {
#pragma unroll
        for (int i = 0; i < C; ++i) g[i] -= sb[i];
    }
#define TV_JUMP(i) ((jmask >> (i)) & 1u)
    // chunk-local pieces: head = samples up to and including the first jump, tail = samples
    // after the last jump; both are the whole chunk when it holds no jump
    bool any = false;
    float head_s = 0.f, head_n = 0.f, tail_s = 0.f, tail_n = 0.f;
#pragma unroll
    for (int i = 0; i < C; ++i) {
        if (!any) { head_s += g[i]; head_n += 1.f; }
        tail_s += g[i]; tail_n += 1.f;
        if (TV_JUMP(i)) { any = true; tail_s = 0.f; tail_n = 0.f; }
    }
    float ls, ln, rs, rn;
    seg_scan<T, G, MCOLS, +1, true>(any, tail_s, tail_n, sm.buf, j, t, ls, ln);   // open part on the left
    seg_scan<T, G, MCOLS, -1, true>(any, head_s, head_n, sm.buf, j, t, rs, rn);   // open part on the right

    // per-sample means: forward pass accumulates, backward pass broadcasts
    float (&mean)[C] = g;
    {
        float s = ls, c = ln;
#pragma unroll
        for (int i = 0; i < C; ++i) {
            s += g[i]; c += 1.f;
            mean[i] = 0.f;
            if (TV_JUMP(i)) { mean[i] = s * __builtin_amdgcn_rcpf(c); s = 0.f; c = 0.f; }
        }
        // trailing open part continues into the next chunks
        const float open_mean = (c > 0.f) ? (s + rs) * __builtin_amdgcn_rcpf(c + rn) : 0.f;
        float carry = open_mean;
#pragma unroll
        for (int i = C - 1; i >= 0; --i) {
            if (TV_JUMP(i)) carry = mean[i];
            mean[i] = carry;
        }
    }
    // a head piece that is closed inside this chunk still needs nothing from the right; a
    // head piece open to the left got (ls, ln) above.  dL/dlam needs the next chunk's first mean.
    TV_EX(1, t) = mean[0];
    Mp::sync();
    const float mnext0 = TV_EX(1, t + 1);
    float gl[1] = {0.f};
#pragma unroll
    for (int i = 0; i < C; ++i) {
        if ((gmask >> i) & 1u) {
            const float mn = (i + 1 < C) ? mean[i + 1] : mnext0;
            const float sg = ((upmask >> i) & 1u) ? 1.f : -1.f;
            gl[0] = fmaf(sg, mean[i] - mn, gl[0]);
        }
    }
    if constexpr (HAS_SUB) {
#pragma unroll
        for (int i = 0; i < C; ++i) mean[i] += sb[i];
    }
    if constexpr (XPOSE) {
#pragma unroll
        for (int i = 0; i < C; ++i) tile[j * TILE_PITCH + t * (C + 1) + i] = mean[i];
        __syncthreads();
        for (int k = xk0; k < T * C; k += T)
            if (xvalid && k < n) p.gy[xoff + (int64_t)k * es] = tile[xj * TILE_PITCH + k + k / C];
    } else {
        chunk_store<C>(p.gy, off, es, k0, n, rvalid, mean, p.L.stream);
    }
    if (p.partial) {
        row_sum<T, G, MCOLS, 1>(gl, sm.red, j, tid);
        if (rvalid && t == 0) p.partial[row] = gl[0];
    }
#undef TV_EX
#undef TV_JUMP
}

// ---------------------------------------------------------------------------------
// Launchers: pick threads-per-row T and samples-per-thread C from the row length.
// ---------------------------------------------------------------------------------
template <int T, int C, int G, bool COLS>
inline hipError_t launch_fwd_long_t(const FwdParams &p, hipStream_t s)
{
    const dim3 grid((p.L.n_rows + G - 1) / G), block(T * G);
    constexpr bool XP = COLS && T <= 64;
    if (p.warm == 2) {
        if constexpr (!COLS && C % kMlFactor == 0)
            hipLaunchKernelGGL((tv1d_fwd_long_kernel<T, C, G, COLS, XP, 2>), grid, block, 0, s, p);
        else
            return hipErrorInvalidValue;
    } else if (p.warm == 3 && T * C > 768) {
        // (cold, with the constant row's dual as a second candidate: rows of 769 samples and more)
        if constexpr (T * C > 768)
            hipLaunchKernelGGL((tv1d_fwd_long_kernel<T, C, G, COLS, XP, 3>), grid, block, 0, s, p);
    } else if (p.warm == 1)
        hipLaunchKernelGGL((tv1d_fwd_long_kernel<T, C, G, COLS, XP, 1>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((tv1d_fwd_long_kernel<T, C, G, COLS, XP, 0>), grid, block, 0, s, p);
    return hipGetLastError();
}

template <int T, int C, int G, bool COLS>
inline hipError_t launch_bwd_long_t(const BwdParams &p, hipStream_t s)
{
    const dim3 grid((p.L.n_rows + G - 1) / G), block(T * G);
    constexpr bool XP = COLS && T <= 64;
    if (p.sub)
        hipLaunchKernelGGL((tv1d_bwd_long_kernel<T, C, G, COLS, XP, true>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((tv1d_bwd_long_kernel<T, C, G, COLS, XP, false>), grid, block, 0, s, p);
    return hipGetLastError();
}

// GX: strided rows of 193-768 samples per workgroup of the transposing kernels.  Forward 8: a
// workgroup of 512 threads (at most 128 registers each) leaves room for a second one on the CU,
// whose loads and transposes then overlap the first one's solve (with 16 rows, 1024 threads, a CU
// holds one workgroup and every phase waits for the slowest wave; 24 images of 512 x 512: column
// pass 61 -> 57 us, K = 4 forward 313 -> 295; 12 of 768 x 768: 48 -> 42, 372 -> 344; columns of
// 769-1024 samples need 139 registers that way and are slower, 44 -> 48).  Backward 16: it is
// bound by memory, and 8 adjacent columns are 32 bytes of every image row (24 images of
// 512 x 512, K = 4 reverse sweep: 205 us with 16 rows, 232 with 8).
#define TV_LONG_DISPATCH(FN, p, s, GX)                                                    \
    do {                                                                                  \
        const int n = (p).L.n;                                                            \
        const bool cols = (p).L.elem_stride != 1;                                         \
        const int64_t wide = tvd::get(tvd::kThreadPerSampleWideRows);                     \
        if (cols) {                                                                       \
            if (n <= 32 && (int64_t)(p).L.n_rows <= wide) return FN<16, 2, 16, true>(p, s);        \
            if (n <= 32) return FN<8, 4, 16, true>(p, s);                                 \
            if (n <= 64) return FN<8, 8, 16, true>(p, s);                                 \
            if (n <= 96) return FN<8, 12, 16, true>(p, s);                                \
            if (n <= 128) return FN<16, 8, 16, true>(p, s);                               \
            if (n <= 192) return FN<16, 12, 16, true>(p, s);                              \
            if (n <= 256) return FN<32, 8, GX, true>(p, s);                               \
            if (n <= 384) return FN<32, 12, GX, true>(p, s);                              \
            if (n <= 512) return FN<64, 8, GX, true>(p, s);                               \
            if (n <= 768) return FN<64, 12, GX, true>(p, s);                              \
            if (n <= 1024) return FN<64, 16, 16, true>(p, s);                             \
            if (n <= 1536) return FN<128, 12, 8, true>(p, s);                             \
            if (n <= 2048) return FN<128, 16, 8, true>(p, s);                             \
            if (n <= 3072) return FN<256, 12, 4, true>(p, s);                             \
            if (n <= 4096) return FN<256, 16, 4, true>(p, s);                             \
            if (n <= 8192) return FN<1024, 8, 1, true>(p, s);                             \
            if (n <= 12288) return FN<1024, 12, 1, true>(p, s);                           \
            return FN<1024, 16, 1, true>(p, s);                                           \
        }                                                                                 \
        if (n <= 32 && (int64_t)(p).L.n_rows <= wide) return FN<16, 2, 16, false>(p, s);           \
        if (n <= 32) return FN<8, 4, 32, false>(p, s);                                    \
        if (n <= 64) return FN<8, 8, 32, false>(p, s);                                    \
        if (n <= 96) return FN<8, 12, 32, false>(p, s);                                   \
        if (n <= 128) return FN<16, 8, 16, false>(p, s);                                  \
        if (n <= 192) return FN<16, 12, 16, false>(p, s);                                 \
        if (n <= 256) return FN<32, 8, 8, false>(p, s);                                   \
        if (n <= 384) return FN<32, 12, 8, false>(p, s);                                  \
        if (n <= 512) return FN<64, 8, 4, false>(p, s);                                   \
        if (n <= 768) return FN<64, 12, 4, false>(p, s);                                  \
        if (n <= 1024) return FN<64, 16, 4, false>(p, s);                                 \
        if (n <= 1536) return FN<128, 12, 2, false>(p, s);                                \
        if (n <= 2048) return FN<256, 8, 1, false>(p, s);                                 \
        if (n <= 3072) return FN<256, 12, 1, false>(p, s);                                \
        if (n <= 4096) return FN<256, 16, 1, false>(p, s);                                \
        if (n <= 6144) return FN<512, 12, 1, false>(p, s);                                \
        if (n <= 8192) return FN<512, 16, 1, false>(p, s);                                \
        if (n <= 12288) return FN<1024, 12, 1, false>(p, s);                              \
        return FN<1024, 16, 1, false>(p, s);                                              \
    } while (0)

inline hipError_t launch_fwd_long(const FwdParams &p, hipStream_t s)
{
    TV_LONG_DISPATCH(launch_fwd_long_t, p, s, 8);
}

// The forward launch with step records (cold start, unit-stride rows): one mapping of each kind
// -- rows inside a wave (wave-level fences, PCR over the wave's separators), and a workgroup per
// row with 256 and with 1024 threads (workgroup barriers, PCR in LDS across waves).
inline hipError_t launch_fwd_long_debug(const FwdParams &p, hipStream_t s)
{
    const int n = p.L.n;
    if (n <= 512)
        hipLaunchKernelGGL((tv1d_fwd_long_kernel<64, 8, 4, false, false, 0, true>), dim3((p.L.n_rows + 3) / 4),
                           dim3(256), 0, s, p);
    else if (n <= 4096)
        hipLaunchKernelGGL((tv1d_fwd_long_kernel<256, 16, 1, false, false, 0, true>), dim3(p.L.n_rows), dim3(256), 0,
                           s, p);
    else
        hipLaunchKernelGGL((tv1d_fwd_long_kernel<1024, 16, 1, false, false, 0, true>), dim3(p.L.n_rows), dim3(1024),
                           0, s, p);
    return hipGetLastError();
}

inline hipError_t launch_bwd_long(const BwdParams &p, hipStream_t s)
{
    TV_LONG_DISPATCH(launch_bwd_long_t, p, s, 16);
}

}  // namespace tvk
