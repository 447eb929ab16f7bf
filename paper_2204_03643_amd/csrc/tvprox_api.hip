// C-ABI entry points of the TV-prox library: argument validation, path selection and
// kernel launches.  Nothing here allocates or synchronises; the only state is the address of
// the static scratch array of tv1d_prox_bwd_noalloc, looked up once per device.
#include "../../include/tvprox.h"

#include <hip/hip_runtime.h>

#include <mutex>
#include <string.h>

#include "tv_common.hpp"
#include "tv_dispatch.hpp"
#include "tv_long.hpp"
#include "tv_small2d.hpp"
#include "tv_plane2d.hpp"
#include "tv_short.hpp"

// Scratch of tv1d_prox_bwd_noalloc (the per-row dL/dlam terms between the backward kernel and
// the per-slot reduction): every GPU the library runs on holds its own copy until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress; kernels are handed
// the address that call returns for the current device.
static __device__ __align__(256) float scratch[TV_NOALLOC_MAX_ROWS];

namespace {

using tvk::BwdParams;
using tvk::FwdParams;
using tvk::Layout;

constexpr int64_t kMaxRows = 0x7fffffff;

inline size_t align16(size_t b) { return (b + 15) & ~(size_t)15; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// ---- validation -------------------------------------------------------------------

// Checks the row set; on TV_OK with *n_rows == 0 there is nothing to do.
int check_rows(const tv_rows &r, int64_t *n_rows)
{
    *n_rows = 0;
    if (r.n_outer < 0 || r.n_inner < 0 || r.length < 1) return TV_ERR_SHAPE;
    if (r.n_outer == 0 || r.n_inner == 0) return TV_OK;
    if (r.n_outer > kMaxRows || r.n_inner > kMaxRows || r.n_outer * r.n_inner > kMaxRows)
        return TV_ERR_SHAPE;
    // Non-overlap: with the (stride, extent) pairs sorted by stride, every stride must
    // cover the full span of the faster-varying ones.
    int64_t st[3] = {r.elem_stride, r.inner_stride, r.outer_stride};
    int64_t ex[3] = {r.length, r.n_inner, r.n_outer};
    int cnt = 0;
    int64_t s[3], e[3];
    for (int i = 0; i < 3; ++i)
        if (ex[i] > 1) {
            if (st[i] < 1) return TV_ERR_STRIDE;
            s[cnt] = st[i]; e[cnt] = ex[i]; ++cnt;
        }
    for (int i = 0; i < cnt; ++i)
        for (int j = i + 1; j < cnt; ++j)
            if (s[j] < s[i]) {
                int64_t t = s[i]; s[i] = s[j]; s[j] = t;
                t = e[i]; e[i] = e[j]; e[j] = t;
            }
    int64_t span = 1;
    for (int i = 0; i < cnt; ++i) {
        if (s[i] < span) return TV_ERR_STRIDE;
        if (e[i] > (INT64_MAX / 8) / s[i]) return TV_ERR_SHAPE;
        span = s[i] * e[i];
    }
    *n_rows = r.n_outer * r.n_inner;
    return TV_OK;
}

int check_lambda(const tv_lambda &l)
{
    if (l.count < 1 || l.div < 1 || l.count > kMaxRows || l.div > kMaxRows) return TV_ERR_LAMBDA;
    return TV_OK;
}

Layout make_layout(const tv_rows &r, const tv_lambda &l, int64_t n_rows)
{
    Layout L;
    L.n_rows = (uint32_t)n_rows;
    L.n_inner = (uint32_t)r.n_inner;
    L.outer_stride = r.outer_stride;
    L.inner_stride = r.inner_stride;
    L.elem_stride = r.elem_stride;
    L.n = (int32_t)r.length;
    L.lam_count = (uint32_t)l.count;
    L.lam_div = (uint32_t)l.div;
    // a tensor of 32 MiB or more does not survive in the caches until it is touched again
    L.stream = (n_rows * r.length >= tvd::get(tvd::kStreamBytes) / 4) ? 1u : 0u;
    return L;
}

// Tiles of 64 rows for the row-per-lane forward kernel: grouped by lambda slot when the slot
// pattern allows it (lam.div a power of two below 64, every slot a whole number of tiles).
tvk::TileMap make_tile_map(const tv_lambda &l, int64_t n_rows)
{
    tvk::TileMap tm = {6u, 0u, 0u, 1u};
    const int64_t div = l.div, count = l.count;
    if (count > 1 && div < 64 && (div & (div - 1)) == 0 && n_rows % (64 * count) == 0 &&
        count * div <= 0x7fffffff && count <= 65535) {
        uint32_t lg = 0;
        while ((1 << lg) < div) ++lg;
        tm.lg = lg;
        tm.hop = (uint32_t)(count * div);
        tm.grouped = 1u;
        tm.count = (uint32_t)count;
    }
    return tm;
}

// Rows are "packed" when row r starts exactly r*length elements after the base.
bool rows_packed(const tv_rows &r)
{
    if (r.length > 1 && r.elem_stride != 1) return false;
    if (r.n_inner > 1 && r.inner_stride != r.length) return false;
    if (r.n_outer > 1 && r.outer_stride != r.n_inner * r.length) return false;
    return true;
}

// Rows that are the columns of contiguous 32 x 32 planes (row id = plane * 32 + column).
bool rows_are_plane_columns(const tv_rows &r)
{
    return r.length == 32 && r.elem_stride == 32 && r.n_inner == 32 && r.inner_stride == 1 &&
           (r.n_outer == 1 || (r.outer_stride >= 1024 && r.outer_stride % 4 == 0));
}

int launch_status()
{
    return hipGetLastError() == hipSuccess ? TV_OK : TV_ERR_HIP;
}

// ---- short rows: one row per lane ---------------------------------------------------

template <int NMAX>
int launch_fwd_short(const FwdParams &p, bool packed_ok, hipStream_t s, bool plane_ok = false,
                     bool ragged_ok = false)
{
    // ragged_ok: packed rows shorter than NMAX in natural order (any 4-byte alignment); rows of up
    // to 8 samples lie so close together that the plain per-lane accesses do as well
    ragged_ok = ragged_ok && NMAX >= 16 && !p.tm.grouped && p.L.n < NMAX;
    static_assert(tvk::kShortBlock == 64, "one tile of 64 rows per workgroup");
    const uint32_t n_tiles = (p.L.n_rows + 63u) / 64u;
    dim3 grid(n_tiles), block(tvk::kShortBlock);
    if (p.tm.grouped) grid = dim3(n_tiles / p.tm.count, p.tm.count);
    const bool full = p.L.n == NMAX;
    if constexpr (NMAX == 32) {
        if (p.io16) {                     // the entry point has checked: packed rows of exactly 32
            hipLaunchKernelGGL((tvk::tv1d_fwd_short_kernel<32, true, true, false, false, true>), grid, block, 0, s, p);
            return launch_status();
        }
        if (p.psearch) {                  // the entry point has checked: no addend, rows of up to 32 samples
            if (full && packed_ok)
                hipLaunchKernelGGL((tvk::tv1d_fwd_short_kernel<32, true, true, false, false, false, false, true>), grid,
                                   block, 0, s, p);
            else
                hipLaunchKernelGGL((tvk::tv1d_fwd_short_kernel<32, false, false, false, false, false, false, true>), grid,
                                   block, 0, s, p);
            return launch_status();
        }
    }
    if constexpr (NMAX == 32) {
        // (the warm-start variant of the plane mode runs out of scalar registers and loses a wave of
        // occupancy to the spill; warm column passes keep the strided accesses)
        if (plane_ok && full && !p.warm) {
            hipLaunchKernelGGL((tvk::tv1d_fwd_short_kernel<32, true, false, false, true>), grid, block, 0, s, p);
            return launch_status();
        }
    }
    if (p.warm) {
        if (full && packed_ok)
            hipLaunchKernelGGL((tvk::tv1d_fwd_short_kernel<NMAX, true, true, true>), grid, block, 0, s, p);
        else if (full)
            hipLaunchKernelGGL((tvk::tv1d_fwd_short_kernel<NMAX, true, false, true>), grid, block, 0, s, p);
        else if (ragged_ok)
            hipLaunchKernelGGL((tvk::tv1d_fwd_short_kernel<NMAX, false, true, true>), grid, block, 0, s, p);
        else
            hipLaunchKernelGGL((tvk::tv1d_fwd_short_kernel<NMAX, false, false, true>), grid, block, 0, s, p);
    } else if (full && packed_ok)
        hipLaunchKernelGGL((tvk::tv1d_fwd_short_kernel<NMAX, true, true>), grid, block, 0, s, p);
    else if (full)
        hipLaunchKernelGGL((tvk::tv1d_fwd_short_kernel<NMAX, true, false>), grid, block, 0, s, p);
    else if (ragged_ok)
        hipLaunchKernelGGL((tvk::tv1d_fwd_short_kernel<NMAX, false, true>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((tvk::tv1d_fwd_short_kernel<NMAX, false, false>), grid, block, 0, s, p);
    return launch_status();
}

template <int NMAX, bool HAS_SUB, bool SEG>
int launch_bwd_short(const BwdParams &p, bool packed_ok, hipStream_t s, bool plane_ok, bool ragged_ok)
{
    ragged_ok = ragged_ok && NMAX >= 16 && p.L.n < NMAX;
    const dim3 grid((p.L.n_rows + tvk::kShortBlock - 1) / tvk::kShortBlock), block(tvk::kShortBlock);
    const bool full = p.L.n == NMAX;
    if constexpr (NMAX == 32 && SEG && !HAS_SUB) {
        if (p.io16) {                     // the entry point has checked: packed rows of exactly 32
            hipLaunchKernelGGL((tvk::tv1d_bwd_short_kernel<32, true, true, false, true, false, true>), grid, block, 0,
                               s, p);
            return launch_status();
        }
    }
    if constexpr (NMAX == 32) {
        if (plane_ok && full) {
            hipLaunchKernelGGL((tvk::tv1d_bwd_short_kernel<32, true, false, HAS_SUB, SEG, true>), grid, block, 0, s, p);
            return launch_status();
        }
    }
    if (full && packed_ok)
        hipLaunchKernelGGL((tvk::tv1d_bwd_short_kernel<NMAX, true, true, HAS_SUB, SEG>), grid, block, 0, s, p);
    else if (full)
        hipLaunchKernelGGL((tvk::tv1d_bwd_short_kernel<NMAX, true, false, HAS_SUB, SEG>), grid, block, 0, s, p);
    else if (ragged_ok)
        hipLaunchKernelGGL((tvk::tv1d_bwd_short_kernel<NMAX, false, true, HAS_SUB, SEG>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((tvk::tv1d_bwd_short_kernel<NMAX, false, false, HAS_SUB, SEG>), grid, block, 0, s, p);
    return launch_status();
}

template <int NMAX>
int launch_bwd_short(const BwdParams &p, bool packed_ok, hipStream_t s, bool plane_ok = false,
                     bool ragged_ok = false)
{
    if (p.seg)
        return p.sub ? launch_bwd_short<NMAX, true, true>(p, packed_ok, s, plane_ok, ragged_ok)
                     : launch_bwd_short<NMAX, false, true>(p, packed_ok, s, plane_ok, ragged_ok);
    return p.sub ? launch_bwd_short<NMAX, true, false>(p, packed_ok, s, plane_ok, ragged_ok)
                 : launch_bwd_short<NMAX, false, false>(p, packed_ok, s, plane_ok, ragged_ok);
}

// ---- slot order for the grouped grid -----------------------------------------------
//
// A tile's cost is its largest Newton step count, which depends mostly on where the slot's
// lambda lies relative to the scale of its rows: one step when every dual ends up on a bound
// (small lambda) or none does (large lambda), many in between.  Workgroups are dispatched in
// grid order, and whatever runs last determines how long the chip drains with idle SIMDs, so
// the expensive slots are dispatched first (longest processing time first).  The cost is
// predicted from a few rows of each slot's first tile: with p the fraction of duals that
// the unconstrained Newton step from u = 0 (the prefix sums of mean(y) - y) puts outside
// the box, the measured step count follows p (1 - p).
constexpr int kOrderMaxSlots = 1024;

// The value of `v` in the lane that the DPP control word names (row-local patterns only).
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

template <int CTRL>
__device__ __forceinline__ int dpp_i(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}

// One workgroup of 1024 threads.
// Step 1, key[slot] = p (1 - p) from sample rows of the slot's first tile (a grouped tile is
// always full).  FAST (packed rows of 32 samples in groups of at least 2 consecutive rows):
// 2 rows per slot, 8 lanes per row with 4 samples each, so one coalesced 16-byte load per
// lane covers 4 slots; prefix sums and counts run across lanes through DPP.  Otherwise
// thread t reads row (t % R) of slot (t / R) sample by sample, R = 1024 / (slots rounded up
// to a power of two) rows per slot, at most 64.
// Step 2: order[rank] = slot, ranks by counting the slots with a larger key (ties by
// index), so equal inputs always give the same order.
template <bool FAST>
__global__ __launch_bounds__(kOrderMaxSlots) void slot_order_kernel(
    const float *__restrict__ y, const float *__restrict__ addend, const float *__restrict__ lam,
    tvk::Layout L, tvk::TileMap tm, uint32_t lgR, uint32_t *__restrict__ order, uint32_t io16)
{
    __shared__ float key[kOrderMaxSlots];
    const uint32_t count = tm.count;
    if constexpr (FAST) {
        const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        const uint32_t sub = lane >> 4, q = lane & 7u;
        constexpr int J = 4;                               // loads in flight per lane
        for (uint32_t c0 = 0; c0 < count; c0 += 64u * J) {
            float4 v[J];
            float lv[J];
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const uint32_t s = c0 + (j * 16u + wave) * 4u + sub;
                v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
                lv[j] = 0.f;
                if (s < count) {
                    lv[j] = lam[s];
                    const size_t a = (size_t)tm.first(0u, s) * 32u + (lane & 15u) * 4u;
                    if (io16) {
                        const uint2 h = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(y) + a);
                        v[j] = make_float4(__uint_as_float(h.x << 16), __uint_as_float(h.x & 0xffff0000u),
                                           __uint_as_float(h.y << 16), __uint_as_float(h.y & 0xffff0000u));
                    } else {
                        v[j] = *reinterpret_cast<const float4 *>(y + a);
                    }
                    if (addend) {
                        const float4 w = *reinterpret_cast<const float4 *>(addend + a);
                        v[j].x += w.x; v[j].y += w.y; v[j].z += w.z; v[j].w += w.w;
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const uint32_t s = c0 + (j * 16u + wave) * 4u + sub;
                float t = (v[j].x + v[j].y) + (v[j].z + v[j].w);
                t += dpp_f<0xB1>(t);            // quad_perm [1,0,3,2]
                t += dpp_f<0x4E>(t);            // quad_perm [2,3,0,1]
                t += dpp_f<0x141>(t);           // row_half_mirror: the other quad of the 8 lanes
                const float mean = t * (1.f / 32.f);
                const float p0 = mean - v[j].x, p1 = p0 + (mean - v[j].y);
                const float p2 = p1 + (mean - v[j].z), p3 = p2 + (mean - v[j].w);
                float inc = p3;                 // inclusive scan over the row's 8 lanes
                { const float up = dpp_f<0x111>(inc); if (q >= 1u) inc += up; }      // row_shr:1
                { const float up = dpp_f<0x112>(inc); if (q >= 2u) inc += up; }      // row_shr:2
                { const float up = dpp_f<0x114>(inc); if (q >= 4u) inc += up; }      // row_shr:4
                const float l = fmaxf(lv[j], 0.f), e = inc - p3;
                int out = (fabsf(e + p0) > l ? 1 : 0) + (fabsf(e + p1) > l ? 1 : 0) +
                          (fabsf(e + p2) > l ? 1 : 0) + ((q < 7u && fabsf(e + p3) > l) ? 1 : 0);
                out += dpp_i<0xB1>(out);
                out += dpp_i<0x4E>(out);
                out += dpp_i<0x141>(out);
                out += dpp_i<0x140>(out);       // row_mirror: the other row of the slot's 16 lanes
                if (s < count && (lane & 15u) == 0u) {
                    const float p = (float)out * (1.f / (2.f * 31.f));
                    key[s] = p * (1.f - p);
                }
            }
        }
    } else {
    const uint32_t R = 1u << lgR;
    const uint32_t s = threadIdx.x >> lgR, i = threadIdx.x & (R - 1u);
    const int n = L.n;                                    // <= 32
    int out = 0;
    if (s < count) {
        const float l = fmaxf(lam[s], 0.f);
        const uint32_t r = tm.row(tm.first(0u, s), i);
        const int64_t off = tvk::row_offset(L, r);
        float v[32];
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            v[j] = 0.f;
            if (j < n) {
                const int64_t a = off + j * L.elem_stride;
                v[j] = io16 ? tvk::bf16_bits_to_f32(reinterpret_cast<const uint16_t *>(y)[a]) : y[a];
                if (addend) v[j] += addend[a];
            }
        }
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < 32; ++j) sum += v[j];         // samples past the row are 0
        const float mean = sum / (float)n;
        float run = 0.f;
#pragma unroll
        for (int j = 0; j < 31; ++j) {
            run += mean - v[j];
            out += (j < n - 1 && fabsf(run) > l) ? 1 : 0;
        }
    }
    for (uint32_t d = 1; d < R; d <<= 1) out += __shfl_xor(out, (int)d);   // R <= 64 lanes, aligned
    if (s < count && i == 0) {
        const float p = (float)out / (float)((int)R * (n > 1 ? n - 1 : 1));
        key[s] = p * (1.f - p);
    }
    }
    __syncthreads();
    // ranks: the 1 << lgR lanes of a slot share the comparisons, reading keys several at a time
    {
        const uint32_t R = 1u << lgR;
        const uint32_t t = threadIdx.x >> lgR, i = threadIdx.x & (R - 1u);
        const float k = t < count ? key[t] : 0.f;
        uint32_t rank = 0;
        if (t < count) {
#pragma unroll 8
            for (uint32_t j = i; j < count; j += R) {
                const float kj = key[j];
                rank += (kj > k || (kj == k && j < t)) ? 1u : 0u;
            }
        }
        for (uint32_t d = 1; d < R; d <<= 1) rank += __shfl_xor(rank, (int)d);
        if (t < count && i == 0) order[rank] = t;
    }
}

bool order_applies(const tvk::TileMap &tm)
{
    return tm.grouped && tm.count <= (uint32_t)kOrderMaxSlots;
}

// ---- multilevel start of long unit-stride rows ------------------------------------------
//
// Projected Newton from the cold start needs 8 to 25 steps on rows of thousands of samples when
// lambda is large against the sample-to-sample variation (few, long segments: the bound set
// changes a little with every step).  The same row averaged in groups of kMlFactor samples,
// with lambda / kMlFactor, is the problem restricted to rows that are constant on the groups;
// its dual, prolonged (see the WARM = 2 kernel), is a start from which the fine level needs
// about 4 steps whatever lambda is.  One level at least, and further ones while a row has more
// than kMlCoarsest samples (by default that leaves the one level: stacking them was measured
// and costs more launches than it saves steps); every level is an ordinary launch of the
// long-row kernel on packed scratch rows.
// Rows whose lambda is small against their variation converge in a few steps anyway and are
// left out (ml_flag = 0): they start cold at the fine level and are skipped at the others.
constexpr int kMlMaxLevels = 8;                // (where it starts and ends: tv_dispatch.hpp)
constexpr float kMlLambdaRatio = 0.5f;     // multilevel start when lambda >= ratio * mean |y[k+1] - y[k]| (2, 4, 8: every kind of row slower; 0.125: 1-2 % slower)
constexpr int kMlProbeGroups = 512;        // ... judged on the row's first 2048 samples

struct MlPlan {
    int levels;                       // coarse levels 1 .. levels (0 = the row itself)
    int64_t n[kMlMaxLevels + 1];
    // scratch in a workspace: every level's rows packed, level after level (byte offsets)
    size_t y_off[kMlMaxLevels + 1], u_off[kMlMaxLevels + 1], flag_off, bytes;
    // scratch inside the output rows: all levels of a row within the row's own n floats (offsets
    // in floats from the start of the row, multiples of 4); row_floats = 0 if they do not fit
    int64_t row_y_off[kMlMaxLevels + 1], row_u_off[kMlMaxLevels + 1], row_flag_off, row_floats;
};

bool ml_plan(const tv_rows &r, int64_t n_rows, MlPlan *pl)
{
    if (r.length < tvd::get(tvd::kMlMinLength) || r.elem_stride != 1) return false;
    pl->levels = 0;
    pl->n[0] = r.length;
    size_t at = 0;
    int64_t in_row = 0;
    do {                                            // one level at least
        const int l = ++pl->levels;
        pl->n[l] = (pl->n[l - 1] + tvk::kMlFactor - 1) / tvk::kMlFactor;
        const size_t bytes = align16((size_t)n_rows * (size_t)pl->n[l] * sizeof(float));
        pl->y_off[l] = at; at += bytes;
        pl->u_off[l] = at; at += bytes;
        const int64_t padded = (pl->n[l] + 3) / 4 * 4;
        pl->row_y_off[l] = in_row; in_row += padded;
        pl->row_u_off[l] = in_row; in_row += padded;
    } while (pl->n[pl->levels] > tvd::get(tvd::kMlCoarsest) && pl->levels < kMlMaxLevels);
    pl->flag_off = at;
    pl->bytes = at + align16((size_t)n_rows * sizeof(uint32_t));
    pl->row_flag_off = in_row;
    pl->row_floats = in_row + 1 <= r.length ? in_row + 1 : 0;
    return pl->levels > 0;
}

// out[row][j] = mean of in[row][kMlFactor j ...] (the samples that exist); one workgroup per row.
// FIRST: `in` is the caller's tensor (rows by L), and the row's flag is decided here from the mean
// absolute difference of neighbouring samples inside the groups; otherwise `in` holds n_in samples
// per row, in_pitch floats apart, and rows with flag 0 are skipped.  out: out_pitch floats apart;
// flag: flag_pitch words apart.
template <bool FIRST>
__global__ __launch_bounds__(256) void ml_average_kernel(const float *__restrict__ in,
                                                         float *__restrict__ out,
                                                         uint32_t *__restrict__ flag,
                                                         const float *__restrict__ lam, tvk::Layout L,
                                                         int32_t n_in, int32_t n_out, int64_t in_pitch,
                                                         int64_t out_pitch, uint32_t flag_pitch)
{
    constexpr int F = tvk::kMlFactor;
    const uint32_t row = blockIdx.x;
    flag += (size_t)row * flag_pitch;
    if (!FIRST && flag[0] == 0) return;
    const float *src = in + (FIRST ? tvk::row_offset(L, row) : (int64_t)row * in_pitch);
    float *dst = out + (int64_t)row * out_pitch;
    const bool vec = ((uintptr_t)src % 16) == 0;
    auto group = [&](int j, float (&v)[F]) {
        const int k = j * F;
        if (vec && k + F <= n_in) {
            const float4 q = *reinterpret_cast<const float4 *>(src + k);
            v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        } else {
#pragma unroll
            for (int r = 0; r < F; ++r) v[r] = (k + r < n_in) ? src[k + r] : 0.f;
        }
    };
    if (FIRST) {
        // the row's variation is judged on its first kMlProbeGroups groups; a row that stays
        // out of the multilevel start needs no averages
        __shared__ float red[256];
        __shared__ uint32_t decision;
        const int probe = n_out < kMlProbeGroups ? n_out : kMlProbeGroups;
        float var = 0.f;
        for (int j = threadIdx.x; j < probe; j += 256) {
            float v[F];
            group(j, v);
#pragma unroll
            for (int r = 0; r + 1 < F; ++r)
                if (j * F + r + 1 < n_in) var += fabsf(v[r + 1] - v[r]);
        }
        red[threadIdx.x] = var;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            // differences counted: F - 1 of every F neighbouring pairs of the probed samples
            const int last = probe * F < n_in ? probe * F : n_in;
            const float pairs = (float)(last - 1) * (float)(F - 1) / (float)F;
            const float l = tvk::load_lambda(lam, L, row);
            decision = (l * pairs >= kMlLambdaRatio * red[0]) ? 1u : 0u;
            flag[0] = decision;
        }
        __syncthreads();
        if (decision == 0) return;
    }
    for (int j = threadIdx.x; j < n_out; j += 256) {
        float v[F];
        group(j, v);
        float sum = 0.f, cnt = 0.f;
#pragma unroll
        for (int r = 0; r < F; ++r)
            if (j * F + r < n_in) { sum += v[r]; cnt += 1.f; }
        dst[j] = sum / cnt;
    }
}
static_assert(tvk::kMlFactor == 4, "ml_average_kernel loads groups as float4");

// The forward call on long rows with the multilevel start; p is the fine level, fully set up.
// ws: the levels' scratch (MlPlan's workspace layout), or null: then every row's levels live in
// that row of the output p.x (MlPlan's in-row layout; packed rows, p.x apart from p.y), which the
// fine level overwrites at its very end, after the one workgroup or wave that owns the row has
// read the row's coarse dual at its start.
int run_fwd_multilevel(FwdParams p, const tv_lambda &l, int64_t n_rows, const MlPlan &pl, char *ws,
                       hipStream_t s)
{
    const bool in_rows = ws == nullptr;
    const int64_t n0 = pl.n[0];
    uint32_t *flag = in_rows ? reinterpret_cast<uint32_t *>(p.x + pl.row_flag_off) : (uint32_t *)(ws + pl.flag_off);
    const uint32_t flag_pitch = in_rows ? (uint32_t)n0 : 1u;
    auto yl = [&](int lv) { return in_rows ? p.x + pl.row_y_off[lv] : (float *)(ws + pl.y_off[lv]); };
    auto ul = [&](int lv) { return in_rows ? p.x + pl.row_u_off[lv] : (float *)(ws + pl.u_off[lv]); };
    auto pitch = [&](int lv) { return in_rows ? n0 : pl.n[lv]; };      // floats between consecutive rows of a level
    const dim3 grid((uint32_t)n_rows), block(256);
    hipLaunchKernelGGL(ml_average_kernel<true>, grid, block, 0, s, p.y, yl(1), flag, l.lam, p.L,
                       (int32_t)pl.n[0], (int32_t)pl.n[1], (int64_t)0, pitch(1), flag_pitch);
    for (int lv = 2; lv <= pl.levels; ++lv)
        hipLaunchKernelGGL(ml_average_kernel<false>, grid, block, 0, s, (const float *)yl(lv - 1), yl(lv), flag,
                           l.lam, p.L, (int32_t)pl.n[lv - 1], (int32_t)pl.n[lv], pitch(lv - 1), pitch(lv), flag_pitch);
    if (launch_status() != TV_OK) return TV_ERR_HIP;
    float scale = 1.0f;
    for (int lv = 1; lv <= pl.levels; ++lv) scale /= (float)tvk::kMlFactor;
    for (int lv = pl.levels; lv >= 1; --lv, scale *= (float)tvk::kMlFactor) {
        FwdParams c = p;
        const tv_rows rc = {1, 0, n_rows, pitch(lv), pl.n[lv], 1};
        c.L = make_layout(rc, l, n_rows);
        c.y = yl(lv); c.addend = nullptr; c.x = nullptr; c.x2 = nullptr; c.resid = nullptr;
        c.info = nullptr; c.seg = nullptr; c.order = nullptr;
        c.dual_out = ul(lv); c.dual_pitch = (int32_t)pitch(lv);
        c.ml_flag = flag; c.flag_pitch = flag_pitch; c.ml_skip = 1;
        c.lam_scale = scale;
        c.warm = lv == pl.levels ? 0u : 2u;
        c.coarse_u = lv == pl.levels ? nullptr : ul(lv + 1);
        c.coarse_n = lv == pl.levels ? 0 : (int32_t)pl.n[lv + 1];
        c.coarse_pitch = lv == pl.levels ? 0 : (int32_t)pitch(lv + 1);
        if (tvk::launch_fwd_long(c, s) != hipSuccess) return TV_ERR_HIP;
    }
    p.warm = 2; p.coarse_u = ul(1); p.coarse_n = (int32_t)pl.n[1]; p.coarse_pitch = (int32_t)pitch(1);
    p.ml_flag = flag; p.flag_pitch = flag_pitch; p.ml_skip = 0;
    return tvk::launch_fwd_long(p, s) == hipSuccess ? TV_OK : TV_ERR_HIP;
}

// ---- dispatch ---------------------------------------------------------------------

// Segment codes read off x (rows of at most 32 samples): what tv1d_fwd_short_kernel builds from its
// registers, for the forward calls that run on the long-row kernels.  x is bit-constant inside a
// segment, so the code follows from x alone.  A thread per row; only small batches come here.
__global__ __launch_bounds__(256) void seg_from_x_kernel(const float *__restrict__ x, uint2 *__restrict__ seg,
                                                         tvk::Layout L)
{
    const uint32_t row = blockIdx.x * 256u + threadIdx.x;
    if (row >= L.n_rows) return;
    const float *xr = x + tvk::row_offset(L, row);
    uint32_t jm = 0, up = 0;
    float prev = xr[0];
    for (int k = 0; k + 1 < L.n; ++k) {
        const float next = xr[(int64_t)(k + 1) * L.elem_stride];
        jm |= (next != prev ? 1u : 0u) << k;
        up |= (next > prev ? 1u : 0u) << k;
        prev = next;
    }
    seg[row] = make_uint2(jm, up);
}

int run_fwd(const float *y, const float *addend, float *x, float *resid, int32_t *info,
            uint2 *seg, uint32_t *order_ws, const tv_rows &r, const tv_lambda &l, int64_t n_rows,
            hipStream_t s, float *x2 = nullptr, bool warm = false, char *ml_ws = nullptr, bool io16 = false,
            bool thread_per_sample = false, bool order_ready = false, bool psearch = false)
{
    FwdParams p;
    p.y = y; p.addend = addend; p.x = x; p.x2 = x2; p.resid = resid; p.lam = l.lam; p.info = info;
    p.seg = seg; p.order = nullptr;
    p.io16 = io16 ? 1u : 0u;
    p.psearch = psearch ? 1u : 0u;
    p.warm = (warm && addend) ? 1u : 0u;
    p.coarse_u = nullptr; p.coarse_n = 0; p.coarse_pitch = 0; p.dual_out = nullptr; p.dual_pitch = 0;
    p.ml_flag = nullptr; p.flag_pitch = 1; p.ml_skip = 0;
    p.lam_scale = 1.0f;
    p.debug = nullptr; p.debug_rows = 0;
    p.L = make_layout(r, l, n_rows);
    p.tm = make_tile_map(l, n_rows);
    // (a few thousand short rows at most: a few threads per row instead of a lane per row; the 2D
    // operator asks for it on small batches of planes, where a lone row-per-lane wave is bound by
    // its dependency chains)
    if (thread_per_sample && r.length >= 2 && r.length <= 32 && !io16) {
        p.seg = nullptr;
        if (tvk::launch_fwd_long(p, s) != hipSuccess) return TV_ERR_HIP;
        if (seg) {
            hipLaunchKernelGGL(seg_from_x_kernel, dim3((uint32_t)((n_rows + 255) / 256)), dim3(256), 0, s, x, seg, p.L);
            if (launch_status() != TV_OK) return TV_ERR_HIP;
        }
        return TV_OK;
    }
    if (order_ws && r.length <= 32 && order_applies(p.tm)) {
        uint32_t lgR = 0;
        while (lgR < 6 && ((uint64_t)p.tm.count << (lgR + 1)) <= (uint64_t)kOrderMaxSlots) ++lgR;
        uint32_t *order = order_ws;
        const bool fast = r.length == 32 && p.tm.lg >= 1 && rows_packed(r) && aligned16(y) &&
                          (!addend || aligned16(addend));
        if (order_ready) {
            // the caller vouches that `order` holds what an earlier call left there
        } else if (fast)
            hipLaunchKernelGGL(slot_order_kernel<true>, dim3(1), dim3(kOrderMaxSlots), 0, s, y, addend,
                               l.lam, p.L, p.tm, lgR, order, io16 ? 1u : 0u);
        else
            hipLaunchKernelGGL(slot_order_kernel<false>, dim3(1), dim3(kOrderMaxSlots), 0, s, y, addend,
                               l.lam, p.L, p.tm, lgR, order, io16 ? 1u : 0u);
        if (launch_status() != TV_OK) return TV_ERR_HIP;
        p.order = order;
    }
    const bool packed = rows_packed(r) && aligned16(y) && aligned16(x) &&
                        (!addend || aligned16(addend)) && (!resid || aligned16(resid));
    const bool ragged = rows_packed(r);
    if (psearch) return launch_fwd_short<32>(p, packed, s, false, false);   // every length up to 32
    if (r.length <= 8) return launch_fwd_short<8>(p, packed, s, false, ragged);
    if (r.length <= 16) return launch_fwd_short<16>(p, packed, s, false, ragged);
    if (r.length <= 32) {
        const bool planes = rows_are_plane_columns(r) && aligned16(y) && aligned16(x) &&
                            (!addend || aligned16(addend)) && (!resid || aligned16(resid)) &&
                            (!x2 || aligned16(x2));
        return launch_fwd_short<32>(p, packed, s, planes, ragged);
    }
    MlPlan pl;
    if (!p.warm && !addend && ml_plan(r, n_rows, &pl)) {
        if (ml_ws) return run_fwd_multilevel(p, l, n_rows, pl, ml_ws, s);
        // no workspace: the levels of a row fit into that row of x (half of it, two thirds with levels stacked), which is the
        // call's to write anyway, if the rows are packed and x and y do not overlap
        const float *y_end = y + n_rows * r.length;
        const float *x_end = x + n_rows * r.length;
        if (pl.row_floats > 0 && rows_packed(r) && (x_end <= y || y_end <= x))
            return run_fwd_multilevel(p, l, n_rows, pl, nullptr, s);
    }
    // long rows that start cold after all (in place, with gaps between them, strided): the cold
    // start with two candidates, which does not run into the step cap when lambda is of the
    // order of the row's lam_max
    if (!p.warm && r.length > 768) p.warm = 3;
    return tvk::launch_fwd_long(p, s) == hipSuccess ? TV_OK : TV_ERR_HIP;
}

// Sums the per-row dL/dlam contributions of every slot: one workgroup per slot, fp64
// accumulation in a fixed order (deterministic).  Four independent loads are kept in
// flight per thread; the walk over the slot's rows needs no division.  `batches` arrays of the
// same shape, `batch_stride` floats apart, are summed together (the passes of a 2D reverse
// sweep).  With few slots and many batches the work of a slot is split over gridDim.y
// workgroups (workgroup j takes batches j, j + gridDim.y, ...), each leaving its fp64 sum in
// `split_out[slot * gridDim.y + j]` for sum_splits_kernel.
template <int kReduceThreads>
__global__ __launch_bounds__(kReduceThreads) void reduce_lambda_kernel(
    const float *__restrict__ partial, float *__restrict__ grad_lam, uint32_t n_rows,
    uint32_t count, uint32_t div, int accumulate, uint32_t batches, uint64_t batch_stride,
    double *__restrict__ split_out)
{
    __shared__ double red[kReduceThreads];
    const uint32_t slot = blockIdx.x;
    // rows of this slot: r = (q*count + slot)*div + i,  i < div,  q = 0, 1, ...
    // thread t visits the pairs (q, i) with q*div + i = t, t + T, t + 2T, ...
    const uint32_t dq = kReduceThreads / div, di = kReduceThreads - dq * div;
    const uint64_t stride = (uint64_t)count * div;
    const uint64_t base = (uint64_t)slot * div;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    partial += blockIdx.y * batch_stride;
    for (uint32_t b = blockIdx.y; b < batches; b += gridDim.y, partial += gridDim.y * batch_stride) {
        uint32_t q = threadIdx.x / div, i = threadIdx.x - q * div;
        bool more = true;
        while (more) {
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // group starts grow with q: once a group starts past the end, nothing follows
                const uint64_t g0 = q * stride + base;
                more = more && (g0 < n_rows);
                v[j] = (more && g0 + i < n_rows) ? partial[g0 + i] : 0.f;
                q += dq; i += di;
                if (i >= div) { i -= div; q += 1; }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] += (double)v[j];
        }
    }
    red[threadIdx.x] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    __syncthreads();
    for (int w = kReduceThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        if (split_out) {
            split_out[slot * gridDim.y + blockIdx.y] = red[0];
        } else {
            const float v = (float)red[0];
            grad_lam[slot] = accumulate ? grad_lam[slot] + v : v;
        }
    }
}

// grad_lam[slot] = the sum, in a fixed order, of the `n` fp64 sums that the split reductions left
// per slot (both directions of a 2D reverse sweep lie side by side: n = 2 * splits).
__global__ __launch_bounds__(64) void sum_splits_kernel(const double *__restrict__ split,
                                                         float *__restrict__ grad_lam, uint32_t count,
                                                         uint32_t splits)
{
    const uint32_t slot = blockIdx.x * 64 + threadIdx.x;
    if (slot >= count) return;
    double acc = 0.0;
    for (uint32_t d = 0; d < 2; ++d)
        for (uint32_t j = 0; j < splits; ++j) acc += split[((uint64_t)d * count + slot) * splits + j];
    grad_lam[slot] = (float)acc;
}

// Slots that own only a handful of rows (e.g. one lambda per row): one thread per slot.
__global__ __launch_bounds__(256) void reduce_lambda_small_kernel(
    const float *__restrict__ partial, float *__restrict__ grad_lam, uint32_t n_rows,
    uint32_t count, uint32_t div, int accumulate, uint32_t batches, uint64_t batch_stride)
{
    const uint32_t slot = blockIdx.x * 256 + threadIdx.x;
    if (slot >= count) return;
    const uint64_t stride = (uint64_t)count * div;
    double acc = 0.0;
    for (uint32_t b = 0; b < batches; ++b, partial += batch_stride)
        for (uint64_t g0 = (uint64_t)slot * div; g0 < n_rows; g0 += stride)
            for (uint32_t i = 0; i < div && g0 + i < n_rows; ++i) acc += (double)partial[g0 + i];
    const float v = (float)acc;
    grad_lam[slot] = accumulate ? grad_lam[slot] + v : v;
}

// The split reduction applies below this many slots (more slots fill the chip by themselves) ...
constexpr uint32_t kSplitMaxSlots = 64;
// ... and uses at most this many workgroups per slot and direction.
constexpr uint32_t kSplitMax = 32;
constexpr size_t kSplitScratchBytes = 2 * (size_t)kSplitMaxSlots * kSplitMax * sizeof(double);

uint32_t reduce_splits(int64_t count, int sweeps)
{
    if (count >= (int64_t)kSplitMaxSlots || sweeps < 2) return 1;
    return (uint32_t)sweeps < kSplitMax ? (uint32_t)sweeps : kSplitMax;
}

// splits > 1: workgroup (slot, j) leaves its fp64 sum in split_out[slot * splits + j]; the rows of
// a slot must then be many enough for the workgroup-per-slot kernel.
int launch_reduce_lambda(const float *partial, float *grad_lam, int64_t n_rows, const tv_lambda &l,
                         int accumulate, hipStream_t s, uint32_t batches = 1, uint64_t batch_stride = 0,
                         uint32_t splits = 1, double *split_out = nullptr)
{
    const uint32_t count = (uint32_t)l.count, div = (uint32_t)l.div, nr = (uint32_t)n_rows;
    const uint64_t groups = ((uint64_t)nr + div - 1) / div;
    const uint64_t rows_per_slot = ((groups + count - 1) / count) * div * ((batches + splits - 1) / splits);
    if (splits > 1) {
        if (rows_per_slot <= 2048)
            hipLaunchKernelGGL(reduce_lambda_kernel<256>, dim3(count, splits), dim3(256), 0, s, partial,
                               grad_lam, nr, count, div, accumulate, batches, batch_stride, split_out);
        else
            hipLaunchKernelGGL(reduce_lambda_kernel<1024>, dim3(count, splits), dim3(1024), 0, s, partial,
                               grad_lam, nr, count, div, accumulate, batches, batch_stride, split_out);
    } else if (rows_per_slot <= 32)
        hipLaunchKernelGGL(reduce_lambda_small_kernel, dim3((count + 255) / 256), dim3(256), 0, s,
                           partial, grad_lam, nr, count, div, accumulate, batches, batch_stride);
    else if (rows_per_slot <= 2048)
        hipLaunchKernelGGL(reduce_lambda_kernel<256>, dim3(count), dim3(256), 0, s, partial, grad_lam,
                           nr, count, div, accumulate, batches, batch_stride, (double *)nullptr);
    else
        hipLaunchKernelGGL(reduce_lambda_kernel<1024>, dim3(count), dim3(1024), 0, s, partial,
                           grad_lam, nr, count, div, accumulate, batches, batch_stride, (double *)nullptr);
    return launch_status();
}

// Row-per-lane kernels add up the dL/dlam terms of neighbouring rows that share a slot before
// they leave the wave: groups of 1 << lg rows, the largest power of two (at most 64) dividing
// div.  What is left for the reduction kernel: red_rows values, red_div of them per slot visit.
struct PartialShape {
    uint32_t lg;
    int64_t  red_rows, red_div;
};

PartialShape partial_shape(const tv_rows &r, const tv_lambda &l, int64_t n_rows)
{
    PartialShape ps = {0, n_rows, l.div};
    if (r.length <= 32) {
        uint32_t lg = 0;
        while (lg < 6 && (l.count == 1 || l.div % ((int64_t)2 << lg) == 0)) ++lg;
        ps.lg = lg;
        ps.red_rows = (n_rows + ((int64_t)1 << lg) - 1) >> lg;
        ps.red_div = l.count == 1 ? 1 : l.div >> lg;
    }
    return ps;
}

// reduce_now = false: the dL/dlam terms stay in `partial` and the caller sums them later.
int run_bwd(const float *g, const float *sub, const float *x, const uint2 *seg, float *gy,
            float *grad_lam, int accumulate, const tv_rows &r, const tv_lambda &l, int64_t n_rows,
            float *partial, hipStream_t s, bool reduce_now = true, bool io16 = false)
{
    BwdParams p;
    p.g = g; p.sub = sub; p.x = x; p.seg = seg; p.gy = gy;
    p.io16 = io16 ? 1u : 0u;
    p.partial = grad_lam ? partial : nullptr;
    p.L = make_layout(r, l, n_rows);
    const bool packed = rows_packed(r) && aligned16(g) && (!x || aligned16(x)) && aligned16(gy) &&
                        (!sub || aligned16(sub));
    int st;
    const PartialShape ps = partial_shape(r, l, n_rows);
    p.part_lg = grad_lam ? ps.lg : 0;
    const int64_t red_rows = ps.red_rows, red_div = ps.red_div;
    const bool ragged = rows_packed(r);
    if (r.length <= 8) st = launch_bwd_short<8>(p, packed, s, false, ragged);
    else if (r.length <= 16) st = launch_bwd_short<16>(p, packed, s, false, ragged);
    else if (r.length <= 32) {
        const bool planes = rows_are_plane_columns(r) && aligned16(g) && (!x || aligned16(x)) &&
                            aligned16(gy) && (!sub || aligned16(sub));
        st = launch_bwd_short<32>(p, packed, s, planes, ragged);
    }
    else st = tvk::launch_bwd_long(p, s) == hipSuccess ? TV_OK : TV_ERR_HIP;
    if (st != TV_OK) return st;
    if (grad_lam && reduce_now) {
        tv_lambda lr = l;
        lr.div = red_div;
        st = launch_reduce_lambda(partial, grad_lam, red_rows, lr, accumulate, s);
    }
    return st;
}

// A fill kernel rather than a memset node, so that callers may capture the call in a graph.
__global__ void zero_floats_kernel(float *p, uint32_t n)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

int zero_floats(float *p, int64_t n, hipStream_t s)
{
    hipLaunchKernelGGL(zero_floats_kernel, dim3((uint32_t)((n + 255) / 256)), dim3(256), 0, s, p,
                       (uint32_t)n);
    return launch_status();
}

// Scratch of the forward call: a uint32 per slot where the slot order applies (rows of up to 32
// samples), the coarse levels where the multilevel start applies (long unit-stride rows).
size_t fwd_workspace_bytes(const tv_rows &rows, const tv_lambda &lam, int64_t n_rows)
{
    MlPlan pl;
    if (ml_plan(rows, n_rows, &pl)) return pl.bytes;
    if (rows.length > 32 || !order_applies(make_tile_map(lam, n_rows))) return 0;
    return align16((size_t)lam.count * sizeof(uint32_t));
}

int fwd_entry(const float *y, float *x, tv_rows rows, tv_lambda lam, const tv_fwd_extra &e,
              hipStream_t s)
{
    int st = check_lambda(lam);
    if (st != TV_OK) return st;
    int64_t n_rows;
    st = check_rows(rows, &n_rows);
    if (st != TV_OK) return st;
    if (n_rows == 0) return TV_OK;
    if (!y || !x || !lam.lam) return TV_ERR_NULL;
    if (rows.length > TV_MAX_LENGTH) return TV_ERR_UNSUPPORTED;
    if (e.seg) {
        if (rows.length > TV_SEG_MAX_LENGTH) return TV_ERR_UNSUPPORTED;
        if ((uintptr_t)e.seg % 8 != 0) return TV_ERR_STRIDE;
    }
    if ((e.flags & TV_FWD_PARALLEL_SEARCH) && rows.length > TV_SEG_MAX_LENGTH) return TV_ERR_UNSUPPORTED;
    uint32_t *order_ws = nullptr;
    if (e.ws) {
        if (!aligned16(e.ws) || e.ws_bytes < fwd_workspace_bytes(rows, lam, n_rows))
            return TV_ERR_WORKSPACE;
        order_ws = (uint32_t *)e.ws;
    }
    // small batches of short rows: a few threads per row (see tv_dispatch.hpp)
    // (not when the caller hands over the slot-order workspace or asks for the parallel step-size
    // search: both belong to the row-per-lane kernels)
    const bool few = n_rows <= tvd::get(tvd::kThreadPerSample1dRows) && !e.ws && !(e.flags & TV_FWD_PARALLEL_SEARCH);
    return run_fwd(y, nullptr, x, nullptr, e.info, reinterpret_cast<uint2 *>(e.seg), order_ws, rows,
                   lam, n_rows, s, nullptr, false, (char *)e.ws, false, few,
                   (e.flags & TV_FWD_ORDER_READY) != 0, (e.flags & TV_FWD_PARALLEL_SEARCH) != 0);
}

// Device address of `scratch` on the current device, resolved on the first call there.
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
float *scratch_ptr[kMaxDevices] = {};

int scratch_of_current_device(float **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TV_ERR_HIP;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TV_ERR_HIP;
        scratch_ptr[dev] = static_cast<float *>(ptr);
    }
    *out = scratch_ptr[dev];
    return TV_OK;
}

// ws == nullptr with static_ws: the dL/dlam terms go through the library's static scratch.
int bwd_entry(const float *g_up, const float *x, const uint64_t *seg, bool with_seg, float *grad_y,
              float *grad_lam, tv_rows rows, tv_lambda lam, void *ws, size_t ws_bytes, hipStream_t stream,
              bool static_ws = false)
{
    int st = check_lambda(lam);
    if (st != TV_OK) return st;
    int64_t n_rows;
    st = check_rows(rows, &n_rows);
    if (st != TV_OK) return st;
    if (n_rows == 0) {
        // no rows: every slot's gradient is zero, which needs a device write
        return grad_lam ? zero_floats(grad_lam, lam.count, stream) : TV_OK;
    }
    if (!g_up || !grad_y || (with_seg ? !seg : !x)) return TV_ERR_NULL;
    if (rows.length > TV_MAX_LENGTH) return TV_ERR_UNSUPPORTED;
    if (with_seg) {
        if (rows.length > TV_SEG_MAX_LENGTH) return TV_ERR_UNSUPPORTED;
        if ((uintptr_t)seg % 8 != 0) return TV_ERR_STRIDE;
    }
    if (static_ws) {
        if (n_rows > (int64_t)TV_NOALLOC_MAX_ROWS) return TV_ERR_SCRATCH;
        if (grad_lam) {
            float *ptr = nullptr;
            st = scratch_of_current_device(&ptr);
            if (st != TV_OK) return st;
            ws = ptr;
        }
    } else if (grad_lam) {
        if (!ws || !aligned16(ws) || ws_bytes < align16((size_t)n_rows * sizeof(float)))
            return TV_ERR_WORKSPACE;
    }
    return run_bwd(g_up, nullptr, with_seg ? nullptr : x,
                   with_seg ? reinterpret_cast<const uint2 *>(seg) : nullptr, grad_y, grad_lam, 0,
                   rows, lam, n_rows, (float *)ws, stream);
}

}  // namespace

extern "C" {

int64_t tv_dispatch_threshold(const char *name)
{
    if (!name) return -1;
    for (int i = 0; i < tvd::kCount; ++i)
        if (strcmp(name, tvd::table[i].name) == 0) return tvd::table[i].value;
    return -1;
}

int tv_dispatch_override(const char *name, int64_t value)
{
    if (!name || value < 0) return TV_ERR_SHAPE;
    for (int i = 0; i < tvd::kCount; ++i)
        if (strcmp(name, tvd::table[i].name) == 0) {
            tvd::table[i].value = value;
            return TV_OK;
        }
    return TV_ERR_UNSUPPORTED;
}

const char *tv_dispatch_name(int index)
{
    return index >= 0 && index < tvd::kCount ? tvd::table[index].name : nullptr;
}

const char *tv_status_str(int status)
{
    switch (status) {
    case TV_OK: return "ok";
    case TV_ERR_NULL: return "null pointer";
    case TV_ERR_SHAPE: return "bad shape";
    case TV_ERR_STRIDE: return "bad stride";
    case TV_ERR_LAMBDA: return "bad lambda descriptor";
    case TV_ERR_WORKSPACE: return "bad workspace";
    case TV_ERR_UNSUPPORTED: return "unsupported size";
    case TV_ERR_HIP: return "HIP runtime error";
    case TV_ERR_SCRATCH: return "more rows than the static scratch buffer holds";
    default: return "unknown status";
    }
}

int tv1d_prox_fwd(const float *y, float *x, tv_rows rows, tv_lambda lam, hipStream_t stream)
{
    return fwd_entry(y, x, rows, lam, tv_fwd_extra{nullptr, nullptr, nullptr, 0, 0}, stream);
}

int tv1d_prox_fwd_info(const float *y, float *x, int32_t *info, tv_rows rows, tv_lambda lam,
                       hipStream_t stream)
{
    return fwd_entry(y, x, rows, lam, tv_fwd_extra{info, nullptr, nullptr, 0, 0}, stream);
}

int tv1d_prox_fwd_seg(const float *y, float *x, uint64_t *seg, tv_rows rows, tv_lambda lam,
                      hipStream_t stream)
{
    if (!seg) {
        int64_t n_rows;
        if (check_lambda(lam) == TV_OK && check_rows(rows, &n_rows) == TV_OK && n_rows > 0)
            return TV_ERR_NULL;
    }
    return fwd_entry(y, x, rows, lam, tv_fwd_extra{nullptr, seg, nullptr, 0, 0}, stream);
}

int tv1d_prox_fwd_ex(const float *y, float *x, tv_rows rows, tv_lambda lam, tv_fwd_extra extra,
                     hipStream_t stream)
{
    return fwd_entry(y, x, rows, lam, extra, stream);
}

size_t tv1d_fwd_steps_floats_per_row(int64_t length)
{
    return length >= 1 && length <= TV_MAX_LENGTH ? (size_t)tvk::step_record_floats(length) : 0;
}

int tv1d_prox_fwd_steps(const float *y, float *x, int32_t *info, float *record, int64_t record_rows,
                        tv_rows rows, tv_lambda lam, hipStream_t stream)
{
    int st = check_lambda(lam);
    if (st != TV_OK) return st;
    int64_t n_rows;
    st = check_rows(rows, &n_rows);
    if (st != TV_OK) return st;
    if (record_rows < 0) return TV_ERR_SHAPE;
    if (n_rows == 0) return TV_OK;
    if (!y || !x || !lam.lam || (record_rows > 0 && !record)) return TV_ERR_NULL;
    if (rows.length > TV_MAX_LENGTH) return TV_ERR_UNSUPPORTED;
    if (rows.length > 32 && rows.elem_stride != 1) return TV_ERR_UNSUPPORTED;
    FwdParams p;
    p.y = y; p.addend = nullptr; p.x = x; p.x2 = nullptr; p.resid = nullptr; p.lam = lam.lam; p.info = info;
    p.seg = nullptr; p.order = nullptr; p.io16 = 0; p.psearch = 0; p.warm = 0;
    p.coarse_u = nullptr; p.coarse_n = 0; p.coarse_pitch = 0; p.dual_out = nullptr; p.dual_pitch = 0;
    p.ml_flag = nullptr; p.flag_pitch = 1; p.ml_skip = 0;
    p.lam_scale = 1.0f;
    p.debug = record;
    p.debug_rows = (uint32_t)(record_rows < n_rows ? record_rows : n_rows);
    p.L = make_layout(rows, lam, n_rows);
    p.tm = tvk::TileMap{6u, 0u, 0u, 1u};
    if (rows.length <= 32) {
        // the general variant of the row-per-lane kernel (any length up to 32, any strides)
        const dim3 grid((uint32_t)((n_rows + 63) / 64)), block(tvk::kShortBlock);
        if (rows.length == 32)
            hipLaunchKernelGGL((tvk::tv1d_fwd_short_kernel<32, true, false, false, false, false, true>), grid, block, 0,
                               stream, p);
        else
            hipLaunchKernelGGL((tvk::tv1d_fwd_short_kernel<32, false, false, false, false, false, true>), grid, block, 0,
                               stream, p);
        return launch_status();
    }
    return tvk::launch_fwd_long_debug(p, stream) == hipSuccess ? TV_OK : TV_ERR_HIP;
}

size_t tv1d_fwd_workspace_bytes(tv_rows rows, tv_lambda lam)
{
    int64_t n_rows;
    if (check_lambda(lam) != TV_OK || check_rows(rows, &n_rows) != TV_OK) return 0;
    return fwd_workspace_bytes(rows, lam, n_rows);
}

size_t tv1d_bwd_workspace_bytes(tv_rows rows, tv_lambda lam)
{
    (void)lam;
    int64_t n_rows;
    if (check_rows(rows, &n_rows) != TV_OK) return 0;
    return align16((size_t)n_rows * sizeof(float));
}

int tv1d_prox_bwd(const float *g_up, const float *x, float *grad_y, float *grad_lam, tv_rows rows,
                  tv_lambda lam, void *ws, size_t ws_bytes, hipStream_t stream)
{
    return bwd_entry(g_up, x, nullptr, false, grad_y, grad_lam, rows, lam, ws, ws_bytes, stream);
}

int tv1d_prox_bwd_seg(const float *g_up, const uint64_t *seg, float *grad_y, float *grad_lam,
                      tv_rows rows, tv_lambda lam, void *ws, size_t ws_bytes, hipStream_t stream)
{
    return bwd_entry(g_up, nullptr, seg, true, grad_y, grad_lam, rows, lam, ws, ws_bytes, stream);
}

int tv1d_prox_bwd_noalloc(const float *g_up, const float *x, float *grad_y, float *grad_lam,
                          tv_rows rows, tv_lambda lam, hipStream_t stream)
{
    return bwd_entry(g_up, x, nullptr, false, grad_y, grad_lam, rows, lam, nullptr, 0, stream, true);
}

// ---- bf16 storage, fp32 arithmetic: packed rows of exactly 32 samples, segment-code pair only --

static int check_bf16(const void *a, const void *b, const uint64_t *seg, tv_rows rows, tv_lambda lam,
                      int64_t *n_rows)
{
    int st = check_lambda(lam);
    if (st != TV_OK) return st;
    st = check_rows(rows, n_rows);
    if (st != TV_OK) return st;
    if (*n_rows == 0) return TV_OK;
    if (!a || !b || !seg || !lam.lam) return TV_ERR_NULL;
    if (rows.length != 32 || !rows_packed(rows)) return TV_ERR_UNSUPPORTED;
    if (!aligned16(a) || !aligned16(b) || (uintptr_t)seg % 8 != 0) return TV_ERR_STRIDE;
    return TV_OK;
}

int tv1d_prox_fwd_seg_bf16(const uint16_t *y, uint16_t *x, uint64_t *seg, tv_rows rows, tv_lambda lam,
                           void *ws, size_t ws_bytes, hipStream_t stream)
{
    int64_t n_rows = 0;
    const int st = check_bf16(y, x, seg, rows, lam, &n_rows);
    if (st != TV_OK || n_rows == 0) return st;
    if (ws && (!aligned16(ws) || ws_bytes < fwd_workspace_bytes(rows, lam, n_rows))) return TV_ERR_WORKSPACE;
    return run_fwd(reinterpret_cast<const float *>(y), nullptr, reinterpret_cast<float *>(x), nullptr, nullptr,
                   reinterpret_cast<uint2 *>(seg), (uint32_t *)ws, rows, lam, n_rows, stream, nullptr, false,
                   nullptr, true);
}

int tv1d_prox_bwd_seg_bf16(const uint16_t *g_up, const uint64_t *seg, uint16_t *grad_y, float *grad_lam,
                           tv_rows rows, tv_lambda lam, void *ws, size_t ws_bytes, hipStream_t stream)
{
    int64_t n_rows = 0;
    const int st = check_bf16(g_up, grad_y, seg, rows, lam, &n_rows);
    if (st != TV_OK) return st;
    if (n_rows == 0) return grad_lam ? zero_floats(grad_lam, lam.count, stream) : TV_OK;
    if (grad_lam && (!ws || !aligned16(ws) || ws_bytes < align16((size_t)n_rows * sizeof(float))))
        return TV_ERR_WORKSPACE;
    return run_bwd(reinterpret_cast<const float *>(g_up), nullptr, nullptr, reinterpret_cast<const uint2 *>(seg),
                   reinterpret_cast<float *>(grad_y), grad_lam, 0, rows, lam, n_rows, (float *)ws, stream, true,
                   true);
}

// ---- 2D: proximal Dykstra (paper Alg. 1) ----------------------------------------------

// Planes whose rows and columns both fit the row-per-lane kernels also keep every pass's
// segment codes (8 bytes per row), which is all the reverse sweep reads of the pass outputs.
static bool small_planes(int64_t H, int64_t W) { return H <= TV_SEG_MAX_LENGTH && W <= TV_SEG_MAX_LENGTH; }

static int check_2d(int64_t planes, int64_t H, int64_t W, int sweeps, size_t *tensor_bytes,
                    size_t *partial_bytes, size_t *code_bytes)
{
    if (planes < 0 || H < 1 || W < 1 || sweeps < 1 || sweeps > 4096) return TV_ERR_SHAPE;
    if (planes > kMaxRows || H > kMaxRows || W > kMaxRows) return TV_ERR_SHAPE;
    if (planes > 0 && (planes * H > kMaxRows || planes * W > kMaxRows)) return TV_ERR_SHAPE;
    if (planes > 0 && H * W > (INT64_MAX / 64) / planes) return TV_ERR_SHAPE;
    *tensor_bytes = align16((size_t)(planes * H * W) * sizeof(float));
    const int64_t mr = planes * (H > W ? H : W);
    *partial_bytes = align16((size_t)mr * sizeof(float));
    *code_bytes = small_planes(H, W) ? align16((size_t)mr * sizeof(uint64_t)) : 0;   // per pass
    return TV_OK;
}

size_t tv2d_workspace_bytes(int64_t planes, int64_t H, int64_t W, int sweeps)
{
    size_t tb, pb, cb;
    if (check_2d(planes, H, W, sweeps, &tb, &pb, &cb) != TV_OK) return 0;
    return tb * (size_t)(2 * sweeps + 2) + (pb + cb) * (size_t)(2 * sweeps) + kSplitScratchBytes;
}

// Planes of at most 32 x 32 are padded to squares of side 8, 16 or 32; a wave holds 64 / side of them.
static int small_side(int64_t H, int64_t W)
{
    const int64_t m = H > W ? H : W;
    return m <= 8 ? 8 : (m <= 16 ? 16 : 32);
}

#define TV_SMALL2D_LAUNCH(KERNEL, q, planes, H, W, stream)                                          \
    do {                                                                                            \
        const int side = small_side(H, W);                                                          \
        const bool full = (H) == side && (W) == side;                                               \
        const dim3 grid((uint32_t)(((planes) + 64 / side - 1) / (64 / side)));                      \
        if (side == 8) {                                                                            \
            if (full) hipLaunchKernelGGL((KERNEL<8, true>), grid, dim3(64), 0, stream, q);          \
            else hipLaunchKernelGGL((KERNEL<8, false>), grid, dim3(64), 0, stream, q);              \
        } else if (side == 16) {                                                                    \
            if (full) hipLaunchKernelGGL((KERNEL<16, true>), grid, dim3(64), 0, stream, q);         \
            else hipLaunchKernelGGL((KERNEL<16, false>), grid, dim3(64), 0, stream, q);             \
        } else {                                                                                    \
            if (full) hipLaunchKernelGGL((KERNEL<32, true>), grid, dim3(64), 0, stream, q);         \
            else hipLaunchKernelGGL((KERNEL<32, false>), grid, dim3(64), 0, stream, q);             \
        }                                                                                           \
    } while (0)

// the same for kernels with further template arguments (bool..., after S and FULL)
#define TV_SMALL2D_LAUNCH_X(KERNEL, q, planes, H, W, stream, ...)                                    \
    do {                                                                                            \
        const int side = small_side(H, W);                                                          \
        const bool full = (H) == side && (W) == side;                                               \
        const dim3 grid((uint32_t)(((planes) + 64 / side - 1) / (64 / side)));                      \
        if (side == 8) {                                                                            \
            if (full) hipLaunchKernelGGL((KERNEL<8, true, __VA_ARGS__>), grid, dim3(64), 0, stream, q);   \
            else hipLaunchKernelGGL((KERNEL<8, false, __VA_ARGS__>), grid, dim3(64), 0, stream, q);       \
        } else if (side == 16) {                                                                    \
            if (full) hipLaunchKernelGGL((KERNEL<16, true, __VA_ARGS__>), grid, dim3(64), 0, stream, q);  \
            else hipLaunchKernelGGL((KERNEL<16, false, __VA_ARGS__>), grid, dim3(64), 0, stream, q);      \
        } else {                                                                                    \
            if (full) hipLaunchKernelGGL((KERNEL<32, true, __VA_ARGS__>), grid, dim3(64), 0, stream, q);  \
            else hipLaunchKernelGGL((KERNEL<32, false, __VA_ARGS__>), grid, dim3(64), 0, stream, q);      \
        }                                                                                           \
    } while (0)

// Small batches of planes of 17-64 samples a side: one launch with a plane per workgroup
// (tv_plane2d.hpp), up to the plane counts of tv_dispatch.hpp.  Planes of at most 32 x 32 leave
// segment codes for the reverse sweep, larger ones their pass outputs.
static bool plane_per_group_2d(int64_t planes, int64_t H, int64_t W, int sweeps)
{
    if (small_planes(H, W)) return small_side(H, W) == 32 && planes <= tvd::get(tvd::kPlanePerGroupPlanes);
    if (H > 64 || W > 64) return false;
    if (sweeps == 1) return planes <= tvd::get(tvd::kPlanePerGroup64Planes);
    if (H == 64 && W == 64)
        return planes <= tvd::get(sweeps == 2 ? tvd::kPlanePerGroup64FullPlanesK2
                                               : (sweeps <= 4 ? tvd::kPlanePerGroup64FullPlanesK3 : tvd::kPlanePerGroup64FullPlanesK5));
    return planes <= tvd::get(tvd::kPlanePerGroup64PlanesK2);
}

// When the one-launch forward kernel is used: while its lower occupancy (17 KB of LDS per wave
// for planes padded to 32 x 32: two waves per SIMD against three) costs less than the launches and
// memory round trips it saves.  The plane counts, and the measurements behind them, are in
// tv_dispatch.hpp; planes of at most 8 x 8 are always better off in one launch.
static bool fused_fwd_applies(int side, bool full, int64_t planes, int sweeps)
{
    // (planes smaller than their 32 x 32 square go pass by pass through the slower general
    // variants of the row-per-lane kernels, so there the one launch wins whenever there is more
    // than one sweep: 28 x 28, 32 768 planes, K = 4: 1.46 ms against 1.94)
    if (side == 32) {
        if (!full) return sweeps >= 2 || planes <= tvd::get(tvd::kFused32RaggedPlanes);
        return planes <= tvd::get(sweeps == 1 ? tvd::kFused32FullPlanes
                                              : (sweeps == 2 ? tvd::kFused32FullPlanesK2 : tvd::kFused32FullPlanesK3));
    }
    if (side == 16) return sweeps >= 2 || planes <= tvd::get(tvd::kFused16OneSweepPlanes);
    return true;
}

int tv2d_prox_fwd(const float *y, float *x, int64_t planes, int64_t H, int64_t W, tv_lambda lam,
                  int sweeps, void *ws, size_t ws_bytes, hipStream_t stream)
{
    if (lam.count < 1 || lam.count > kMaxRows) return TV_ERR_LAMBDA;
    size_t tb, pb, cb;
    int st = check_2d(planes, H, W, sweeps, &tb, &pb, &cb);
    if (st != TV_OK) return st;
    if (planes == 0) return TV_OK;
    if (!y || !x || !lam.lam) return TV_ERR_NULL;
    if (H > TV_MAX_LENGTH || W > TV_MAX_LENGTH) return TV_ERR_UNSUPPORTED;
    if (!ws || !aligned16(ws) || ws_bytes < tb * (size_t)(2 * sweeps + 2) + (pb + cb) * (size_t)(2 * sweeps) + kSplitScratchBytes)
        return TV_ERR_WORKSPACE;

    char *base = (char *)ws;
    auto saved = [&](int i) { return (float *)(base + tb * (size_t)i); };
    float *P = saved(2 * sweeps), *Q = saved(2 * sweeps + 1);
    auto codes = [&](int pass) -> uint2 * {
        return cb ? (uint2 *)(base + tb * (size_t)(2 * sweeps + 2) + pb * (size_t)(2 * sweeps) + cb * (size_t)pass)
                  : nullptr;
    };
    const tv_rows rrow = {planes, H * W, H, W, W, 1};
    const tv_rows rcol = {planes, H * W, W, 1, H, W};
    const tv_lambda lrow = {lam.lam, lam.count, H};
    const tv_lambda lcol = {lam.lam, lam.count, W};

    if (plane_per_group_2d(planes, H, W, sweeps)) {
        // a small batch of planes of 17-64 samples a side: one launch, a plane per workgroup
        tvk::Small2dFwdParams q;
        q.y = y; q.x = x; q.saved = saved(0); q.saved_stride = tb / sizeof(float); q.keep_passes = tvd::get(tvd::kFusedKeepsPasses) != 0 ? 1u : 0u;
        q.codes = codes(0); q.code_stride = cb / sizeof(uint2);
        q.lam = lam.lam; q.lam_count = lam.count;
        q.planes = (int32_t)planes; q.H = (int32_t)H; q.W = (int32_t)W; q.sweeps = sweeps;
        q.stream = 0u;
        const dim3 grid((uint32_t)planes);
        if (cb) hipLaunchKernelGGL((tvk::tv2d_fwd_plane_kernel<16, 2>), grid, dim3(512), 0, stream, q);
        else hipLaunchKernelGGL((tvk::tv2d_fwd_plane_kernel<8, 8>), grid, dim3(512), 0, stream, q);
        return launch_status();
    }
    if (cb && fused_fwd_applies(small_side(H, W), H == small_side(H, W) && W == H, planes, sweeps)) {
        // planes of at most 32 x 32: all passes in one launch, the planes resident in LDS
        tvk::Small2dFwdParams q;
        q.y = y; q.x = x; q.saved = saved(0); q.saved_stride = tb / sizeof(float); q.keep_passes = tvd::get(tvd::kFusedKeepsPasses) != 0 ? 1u : 0u;
        q.codes = codes(0); q.code_stride = cb / sizeof(uint2);
        q.lam = lam.lam; q.lam_count = lam.count;
        q.planes = (int32_t)planes; q.H = (int32_t)H; q.W = (int32_t)W; q.sweeps = sweeps;
        q.stream = (planes * H * W >= tvd::get(tvd::kStreamBytes) / 4) ? 1u : 0u;
        if (small_side(H, W) == 16 && planes >= tvd::get(tvd::kFused16DensePlanes)) {
            const dim3 grid((uint32_t)((planes + 3) / 4));
            if (H == 16 && W == 16) hipLaunchKernelGGL((tvk::tv2d_fwd_small_kernel<16, true, false, true>), grid, dim3(64), 0, stream, q);
            else hipLaunchKernelGGL((tvk::tv2d_fwd_small_kernel<16, false, false, true>), grid, dim3(64), 0, stream, q);
            return launch_status();
        }
        TV_SMALL2D_LAUNCH(tvk::tv2d_fwd_small_kernel, q, planes, H, W, stream);
        return launch_status();
    }
    for (int k = 0; k < sweeps; ++k) {
        const bool last = (k == sweeps - 1);
        const float *Yk = (k == 0) ? y : saved(2 * k - 1);
        float *Z = saved(2 * k), *Yn = saved(2 * k + 1);
        // Z = proxRows(Y + P);  P <- (Y + P) - Z      (P = 0 in the first sweep)
        // From the second sweep on, P = D^T u of the row pass one sweep earlier (x = y - D^T u),
        // and likewise Q for the columns: each pass starts from that dual.
        st = run_fwd(Yk, k == 0 ? nullptr : P, Z, last ? nullptr : P, nullptr, codes(2 * k), nullptr,
                     rrow, lrow, planes * H, stream, nullptr, true);
        if (st != TV_OK) return st;
        // Y' = proxCols(Z + Q);  Q <- (Z + Q) - Y'
        // the last pass writes its output twice: where the reverse sweep will look for it, and to x
        st = run_fwd(Z, k == 0 ? nullptr : Q, Yn, last ? nullptr : Q, nullptr, codes(2 * k + 1), nullptr,
                     rcol, lcol, planes * W, stream, last ? x : nullptr, true);
        if (st != TV_OK) return st;
    }
    return TV_OK;
}

// ---- the 2D operator with bf16 storage of y, x, g_up and grad_y (planes of at most 32 x 32): always
//      one launch each way (small batches of planes of 17-32 samples a side with a plane per
//      workgroup, a row per lane otherwise); the workspace (saved pass outputs, segment codes) is
//      as for fp32.
int tv2d_prox_fwd_bf16(const uint16_t *y, uint16_t *x, int64_t planes, int64_t H, int64_t W, tv_lambda lam,
                       int sweeps, void *ws, size_t ws_bytes, hipStream_t stream)
{
    if (lam.count < 1 || lam.count > kMaxRows) return TV_ERR_LAMBDA;
    size_t tb, pb, cb;
    int st = check_2d(planes, H, W, sweeps, &tb, &pb, &cb);
    if (st != TV_OK) return st;
    if (planes == 0) return TV_OK;
    if (!y || !x || !lam.lam) return TV_ERR_NULL;
    if (!small_planes(H, W)) return TV_ERR_UNSUPPORTED;
    if (((uintptr_t)y | (uintptr_t)x) % 2 != 0) return TV_ERR_STRIDE;
    if (!ws || !aligned16(ws) || ws_bytes < tb * (size_t)(2 * sweeps + 2) + (pb + cb) * (size_t)(2 * sweeps) + kSplitScratchBytes)
        return TV_ERR_WORKSPACE;
    char *base = (char *)ws;
    tvk::Small2dFwdParams q;
    q.y = reinterpret_cast<const float *>(y); q.x = reinterpret_cast<float *>(x);
    q.saved = (float *)base; q.saved_stride = tb / sizeof(float); q.keep_passes = tvd::get(tvd::kFusedKeepsPasses) != 0 ? 1u : 0u;
    q.codes = (uint2 *)(base + tb * (size_t)(2 * sweeps + 2) + pb * (size_t)(2 * sweeps));
    q.code_stride = cb / sizeof(uint2);
    q.lam = lam.lam; q.lam_count = lam.count;
    q.planes = (int32_t)planes; q.H = (int32_t)H; q.W = (int32_t)W; q.sweeps = sweeps;
    q.stream = (planes * H * W >= tvd::get(tvd::kStreamBytes) / 4) ? 1u : 0u;
    if (plane_per_group_2d(planes, H, W, sweeps))       // a small batch: a plane per workgroup
        hipLaunchKernelGGL((tvk::tv2d_fwd_plane_kernel<16, 2, true>), dim3((uint32_t)planes), dim3(512), 0, stream, q);
    else
        TV_SMALL2D_LAUNCH_X(tvk::tv2d_fwd_small_kernel, q, planes, H, W, stream, true);
    return launch_status();
}

int tv2d_prox_bwd_bf16(const uint16_t *g_up, uint16_t *grad_y, float *grad_lam, int64_t planes, int64_t H,
                       int64_t W, tv_lambda lam, int sweeps, void *ws, size_t ws_bytes, hipStream_t stream)
{
    if (lam.count < 1 || lam.count > kMaxRows) return TV_ERR_LAMBDA;
    size_t tb, pb, cb;
    int st = check_2d(planes, H, W, sweeps, &tb, &pb, &cb);
    if (st != TV_OK) return st;
    if (planes == 0) return grad_lam ? zero_floats(grad_lam, lam.count, stream) : TV_OK;
    if (!g_up || !grad_y) return TV_ERR_NULL;
    if (!small_planes(H, W)) return TV_ERR_UNSUPPORTED;
    if (((uintptr_t)g_up | (uintptr_t)grad_y) % 2 != 0) return TV_ERR_STRIDE;
    if (!ws || !aligned16(ws) || ws_bytes < tb * (size_t)(2 * sweeps + 2) + (pb + cb) * (size_t)(2 * sweeps) + kSplitScratchBytes)
        return TV_ERR_WORKSPACE;
    char *base = (char *)ws;
    float *partial = (float *)(base + tb * (size_t)(2 * sweeps + 2));
    tvk::Small2dBwdParams q;
    q.g_up = reinterpret_cast<const float *>(g_up); q.gy = reinterpret_cast<float *>(grad_y);
    q.codes = (const uint2 *)(base + tb * (size_t)(2 * sweeps + 2) + pb * (size_t)(2 * sweeps));
    q.code_stride = cb / sizeof(uint2);
    q.saved = (const float *)base; q.saved_stride = tb / sizeof(float);
    q.partial = grad_lam ? partial : nullptr;
    q.planes = (int32_t)planes; q.H = (int32_t)H; q.W = (int32_t)W; q.sweeps = sweeps;
    q.stream = (planes * H * W >= tvd::get(tvd::kStreamBytes) / 4) ? 1u : 0u;
    if (small_side(H, W) == 32 && planes <= tvd::get(tvd::kPlanePerGroupBwdPlanes))
        hipLaunchKernelGGL((tvk::tv2d_bwd_plane_kernel<16, 2, true>), dim3((uint32_t)planes), dim3(512), 0, stream, q);
    else
        TV_SMALL2D_LAUNCH_X(tvk::tv2d_bwd_small_kernel, q, planes, H, W, stream, false, true);
    if (launch_status() != TV_OK) return TV_ERR_HIP;
    if (!grad_lam) return TV_OK;
    const tv_lambda lp = {lam.lam, lam.count, 1};
    return launch_reduce_lambda(partial, grad_lam, planes, lp, 0, stream);
}

int tv2d_prox_bwd(const float *g_up, float *grad_y, float *grad_lam, int64_t planes, int64_t H,
                  int64_t W, tv_lambda lam, int sweeps, void *ws, size_t ws_bytes,
                  hipStream_t stream)
{
    if (lam.count < 1 || lam.count > kMaxRows) return TV_ERR_LAMBDA;
    size_t tb, pb, cb;
    int st = check_2d(planes, H, W, sweeps, &tb, &pb, &cb);
    if (st != TV_OK) return st;
    if (planes == 0) {
        return grad_lam ? zero_floats(grad_lam, lam.count, stream) : TV_OK;
    }
    if (!g_up || !grad_y) return TV_ERR_NULL;
    if (H > TV_MAX_LENGTH || W > TV_MAX_LENGTH) return TV_ERR_UNSUPPORTED;
    if (!ws || !aligned16(ws) || ws_bytes < tb * (size_t)(2 * sweeps + 2) + (pb + cb) * (size_t)(2 * sweeps) + kSplitScratchBytes)
        return TV_ERR_WORKSPACE;

    char *base = (char *)ws;
    auto saved = [&](int i) { return (float *)(base + tb * (size_t)i); };
    float *Ab = saved(2 * sweeps), *Bb = saved(2 * sweeps + 1);
    // dL/dlam terms of pass i; summed over all passes at the end, one launch per direction
    auto partial = [&](int pass) { return (float *)(base + tb * (size_t)(2 * sweeps + 2) + pb * (size_t)pass); };
    auto codes = [&](int pass) -> const uint2 * {
        return cb ? (const uint2 *)(base + tb * (size_t)(2 * sweeps + 2) + pb * (size_t)(2 * sweeps) +
                                    cb * (size_t)pass)
                  : nullptr;
    };
    const tv_rows rrow = {planes, H * W, H, W, W, 1};
    const tv_rows rcol = {planes, H * W, W, 1, H, W};
    const tv_lambda lrow = {lam.lam, lam.count, H};
    const tv_lambda lcol = {lam.lam, lam.count, W};

    // Adjoint of one sweep (A = Y + P, Z = R(A), P' = A - Z, B = Z + Q, Y' = C(B), Q' = B - Y'):
    //   Bbar = Qbar' + C^T(Ybar' - Qbar'),   Qbar = Bbar,
    //   Abar = Pbar' + R^T(Bbar - Pbar'),    Ybar = Pbar = Abar.
    // Ybar and Pbar coincide from the second reverse step on, so two tensors carry the state.
    if ((cb && small_side(H, W) == 32 && planes <= tvd::get(tvd::kPlanePerGroupBwdPlanes)) ||
        (!cb && H <= 64 && W <= 64 &&
         planes <= tvd::get((H == 64 && W == 64) ? tvd::kPlanePerGroup64BwdPlanes
                                                 : (sweeps == 1 ? tvd::kPlanePerGroup64BwdRaggedPlanes
                                                                : tvd::kPlanePerGroup64BwdRaggedPlanesK2)))) {
        // a small batch of planes of 17-64 samples a side: one launch, a plane per workgroup
        tvk::Small2dBwdParams q;
        q.g_up = g_up; q.gy = grad_y; q.codes = codes(0); q.code_stride = cb / sizeof(uint2);
        q.saved = saved(0); q.saved_stride = tb / sizeof(float);
        q.partial = grad_lam ? partial(0) : nullptr;
        q.planes = (int32_t)planes; q.H = (int32_t)H; q.W = (int32_t)W; q.sweeps = sweeps;
        q.stream = 0u;
        const dim3 grid((uint32_t)planes);
        if (cb) hipLaunchKernelGGL((tvk::tv2d_bwd_plane_kernel<16, 2>), grid, dim3(512), 0, stream, q);
        else hipLaunchKernelGGL((tvk::tv2d_bwd_plane_kernel<8, 8>), grid, dim3(512), 0, stream, q);
        if (launch_status() != TV_OK) return TV_ERR_HIP;
        if (!grad_lam) return TV_OK;
        const tv_lambda lp = {lam.lam, lam.count, 1};
        return launch_reduce_lambda(partial(0), grad_lam, planes, lp, 0, stream);
    }
    if (cb || (H == 64 && W == 64)) {
        // planes of at most 32 x 32, or of 64 x 64: the whole reverse sweep in one launch, state
        // resident in LDS (up to 32 x 32 the segments come from the codes, at 64 x 64 from the saved
        // pass outputs; other planes of 33-64 samples a side are faster pass by pass: 40 x 40,
        // K = 1, 44 us against 116)
        tvk::Small2dBwdParams q;
        q.g_up = g_up; q.gy = grad_y; q.codes = codes(0); q.code_stride = cb / sizeof(uint2);
        q.saved = saved(0); q.saved_stride = tb / sizeof(float);
        q.partial = grad_lam ? partial(0) : nullptr;
        q.planes = (int32_t)planes; q.H = (int32_t)H; q.W = (int32_t)W; q.sweeps = sweeps;
        q.stream = (planes * H * W >= tvd::get(tvd::kStreamBytes) / 4) ? 1u : 0u;
        if (cb) {
            TV_SMALL2D_LAUNCH(tvk::tv2d_bwd_small_kernel, q, planes, H, W, stream);
        } else {
            hipLaunchKernelGGL((tvk::tv2d_bwd_small_kernel<64, true>), dim3((uint32_t)planes), dim3(64), 0, stream, q);
        }
        if (launch_status() != TV_OK) return TV_ERR_HIP;
        if (!grad_lam) return TV_OK;
        const tv_lambda lp = {lam.lam, lam.count, 1};
        return launch_reduce_lambda(partial(0), grad_lam, planes, lp, 0, stream);
    }
    for (int k = sweeps - 1; k >= 0; --k) {
        const bool first = (k == sweeps - 1);
        st = run_bwd(first ? g_up : Ab, first ? nullptr : Bb, cb ? nullptr : saved(2 * k + 1), codes(2 * k + 1),
                     Bb, grad_lam, 0, rcol, lcol, planes * W, partial(2 * k + 1), stream, false);
        if (st != TV_OK) return st;
        st = run_bwd(Bb, first ? nullptr : Ab, cb ? nullptr : saved(2 * k), codes(2 * k), k == 0 ? grad_y : Ab,
                     grad_lam, 0, rrow, lrow, planes * H, partial(2 * k), stream, false);
        if (st != TV_OK) return st;
    }
    if (grad_lam) {
        const uint64_t two_passes = 2 * (uint64_t)(pb / sizeof(float));
        const PartialShape pr = partial_shape(rrow, lrow, planes * H), pc = partial_shape(rcol, lcol, planes * W);
        tv_lambda lr = lrow, lc = lcol;
        lr.div = pr.red_div; lc.div = pc.red_div;
        const uint32_t splits = reduce_splits(lam.count, sweeps);
        double *split = (double *)(base + tb * (size_t)(2 * sweeps + 2) + (pb + cb) * (size_t)(2 * sweeps));
        st = launch_reduce_lambda(partial(0), grad_lam, pr.red_rows, lr, 0, stream, (uint32_t)sweeps, two_passes,
                                  splits, splits > 1 ? split : nullptr);
        if (st != TV_OK) return st;
        st = launch_reduce_lambda(partial(1), grad_lam, pc.red_rows, lc, 1, stream, (uint32_t)sweeps, two_passes,
                                  splits, splits > 1 ? split + (size_t)lam.count * splits : nullptr);
        if (st != TV_OK) return st;
        if (splits > 1) {
            hipLaunchKernelGGL(sum_splits_kernel, dim3((uint32_t)((lam.count + 63) / 64)), dim3(64), 0, stream,
                               split, grad_lam, (uint32_t)lam.count, splits);
            if (launch_status() != TV_OK) return TV_ERR_HIP;
        }
    }
    return TV_OK;
}

}  // extern "C"
