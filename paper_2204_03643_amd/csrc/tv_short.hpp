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

#ifndef TV_FWD_ATTR
#define TV_FWD_ATTR
#endif
constexpr int kShortBlock = 64;    // one wave of 64 rows per workgroup: a finished wave frees its slot at once

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
    const int t = threadIdx.x;
    if (t <= NMAX) {
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

template <int NMAX>
struct TileRegs {
    float4 q[NMAX / 4];
};

// Global -> registers, in tile order (coalesced).  Rows past the end of the batch read as 0.
template <int NMAX>
__device__ __forceinline__ void tile_fetch(const float *__restrict__ src, uint32_t r0,
                                           uint32_t n_rows, int lane, TileRegs<NMAX> &t)
{
    const uint32_t valid_rows = r0 < n_rows ? min(64u, n_rows - r0) : 0u;
    const float4 *s4 = reinterpret_cast<const float4 *>(src + (size_t)r0 * NMAX);
#pragma unroll
    for (int i = 0; i < NMAX / 4; ++i) {
        const int e4 = i * 64 + lane;
        const uint32_t row = (uint32_t)(e4 * 4) / NMAX;
        t.q[i] = row < valid_rows ? s4[e4] : make_float4(0.f, 0.f, 0.f, 0.f);
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
__device__ __forceinline__ void tile_put(float *__restrict__ dst, uint32_t r0, uint32_t n_rows,
                                         int lane, const TileRegs<NMAX> &t)
{
    const uint32_t valid_rows = r0 < n_rows ? min(64u, n_rows - r0) : 0u;
    float4 *d4 = reinterpret_cast<float4 *>(dst + (size_t)r0 * NMAX);
#pragma unroll
    for (int i = 0; i < NMAX / 4; ++i) {
        const int e4 = i * 64 + lane;
        if ((uint32_t)(e4 * 4) / NMAX < valid_rows) d4[e4] = t.q[i];
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
// The dual u, the Newton direction and the pivots live in registers.  The input row is
// read-only after the start, so it is parked in LDS, sample-major: yl[k * 64] is sample k
// of this lane's row (consecutive lanes -> consecutive banks, no conflicts); that keeps the
// kernel at four waves per SIMD.  Samples k >= n must be 0.  On return xs holds the minimiser of paper Eq. 1.
// ---------------------------------------------------------------------------------
template <int NMAX, bool FULL>
__device__ __forceinline__ int pn_solve_row(const float *yl,
                                            float (&xs)[NMAX], float lam, int n, bool valid,
                                            const float *gtab, const float *rtab)
{
    constexpr int M = NMAX - 1;
    const int m = n - 1;
    // duals past the end of a shorter row get an empty box and never move
#define TV_LK(k) ((FULL || (k) < m) ? lam : 0.0f)
#define TV_Y(k) yl[(k) * 64]
#define TV_TAB(tab, off4) (*reinterpret_cast<const float *>(reinterpret_cast<const char *>(tab) + (off4)))
    // The parked row must be re-read in every pass; without this the compiler hoists the
    // (loop-invariant) LDS loads back into registers and the occupancy gain is lost.
#define TV_REREAD() asm volatile("" ::: "memory")

    float u[M > 0 ? M : 1];
    float X[NMAX];          // x(u) = y - D^T u for the current dual, carried between passes
    float fcur;

    // ---- starting point, one of two feasible candidates:
    //      A = one full Newton step from u = 0 with every dual free, clipped into the box
    //          (exact whenever lam >= lam_max = max_k |prefix_k(mean(y) - y)|);
    //      B = every dual at the bound its local difference points to (exact for small lam).
    //      A is taken when lam >= lam_max / 4, which picks the candidate with the lower dual
    //      objective in all but a few percent of rows (measured on the five workloads).
    {
        TV_REREAD();
        float sum = 0.f;
#pragma unroll
        for (int k = 0; k < NMAX; ++k) sum += TV_Y(k);
        const float ybar = sum * rtab[n];
        float uB[M > 0 ? M : 1];
        float run = 0.f, rmax = 0.f;
        TV_REREAD();
        float yk = TV_Y(0);
#pragma unroll
        for (int k = 0; k < M; ++k) {
            const float l = TV_LK(k);
            const float yn = TV_Y(k + 1);
            run += ybar - yk;
            if (FULL || k < m) rmax = fmaxf(rmax, fabsf(run));
            u[k] = __builtin_amdgcn_fmed3f(run, -l, l);
            uB[k] = __builtin_amdgcn_fmed3f((yn - yk) * 1e30f, -l, l);
            yk = yn;
        }
        const bool pickA = lam >= 0.25f * rmax;
        TV_REREAD();
        float acc = 0.f, prev = 0.f;
#pragma unroll
        for (int k = 0; k < M; ++k) {
            const float c = pickA ? u[k] : uB[k];
            const float xc = TV_Y(k) + c - prev;
            acc = fmaf(xc, xc, acc);
            u[k] = c; X[k] = xc; prev = c;
        }
        {
            const float xc = TV_Y(M) - prev;
            acc = fmaf(xc, xc, acc);
            X[M] = xc;
        }
        fcur = 0.5f * acc;
    }

    bool active = valid;
    bool prev_unclipped = false;
    int steps = 0, flags = 0, nfail = 0;
    float alpha_try = 1.f;
    // D: gamma*w after the forward elimination, then the Newton direction.  G: the pivots
    // gamma (0 exactly at bound duals); during the line search it keeps the previous dual.
    float D[M > 0 ? M : 1], G[M > 0 ? M : 1];

    for (int it = 0;; ++it) {
        // ---- gradient, bound set (Bertsekas' sign test with exact comparisons: a clipped
        //      dual is bit-equal to +-lam), optimality test, Thomas forward elimination
        //      w_k = g_k + gamma_{k-1} w_{k-1}, kept as t_k = gamma_k w_k
        bool vio = false;
        float dec = 0.f, tprev = 0.f;
        int pos4 = 0;                               // 4 * position inside the free run
#pragma unroll
        for (int k = 0; k < M; ++k) {
            const float g = X[k] - X[k + 1];
            const float s = copysignf(TV_LK(k), g);
            const bool bnd = (u[k] == -s);          // at a bound and pushed outwards
            if (FULL || k < m) vio |= (u[k] == s) && (g != 0.f);  // at a bound, pushed inwards
            pos4 = bnd ? 0 : pos4 + 4;
            const float gam = TV_TAB(gtab, pos4);
            const float w = g + tprev;
            const float t = gam * w;
            dec = fmaf(t, w, dec);                  // accumulates g^T H_S^-1 g
            D[k] = t; G[k] = gam;
            tprev = t;
        }
        // A full, unclipped Newton step zeroes the gradient on the free set; if no dual
        // sits on a bound with the gradient pointing inwards, the KKT conditions hold.
        if (active && prev_unclipped && !vio) { active = false; flags = kInfoConverged; }
        if (active && it >= kMaxNewtonSteps) { active = false; flags = kInfoCapped; }
        if (!__any(active)) break;
        steps += active ? 1 : 0;

        // ---- back substitution d_k = gamma_k (w_k + d_{k+1}) = t_k + gamma_k d_{k+1}
        {
            float dn = 0.f;
#pragma unroll
            for (int k = M - 1; k >= 0; --k) {
                dn = fmaf(G[k], dn, D[k]);
                D[k] = dn;
            }
        }

        // ---- projected step u(alpha) = clip(u - alpha d); alpha = 1 is taken outright when
        //      nothing clips (it is the exact minimiser over the free subspace), otherwise it
        //      must pass the Armijo test (paper Sec. 3.2).  The trial moves the previous dual
        //      into G (the pivots are spent once d is known) and writes the new dual and its x
        //      in place.  A row that fails the test takes its dual back and retries in the next
        //      round with a step length from quadratic interpolation; that is rare (under one
        //      row in a hundred), so the direction is simply recomputed there.
        const float alpha = active ? alpha_try : 0.f;
        bool changed = false;
        float acc = 0.f, prev = 0.f, tmax = 0.f;
        TV_REREAD();
#pragma unroll
        for (int k = 0; k < M; ++k) {
            const float l = TV_LK(k);
            const float uo = u[k];
            const float t = fmaf(-alpha, D[k], uo);
            const float c = __builtin_amdgcn_fmed3f(t, -l, l);
            tmax = fmaxf(tmax, fabsf(t));
            changed |= (c != uo);
            const float xc = TV_Y(k) + c - prev;
            acc = fmaf(xc, xc, acc);
            G[k] = uo; u[k] = c; X[k] = xc; prev = c;
        }
        {
            const float xc = TV_Y(M) - prev;
            acc = fmaf(xc, xc, acc);
            X[M] = xc;
        }
        const bool clipped = tmax > lam;
        const float fc = 0.5f * acc;
        const bool ok = !active || (alpha == 1.f && !clipped) ||
                        (fc <= fcur - kArmijoSigma * alpha * dec + kArmijoSlackEps * fabsf(fcur));
        if (__any(!ok)) {
            TV_REREAD();
            float pv = 0.f;
#pragma unroll
            for (int k = 0; k < M; ++k) {
                const float c = ok ? u[k] : G[k];
                u[k] = c;
                X[k] = TV_Y(k) + c - pv;
                pv = c;
            }
            X[M] = TV_Y(M) - pv;
            if (!ok) {
                const float den = 2.f * (fc - fcur + dec * alpha);
                const float an = den > 0.f ? dec * alpha * alpha / den : 0.5f * alpha;
                alpha_try = fminf(fmaxf(an, 0.1f * alpha), 0.5f * alpha);
                prev_unclipped = false;
                if (++nfail > kMaxBacktracks) { active = false; flags = kInfoStalled | kInfoPlain; }
            }
        }
        if (ok && active) {
            fcur = fc;
            prev_unclipped = (alpha == 1.f) && !clipped;
            alpha_try = 1.f;
            nfail = 0;
            if (!changed) {
                // a step that moves nothing: a KKT point if it was a full step with no dual
                // held against an inward gradient; otherwise the line search has run dry
                active = false;
                flags = kInfoStalled | ((alpha == 1.f && !vio) ? 0 : kInfoPlain);
            }
        }
        if (!__any(active)) {
            // G holds the previous dual now: rebuild the bound flags of the final iterate
#pragma unroll
            for (int k = 0; k < M; ++k) {
                const float g = X[k] - X[k + 1];
                G[k] = (u[k] == -copysignf(TV_LK(k), g)) ? 0.f : 1.f;
            }
            break;
        }
    }

    // ---- primal recovery.  X is x = y - D^T u at the final dual, and G[k] == 0 exactly at
    //      its bound duals.  Between two bound duals x is constant up to rounding; every
    //      sample takes the value of the first sample of its block, so that constant runs are
    //      bit-identical, which is what the backward pass keys on.  Rows that stopped without
    //      reaching a KKT point (iteration cap, failed line search) keep the plain x.
    {
        const bool plain = (flags & (kInfoCapped | kInfoPlain)) != 0;
        float val = X[0];
        xs[0] = val;
#pragma unroll
        for (int k = 1; k < NMAX; ++k) {
            const bool start = plain || (G[k - 1] == 0.f);
            val = start ? X[k] : val;
            xs[k] = val;
        }
    }
#undef TV_LK
#undef TV_Y
#undef TV_TAB
#undef TV_REREAD
    return steps | flags;
}

// ---------------------------------------------------------------------------------
// Forward kernel: one row per lane, one wave per workgroup.
// ---------------------------------------------------------------------------------
template <int NMAX, bool FULL, bool PACKED>
__global__ __launch_bounds__(kShortBlock) TV_FWD_ATTR void tv1d_fwd_short_kernel(FwdParams p)
{
    using S = ShortSmem<NMAX>;
    __shared__ float smem[S::kFloats];
    const int lane = threadIdx.x;
    float *tile = smem;
    float *gtab = smem + S::kTileFloats;
    float *rtab = gtab + S::kTabFloats;
    fill_tables<NMAX>(gtab, rtab);

    const uint32_t row = blockIdx.x * kShortBlock + threadIdx.x;
    const uint32_t r0 = row - lane;
    const bool valid = row < p.L.n_rows;
    const int n = FULL ? NMAX : p.L.n;
    const float lam = valid ? load_lambda(p.lam, p.L, row) : 0.f;
    const int64_t off = (!PACKED && valid) ? row_offset(p.L, row) : 0;

    float y[NMAX], xs[NMAX];
    if constexpr (PACKED) {
        TileRegs<NMAX> t;
        tile_fetch<NMAX>(p.y, r0, p.L.n_rows, lane, t);
        if (p.addend) {
            TileRegs<NMAX> a;
            tile_fetch<NMAX>(p.addend, r0, p.L.n_rows, lane, a);
            tile_add<NMAX>(t, a, 1.f);
        }
        tile_to_rows<NMAX>(t, tile, lane, y);
    } else {
        row_load_strided<NMAX, FULL>(p.y, p.addend, off, p.L.elem_stride, n, valid, y);
    }
    // park the row in LDS, sample-major
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < NMAX; ++k) tile[k * 64 + lane] = y[k];
    wave_lds_sync();

    const int info = pn_solve_row<NMAX, FULL>(tile + lane, xs, lam, n, valid, gtab, rtab);

    const bool want_resid = p.resid != nullptr;
    float rs[NMAX];
    if (want_resid) {
#pragma unroll
        for (int k = 0; k < NMAX; ++k) rs[k] = tile[k * 64 + lane] - xs[k];
    }
    if constexpr (PACKED) {
        TileRegs<NMAX> t;
        rows_to_tile<NMAX>(xs, tile, lane, t);
        tile_put<NMAX>(p.x, r0, p.L.n_rows, lane, t);
        if (want_resid) {
            rows_to_tile<NMAX>(rs, tile, lane, t);
            tile_put<NMAX>(p.resid, r0, p.L.n_rows, lane, t);
        }
    } else {
        row_store_strided<NMAX, FULL>(p.x, off, p.L.elem_stride, n, valid, xs);
        if (want_resid) row_store_strided<NMAX, FULL>(p.resid, off, p.L.elem_stride, n, valid, rs);
    }
    if (p.info && valid) p.info[row] = info;
}

// ---------------------------------------------------------------------------------
// Backward kernel (paper Eq. 5-6 as segment averaging): one row per lane.
//   segments = maximal runs of bit-equal neighbours in the forward output x;
//   grad_y   = per-segment mean of (g - sub), plus sub;
//   dL/dlam  = sum over jumps k of sign(x[k+1]-x[k]) * (mean_left - mean_right).
// ---------------------------------------------------------------------------------
template <int NMAX, bool FULL, bool PACKED, bool HAS_SUB>
__global__ __launch_bounds__(kShortBlock) void tv1d_bwd_short_kernel(BwdParams p)
{
    using S = ShortSmem<NMAX>;
    __shared__ float smem[S::kFloats];
    const int lane = threadIdx.x;
    float *tile = smem;
    float *gtab = smem + S::kTileFloats;
    float *rtab = gtab + S::kTabFloats;
    fill_tables<NMAX>(gtab, rtab);

    const uint32_t row = blockIdx.x * kShortBlock + threadIdx.x;
    const uint32_t r0 = row - lane;
    const bool valid = row < p.L.n_rows;
    const int n = FULL ? NMAX : p.L.n;
    const int64_t off = (!PACKED && valid) ? row_offset(p.L, row) : 0;

    float g[NMAX], x[NMAX];
    float sb[NMAX];                   // sub per row (strided path)
    TileRegs<NMAX> st;                // sub in tile order, kept until the store (packed path)
    if constexpr (PACKED) {
        TileRegs<NMAX> tg, tx;
        tile_fetch<NMAX>(p.g, r0, p.L.n_rows, lane, tg);
        tile_fetch<NMAX>(p.x, r0, p.L.n_rows, lane, tx);
        if constexpr (HAS_SUB) {
            tile_fetch<NMAX>(p.sub, r0, p.L.n_rows, lane, st);
            tile_add<NMAX>(tg, st, -1.f);
        }
        tile_to_rows<NMAX>(tg, tile, lane, g);
        tile_to_rows<NMAX>(tx, tile, lane, x);
    } else {
        row_load_strided<NMAX, FULL>(p.g, nullptr, off, p.L.elem_stride, n, valid, g);
        row_load_strided<NMAX, FULL>(p.x, nullptr, off, p.L.elem_stride, n, valid, x);
        if constexpr (HAS_SUB) {
            row_load_strided<NMAX, FULL>(p.sub, nullptr, off, p.L.elem_stride, n, valid, sb);
#pragma unroll
            for (int k = 0; k < NMAX; ++k) g[k] -= sb[k];
        }
        wave_lds_sync();                  // the tables are ready
    }

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
            const bool end = last || (k + 1 < NMAX && x[k + 1] != x[k]);
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
            const bool end = last || (k + 1 < NMAX && x[k + 1] != x[k]);
            carry = end ? g[k] : carry;
            g[k] = carry;
            if (k + 1 < NMAX && (FULL || k < n - 1)) {
                const float dx = x[k + 1] - x[k];
                glam = fmaf(copysignf(1.f, dx), carry - right, glam);
            }
        }
    }
    if constexpr (PACKED) {
        TileRegs<NMAX> t;
        rows_to_tile<NMAX>(g, tile, lane, t);
        if constexpr (HAS_SUB) tile_add<NMAX>(t, st, 1.f);
        tile_put<NMAX>(p.gy, r0, p.L.n_rows, lane, t);
    } else {
        if constexpr (HAS_SUB) {
#pragma unroll
            for (int k = 0; k < NMAX; ++k) g[k] += sb[k];
        }
        row_store_strided<NMAX, FULL>(p.gy, off, p.L.elem_stride, n, valid, g);
    }
    if (p.partial && valid) p.partial[row] = glam;
}

}  // namespace tvk
