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

constexpr int kShortBlock = 256;   // 4 waves of 64 rows

template <int NMAX>
struct ShortSmem {
    static constexpr int kPitch      = NMAX + 1;
    static constexpr int kTileFloats = 64 * kPitch;
    static constexpr int kTabFloats  = NMAX + 2;
    static constexpr int kFloats     = (kShortBlock / 64) * kTileFloats + 2 * kTabFloats;
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
// Tile movers.  A wave's 64 packed rows form one contiguous block of 64*NMAX floats.
// ---------------------------------------------------------------------------------
template <int NMAX>
__device__ __forceinline__ void tile_load_packed(const float *__restrict__ src,
                                                 const float *__restrict__ add, uint32_t r0,
                                                 uint32_t n_rows, float *tile, int lane,
                                                 float (&v)[NMAX])
{
    constexpr int P = NMAX + 1;
    const uint32_t valid_rows = r0 < n_rows ? min(64u, n_rows - r0) : 0u;
    const float4 *s4 = reinterpret_cast<const float4 *>(src + (size_t)r0 * NMAX);
    const float4 *a4 = reinterpret_cast<const float4 *>(add + (size_t)r0 * NMAX);
#pragma unroll
    for (int i = 0; i < NMAX / 4; ++i) {
        const int e4 = i * 64 + lane;
        const uint32_t row = (uint32_t)(e4 * 4) / NMAX;
        const int col = (e4 * 4) % NMAX;
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < valid_rows) {
            t = s4[e4];
            if (add) {
                const float4 q = a4[e4];
                t.x += q.x; t.y += q.y; t.z += q.z; t.w += q.w;
            }
        }
        float *d = tile + row * P + col;
        d[0] = t.x; d[1] = t.y; d[2] = t.z; d[3] = t.w;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < NMAX; ++k) v[k] = tile[lane * P + k];
    __syncthreads();
}

template <int NMAX>
__device__ __forceinline__ void tile_store_packed(float *__restrict__ dst, uint32_t r0,
                                                  uint32_t n_rows, float *tile, int lane,
                                                  const float (&v)[NMAX])
{
    constexpr int P = NMAX + 1;
    const uint32_t valid_rows = r0 < n_rows ? min(64u, n_rows - r0) : 0u;
#pragma unroll
    for (int k = 0; k < NMAX; ++k) tile[lane * P + k] = v[k];
    __syncthreads();
    float4 *d4 = reinterpret_cast<float4 *>(dst + (size_t)r0 * NMAX);
#pragma unroll
    for (int i = 0; i < NMAX / 4; ++i) {
        const int e4 = i * 64 + lane;
        const uint32_t row = (uint32_t)(e4 * 4) / NMAX;
        const int col = (e4 * 4) % NMAX;
        const float *s = tile + row * P + col;
        if (row < valid_rows) d4[e4] = make_float4(s[0], s[1], s[2], s[3]);
    }
    __syncthreads();
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
// Projected Newton on the dual of one row held in registers (paper Eq. 3-4).
//
//   dual (minimisation form): f(u) = 1/2 ||x(u)||^2 - 1/2 ||y||^2,  x(u) = y - D^T u,
//   |u_k| <= lam; gradient g_k = x_k - x_{k+1}; Hessian tridiag(-1, 2, -1).
//
// y[k] must be 0 for k >= n.  On return xs holds the minimiser of paper Eq. 1.
// ---------------------------------------------------------------------------------
template <int NMAX, bool FULL>
__device__ __forceinline__ int pn_solve_row(const float (&y)[NMAX], float (&xs)[NMAX], float lam,
                                            int n, bool valid, const float *gtab,
                                            const float *rtab)
{
    constexpr int M = NMAX - 1;
    const int m = n - 1;
    // duals past the end of a shorter row get an empty box and never move
#define TV_LK(k) ((FULL || (k) < m) ? lam : 0.0f)

    float u[M > 0 ? M : 1];
    float fcur;

    // ---- starting point: the better (lower dual objective) of two feasible candidates:
    //      A = one full Newton step from u = 0 with every dual free, clipped into the box
    //          (exact whenever lam >= lam_max);
    //      B = every dual at the bound its local difference points to (exact for small lam).
    {
        float sum = 0.f;
#pragma unroll
        for (int k = 0; k < NMAX; ++k) sum += y[k];
        const float ybar = sum * rtab[n];
        float uA[M > 0 ? M : 1], uB[M > 0 ? M : 1];
        float run = 0.f, fA = 0.f, fB = 0.f, pa = 0.f, pb = 0.f;
#pragma unroll
        for (int k = 0; k < M; ++k) {
            const float l = TV_LK(k);
            run += ybar - y[k];
            const float a = __builtin_amdgcn_fmed3f(run, -l, l);
            const float b = __builtin_amdgcn_fmed3f((y[k + 1] - y[k]) * 1e30f, -l, l);
            const float xa = y[k] + a - pa;
            const float xb = y[k] + b - pb;
            fA = fmaf(xa, xa, fA);
            fB = fmaf(xb, xb, fB);
            uA[k] = a; uB[k] = b; pa = a; pb = b;
        }
        {
            const float xa = y[M] - pa, xb = y[M] - pb;
            fA = fmaf(xa, xa, fA);
            fB = fmaf(xb, xb, fB);
        }
        const bool pickA = fA <= fB;
#pragma unroll
        for (int k = 0; k < M; ++k) u[k] = pickA ? uA[k] : uB[k];
        fcur = 0.5f * (pickA ? fA : fB);
    }

    bool active = valid;
    bool prev_unclipped = false;
    int steps = 0, flags = 0;
    float W[M > 0 ? M : 1], G[M > 0 ? M : 1];

    for (int it = 0;; ++it) {
        // ---- gradient, bound set (Bertsekas' sign test with exact comparisons: a clipped
        //      dual is bit-equal to +-lam), optimality test, Thomas forward elimination
        bool vio = false;
        float dec = 0.f, wprev = 0.f, gprev = 0.f;
        int pos = 0;
        float xk = y[0] + (M > 0 ? u[0] : 0.f);
#pragma unroll
        for (int k = 0; k < M; ++k) {
            const float un = (k + 1 < M) ? u[k + 1] : 0.f;
            const float xn = y[k + 1] + un - u[k];
            const float g = xk - xn;
            const float s = copysignf(TV_LK(k), g);
            const bool bnd = (u[k] == -s);          // at a bound and pushed outwards
            if (FULL || k < m) vio |= (u[k] == s) && (g != 0.f);  // at a bound, pushed inwards
            pos = bnd ? 0 : pos + 1;
            const float gam = gtab[pos];
            const float w = fmaf(gprev, wprev, g);
            dec = fmaf(gam * w, w, dec);            // accumulates g^T H_S^-1 g
            W[k] = w; G[k] = gam;
            wprev = w; gprev = gam; xk = xn;
        }
        // A full, unclipped Newton step zeroes the gradient on the free set; if no dual
        // sits on a bound with the gradient pointing inwards, the KKT conditions hold.
        if (active && prev_unclipped && !vio) { active = false; flags = kInfoConverged; }
        if (active && it >= kMaxNewtonSteps) { active = false; flags = kInfoCapped; }
        if (!__any(active)) break;
        steps += active ? 1 : 0;

        // ---- back substitution: W becomes the Newton direction d (0 on the bound set)
        {
            float dn = 0.f;
#pragma unroll
            for (int k = M - 1; k >= 0; --k) {
                dn = G[k] * (W[k] + dn);
                W[k] = dn;
            }
        }

        // ---- projected step u(alpha) = clip(u - alpha d); alpha = 1 is taken outright when
        //      nothing clips (it is the exact minimiser over the free subspace), otherwise
        //      Armijo with quadratic-interpolation backtracking (paper Sec. 3.2)
        float alpha = active ? 1.f : 0.f;
        float uc[M > 0 ? M : 1];
        float fc;
        bool clipped, changed;
        for (int ls = 0;; ++ls) {
            clipped = false; changed = false;
            float acc = 0.f, prev = 0.f;
#pragma unroll
            for (int k = 0; k < M; ++k) {
                const float l = TV_LK(k);
                const float t = fmaf(-alpha, W[k], u[k]);
                const float c = __builtin_amdgcn_fmed3f(t, -l, l);
                clipped |= (c != t);
                changed |= (c != u[k]);
                const float xc = y[k] + c - prev;
                acc = fmaf(xc, xc, acc);
                uc[k] = c; prev = c;
            }
            {
                const float xc = y[M] - prev;
                acc = fmaf(xc, xc, acc);
            }
            fc = 0.5f * acc;
            const bool ok = !active || alpha == 0.f || (alpha == 1.f && !clipped) ||
                            (fc <= fcur - kArmijoSigma * alpha * dec + kArmijoSlackEps * fabsf(fcur));
            if (__all(ok)) break;
            if (!ok) {
                if (ls >= kMaxBacktracks) {
                    alpha = 0.f;
                } else {
                    const float den = 2.f * (fc - fcur + dec * alpha);
                    float an = den > 0.f ? dec * alpha * alpha / den : 0.5f * alpha;
                    alpha = fminf(fmaxf(an, 0.1f * alpha), 0.5f * alpha);
                }
            }
        }
#pragma unroll
        for (int k = 0; k < M; ++k) u[k] = uc[k];
        prev_unclipped = (alpha == 1.f) && !clipped;
        if (active) fcur = fc;
        if (active && !changed) { active = false; flags = kInfoStalled; }
        if (!__any(active)) break;
    }

    // ---- primal recovery.  Plain form x = y - D^T u, and the segment form: on a block
    //      between two bound duals p < q,  x = (sum of y over the block + u_q - u_p) / size,
    //      which is bit-identical inside a block.  The segment form is kept when it agrees
    //      with the plain one (it always does at a KKT point).
    float V[NMAX];
    bool endk[NMAX];
    float dev = 0.f, ymax = 0.f;
    {
        float s = 0.f, up = 0.f;
        int c = 0;
        float xk = y[0] + (M > 0 ? u[0] : 0.f);
#pragma unroll
        for (int k = 0; k < NMAX; ++k) {
            s += y[k];
            c += 1;
            bool end = true;
            float ub = 0.f;
            if (k < M) {
                const float un = (k + 1 < M) ? u[k + 1] : 0.f;
                const float xn = y[k + 1] + un - u[k];
                const float g = xk - xn;
                end = (u[k] == -copysignf(TV_LK(k), g));
                ub = u[k];
                xs[k] = xk;          // plain form, replaced below
                xk = xn;
            } else {
                xs[k] = xk;
            }
            V[k] = (s + ub - up) * rtab[c];
            endk[k] = end;
            if (end) { s = 0.f; c = 0; up = ub; }
            ymax = fmaxf(ymax, fabsf(y[k]));
        }
        float carry = 0.f;
#pragma unroll
        for (int k = NMAX - 1; k >= 0; --k) {
            carry = endk[k] ? V[k] : carry;
            V[k] = carry;
            dev = fmaxf(dev, fabsf(carry - xs[k]));
        }
    }
    const bool use_segments = !(flags & kInfoCapped) && dev <= 2e-5f * (1.f + ymax + lam);
    if (use_segments) {
#pragma unroll
        for (int k = 0; k < NMAX; ++k) xs[k] = V[k];
    } else {
        flags |= 1 << 19;
    }
#undef TV_LK
    return steps | flags;
}

// ---------------------------------------------------------------------------------
// Forward kernel: one row per lane.
// ---------------------------------------------------------------------------------
template <int NMAX, bool FULL, bool PACKED>
__global__ __launch_bounds__(kShortBlock) void tv1d_fwd_short_kernel(FwdParams p)
{
    using S = ShortSmem<NMAX>;
    __shared__ float smem[S::kFloats];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float *tile = smem + wave * S::kTileFloats;
    float *gtab = smem + (kShortBlock / 64) * S::kTileFloats;
    float *rtab = gtab + S::kTabFloats;
    fill_tables<NMAX>(gtab, rtab);

    const uint32_t row = blockIdx.x * kShortBlock + threadIdx.x;
    const uint32_t r0 = row - lane;
    const bool valid = row < p.L.n_rows;
    const int n = FULL ? NMAX : p.L.n;
    const float lam = valid ? load_lambda(p.lam, p.L, row) : 0.f;
    const int64_t off = (!PACKED && valid) ? row_offset(p.L, row) : 0;

    float y[NMAX], xs[NMAX];
    if (PACKED) {
        tile_load_packed<NMAX>(p.y, p.addend, r0, p.L.n_rows, tile, lane, y);   // syncs: tables ready
    } else {
        row_load_strided<NMAX, FULL>(p.y, p.addend, off, p.L.elem_stride, n, valid, y);
        __syncthreads();
    }

    const int info = pn_solve_row<NMAX, FULL>(y, xs, lam, n, valid, gtab, rtab);

    if (PACKED) {
        tile_store_packed<NMAX>(p.x, r0, p.L.n_rows, tile, lane, xs);
        if (p.resid) {
#pragma unroll
            for (int k = 0; k < NMAX; ++k) xs[k] = y[k] - xs[k];
            tile_store_packed<NMAX>(p.resid, r0, p.L.n_rows, tile, lane, xs);
        }
    } else {
        row_store_strided<NMAX, FULL>(p.x, off, p.L.elem_stride, n, valid, xs);
        if (p.resid) {
#pragma unroll
            for (int k = 0; k < NMAX; ++k) xs[k] = y[k] - xs[k];
            row_store_strided<NMAX, FULL>(p.resid, off, p.L.elem_stride, n, valid, xs);
        }
    }
    if (p.info && valid) p.info[row] = info;
}

// ---------------------------------------------------------------------------------
// Backward kernel (paper Eq. 5-6 as segment averaging): one row per lane.
//   segments = maximal runs of bit-equal neighbours in the forward output x;
//   grad_y   = per-segment mean of (g - sub), plus sub;
//   dL/dlam  = sum over jumps k of sign(x[k+1]-x[k]) * (mean_left - mean_right).
// ---------------------------------------------------------------------------------
template <int NMAX, bool FULL, bool PACKED>
__global__ __launch_bounds__(kShortBlock) void tv1d_bwd_short_kernel(BwdParams p)
{
    using S = ShortSmem<NMAX>;
    __shared__ float smem[S::kFloats];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float *tile = smem + wave * S::kTileFloats;
    float *gtab = smem + (kShortBlock / 64) * S::kTileFloats;
    float *rtab = gtab + S::kTabFloats;
    fill_tables<NMAX>(gtab, rtab);

    const uint32_t row = blockIdx.x * kShortBlock + threadIdx.x;
    const uint32_t r0 = row - lane;
    const bool valid = row < p.L.n_rows;
    const int n = FULL ? NMAX : p.L.n;
    const int64_t off = (!PACKED && valid) ? row_offset(p.L, row) : 0;

    float g[NMAX], x[NMAX], sb[NMAX];
    if (PACKED) {
        tile_load_packed<NMAX>(p.g, nullptr, r0, p.L.n_rows, tile, lane, g);
        tile_load_packed<NMAX>(p.x, nullptr, r0, p.L.n_rows, tile, lane, x);
        if (p.sub) tile_load_packed<NMAX>(p.sub, nullptr, r0, p.L.n_rows, tile, lane, sb);
    } else {
        row_load_strided<NMAX, FULL>(p.g, nullptr, off, p.L.elem_stride, n, valid, g);
        row_load_strided<NMAX, FULL>(p.x, nullptr, off, p.L.elem_stride, n, valid, x);
        if (p.sub) row_load_strided<NMAX, FULL>(p.sub, nullptr, off, p.L.elem_stride, n, valid, sb);
        __syncthreads();
    }
    if (p.sub) {
#pragma unroll
        for (int k = 0; k < NMAX; ++k) g[k] -= sb[k];
    }

    // forward sweep: segment sums; a segment ends at k when x jumps after k (or the row ends)
    float V[NMAX];
    bool endk[NMAX];
    {
        float s = 0.f;
        int c = 0;
#pragma unroll
        for (int k = 0; k < NMAX; ++k) {
            s += g[k];
            c += 1;
            const bool last = FULL ? (k == NMAX - 1) : (k >= n - 1);
            const bool end = last || (k + 1 < NMAX && x[k + 1] != x[k]);
            V[k] = s * rtab[c];
            endk[k] = end;
            if (end) { s = 0.f; c = 0; }
        }
    }
    // backward sweep: broadcast each segment's mean; accumulate dL/dlam at the jumps
    float glam = 0.f;
    {
        float carry = 0.f;
#pragma unroll
        for (int k = NMAX - 1; k >= 0; --k) {
            const float right = carry;                // mean of the segment to the right
            carry = endk[k] ? V[k] : carry;
            V[k] = carry;
            if (k + 1 < NMAX && (FULL || k < n - 1)) {
                const float dx = x[k + 1] - x[k];
                const float sg = (dx > 0.f) ? 1.f : ((dx < 0.f) ? -1.f : 0.f);
                glam = fmaf(sg, carry - right, glam);
            }
        }
    }
    if (p.sub) {
#pragma unroll
        for (int k = 0; k < NMAX; ++k) V[k] += sb[k];
    }
    if (PACKED) {
        tile_store_packed<NMAX>(p.gy, r0, p.L.n_rows, tile, lane, V);
    } else {
        row_store_strided<NMAX, FULL>(p.gy, off, p.L.elem_stride, n, valid, V);
    }
    if (p.partial && valid) p.partial[row] = glam;
}

}  // namespace tvk
