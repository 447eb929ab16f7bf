// The 2D operator (paper Alg. 1) and its reverse sweep (Sec. 3.2) for small batches of planes of
// at most 64 x 64: one plane per workgroup, resident in LDS for all 2K passes of a call, each row
// (or column) of a pass handled by T neighbouring lanes with C samples each.  Forward kernel
// first, reverse sweep at the end of the file.
//
// With a few hundred planes the row-per-lane kernels of tv_small2d.hpp fill a fraction of the
// chip with long dependent chains (one wave per one or two planes), and the pass-by-pass route
// pays a launch and a trip through memory per pass for a few microseconds of arithmetic.  Here a
// workgroup of 512 threads holds the plane; the row and the column view read the same tile of
// odd pitch, a thread touches the same tile elements going in and coming out of a pass, so one
// barrier per pass is all the synchronisation there is, and the correction terms of paper Alg. 1
// (P for the rows, Q for the columns) never leave the registers of the threads that own them.
//
// The solve is the method of tv_long.hpp (chunk-local Thomas recurrences with table pivots, the
// chunks' last duals as separators, a cyclic reduction of the separator system, Armijo
// backtracking on the projected step) restricted to rows inside one 16-lane DPP row: every
// exchange between the threads of a row is a row shift or a butterfly inside the wave, and
// nothing but the pivot tables is read from LDS during a solve.
#pragma once
#include "tv_long.hpp"
#include "tv_small2d.hpp"

namespace tvk {

// OR over the T <= 16 lanes of a row (rows are aligned groups of T lanes), the result in all of them.
template <int T>
__device__ __forceinline__ uint32_t row_or_all(uint32_t v)
{
    static_assert(T == 8 || T == 16, "butterflies inside a 16-lane DPP row");
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, true);     // quad_perm [1,0,3,2]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, true);     // quad_perm [2,3,0,1]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, true);    // mirror within 8
    if (T > 8) v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xf, 0xf, true);   // within 16
    return v;
}

// Does any of the T lanes of this lane's row pass `pred`?  (A wave-wide ballot, of which every
// lane looks at its own row's bits.)
template <int T>
__device__ __forceinline__ bool row_any(bool pred)
{
    const uint64_t b = __ballot(pred ? 1 : 0);
    const int first = (int)(threadIdx.x & 63u & ~(uint32_t)(T - 1));
    return ((uint32_t)(b >> first) & ((1u << T) - 1u)) != 0u;
}

// Maximum over the T lanes of a row, the result in all of them.
template <int T>
__device__ __forceinline__ float row_max_all(float v)
{
    static_assert(T == 8 || T == 16, "butterflies inside a 16-lane DPP row");
    v = fmaxf(v, long_dpp<0xB1>(v));
    v = fmaxf(v, long_dpp<0x4E>(v));
    v = fmaxf(v, long_dpp<0x141>(v));
    if (T > 8) v = fmaxf(v, long_dpp<0x140>(v));
    return v;
}

// Sum of v over the threads of the row before this one (0 for the first), by row shifts.
template <int T>
__device__ __forceinline__ float row_sum_before(float v, int t)
{
    v += from_left<T, 1>(v, t);
    v += from_left<T, 2>(v, t);
    v += from_left<T, 4>(v, t);
    if constexpr (T > 8) v += from_left<T, 8>(v, t);
    return from_left<T, 1>(v, t);
}

// The value s of the nearest thread before this one in the row that has `closed` set (thread 0
// of a row must have it set; its own result is unused).
template <int T>
__device__ __forceinline__ float row_copy_before(bool closed, float s, int t)
{
    float f = closed ? 1.f : 0.f;
#define TV_STEP(D)                                                              \
    if constexpr ((D) < T) {                                                    \
        const float of = from_left<T, (D) < T ? (D) : 1>(f, t), os = from_left<T, (D) < T ? (D) : 1>(s, t); \
        if (t >= (D) && f == 0.f) { s = os; f = of; }                           \
    }
    TV_STEP(1) TV_STEP(2) TV_STEP(4) TV_STEP(8)
#undef TV_STEP
    return from_left<T, 1>(s, t);
}

// One row solved by the T lanes that hold it (paper Eq. 3-4).  y: the thread's chunk of the
// row (zero past the end, n samples in the row).  WARM: u holds the negated running sums of the
// chunk's part of D^T u0 for a starting dual u0, wsum the last of them (the chunks before are
// added here).  Every lane of the wave must call, rows that do not exist with valid = false.
// Returns the step count and flags of FwdParams::info; xs is the chunk of the minimiser.
template <int T, int C, bool WARM>
__device__ __forceinline__ int lanes_row_solve(const float (&y)[C], float (&u)[C], float wsum, float lam, int n,
                                               int t, bool valid, const float *gtab, const float *rtab,
                                               float (&xs)[C])
{
    static_assert(T <= 16, "the row must lie inside one 16-lane DPP row");
    const int k0 = t * C;
    // rounding floor of a difference of two x values (|x| <= max|y|, |u| <= lam)
    float gtol;
    {
        float ym = 0.f;
#pragma unroll
        for (int i = 0; i < C; ++i) ym = fmaxf(ym, fabsf(y[i]));
        ym = row_max_all<T>(ym);
        // every lambda from lam_max <= n / 2 max|y| on gives the row's mean; the cold start puts
        // the duals on the bounds, so the box is kept at the scale of the data
        if constexpr (!WARM) lam = fminf(lam, 0.51f * (float)n * ym);
        gtol = kGradNoise * (ym + lam);
    }
    // duals past the end of the row get an empty box and never move
    const int nv = min(max(n - 1 - k0, 0), C);
#define TV_LK(i) (((i) < nv) ? lam : 0.0f)
    const float ynext0 = from_right<T, 1>(y[0], t);
    float hd[C];                   // half the local differences of y (the Gauss-Seidel polish)
#pragma unroll
    for (int i = 0; i < C; ++i) hd[i] = 0.5f * (((i + 1 < C) ? y[i + 1] : ynext0) - y[i]);

    // ---- starting point: every dual at the bound its local difference points to, or the given
    //      dual brought into the box (duals within rounding distance of a bound onto it)
    float fcur, edge_l, edge_r;
    {
        if constexpr (WARM) {
            const float before = row_sum_before<T>(wsum, t);
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
        }
        edge_l = from_left<T, 1>(u[C - 1], t);
        edge_r = from_right<T, 1>(u[0], t);
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < C; ++i) {
            const float xi = y[i] + u[i] - (i > 0 ? u[i - 1] : edge_l);
            acc = fmaf(xi, xi, acc);
        }
        fcur = 0.5f * wave_sum_all<T>(acc);
    }

    bool active = valid;
    bool prev_unclipped = false;
    int steps = 0, flags = 0;

    for (int it = 0;; ++it) {
        const float uleft = edge_l, unext0 = edge_r;

        // ---- gradient, bound set, optimality test, interior elimination (Thomas, pass 1)
        float g[C], gam[C > 1 ? C - 1 : 1], w[C];
        bool bsep = false;
        int pos = 0, a = 0;
        bool seen_bound = false;
        float viof = 0.f;
        {
            float wprev = 0.f, gprev = 0.f;
            float xi = y[0] + u[0] - uleft;
#pragma unroll
            for (int i = 0; i < C; ++i) {
                const float xn = (i + 1 < C) ? (y[i + 1] + u[i + 1] - u[i]) : (ynext0 + unext0 - u[C - 1]);
                const float gi = xi - xn;
                g[i] = gi;
                const float s = copysignf(TV_LK(i), gi);
                const bool bnd = (u[i] == -s);
                if (i < nv && u[i] == s && fabsf(gi) > gtol) viof += 1.f;
                if (i < C - 1) {
                    pos = bnd ? 0 : pos + 1;
                    // (two samples per thread: the one interior dual is bound or a free run of one,
                    // and a select keeps the table's LDS latency off the critical path)
                    const float gm = C == 2 ? (pos == 0 ? 0.f : 0.5f) : gtab[pos];
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
        float p0 = 0.f, pl = 0.f;
#pragma unroll
        for (int i = C - 2; i >= 0; --i) {
            p0 = gam[i] * (w[i] + p0);
            if (i == C - 2) pl = p0;
        }
        // separator diagonal 2 - (A^-1)_{last,last} of this chunk's interior block -
        // (A^-1)_{first,first} of the next one's, carried as 1 - a / (a + 1) = 1 / (a + 1)
        const float c_alpha = C == 2 ? (a == 0 ? 1.f : 0.5f) : rtab[a];
        const float c_delta = C == 2 ? (pos == 0 ? 1.f : 0.5f) : rtab[pos];
        const float c_beta = (a == C - 1) ? (1.0f / (float)C) : 0.f;
        const bool vio = row_any<T>(viof != 0.f);
        const float p0n = from_right<T, 1>(p0, t), alphan = from_right<T, 1>(c_alpha, t),
                    betan = from_right<T, 1>(c_beta, t);

        if (active && prev_unclipped && !vio) { active = false; flags = kInfoConverged; }
        if (active && it >= kMaxNewtonSteps) { active = false; flags = kInfoCapped; }
        if (!__any(active ? 1 : 0)) break;

        // ---- separator system (normalised to unit diagonal), cyclic reduction by row shifts
        float ea = 0.f, ec = 0.f, er = 0.f;
        if (!bsep) {
            const float inv = __builtin_amdgcn_rcpf(c_delta + alphan);
            ea = -c_beta * inv;
            ec = -betan * inv;
            er = (g[C - 1] + pl + p0n) * inv;
        }
        // (every step is taken: with the row in one wave a vote on "all decoupled" costs as much
        // as the step it would save)
#define TV_PCR_STEP(S)                                                                                  \
        if constexpr ((S) < T) {                                                                        \
            constexpr int SS = (S) < T ? (S) : 1;                                                       \
            const float la = from_left<T, SS>(ea, t), lc = from_left<T, SS>(ec, t),                     \
                        lr = from_left<T, SS>(er, t);                                                   \
            const float ra = from_right<T, SS>(ea, t), rc = from_right<T, SS>(ec, t),                   \
                        rr = from_right<T, SS>(er, t);                                                  \
            const float inv = __builtin_amdgcn_rcpf(1.0f - ea * lc - ec * ra);                          \
            er = (er - ea * lr - ec * rr) * inv;                                                        \
            const float na = -ea * la * inv, nc = -ec * rc * inv;                                       \
            ea = na; ec = nc;                                                                           \
        }
        TV_PCR_STEP(1) TV_PCR_STEP(2) TV_PCR_STEP(4) TV_PCR_STEP(8)
#undef TV_PCR_STEP
        const float sleft = from_left<T, 1>(er, t);
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

        // ---- projected step with Armijo backtracking (quadratic interpolation)
        const float dec = wave_sum_all<T>(decp);
        // Newton decrement g^T d = |D^T d|^2, the squared length of the move of x that the step
        // about to be tried would make: once no sample would move by more than the rounding
        // floor of a difference of two x values, and no bound dual wants to leave its bound,
        // the row is done (without this a polished point and the Newton step from it can swap
        // a last ulp for ever)
        if (active && !vio && dec <= gtol * gtol) { active = false; flags = kInfoConverged; }
        if (!__any(active ? 1 : 0)) break;
        steps += active ? 1 : 0;
        float alpha = active ? 1.f : 0.f;
        float uc[C];
        float fc = 0.f;
        bool clipped = false, changed = false;
        for (int ls = 0;; ++ls) {
            bool cl = false, ch = false;
#pragma unroll
            for (int i = 0; i < C; ++i) {
                const float l = TV_LK(i);
                const float tt = fmaf(-alpha, w[i], u[i]);
                const float cc = __builtin_amdgcn_fmed3f(tt, -l, l);
                cl |= (cc != tt);
                uc[i] = cc;
            }
            float ucleft = from_left<T, 1>(uc[C - 1], t);
            float ucright = from_right<T, 1>(uc[0], t);
            clipped = row_any<T>(cl);
            // A clipped trial point is polished by two Gauss-Seidel sweeps (exact minimisation
            // of the dual objective over one dual at a time, inside the box), each thread over
            // its own chunk with its neighbours' trial values held: the duals that the clip
            // stopped at a bound let go of the ones next to them, which Newton's direction for
            // the old bound set could not know.  The result goes through the Armijo test like
            // any clipped step.  (CPU prototype, 32 x 32 feature maps: 14 % fewer trips of the
            // slowest row of a pass, and hardly any backtracking.)
            if (__any((clipped && active) ? 1 : 0)) {
                if (clipped && active) {                // (in place: no lane of another row takes part)
#pragma unroll
                    for (int i = 0; i < C; ++i) {
                        const float l = TV_LK(i);
                        const float nb = (i > 0 ? uc[i - 1] : ucleft) + (i + 1 < C ? uc[i + 1] : ucright);
                        uc[i] = __builtin_amdgcn_fmed3f(fmaf(0.5f, nb, hd[i]), -l, l);
                    }
#pragma unroll
                    for (int i = C - 1; i >= 0; --i) {
                        const float l = TV_LK(i);
                        const float nb = (i > 0 ? uc[i - 1] : ucleft) + (i + 1 < C ? uc[i + 1] : ucright);
                        uc[i] = __builtin_amdgcn_fmed3f(fmaf(0.5f, nb, hd[i]), -l, l);
                    }
                }
                ucleft = from_left<T, 1>(uc[C - 1], t);
                ucright = from_right<T, 1>(uc[0], t);
            }
            edge_l = ucleft;
            edge_r = ucright;
            float v0 = 0.f;
#pragma unroll
            for (int i = 0; i < C; ++i) {
                ch |= (uc[i] != u[i]);
                const float xc = y[i] + uc[i] - (i > 0 ? uc[i - 1] : ucleft);
                v0 = fmaf(xc, xc, v0);
            }
            fc = 0.5f * wave_sum_all<T>(v0);
            changed = row_any<T>(ch);
            const bool ok = !active || alpha == 0.f || (alpha == 1.f && !clipped) ||
                            (fc <= fcur - kArmijoSigma * alpha * dec + kArmijoSlackEps * fabsf(fcur));
            if (!__any(ok ? 0 : 1)) break;
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
        if (active) fcur = fc;
        if (active && !changed) { active = false; flags = kInfoStalled; }
        if (!__any(active ? 1 : 0)) break;
    }

    // ---- primal recovery x = y - D^T u, then every block between two bound duals takes the
    //      value of its first sample, so that constant runs are bit-identical
    {
        const float uleft = from_left<T, 1>(u[C - 1], t);
        const float unext0 = from_right<T, 1>(u[0], t);
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
        // (the shift is fetched by all lanes before any of them branches)
        const float left_bound = from_left<T, 1>(bnd[C - 1] ? 1.f : 0.f, t);
        const bool start0 = (t == 0) || (left_bound != 0.f);
        bool closed = start0;
        float last = xs[0];
#pragma unroll
        for (int i = 1; i < C; ++i)
            if (bnd[i - 1]) { closed = true; last = xs[i]; }
        const float cv = row_copy_before<T>(closed, last, t);
        float val = start0 ? xs[0] : cv;
        float dev = 0.f;
        float blk[C];
#pragma unroll
        for (int i = 0; i < C; ++i) {
            if (i > 0 && bnd[i - 1]) val = xs[i];
            // (a row that stopped on its Newton decrement has every sample within gtol of where
            // the next step would put it, whatever the size of the samples next to it)
            // (a NaN counts as a deviation: the sweeps of the polish do not carry a NaN of y into
            // the dual, and the row's output must still show it)
            if (!(fabsf(val - xs[i]) <= fmaxf(2e-5f * (1.f + fabsf(y[i]) + lam), 4.f * gtol))) dev += 1.f;
            blk[i] = val;
        }
        dev = wave_sum_all<T>(dev);
        // (an infinite sample makes the floor infinite: such a row keeps its plain output, which shows it)
        if (!(flags & kInfoCapped) && dev == 0.f && gtol <= 3.0e38f) {
#pragma unroll
            for (int i = 0; i < C; ++i) xs[i] = blk[i];
        } else {
            flags |= kInfoPlain;
        }
    }
#undef TV_LK
    return steps | flags;
}

// T threads per row, C samples per thread: planes of at most S x S, S = T * C (16 x 2: up to
// 32 x 32, with segment codes for the reverse sweep; 8 x 8: up to 64 x 64, whose reverse sweep
// reads the saved pass outputs).  One plane per workgroup of S * T = 512 threads.
// (32 x 32 with 8 threads x 4 samples, 256 threads: 256 planes, K = 4, 52 us against 38 with
// 16 x 2, whose chains are shorter; from 1500 planes on 8 x 4 is 5-10 % ahead, where the
// row-per-lane kernels take over anyway.)
// IO16: y and x are bf16 in memory (fp32 in the tile and in all arithmetic; the saved pass outputs
// stay fp32).
template <int T, int C, bool IO16 = false>
__global__ __launch_bounds__(T * T * C, C <= 4 ? 8 : 4) void tv2d_fwd_plane_kernel(Small2dFwdParams p)
{
    constexpr int S = T * C, P = S + 1, NT = S * T;
    static_assert(NT % 64 == 0 && NT <= 1024, "whole waves");
    __shared__ float X[S * P], gtab[C + 2], rtab[C + 2];
    const int tid = threadIdx.x;
    const int j = tid / T, t = tid % T, k0 = t * C;
    const int H = p.H, W = p.W, HW = H * W;
    const int64_t plane = blockIdx.x;
    if (tid <= C) {
        gtab[tid] = (float)tid / (float)(tid + 1);
        rtab[tid] = 1.0f / (float)(tid + 1);
    }
    const float lam = fmaxf(p.lam[plane % p.lam_count], 0.f);
    if constexpr (IO16) {
        const uint16_t *src = reinterpret_cast<const uint16_t *>(p.y) + plane * HW;
        for (int e = tid; e < HW; e += NT) X[(e / W) * P + e % W] = bf16_bits_to_f32(src[e]);
    } else {
        const float *src = p.y + plane * HW;
        for (int e = tid; e < HW; e += NT) X[(e / W) * P + e % W] = src[e];
    }
    __syncthreads();
    auto put_plane = [&](float *dst) {
        for (int e = tid; e < HW; e += NT) dst[e] = X[(e / W) * P + e % W];
    };

    // the correction terms of the thread's row chunk and of its column chunk (paper Alg. 1)
    float corr_r[C], corr_c[C];
    const int n_pass = 2 * p.sweeps;
    for (int i = 0; i < n_pass; ++i) {
        const bool col = (i & 1) != 0;
        const int n = col ? H : W, rows = col ? W : H;
        const bool valid = j < rows;
        // sample k of the thread's row: X[j][k] in a row pass, X[k][j] in a column pass
        const int base = col ? j : j * P, step = col ? P : 1;
        float y[C], u[C], xs[C];
#pragma unroll
        for (int c = 0; c < C; ++c) {
            y[c] = (valid && k0 + c < n) ? X[base + (k0 + c) * step] : 0.f;
            u[c] = 0.f;
        }
        int info;
        if (i < 2) {
            info = lanes_row_solve<T, C, false>(y, u, 0.f, lam, n, t, valid, gtab, rtab, xs);
        } else {
            // input = the other direction's output plus this direction's correction term, which
            // is D^T u of this direction's pass one sweep earlier: start from that dual
            float wsum = 0.f;
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const float cr = col ? corr_c[c] : corr_r[c];
                y[c] += cr;
                wsum -= cr;
                u[c] = wsum;
            }
            info = lanes_row_solve<T, C, true>(y, u, wsum, lam, n, t, valid, gtab, rtab, xs);
        }
        (void)info;
        if (i + 2 < n_pass) {
#pragma unroll
            for (int c = 0; c < C; ++c) {
                if (col) corr_c[c] = y[c] - xs[c];
                else corr_r[c] = y[c] - xs[c];
            }
        }
#pragma unroll
        for (int c = 0; c < C; ++c)
            if (valid && k0 + c < n) X[base + (k0 + c) * step] = xs[c];

        if constexpr (S <= 32) {
            // segment code of the row: bit k = x jumps behind sample k / rises there
            const float xnext0 = from_right<T, 1>(xs[0], t);
            uint32_t jm = 0, up = 0;
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const float d = xs[c] - ((c + 1 < C) ? xs[c + 1] : xnext0);
                if (k0 + c < n - 1) {
                    if (d != 0.f) jm |= 1u << (k0 + c);
                    if (d < 0.f) up |= 1u << (k0 + c);
                }
            }
            jm = row_or_all<T>(jm);
            up = row_or_all<T>(up);
            if (valid && t == 0)
                p.codes[(size_t)i * p.code_stride + (size_t)plane * rows + j] = make_uint2(jm, up);
        }
        __syncthreads();
        // (planes of at most 32 x 32: the reverse sweep reads the codes written above)
        if (S > 32 || p.keep_passes) {
            put_plane(p.saved + (size_t)i * p.saved_stride + plane * HW);
            if (i + 1 < n_pass) __syncthreads();      // the next pass writes into the tile
        }
    }
    if constexpr (IO16) {
        uint16_t *dst = reinterpret_cast<uint16_t *>(p.x) + plane * HW;
        for (int e = tid; e < HW; e += NT) dst[e] = f32_to_bf16_bits(X[(e / W) * P + e % W]);
    } else {
        put_plane(p.x + plane * HW);
    }
}

// ---------------------------------------------------------------------------------
// Reverse sweep through paper Alg. 1 (Sec. 3.2) for small batches: one plane per workgroup, the
// two adjoint state tensors resident in LDS for all 2K passes, T threads x C samples per row.
// ---------------------------------------------------------------------------------

// Segmented exclusive sums over the T threads of a row, from thread 0 upwards (DIR = +1) or from
// thread T - 1 downwards (DIR = -1), by row shifts: each thread contributes (closed, s, n) as in
// seg_scan of tv_long.hpp (closed: its chunk holds a segment boundary; (s, n): sum and count of
// the part of its chunk beyond the last boundary in scan direction) and gets the sum and count
// of the open part that arrives at it (zero at the origin).
template <int T, int DIR>
__device__ __forceinline__ void row_open_part_before(bool closed, float s, float n, int t, float &cs, float &cn)
{
    float f = closed ? 1.f : 0.f;
#define TV_STEP(D)                                                                                  \
    if constexpr ((D) < T) {                                                                        \
        constexpr int DD = (D) < T ? (D) : 1;                                                       \
        const float of = DIR > 0 ? from_left<T, DD>(f, t) : from_right<T, DD>(f, t);                \
        const float os = DIR > 0 ? from_left<T, DD>(s, t) : from_right<T, DD>(s, t);                \
        const float on = DIR > 0 ? from_left<T, DD>(n, t) : from_right<T, DD>(n, t);                \
        const bool has = DIR > 0 ? (t >= (D)) : (t + (D) < T);                                      \
        if (has && f == 0.f) { s += os; n += on; f = of; }                                          \
    }
    TV_STEP(1) TV_STEP(2) TV_STEP(4) TV_STEP(8)
#undef TV_STEP
    cs = DIR > 0 ? from_left<T, 1>(s, t) : from_right<T, 1>(s, t);
    cn = DIR > 0 ? from_left<T, 1>(n, t) : from_right<T, 1>(n, t);
}

// Segment means of one row held by T threads (paper Eq. 5-6 as segment averaging): g is the
// thread's chunk of the averaged quantity on entry (zero past the end of the row) and of the
// means on return.  Bit i of jm: the row's output jumps behind sample k0 + i; of up: it rises
// there (only duals inside the row are looked at).  Returns the thread's part of the row's
// dL/dlam term  sum over jumps of sign(x[k+1] - x[k]) (mean_left - mean_right).
template <int T, int C>
__device__ __forceinline__ float lanes_segment_means(float (&g)[C], uint32_t jm, uint32_t up, int n, int t)
{
    const int k0 = t * C;
    const int nv = min(max(n - 1 - k0, 0), C);             // duals of this chunk inside the row
    const uint32_t inrow = (1u << nv) - 1u;
    const uint32_t gmask = jm & inrow;                      // jumps that count for dL/dlam
    // the end of the row closes a segment, and samples past it are segments of their own
    const uint32_t jmask = (jm & inrow) | ~inrow;
#define TV_JUMP(i) ((jmask >> (i)) & 1u)
    bool any = false;
    float head_s = 0.f, head_n = 0.f, tail_s = 0.f, tail_n = 0.f;
#pragma unroll
    for (int i = 0; i < C; ++i) {
        if (!any) { head_s += g[i]; head_n += 1.f; }
        tail_s += g[i]; tail_n += 1.f;
        if (TV_JUMP(i)) { any = true; tail_s = 0.f; tail_n = 0.f; }
    }
    float ls, ln, rs, rn;
    row_open_part_before<T, +1>(any, tail_s, tail_n, t, ls, ln);       // open part on the left
    row_open_part_before<T, -1>(any, head_s, head_n, t, rs, rn);       // open part on the right
    {
        float s = ls, c = ln;
#pragma unroll
        for (int i = 0; i < C; ++i) {
            s += g[i]; c += 1.f;
            g[i] = 0.f;
            if (TV_JUMP(i)) { g[i] = s * __builtin_amdgcn_rcpf(c); s = 0.f; c = 0.f; }
        }
        // the trailing open part continues into the next chunks
        float carry = (c > 0.f) ? (s + rs) * __builtin_amdgcn_rcpf(c + rn) : 0.f;
#pragma unroll
        for (int i = C - 1; i >= 0; --i) {
            if (TV_JUMP(i)) carry = g[i];
            g[i] = carry;
        }
    }
#undef TV_JUMP
    const float mnext0 = from_right<T, 1>(g[0], t);
    float gl = 0.f;
#pragma unroll
    for (int i = 0; i < C; ++i) {
        if ((gmask >> i) & 1u) {
            const float mn = (i + 1 < C) ? g[i + 1] : mnext0;
            const float d = g[i] - mn;
            gl += ((up >> i) & 1u) ? d : -d;
        }
    }
    return gl;
}

// T, C as in the forward kernel.  Planes of at most 32 x 32 read the segments of a pass from its
// 8-byte codes, larger ones from its saved output.  p.partial gets one dL/dlam term per plane.
// IO16: the upstream gradient and grad_y are bf16 in memory.
template <int T, int C, bool IO16 = false>
__global__ __launch_bounds__(T * T * C, C <= 4 ? 8 : 4) void tv2d_bwd_plane_kernel(Small2dBwdParams p)
{
    constexpr int S = T * C, P = S + 1, NT = S * T, NW = NT / 64;
    static_assert(NT % 64 == 0 && NT <= 1024, "whole waves");
    __shared__ float A[S * P], B[S * P], part[NW];
    const int tid = threadIdx.x;
    const int j = tid / T, t = tid % T, k0 = t * C;
    const int H = p.H, W = p.W, HW = H * W;
    const int64_t plane = blockIdx.x;
    if constexpr (IO16) {
        const uint16_t *src = reinterpret_cast<const uint16_t *>(p.g_up) + plane * HW;
        for (int e = tid; e < HW; e += NT) A[(e / W) * P + e % W] = bf16_bits_to_f32(src[e]);
    } else {
        const float *src = p.g_up + plane * HW;
        for (int e = tid; e < HW; e += NT) A[(e / W) * P + e % W] = src[e];
    }

    // Segments of pass `pass` for the thread's chunk of its row (row pass) or column (column
    // pass); fetched one pass ahead, so that the latency hides behind the pass before.
    auto fetch = [&](int pass, uint32_t &jm, uint32_t &up) {
        jm = 0u; up = 0u;
        if (pass < 0) return;
        const bool col = (pass & 1) != 0;
        const int n = col ? H : W, rows = col ? W : H;
        const bool valid = j < rows;
        if constexpr (S <= 32) {
            if (valid) {
                const uint2 c = p.codes[(size_t)pass * p.code_stride + (size_t)plane * rows + j];
                jm = (c.x >> k0) & ((1u << C) - 1u);
                up = (c.y >> k0) & ((1u << C) - 1u);
            }
        } else {
            const float *xs = p.saved + (size_t)pass * p.saved_stride + (size_t)plane * HW;
            float x[C];
#pragma unroll
            for (int c = 0; c < C; ++c)
                x[c] = (valid && k0 + c < n) ? (col ? xs[(k0 + c) * W + j] : xs[j * W + k0 + c]) : 0.f;
            const float xnext0 = from_right<T, 1>(x[0], t);
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const float xn = (c + 1 < C) ? x[c + 1] : xnext0;
                if (xn != x[c]) jm |= 1u << c;
                if (xn > x[c]) up |= 1u << c;
            }
        }
    };

    float glam = 0.f;
    uint32_t jm_next, up_next;
    fetch(2 * p.sweeps - 1, jm_next, up_next);
    __syncthreads();
    // Adjoint of one sweep (A = Y + P, Z = R(A), P' = A - Z, B = Z + Q, Y' = C(B), Q' = B - Y'):
    //   Bbar = Qbar' + C^T(Ybar' - Qbar'),   Abar = Pbar' + R^T(Bbar - Pbar'),   Ybar = Pbar = Abar;
    // tile A carries Ybar = Pbar, tile B carries Qbar = Bbar.  A thread reads and writes only its
    // own tile elements in a pass, so one barrier per pass suffices.
    for (int k = p.sweeps - 1; k >= 0; --k) {
        const bool first = (k == p.sweeps - 1);
#pragma unroll
        for (int dir = 1; dir >= 0; --dir) {
            const bool col = dir != 0;
            const int n = col ? H : W, rows = col ? W : H;
            const bool valid = j < rows;
            const int base = col ? j : j * P, step = col ? P : 1;
            const uint32_t jm = jm_next, up = up_next;
            fetch(2 * k + dir - 1, jm_next, up_next);
            float *dst = col ? B : A;                    // column pass: B <- C^T(A - B) + B
            const float *src = col ? A : B;              // row pass:    A <- R^T(B - A) + A
            float v[C], old[C];
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const bool in = valid && k0 + c < n;
                const int e = base + (k0 + c) * step;
                old[c] = (in && !first) ? dst[e] : 0.f;
                v[c] = in ? src[e] - old[c] : 0.f;
            }
            const float gl = lanes_segment_means<T, C>(v, jm, up, n, t);
            if (valid) glam += gl;
#pragma unroll
            for (int c = 0; c < C; ++c)
                if (valid && k0 + c < n) dst[base + (k0 + c) * step] = old[c] + v[c];
            __syncthreads();
        }
    }
    if constexpr (IO16) {
        uint16_t *dst = reinterpret_cast<uint16_t *>(p.gy) + plane * HW;
        for (int e = tid; e < HW; e += NT) dst[e] = f32_to_bf16_bits(A[(e / W) * P + e % W]);
    } else {
        float *dst = p.gy + plane * HW;
        for (int e = tid; e < HW; e += NT) dst[e] = A[(e / W) * P + e % W];
    }
    if (p.partial) {
        // the plane's term: waves in a fixed order
        const float s = wave_sum_all<64>(glam);
        if ((tid & 63) == 0) part[tid >> 6] = s;
        __syncthreads();
        if (tid == 0) {
            float tot = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) tot += part[w];
            p.partial[plane] = tot;
        }
    }
}

}  // namespace tvk
