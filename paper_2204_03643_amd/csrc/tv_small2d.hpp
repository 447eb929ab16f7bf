// The 2D operator (paper Alg. 1) and its reverse sweep (Sec. 3.2) for planes of at most 32 x 32,
// all 2K passes of a call in one launch; planes of at most 16 x 16 or 8 x 8 are packed four or
// eight to a wave.  Forward kernel: at the end of this file.
//
// Reverse sweep.
// The backward pass of a 1D prox is segment averaging (paper Eq. 5-6) and moves 12 bytes per
// sample for a few dozen instructions, so the pass-by-pass reverse sweep is bound by memory:
// 2K passes read and write the two adjoint state tensors again and again.  Here a wave keeps the
// state of its planes (two of up to 32 x 32, four of up to 16 x 16, eight of up to 8 x 8) in LDS for the whole sweep: the upstream gradient is read once, grad_y is
// written once, and per pass only the rows' 8-byte segment codes come from memory.  Both views of
// a plane (a row per lane, a column per lane) read the same tile of odd pitch without bank
// conflicts, so no transpose is needed between the row and the column passes.
#pragma once
#include "tv_short.hpp"

namespace tvk {

struct Small2dBwdParams {
    const float *g_up;
    float       *gy;
    const uint2 *codes;        // pass i (row pass of sweep k: 2k, column pass: 2k + 1) at codes + i * code_stride
    size_t       code_stride;  // in uint2
    float       *partial;      // optional: one dL/dlam term per plane (all passes summed)
    int32_t      planes, H, W, sweeps;
    uint32_t     stream;       // tensors too large to stay in cache: non-temporal accesses
};

// Segment means of g[0 .. n-1] in place, segments given by the code's jump bits; returns the
// row's dL/dlam term  sum over jumps k of sign(x[k+1] - x[k]) (mean_left - mean_right).
// FULL: n = S at compile time.
template <int S, bool FULL>
__device__ __forceinline__ float small2d_segment_means(float (&g)[S], uint2 code, int n, const float *rtab)
{
    {
        float s = 0.f;
        int c4 = 0;
#pragma unroll
        for (int k = 0; k < S; ++k) {
            s += g[k];
            c4 += 4;
            const bool last = FULL ? (k == S - 1) : (k >= n - 1);
            const bool end = last || (k + 1 < S && (code.x & (1u << k)) != 0u);
            g[k] = s * *reinterpret_cast<const float *>(reinterpret_cast<const char *>(rtab) + c4);
            if (end) { s = 0.f; c4 = 0; }
        }
    }
    float glam = 0.f;
    float carry = 0.f;
#pragma unroll
    for (int k = S - 1; k >= 0; --k) {
        const float right = carry;
        const bool last = FULL ? (k == S - 1) : (k >= n - 1);
        const bool end = last || (k + 1 < S && (code.x & (1u << k)) != 0u);
        carry = end ? g[k] : carry;
        g[k] = carry;
        if (k + 1 < S && (FULL || k < n - 1)) {
            const float d = carry - right;
            glam += (code.y & (1u << k)) != 0u ? d : -d;
        }
    }
    return glam;
}

// S = 8, 16 or 32: the side of the square a plane is padded to; a wave holds 64 / S planes, one
// row or column per lane.  FULL: planes of exactly S x S.
template <int S, bool FULL>
__global__ __launch_bounds__(64) void tv2d_bwd_small_kernel(Small2dBwdParams p)
{
    constexpr int P = S + 1;                        // tile pitch
    constexpr int PP = 64 / S;                      // planes per wave
    __shared__ float A[64 * P], B[64 * P], rtab[S + 2];
    const int lane = threadIdx.x;
    if (lane <= S) rtab[lane] = lane > 0 ? 1.0f / (float)lane : 0.0f;
    const int h = lane / S, idx = lane % S;         // which of the wave's planes; row or column
    const int H = FULL ? S : p.H, W = FULL ? S : p.W, HW = H * W;
    const int64_t plane0 = (int64_t)blockIdx.x * PP;
    const int64_t plane = plane0 + h;
    const bool pvalid = plane < p.planes;
    const int n_here = (int)((p.planes - plane0 < PP) ? (p.planes - plane0) : PP);

    // the upstream gradient of the wave's planes -> A
    {
        const float *src = p.g_up + plane0 * HW;
        if (FULL && ((uintptr_t)src % 16) == 0) {
#pragma unroll
            for (int i = 0; i < S / 4; ++i) {
                const int e = (i * 64 + lane) * 4;              // 0 .. 64 S - 1
                float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
                if (e / (S * S) < n_here) q = load16(src + e, p.stream != 0);
                float *d = A + (e / S) * P + (e % S);
                d[0] = q.x; d[1] = q.y; d[2] = q.z; d[3] = q.w;
            }
        } else {
            for (int e = lane; e < n_here * HW; e += 64) {
                const int hh = e / HW, rem = e - hh * HW, r = rem / W, c = rem - r * W;
                A[(hh * S + r) * P + c] = src[e];
            }
        }
    }
    wave_lds_sync();

    float glam = 0.f;
    float v[S];
    // the segment code of a pass is fetched one pass ahead, so that its latency hides behind
    // the pass before
    const bool cvalid = pvalid && (FULL || idx < W), rvalid = pvalid && (FULL || idx < H);
    auto fetch_code = [&](int pass) -> uint2 {
        if (pass < 0) return make_uint2(0u, 0u);
        const bool col = (pass & 1) != 0;
        if (!(col ? cvalid : rvalid)) return make_uint2(0u, 0u);
        return p.codes[(size_t)pass * p.code_stride + (size_t)plane * (col ? W : H) + idx];
    };
    uint2 code_next = fetch_code(2 * p.sweeps - 1);
    for (int k = p.sweeps - 1; k >= 0; --k) {
        const bool first = (k == p.sweeps - 1);
        // ---- adjoint of the column pass: B <- C^T(A - B) + B  (B = 0 in the first reverse step);
        //      a lane holds column idx of its plane
        {
            const bool valid = cvalid;
            const uint2 code = code_next;
            code_next = fetch_code(2 * k);
            const float *a = A + (h * S) * P + idx;
            float *b = B + (h * S) * P + idx;
            // (tile entries outside H x W, and the tile half of a plane that does not exist, hold
            // garbage that stays where it is: a segment never extends past the row's end)
            if (first) {
#pragma unroll
                for (int r = 0; r < S; ++r) v[r] = a[r * P];
            } else {
#pragma unroll
                for (int r = 0; r < S; ++r) v[r] = a[r * P] - b[r * P];
            }
            const float t = small2d_segment_means<S, FULL>(v, code, H, rtab);
            if (valid) glam += t;
            if (first) {
#pragma unroll
                for (int r = 0; r < S; ++r) b[r * P] = v[r];
            } else {
#pragma unroll
                for (int r = 0; r < S; ++r) b[r * P] += v[r];
            }
        }
        wave_lds_sync();
        // ---- adjoint of the row pass: A <- R^T(B - A) + A  (without A in the first reverse step);
        //      a lane holds row idx of its plane
        {
            const bool valid = rvalid;
            const uint2 code = code_next;
            code_next = fetch_code(2 * k - 1);
            float *a = A + (h * S + idx) * P;
            const float *b = B + (h * S + idx) * P;
            if (first) {
#pragma unroll
                for (int c = 0; c < S; ++c) v[c] = b[c];
            } else {
#pragma unroll
                for (int c = 0; c < S; ++c) v[c] = b[c] - a[c];
            }
            const float t = small2d_segment_means<S, FULL>(v, code, W, rtab);
            if (valid) glam += t;
            if (first) {
#pragma unroll
                for (int c = 0; c < S; ++c) a[c] = v[c];
            } else {
#pragma unroll
                for (int c = 0; c < S; ++c) a[c] += v[c];
            }
        }
        wave_lds_sync();
    }

    // grad_y = A
    {
        float *dst = p.gy + plane0 * HW;
        if (FULL && ((uintptr_t)dst % 16) == 0) {
#pragma unroll
            for (int i = 0; i < S / 4; ++i) {
                const int e = (i * 64 + lane) * 4;
                const float *s = A + (e / S) * P + (e % S);
                if (e / (S * S) < n_here) store16(dst + e, make_float4(s[0], s[1], s[2], s[3]), p.stream != 0);
            }
        } else {
            for (int e = lane; e < n_here * HW; e += 64) {
                const int hh = e / HW, rem = e - hh * HW, r = rem / W, c = rem - r * W;
                dst[e] = A[(hh * S + r) * P + c];
            }
        }
    }
    if (p.partial) {
        // sum over the S lanes of each plane, in a fixed order
        float s = glam;
#pragma unroll
        for (int d = 1; d < S; d <<= 1) s += __shfl_xor(s, d);
        if (pvalid && idx == 0) p.partial[plane] = s;
    }
}

// ---------------------------------------------------------------------------------
// Forward: K sweeps of paper Alg. 1 on planes of at most 32 x 32 in one launch.
//
// A wave owns its planes (two, four or eight, as in the reverse sweep) for the whole call.  A row pass gives each lane a row of its plane, a
// column pass a column; either way the lane solves its 1D problem exactly as the short-row
// kernel does (same RowSolver, row in registers).  Between passes the plane changes hands
// through one LDS tile of odd pitch (side + 1), which both views read and write without bank conflicts.
// The correction terms P (rows) and Q (columns) are only ever touched by the lane that owns
// the row or column, so they live in a lane-private LDS column; one such column suffices,
// because P is consumed (A = Y + P) just before the new Q has to be put away and the other way
// round.  From the second sweep on a pass starts from the dual its correction term encodes
// (P = D^T u of the row pass one sweep earlier, likewise Q).
//
// Memory traffic: y is read once; every pass writes its output (the reverse sweep's tests and
// the caller's workspace contract want them) and one 8-byte segment code per row or column.
// ---------------------------------------------------------------------------------
struct Small2dFwdParams {
    const float *y;
    float       *x;
    float       *saved;        // output of pass i at saved + i * saved_stride (floats)
    size_t       saved_stride;
    uint2       *codes;        // as in Small2dBwdParams
    size_t       code_stride;
    const float *lam;          // plane p uses lam[p % lam_count]
    int64_t      lam_count;
    int32_t      planes, H, W, sweeps;
    uint32_t     stream;
};

// S, FULL: as in the reverse sweep (a wave holds 64 / S planes).
template <int S, bool FULL>
__global__ __launch_bounds__(64, 2) void tv2d_fwd_small_kernel(Small2dFwdParams p)
{
    constexpr int P = S + 1;
    constexpr int PP = 64 / S;
    __shared__ float T1[64 * P], T2[64 * S], gtab[S + 2], rtab[S + 2];
    const int lane = threadIdx.x;
    fill_tables<S>(gtab, rtab);
    const int h = lane / S, idx = lane % S;
    const int H = FULL ? S : p.H, W = FULL ? S : p.W, HW = H * W;
    const int64_t plane0 = (int64_t)blockIdx.x * PP;
    const int64_t plane = plane0 + h;
    const bool pvalid = plane < p.planes;
    const int n_here = (int)((p.planes - plane0 < PP) ? (p.planes - plane0) : PP);
    float lam = 0.f;
    if (pvalid) lam = fmaxf(p.lam[plane % p.lam_count], 0.f);

    float *rowp = T1 + (h * S + idx) * P;      // row idx of the lane's plane, unit step
    float *colp = T1 + (h * S) * P + idx;      // column idx, step P
    float *park = T1 + lane;                    // the solver's read-only copy of its input, step 64
    float *mine = T2 + lane;                    // lane-private: the correction term, step 64

    // the two planes -> T1 (memory rows at pitch P)
    {
        const float *src = p.y + plane0 * HW;
        if (FULL && ((uintptr_t)src % 16) == 0) {
#pragma unroll
            for (int i = 0; i < S / 4; ++i) {
                const int e = (i * 64 + lane) * 4;
                float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
                if (e / (S * S) < n_here) q = load16(src + e, p.stream != 0);
                float *d = T1 + (e / S) * P + (e % S);
                d[0] = q.x; d[1] = q.y; d[2] = q.z; d[3] = q.w;
            }
        } else {
            for (int e = lane; e < n_here * HW; e += 64) {
                const int hh = e / HW, rem = e - hh * HW, r = rem / W, c = rem - r * W;
                T1[(hh * S + r) * P + c] = src[e];
            }
        }
    }
    wave_lds_sync();

    // a pass's output, T1 -> memory in plane order
    auto put_planes = [&](float *dst) {
        if (FULL && ((uintptr_t)dst % 16) == 0) {
#pragma unroll
            for (int i = 0; i < S / 4; ++i) {
                const int e = (i * 64 + lane) * 4;
                const float *s = T1 + (e / S) * P + (e % S);
                if (e / (S * S) < n_here) store16(dst + e, make_float4(s[0], s[1], s[2], s[3]), p.stream != 0);
            }
        } else {
            for (int e = lane; e < n_here * HW; e += 64) {
                const int hh = e / HW, rem = e - hh * HW, r = rem / W, c = rem - r * W;
                dst[e] = T1[(hh * S + r) * P + c];
            }
        }
    };

    float v[S], xs[S];
    RowSolver<S, FULL> sv;
    bool valid = pvalid && (FULL || idx < H);   // first pass: rows, of W samples
    int n = W;
#pragma unroll
    for (int k = 0; k < S; ++k) v[k] = (valid && (FULL || k < n)) ? rowp[k] : 0.f;

    const int n_pass = 2 * p.sweeps;
    for (int i = 0; i < n_pass; ++i) {
        const bool col = (i & 1) != 0;
        wave_lds_sync();                        // every lane has taken its input out of T1
#pragma unroll
        for (int k = 0; k < S; ++k) park[k * 64] = v[k];
        wave_lds_sync();

        sv.yl = park; sv.gtab = gtab; sv.lam = lam; sv.m = n - 1;
        sv.alpha_try = 1.f; sv.steps = 0; sv.flags = 0; sv.nfail = 0;
        sv.active = valid; sv.prev_unclipped = false;
        if (i < 2) sv.start(v, rtab[n]);        // first sweep: no correction term yet
        else sv.start_warm(v);
        for (int it = 0; !sv.iterate(it); ++it) {}
        sv.recover(xs);

        {   // segment code of the row / column (as the short-row kernel builds it)
            uint32_t jm = 0, up = 0;
#pragma unroll
            for (int k = S - 2; k >= 0; --k) {
                const float d = xs[k] - xs[k + 1];
                up = __builtin_amdgcn_alignbit(up, __float_as_uint(d), 31);
                jm = __builtin_amdgcn_alignbit(jm, __float_as_uint(0.0f - fabsf(d)), 31);
            }
            if (!FULL) {
                const uint32_t in = n > 1 ? (0xffffffffu >> (33 - n)) : 0u;
                jm &= in; up &= in;
            }
            if (valid) p.codes[(size_t)i * p.code_stride + (size_t)plane * (col ? W : H) + idx] = make_uint2(jm, up);
        }

        // the pass's new correction term (input - output); needed by the same direction's pass
        // of the next sweep
        const bool keep = i + 2 < n_pass;
        if (keep) {
#pragma unroll
            for (int k = 0; k < S; ++k) v[k] = park[k * 64] - xs[k];
        }
        wave_lds_sync();                        // the parked inputs have been read
        if (col) {
#pragma unroll
            for (int k = 0; k < S; ++k) colp[k * P] = xs[k];
        } else {
#pragma unroll
            for (int k = 0; k < S; ++k) rowp[k] = xs[k];
        }
        wave_lds_sync();
        put_planes(p.saved + (size_t)i * p.saved_stride + plane0 * HW);
        if (i + 1 == n_pass) {
            put_planes(p.x + plane0 * HW);
            break;
        }

        // input of the next pass: this output seen the other way, plus that direction's
        // correction term, whose negated running sum is the dual to start from
        valid = pvalid && (FULL || idx < (col ? H : W));
        n = col ? W : H;
        float t[S];
        if (col) {
#pragma unroll
            for (int k = 0; k < S; ++k) t[k] = (valid && (FULL || k < n)) ? rowp[k] : 0.f;
        } else {
#pragma unroll
            for (int k = 0; k < S; ++k) t[k] = (valid && (FULL || k < n)) ? colp[k * P] : 0.f;
        }
        if (i >= 1) {
            float run = 0.f;
#pragma unroll
            for (int k = 0; k < S; ++k) {
                const float c = mine[k * 64];
                t[k] += c;
                run -= c;
                if (k < S - 1) sv.u[k] = run;
            }
        }
        if (keep) {
#pragma unroll
            for (int k = 0; k < S; ++k) mine[k * 64] = v[k];
        }
#pragma unroll
        for (int k = 0; k < S; ++k) v[k] = t[k];
    }
}

}  // namespace tvk
