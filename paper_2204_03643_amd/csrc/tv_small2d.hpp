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

// ---- bf16 storage of the planes (fp32 everywhere inside): the wave's planes between memory (bf16
//      bit patterns, plane after plane) and an LDS tile of fp32 rows at pitch P.
// FULL planes (S x S, 16-byte aligned block): eight samples per 16-byte access.
template <int S>
__device__ __forceinline__ void planes16_into_tile(const uint16_t *__restrict__ src, int n_here, int lane,
                                                   float *tile, bool stream)
{
    constexpr int P = S + 1;
#pragma unroll
    for (int i = 0; i < S / 8; ++i) {
        const int e = (i * 64 + lane) * 8;                 // sample index inside the wave's block
        float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
        if (e / (S * S) < n_here) q = load16(reinterpret_cast<const float *>(src + e), stream);
        const uint32_t w[4] = {__float_as_uint(q.x), __float_as_uint(q.y), __float_as_uint(q.z), __float_as_uint(q.w)};
        float *d = tile + (e / S) * P + (e % S);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            d[2 * j] = __uint_as_float(w[j] << 16);
            d[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
        }
    }
}
template <int S>
__device__ __forceinline__ void tile_into_planes16(const float *tile, uint16_t *__restrict__ dst, int n_here,
                                                   int lane, bool stream)
{
    constexpr int P = S + 1;
#pragma unroll
    for (int i = 0; i < S / 8; ++i) {
        const int e = (i * 64 + lane) * 8;
        const float *sp = tile + (e / S) * P + (e % S);
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = f32x2_to_bf16x2(sp[2 * j], sp[2 * j + 1]);
        if (e / (S * S) < n_here)
            store16(reinterpret_cast<float *>(dst + e),
                    make_float4(__uint_as_float(w[0]), __uint_as_float(w[1]), __uint_as_float(w[2]), __uint_as_float(w[3])),
                    stream);
    }
}
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float v) { return (uint16_t)(f32x2_to_bf16x2(v, 0.f) & 0xffffu); }

struct Small2dBwdParams {
    const float *g_up;
    float       *gy;
    const uint2 *codes;        // pass i (row pass of sweep k: 2k, column pass: 2k + 1) at codes + i * code_stride
    size_t       code_stride;  // in uint2
    const float *saved;        // planes of 33-64 samples a side have no codes: the output of pass i,
    size_t       saved_stride; // at saved + i * saved_stride (floats), is read instead
    float       *partial;      // optional: one dL/dlam term per plane (all passes summed)
    int32_t      planes, H, W, sweeps;
    uint32_t     stream;       // tensors too large to stay in cache: non-temporal accesses
};                             // (IO16 kernels: g_up and gy point to bf16 bit patterns)

// Bit k of a row's segment code: x = jump bits 0-31, y = direction bits 0-31, z and w = the same
// for duals 32-62 (rows of more than 32 samples).
template <int K>
__device__ __forceinline__ bool code_jump(const uint4 &c) { return ((K < 32 ? c.x : c.z) & (1u << (K & 31))) != 0u; }
template <int K>
__device__ __forceinline__ bool code_up(const uint4 &c) { return ((K < 32 ? c.y : c.w) & (1u << (K & 31))) != 0u; }

// Segment means of g[0 .. n-1] in place, segments given by the code's jump bits; returns the
// row's dL/dlam term  sum over jumps k of sign(x[k+1] - x[k]) (mean_left - mean_right).
// FULL: n = S at compile time.
template <int S, bool FULL, int K = 0>
__device__ __forceinline__ void small2d_means_up(float (&g)[S], const uint4 &code, int n, const float *rtab,
                                                 float &s, int &c4)
{
    if constexpr (K < S) {
        s += g[K];
        c4 += 4;
        const bool last = FULL ? (K == S - 1) : (K >= n - 1);
        bool end = last;
        if constexpr (K + 1 < S) end = end || code_jump<K>(code);
        g[K] = s * *reinterpret_cast<const float *>(reinterpret_cast<const char *>(rtab) + c4);
        if (end) { s = 0.f; c4 = 0; }
        small2d_means_up<S, FULL, K + 1>(g, code, n, rtab, s, c4);
    }
}
template <int S, bool FULL, int K = S - 1>
__device__ __forceinline__ void small2d_means_down(float (&g)[S], const uint4 &code, int n, float &carry,
                                                   float &glam)
{
    if constexpr (K >= 0) {
        const float right = carry;
        const bool last = FULL ? (K == S - 1) : (K >= n - 1);
        bool end = last;
        if constexpr (K + 1 < S) end = end || code_jump<K>(code);
        carry = end ? g[K] : carry;
        g[K] = carry;
        if constexpr (K + 1 < S) {
            if (FULL || K < n - 1) {
                const float d = carry - right;
                glam += code_up<K>(code) ? d : -d;
            }
        }
        small2d_means_down<S, FULL, K - 1>(g, code, n, carry, glam);
    }
}
template <int S, bool FULL>
__device__ __forceinline__ float small2d_segment_means(float (&g)[S], const uint4 &code, int n, const float *rtab)
{
    float s = 0.f, carry = 0.f, glam = 0.f;
    int c4 = 0;
    // the row length in a vector register: as a wave-uniform value every "k is past the end"
    // predicate of the unrolled loops would be kept in scalar registers, 2 S pairs of them
    if (!FULL) asm volatile("" : "+v"(n));
    small2d_means_up<S, FULL>(g, code, n, rtab, s, c4);
    small2d_means_down<S, FULL>(g, code, n, carry, glam);
    return glam;
}
// S = 8, 16, 32 or 64: the side of the square a plane is padded to; a wave holds 64 / S planes,
// one row or column per lane.  FULL: planes of exactly S x S.  S = 64: the segments of a pass are
// read off its saved output (the forward kernels for rows of more than 32 samples write no codes).
// FROM_X: the segments of a pass are read off its saved output instead of its codes.
// IO16: the upstream gradient and grad_y are bf16 in memory (fp32 in the tiles and in all arithmetic).
template <int S, bool FULL, bool FROM_X = (S > 32), bool IO16 = false>
__global__ __launch_bounds__(64) void tv2d_bwd_small_kernel(Small2dBwdParams p)
{
    constexpr int P = S + 1;                        // tile pitch
    constexpr int PP = 64 / S;                      // planes per wave
    __shared__ float A[64 * P], B[64 * P], rtab[S + 2];
    const int lane = threadIdx.x;
    for (int i = lane; i <= S; i += 64) rtab[i] = i > 0 ? 1.0f / (float)i : 0.0f;
    const int h = lane / S, idx = lane % S;         // which of the wave's planes; row or column
    const int H = FULL ? S : p.H, W = FULL ? S : p.W, HW = H * W;
    const int64_t plane0 = (int64_t)blockIdx.x * PP;
    const int64_t plane = plane0 + h;
    const bool pvalid = plane < p.planes;
    const int n_here = (int)((p.planes - plane0 < PP) ? (p.planes - plane0) : PP);

    // the upstream gradient of the wave's planes -> A
    if constexpr (IO16) {
        const uint16_t *src = reinterpret_cast<const uint16_t *>(p.g_up) + plane0 * HW;
        if (FULL && ((uintptr_t)src % 16) == 0) {
            planes16_into_tile<S>(src, n_here, lane, A, p.stream != 0);
        } else if (pvalid && idx < W) {
            const uint16_t *col = src + h * HW + idx;
            for (int r = 0; r < H; ++r) A[(h * S + r) * P + idx] = bf16_bits_to_f32(col[r * W]);
        }
    } else {
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
            // lane (h, idx) moves column idx of its plane: W contiguous floats per memory row
            if (pvalid && idx < W) {
                const float *col = src + h * HW + idx;
                for (int r = 0; r < H; ++r) A[(h * S + r) * P + idx] = col[r * W];
            }
        }
    }
    wave_lds_sync();

    float glam = 0.f;
    float v[S];
    // the segment code of a pass is fetched one pass ahead, so that its latency hides behind
    // the pass before
    const bool cvalid = pvalid && (FULL || idx < W), rvalid = pvalid && (FULL || idx < H);
    auto fetch_code = [&](int pass) -> uint4 {
        if (pass < 0) return make_uint4(0u, 0u, 0u, 0u);
        const bool col = (pass & 1) != 0;
        if constexpr (!FROM_X) {
            if (!(col ? cvalid : rvalid)) return make_uint4(0u, 0u, 0u, 0u);
            const uint2 c = p.codes[(size_t)pass * p.code_stride + (size_t)plane * (col ? W : H) + idx];
            return make_uint4(c.x, c.y, 0u, 0u);
        } else {
            // the lane's row or column of the pass's output, then one bit per neighbour pair
            const float *xs = p.saved + (size_t)pass * p.saved_stride + (size_t)plane * HW;
            float xv[S];
            if (col) {
#pragma unroll
                for (int r = 0; r < S; ++r) xv[r] = (cvalid && (FULL || r < H)) ? xs[r * W + idx] : 0.f;
            } else if (FULL && ((uintptr_t)xs % 16) == 0) {
#pragma unroll
                for (int c = 0; c < S; c += 4) {
                    float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (rvalid) q = *reinterpret_cast<const float4 *>(xs + idx * S + c);
                    xv[c] = q.x; xv[c + 1] = q.y; xv[c + 2] = q.z; xv[c + 3] = q.w;
                }
            } else {
#pragma unroll
                for (int c = 0; c < S; ++c) xv[c] = (rvalid && (FULL || c < W)) ? xs[idx * W + c] : 0.f;
            }
            // built from the highest dual of each word down, one shift-in per dual, so that dual k
            // ends up at bit k & 31; the sign of x[k] - x[k+1] says "rises", that of -|.| "differs"
            uint4 c = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int k = S - 2; k >= 32; --k) {
                const float d = xv[k] - xv[k + 1];
                c.w = __builtin_amdgcn_alignbit(c.w, __float_as_uint(d), 31);
                c.z = __builtin_amdgcn_alignbit(c.z, __float_as_uint(0.0f - fabsf(d)), 31);
            }
#pragma unroll
            for (int k = (S - 2 < 31 ? S - 2 : 31); k >= 0; --k) {
                const float d = xv[k] - xv[k + 1];
                c.y = __builtin_amdgcn_alignbit(c.y, __float_as_uint(d), 31);
                c.x = __builtin_amdgcn_alignbit(c.x, __float_as_uint(0.0f - fabsf(d)), 31);
            }
            return c;
        }
    };
    uint4 code_next = fetch_code(2 * p.sweeps - 1);
    for (int k = p.sweeps - 1; k >= 0; --k) {
        const bool first = (k == p.sweeps - 1);
        // ---- adjoint of the column pass: B <- C^T(A - B) + B  (B = 0 in the first reverse step);
        //      a lane holds column idx of its plane
        {
            const bool valid = cvalid;
            const uint4 code = code_next;
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
            const uint4 code = code_next;
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
    if constexpr (IO16) {
        uint16_t *dst = reinterpret_cast<uint16_t *>(p.gy) + plane0 * HW;
        if (FULL && ((uintptr_t)dst % 16) == 0) {
            tile_into_planes16<S>(A, dst, n_here, lane, p.stream != 0);
        } else if (pvalid && idx < W) {
            uint16_t *col = dst + h * HW + idx;
            for (int r = 0; r < H; ++r) col[r * W] = f32_to_bf16_bits(A[(h * S + r) * P + idx]);
        }
    } else {
        float *dst = p.gy + plane0 * HW;
        if (FULL && ((uintptr_t)dst % 16) == 0) {
#pragma unroll
            for (int i = 0; i < S / 4; ++i) {
                const int e = (i * 64 + lane) * 4;
                const float *s = A + (e / S) * P + (e % S);
                if (e / (S * S) < n_here) store16(dst + e, make_float4(s[0], s[1], s[2], s[3]), p.stream != 0);
            }
        } else {
            if (pvalid && idx < W) {
                float *col = dst + h * HW + idx;
                for (int r = 0; r < H; ++r) col[r * W] = A[(h * S + r) * P + idx];
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
    uint32_t     keep_passes;  // planes of at most 32 x 32: 0 = write the codes only, not the pass outputs
    uint2       *codes;        // as in Small2dBwdParams
    size_t       code_stride;
    const float *lam;          // plane p uses lam[p % lam_count]
    int64_t      lam_count;
    int32_t      planes, H, W, sweeps;
    uint32_t     stream;
};

// S, FULL: as in the reverse sweep (a wave holds 64 / S planes), S <= 32.
// IO16: y and x are bf16 in memory; the saved pass outputs stay fp32.
// (Planes of 33-64 samples a side: tv_plane2d.hpp.  A row of 64 samples per lane would take four
// arrays of 64 registers, the whole register file of a SIMD lane, for one wave per SIMD.)
// Waves per SIMD asked of the register allocator: two at least; six for planes of 8 x 8 (80 VGPRs
// instead of 87-96 at the price of 3-5 spilled registers: 65 536 planes, K = 4: 98 -> 95 us).
// Four for planes of 16 x 16 (128 VGPRs instead of 145-168, 16-54 spilled) take 65 536 planes
// with K = 4 from 334 to 302 us but 8192 planes with K = 2, which do not fill three waves per SIMD
// anyway, from 43 to 45: that is the variant DENSE, which the dispatch takes for large batches.
template <int S, bool FULL, bool IO16 = false, bool DENSE = false>
__global__ __launch_bounds__(64, (S == 8 ? 6 : ((S == 16 && DENSE) ? 4 : 2))) void tv2d_fwd_small_kernel(Small2dFwdParams p)
{
    static_assert(S <= 32, "a row or column per lane: planes of at most 32 x 32");
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

    // the wave's planes -> T1 (memory rows at pitch P)
    if constexpr (IO16) {
        const uint16_t *src = reinterpret_cast<const uint16_t *>(p.y) + plane0 * HW;
        if (FULL && ((uintptr_t)src % 16) == 0) {
            planes16_into_tile<S>(src, n_here, lane, T1, p.stream != 0);
        } else if (pvalid && idx < W) {
            const uint16_t *col = src + h * HW + idx;
            for (int r = 0; r < H; ++r) T1[(h * S + r) * P + idx] = bf16_bits_to_f32(col[r * W]);
        }
    } else {
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
            // lane (h, idx) moves column idx of its plane: W contiguous floats per memory row
            if (pvalid && idx < W) {
                const float *col = src + h * HW + idx;
                for (int r = 0; r < H; ++r) T1[(h * S + r) * P + idx] = col[r * W];
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
            if (pvalid && idx < W) {
                float *col = dst + h * HW + idx;
                for (int r = 0; r < H; ++r) col[r * W] = T1[(h * S + r) * P + idx];
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
        // (planes of at most 32 x 32: the reverse sweep reads the codes written above)
        if (p.keep_passes) put_planes(p.saved + (size_t)i * p.saved_stride + plane0 * HW);
        if (i + 1 == n_pass) {
            if constexpr (IO16) {
                uint16_t *dst = reinterpret_cast<uint16_t *>(p.x) + plane0 * HW;
                if (FULL && ((uintptr_t)dst % 16) == 0) {
                    tile_into_planes16<S>(T1, dst, n_here, lane, p.stream != 0);
                } else if (pvalid && idx < W) {
                    uint16_t *colo = dst + h * HW + idx;
                    for (int r = 0; r < H; ++r) colo[r * W] = f32_to_bf16_bits(T1[(h * S + r) * P + idx]);
                }
            } else {
                put_planes(p.x + plane0 * HW);
            }
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
