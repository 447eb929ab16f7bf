// Reverse sweep of the 2D operator (paper Alg. 1, Sec. 3.2) for planes of at most 32 x 32, all
// 2K passes in one launch.
//
// The backward pass of a 1D prox is segment averaging (paper Eq. 5-6) and moves 12 bytes per
// sample for a few dozen instructions, so the pass-by-pass reverse sweep is bound by memory:
// 2K passes read and write the two adjoint state tensors again and again.  Here a wave keeps the
// state of two planes in LDS for the whole sweep: the upstream gradient is read once, grad_y is
// written once, and per pass only the rows' 8-byte segment codes come from memory.  Both views of
// a plane (a row per lane, a column per lane) read the same tile of pitch 33 without bank
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
// FULL: n = 32 at compile time.
template <bool FULL>
__device__ __forceinline__ float small2d_segment_means(float (&g)[32], uint2 code, int n, const float *rtab)
{
    {
        float s = 0.f;
        int c4 = 0;
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            s += g[k];
            c4 += 4;
            const bool last = FULL ? (k == 31) : (k >= n - 1);
            const bool end = last || (k + 1 < 32 && (code.x & (1u << k)) != 0u);
            g[k] = s * *reinterpret_cast<const float *>(reinterpret_cast<const char *>(rtab) + c4);
            if (end) { s = 0.f; c4 = 0; }
        }
    }
    float glam = 0.f;
    float carry = 0.f;
#pragma unroll
    for (int k = 31; k >= 0; --k) {
        const float right = carry;
        const bool last = FULL ? (k == 31) : (k >= n - 1);
        const bool end = last || (k + 1 < 32 && (code.x & (1u << k)) != 0u);
        carry = end ? g[k] : carry;
        g[k] = carry;
        if (k + 1 < 32 && (FULL || k < n - 1)) {
            const float d = carry - right;
            glam += (code.y & (1u << k)) != 0u ? d : -d;
        }
    }
    return glam;
}

// FULL: planes of exactly 32 x 32.
template <bool FULL>
__global__ __launch_bounds__(64) void tv2d_bwd_small_kernel(Small2dBwdParams p)
{
    constexpr int P = 33;                           // tile pitch
    __shared__ float A[64 * P], B[64 * P], rtab[34];
    const int lane = threadIdx.x;
    if (lane <= 32) rtab[lane] = lane > 0 ? 1.0f / (float)lane : 0.0f;
    const int h = lane >> 5, idx = lane & 31;       // which of the wave's two planes; row or column
    const int H = FULL ? 32 : p.H, W = FULL ? 32 : p.W, HW = H * W;
    const int64_t plane0 = (int64_t)blockIdx.x * 2;
    const int64_t plane = plane0 + h;
    const bool pvalid = plane < p.planes;
    const int n_here = (plane0 + 1 < p.planes) ? 2 : 1;

    // the upstream gradient of the two planes -> A
    {
        const float *src = p.g_up + plane0 * HW;
        if (FULL && ((uintptr_t)src % 16) == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = (i * 64 + lane) * 4;              // 0 .. 2047
                float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
                if ((e >> 10) < n_here) q = load16(src + e, p.stream != 0);
                float *d = A + (e >> 5) * P + (e & 31);
                d[0] = q.x; d[1] = q.y; d[2] = q.z; d[3] = q.w;
            }
        } else {
            for (int e = lane; e < n_here * HW; e += 64) {
                const int hh = e / HW, rem = e - hh * HW, r = rem / W, c = rem - r * W;
                A[(hh * 32 + r) * P + c] = src[e];
            }
        }
    }
    wave_lds_sync();

    float glam = 0.f;
    float v[32];
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
            const float *a = A + (h * 32) * P + idx;
            float *b = B + (h * 32) * P + idx;
            // (tile entries outside H x W, and the tile half of a plane that does not exist, hold
            // garbage that stays where it is: a segment never extends past the row's end)
            if (first) {
#pragma unroll
                for (int r = 0; r < 32; ++r) v[r] = a[r * P];
            } else {
#pragma unroll
                for (int r = 0; r < 32; ++r) v[r] = a[r * P] - b[r * P];
            }
            const float t = small2d_segment_means<FULL>(v, code, H, rtab);
            if (valid) glam += t;
            if (first) {
#pragma unroll
                for (int r = 0; r < 32; ++r) b[r * P] = v[r];
            } else {
#pragma unroll
                for (int r = 0; r < 32; ++r) b[r * P] += v[r];
            }
        }
        wave_lds_sync();
        // ---- adjoint of the row pass: A <- R^T(B - A) + A  (without A in the first reverse step);
        //      a lane holds row idx of its plane
        {
            const bool valid = rvalid;
            const uint2 code = code_next;
            code_next = fetch_code(2 * k - 1);
            float *a = A + (h * 32 + idx) * P;
            const float *b = B + (h * 32 + idx) * P;
            if (first) {
#pragma unroll
                for (int c = 0; c < 32; ++c) v[c] = b[c];
            } else {
#pragma unroll
                for (int c = 0; c < 32; ++c) v[c] = b[c] - a[c];
            }
            const float t = small2d_segment_means<FULL>(v, code, W, rtab);
            if (valid) glam += t;
            if (first) {
#pragma unroll
                for (int c = 0; c < 32; ++c) a[c] = v[c];
            } else {
#pragma unroll
                for (int c = 0; c < 32; ++c) a[c] += v[c];
            }
        }
        wave_lds_sync();
    }

    // grad_y = A
    {
        float *dst = p.gy + plane0 * HW;
        if (FULL && ((uintptr_t)dst % 16) == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = (i * 64 + lane) * 4;
                const float *s = A + (e >> 5) * P + (e & 31);
                if ((e >> 10) < n_here) store16(dst + e, make_float4(s[0], s[1], s[2], s[3]), p.stream != 0);
            }
        } else {
            for (int e = lane; e < n_here * HW; e += 64) {
                const int hh = e / HW, rem = e - hh * HW, r = rem / W, c = rem - r * W;
                dst[e] = A[(hh * 32 + r) * P + c];
            }
        }
    }
    if (p.partial) {
        // sum over the 32 lanes of each plane, in a fixed order
        float s = glam;
#pragma unroll
        for (int d = 1; d < 32; d <<= 1) s += __shfl_xor(s, d);
        if (pvalid && idx == 0) p.partial[plane] = s;
    }
}

}  // namespace tvk
