/*
 * CPU oracle for the total-variation proximal operator (TEST INFRASTRUCTURE ONLY).
 *
 * Plain double-precision C.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call this; the product path (the HIP library) shares no
 * code with it and never falls back to it.
 *
 * Naming follows the build's convention: y = input row, x = output row,
 * lam = lambda >= 0, N = row length.  (The paper's Eq. 1 writes the input as x
 * and the output as y; only the letters differ.)
 *
 *   x* = argmin_x 1/2 ||x - y||^2 + lam * sum_k |x[k+1] - x[k]|        (paper Eq. 1)
 *
 * Forward: the minimiser is unique (strictly convex), so the oracle computes it
 * by an exact direct method (Condat's 2013 taut-string style scan) rather than by
 * the iterative projected-Newton method the GPU path uses.  It is pinned in
 * tests/ by brute force over sign patterns, closed forms, invariants and a
 * duality-gap certificate.
 *
 * Backward: paper Eq. 5-6.  The columns of the lower-triangular all-ones matrix
 * selected by the jump set (plus the constant column) span the vectors that are
 * constant on the segments of x*, so M L^T is the orthogonal projector onto
 * them: the gradient w.r.t. y is the upstream gradient averaged per segment,
 * and the gradient w.r.t. lam is sum over segments of
 * mean(g_up) * (sign of right jump - sign of left jump).
 *
 * 2D: K sweeps of the proximal Dykstra iteration of paper Alg. 1 (rows, then
 * columns, with correction terms P and Q), and the hand-derived reverse sweep
 * that replaces autograd through Alg. 1.
 */
#include <stdlib.h>
#include <string.h>
#include <math.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------- */
/* 1D forward: exact minimiser of paper Eq. 1 for one row.                    */
/* y, x: n doubles with element stride `es` (in doubles).  Returns 0, or      */
/* nonzero for invalid arguments (n < 1 or lam < 0 or not finite).            */
/* ------------------------------------------------------------------------- */
static void fill(double *x, long es, long a, long b, double v)
{
    for (long i = a; i <= b; ++i) x[i * es] = v;
}

int tvo_prox1d(const double *y, double *x, long n, long es, double lam)
{
    if (n < 1 || !(lam >= 0.0) || isinf(lam)) return 1;
    if (n == 1) { x[0] = y[0]; return 0; }

    /* The scan grows one segment [k0 .. k] at a time.  lo / hi are the lowest
     * and highest value the segment could still take; ulo / uhi are the values
     * the (sign-flipped) dual would have at k if the segment took lo / hi;
     * klo / khi are the last positions at which ulo / uhi sat on their bound,
     * i.e. where the segment would have to end if lo / hi became binding.     */
    long k = 0, k0 = 0, klo = 0, khi = 0;
    double lo = y[0] - lam, hi = y[0] + lam;
    double ulo = lam, uhi = -lam;

    for (;;) {
        if (k == n - 1) {
            /* End of the row: the dual must return to zero. */
            if (ulo < 0.0) {
                /* lo is too high to close the row: the segment ends at klo
                 * with value lo and the signal jumps down after it. */
                fill(x, es, k0, klo, lo);
                k = k0 = klo = klo + 1;
                lo = y[k * es];
                ulo = lam;
                uhi = y[k * es] + lam - hi;
            } else if (uhi > 0.0) {
                /* hi is too low: segment ends at khi with value hi, jump up. */
                fill(x, es, k0, khi, hi);
                k = k0 = khi = khi + 1;
                hi = y[k * es];
                uhi = -lam;
                ulo = y[k * es] - lam - lo;
            } else {
                /* A common value closes the row with zero dual at the end. */
                fill(x, es, k0, n - 1, lo + ulo / (double)(k - k0 + 1));
                return 0;
            }
        } else {
            double ynext = y[(k + 1) * es];
            if (ynext + ulo < lo - lam) {
                /* Next sample is so low that even lo cannot follow: negative jump. */
                fill(x, es, k0, klo, lo);
                k = k0 = klo = khi = klo + 1;
                lo = y[k * es];
                hi = y[k * es] + 2.0 * lam;
                ulo = lam;
                uhi = -lam;
            } else if (ynext + uhi > hi + lam) {
                /* Next sample is so high that even hi cannot follow: positive jump. */
                fill(x, es, k0, khi, hi);
                k = k0 = klo = khi = khi + 1;
                hi = y[k * es];
                lo = y[k * es] - 2.0 * lam;
                ulo = lam;
                uhi = -lam;
            } else {
                /* Extend the segment by one sample and tighten lo / hi. */
                k += 1;
                ulo += y[k * es] - lo;
                uhi += y[k * es] - hi;
                if (ulo >= lam) {
                    lo += (ulo - lam) / (double)(k - k0 + 1);
                    ulo = lam;
                    klo = k;
                }
                if (uhi <= -lam) {
                    hi += (uhi + lam) / (double)(k - k0 + 1);
                    uhi = -lam;
                    khi = k;
                }
            }
        }
    }
}

/* ------------------------------------------------------------------------- */
/* 1D backward for one row (paper Eq. 5-6 as segment averaging).              */
/* g: upstream gradient, x: the forward OUTPUT (segments = maximal runs of    */
/* exactly equal neighbours).  gy receives dL/dy.  Returns this row's         */
/* contribution to dL/dlam.                                                   */
/* ------------------------------------------------------------------------- */
static double sgn(double v) { return (v > 0.0) - (v < 0.0); }

double tvo_prox1d_bwd(const double *g, const double *x, double *gy, long n, long es)
{
    double glam = 0.0;
    long a = 0;
    while (a < n) {
        long b = a;
        double s = g[a * es];
        while (b + 1 < n && x[(b + 1) * es] == x[b * es]) { b += 1; s += g[b * es]; }
        double mean = s / (double)(b - a + 1);
        for (long i = a; i <= b; ++i) gy[i * es] = mean;
        double s_left  = (a > 0)     ? sgn(x[a * es] - x[(a - 1) * es]) : 0.0;
        double s_right = (b + 1 < n) ? sgn(x[(b + 1) * es] - x[b * es]) : 0.0;
        glam += mean * (s_right - s_left);
        a = b + 1;
    }
    return glam;
}

/* ------------------------------------------------------------------------- */
/* Batched 1D calls over a strided set of rows.                               */
/* row id r = outer * n_inner + inner lives at                                */
/*   base + outer*outer_stride + inner*inner_stride, element stride es.       */
/* lambda slot of row r = (r / lam_div) % lam_count.                          */
/* ------------------------------------------------------------------------- */
int tvo_prox1d_batch(const double *y, double *x,
                     long n_outer, long outer_stride, long n_inner, long inner_stride,
                     long n, long es, const double *lam, long lam_count, long lam_div)
{
    long rows = n_outer * n_inner;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(|:bad)
    for (long r = 0; r < rows; ++r) {
        long off = (r / n_inner) * outer_stride + (r % n_inner) * inner_stride;
        double l = lam[(r / lam_div) % lam_count];
        bad |= tvo_prox1d(y + off, x + off, n, es, l);
    }
    return bad;
}

/* grad_lam (lam_count doubles) is ACCUMULATED into; the caller zeroes it.    */
void tvo_prox1d_bwd_batch(const double *g, const double *x, double *gy, double *grad_lam,
                          long n_outer, long outer_stride, long n_inner, long inner_stride,
                          long n, long es, long lam_count, long lam_div)
{
    long rows = n_outer * n_inner;
    double *part = (double *)malloc(sizeof(double) * (size_t)(rows > 0 ? rows : 1));
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        long off = (r / n_inner) * outer_stride + (r % n_inner) * inner_stride;
        part[r] = tvo_prox1d_bwd(g + off, x + off, gy + off, n, es);
    }
    if (grad_lam)
        for (long r = 0; r < rows; ++r) grad_lam[(r / lam_div) % lam_count] += part[r];
    free(part);
}

/* ------------------------------------------------------------------------- */
/* 2D: K sweeps of paper Alg. 1 over `planes` images of H x W (row-major).    */
/* lam slot of a plane = plane % lam_count.                                   */
/* saved (may be NULL): 2*K*planes*H*W doubles; pass 2k holds Z^(k) (row-pass */
/* output), pass 2k+1 holds Y^(k+1) (column-pass output) -- what the reverse  */
/* sweep needs.                                                               */
/* ------------------------------------------------------------------------- */
int tvo_prox2d_fwd(const double *y, double *x, long planes, long H, long W,
                   const double *lam, long lam_count, int K, double *saved)
{
    long hw = H * W, tot = planes * hw;
    double *Y = (double *)malloc(sizeof(double) * (size_t)tot);
    double *P = (double *)calloc((size_t)tot, sizeof(double));
    double *Q = (double *)calloc((size_t)tot, sizeof(double));
    double *A = (double *)malloc(sizeof(double) * (size_t)tot);
    double *Z = (double *)malloc(sizeof(double) * (size_t)tot);
    int bad = 0;
    memcpy(Y, y, sizeof(double) * (size_t)tot);
    for (int k = 0; k < K; ++k) {
        /* Z = proxRows(Y + P);  P += Y - Z */
        for (long i = 0; i < tot; ++i) A[i] = Y[i] + P[i];
        bad |= tvo_prox1d_batch(A, Z, planes, hw, H, W, W, 1, lam, lam_count, H);
        for (long i = 0; i < tot; ++i) P[i] = A[i] - Z[i];
        if (saved) memcpy(saved + (size_t)(2 * k) * tot, Z, sizeof(double) * (size_t)tot);
        /* Y = proxCols(Z + Q);  Q += Z - Y */
        for (long i = 0; i < tot; ++i) A[i] = Z[i] + Q[i];
        bad |= tvo_prox1d_batch(A, Y, planes, hw, W, 1, H, W, lam, lam_count, W);
        for (long i = 0; i < tot; ++i) Q[i] = A[i] - Y[i];
        if (saved) memcpy(saved + (size_t)(2 * k + 1) * tot, Y, sizeof(double) * (size_t)tot);
    }
    memcpy(x, Y, sizeof(double) * (size_t)tot);
    free(Y); free(P); free(Q); free(A); free(Z);
    return bad;
}

/* Reverse sweep through Alg. 1.  grad_lam (lam_count doubles) is overwritten. */
void tvo_prox2d_bwd(const double *g_up, double *grad_y, double *grad_lam,
                    long planes, long H, long W, long lam_count, int K, const double *saved)
{
    long hw = H * W, tot = planes * hw;
    double *Yb = (double *)malloc(sizeof(double) * (size_t)tot);
    double *Pb = (double *)calloc((size_t)tot, sizeof(double));
    double *Qb = (double *)calloc((size_t)tot, sizeof(double));
    double *T  = (double *)malloc(sizeof(double) * (size_t)tot);
    double *R  = (double *)malloc(sizeof(double) * (size_t)tot);
    memcpy(Yb, g_up, sizeof(double) * (size_t)tot);
    for (long s = 0; s < lam_count; ++s) grad_lam[s] = 0.0;
    for (int k = K - 1; k >= 0; --k) {
        const double *Ycol = saved + (size_t)(2 * k + 1) * tot;   /* Y^(k+1) */
        const double *Zrow = saved + (size_t)(2 * k) * tot;       /* Z^(k)   */
        /* Q' = B - Y', Y' = proxCols(B), B = Z + Q */
        for (long i = 0; i < tot; ++i) T[i] = Yb[i] - Qb[i];
        tvo_prox1d_bwd_batch(T, Ycol, R, grad_lam, planes, hw, W, 1, H, W, lam_count, W);
        for (long i = 0; i < tot; ++i) { R[i] += Qb[i]; Qb[i] = R[i]; }   /* R = B-bar */
        /* P' = A - Z, Z = proxRows(A), A = Y + P */
        for (long i = 0; i < tot; ++i) T[i] = R[i] - Pb[i];
        tvo_prox1d_bwd_batch(T, Zrow, R, grad_lam, planes, hw, H, W, W, 1, lam_count, H);
        for (long i = 0; i < tot; ++i) { R[i] += Pb[i]; Yb[i] = R[i]; Pb[i] = R[i]; }
    }
    memcpy(grad_y, Yb, sizeof(double) * (size_t)tot);
    free(Yb); free(Pb); free(Qb); free(T); free(R);
}

int tvo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Thread count of the batch loops from now on (timing only: the arithmetic per row does not
 * depend on it).  n < 1 is ignored. */
void tvo_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
