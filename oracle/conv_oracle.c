/*
 * conv_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * Plain, slow, obviously-correct CPU evaluation of the two definitions the
 * paper's systolic designs all compute:
 *
 *   1-D (paper Eq. 2, Section 3.1):   Z(c)   = sum_q          x(c+q)     * w(q)
 *   2-D (paper Eq. 3, Section 5):     Z(c,r) = sum_q sum_p    x(c+q,r+p) * w(q,p)
 *
 * and the strided 1-D form that the stride-2 FBS design of Table 2 (row 3 right)
 * computes:                            Z(c)   = sum_q          x(S*c+q)   * w(q)
 * and its 2-D analogue (the stride of the paper's Section 6 experiment applied to
 * both axes):                          Z(c,r) = sum_q sum_p    x(S*c+q,S*r+p) * w(q,p)
 *
 * Readings taken where the paper is silent:
 *   - no filter flip (the equations index x(c+q), so this is cross-correlation);
 *   - "valid" extent: the recurrences load x(c+q) for c = C-1, q = Q-1, so the
 *     input has C+Q-1 elements and there is no padding;
 *   - stride S: the table prints x(c+q) for the stride-2 design too, but its
 *     dependence X(c,q) = X(c+1,q-2) only holds for x(2c+q) (x(2(c+1)+q-2) is the
 *     same element), so that is the definition taken; outputs exist for every c
 *     with S*c + k - 1 < n, i.e. floor((n-k)/S) + 1 of them;
 *   - the paper's fast (systolic) axis c,q is the column of a row-major image
 *     and r,p is the row:  y[r][c] = sum_p sum_q f[p][q] * x[r+p][c+q].
 *
 * Inputs are fp32 (the paper's data type); every product and sum is taken in
 * fp64, so each product is exact and the only rounding is in the additions.
 * Loop order is the definition's: taps ascending, rows of the filter outer.
 * There is no blocking, no vector code and no reordering here on purpose.
 *
 * Nothing in the GPU library includes, links or calls this file.  Only the
 * tests, the smoke check and the benchmark's CPU-baseline leg may use it.
 *
 * Threads: the loop over outputs may be split with OpenMP (every output is
 * independent, so the result does not depend on the thread count).
 */
#include <stddef.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Status codes of this file only. */
enum { ORACLE_OK = 0, ORACLE_BAD_ARG = 1 };

static int clamp_threads(int nthreads)
{
    if (nthreads < 1) nthreads = 1;
#ifdef _OPENMP
    return nthreads;
#else
    return 1;
#endif
}

/* How many threads a call with this request would really use. */
int oracle_threads(int nthreads)
{
    return clamp_threads(nthreads);
}

/*
 * Eq. 2.  x: n floats, w: k floats, y: n-k+1 doubles.
 */
int oracle_conv1d(const float *x, size_t n, const float *w, int k,
                  double *y, int nthreads)
{
    if (!x || !w || !y || k < 1 || (size_t)k > n) return ORACLE_BAD_ARG;
    const long long m = (long long)(n - (size_t)k + 1);
    const int nt = clamp_threads(nthreads);
    (void)nt;
#ifdef _OPENMP
#pragma omp parallel for num_threads(nt) schedule(static)
#endif
    for (long long c = 0; c < m; ++c) {
        double z = 0.0;
        for (int q = 0; q < k; ++q)
            z += (double)x[c + q] * (double)w[q];
        y[c] = z;
    }
    return ORACLE_OK;
}

/*
 * Strided Eq. 2 (Table 2, row 3 right, read with x(S*c+q)).
 * x: n floats, w: k floats, y: (n-k)/stride + 1 doubles.  stride 1 is Eq. 2.
 */
int oracle_conv1d_strided(const float *x, size_t n, const float *w, int k, int stride,
                          double *y, int nthreads)
{
    if (!x || !w || !y || k < 1 || (size_t)k > n || stride < 1) return ORACLE_BAD_ARG;
    const long long m = (long long)((n - (size_t)k) / (size_t)stride + 1);
    const int nt = clamp_threads(nthreads);
    (void)nt;
#ifdef _OPENMP
#pragma omp parallel for num_threads(nt) schedule(static)
#endif
    for (long long c = 0; c < m; ++c) {
        double z = 0.0;
        for (int q = 0; q < k; ++q)
            z += (double)x[(long long)stride * c + q] * (double)w[q];
        y[c] = z;
    }
    return ORACLE_OK;
}

/*
 * Eq. 3.  x: h rows of w_img floats, row stride x_pitch elements.
 * f: kh*kw floats, row-major.  y: (h-kh+1) rows of (w_img-kw+1) doubles,
 * row stride y_pitch elements.
 */
int oracle_conv2d(const float *x, int h, int w_img, size_t x_pitch,
                  const float *f, int kh, int kw,
                  double *y, size_t y_pitch, int nthreads)
{
    if (!x || !f || !y || kh < 1 || kw < 1 || kh > h || kw > w_img) return ORACLE_BAD_ARG;
    if (x_pitch < (size_t)w_img) return ORACLE_BAD_ARG;
    const int oh = h - kh + 1;
    const int ow = w_img - kw + 1;
    if (y_pitch < (size_t)ow) return ORACLE_BAD_ARG;
    const int nt = clamp_threads(nthreads);
    (void)nt;
#ifdef _OPENMP
#pragma omp parallel for num_threads(nt) schedule(static)
#endif
    for (int r = 0; r < oh; ++r) {
        for (int c = 0; c < ow; ++c) {
            double z = 0.0;
            for (int p = 0; p < kh; ++p)
                for (int q = 0; q < kw; ++q)
                    z += (double)x[(size_t)(r + p) * x_pitch + (size_t)(c + q)]
                       * (double)f[p * kw + q];
            y[(size_t)r * y_pitch + (size_t)c] = z;
        }
    }
    return ORACLE_OK;
}

/*
 * Strided Eq. 3: y[r][c] = sum_p sum_q f[p][q] * x[S*r+p][S*c+q], the same stride on both
 * axes; (h-kh)/S + 1 rows of (w_img-kw)/S + 1 outputs.  stride 1 is Eq. 3.
 */
int oracle_conv2d_strided(const float *x, int h, int w_img, size_t x_pitch,
                          const float *f, int kh, int kw, int stride,
                          double *y, size_t y_pitch, int nthreads)
{
    if (!x || !f || !y || kh < 1 || kw < 1 || kh > h || kw > w_img || stride < 1) return ORACLE_BAD_ARG;
    if (x_pitch < (size_t)w_img) return ORACLE_BAD_ARG;
    const int oh = (h - kh) / stride + 1;
    const int ow = (w_img - kw) / stride + 1;
    if (y_pitch < (size_t)ow) return ORACLE_BAD_ARG;
    const int nt = clamp_threads(nthreads);
    (void)nt;
#ifdef _OPENMP
#pragma omp parallel for num_threads(nt) schedule(static)
#endif
    for (int r = 0; r < oh; ++r) {
        for (int c = 0; c < ow; ++c) {
            double z = 0.0;
            for (int p = 0; p < kh; ++p)
                for (int q = 0; q < kw; ++q)
                    z += (double)x[(size_t)(stride * r + p) * x_pitch + (size_t)(stride * c + q)]
                       * (double)f[p * kw + q];
            y[(size_t)r * y_pitch + (size_t)c] = z;
        }
    }
    return ORACLE_OK;
}

int oracle_absdot2d_strided(const float *x, int h, int w_img, size_t x_pitch,
                            const float *f, int kh, int kw, int stride,
                            double *s, size_t s_pitch, int nthreads)
{
    if (!x || !f || !s || kh < 1 || kw < 1 || kh > h || kw > w_img || stride < 1) return ORACLE_BAD_ARG;
    if (x_pitch < (size_t)w_img) return ORACLE_BAD_ARG;
    const int oh = (h - kh) / stride + 1;
    const int ow = (w_img - kw) / stride + 1;
    if (s_pitch < (size_t)ow) return ORACLE_BAD_ARG;
    const int nt = clamp_threads(nthreads);
    (void)nt;
#ifdef _OPENMP
#pragma omp parallel for num_threads(nt) schedule(static)
#endif
    for (int r = 0; r < oh; ++r) {
        for (int c = 0; c < ow; ++c) {
            double z = 0.0;
            for (int p = 0; p < kh; ++p)
                for (int q = 0; q < kw; ++q) {
                    double xv = (double)x[(size_t)(stride * r + p) * x_pitch + (size_t)(stride * c + q)];
                    double wv = (double)f[p * kw + q];
                    z += (xv < 0 ? -xv : xv) * (wv < 0 ? -wv : wv);
                }
            s[(size_t)r * s_pitch + (size_t)c] = z;
        }
    }
    return ORACLE_OK;
}

/*
 * The scale the parity metric divides by:  sum |w||x| over the same window,
 * also in fp64.  Written out separately (not by calling the functions above
 * on pre-processed data) so the metric can be read by eye.
 */
int oracle_absdot1d(const float *x, size_t n, const float *w, int k,
                    double *s, int nthreads)
{
    if (!x || !w || !s || k < 1 || (size_t)k > n) return ORACLE_BAD_ARG;
    const long long m = (long long)(n - (size_t)k + 1);
    const int nt = clamp_threads(nthreads);
    (void)nt;
#ifdef _OPENMP
#pragma omp parallel for num_threads(nt) schedule(static)
#endif
    for (long long c = 0; c < m; ++c) {
        double z = 0.0;
        for (int q = 0; q < k; ++q) {
            double xv = (double)x[c + q], wv = (double)w[q];
            z += (xv < 0 ? -xv : xv) * (wv < 0 ? -wv : wv);
        }
        s[c] = z;
    }
    return ORACLE_OK;
}

int oracle_absdot1d_strided(const float *x, size_t n, const float *w, int k, int stride,
                            double *s, int nthreads)
{
    if (!x || !w || !s || k < 1 || (size_t)k > n || stride < 1) return ORACLE_BAD_ARG;
    const long long m = (long long)((n - (size_t)k) / (size_t)stride + 1);
    const int nt = clamp_threads(nthreads);
    (void)nt;
#ifdef _OPENMP
#pragma omp parallel for num_threads(nt) schedule(static)
#endif
    for (long long c = 0; c < m; ++c) {
        double z = 0.0;
        for (int q = 0; q < k; ++q) {
            double xv = (double)x[(long long)stride * c + q], wv = (double)w[q];
            z += (xv < 0 ? -xv : xv) * (wv < 0 ? -wv : wv);
        }
        s[c] = z;
    }
    return ORACLE_OK;
}

int oracle_absdot2d(const float *x, int h, int w_img, size_t x_pitch,
                    const float *f, int kh, int kw,
                    double *s, size_t s_pitch, int nthreads)
{
    if (!x || !f || !s || kh < 1 || kw < 1 || kh > h || kw > w_img) return ORACLE_BAD_ARG;
    if (x_pitch < (size_t)w_img) return ORACLE_BAD_ARG;
    const int oh = h - kh + 1;
    const int ow = w_img - kw + 1;
    if (s_pitch < (size_t)ow) return ORACLE_BAD_ARG;
    const int nt = clamp_threads(nthreads);
    (void)nt;
#ifdef _OPENMP
#pragma omp parallel for num_threads(nt) schedule(static)
#endif
    for (int r = 0; r < oh; ++r) {
        for (int c = 0; c < ow; ++c) {
            double z = 0.0;
            for (int p = 0; p < kh; ++p)
                for (int q = 0; q < kw; ++q) {
                    double xv = (double)x[(size_t)(r + p) * x_pitch + (size_t)(c + q)];
                    double wv = (double)f[p * kw + q];
                    z += (xv < 0 ? -xv : xv) * (wv < 0 ? -wv : wv);
                }
            s[(size_t)r * s_pitch + (size_t)c] = z;
        }
    }
    return ORACLE_OK;
}
