/*
 * san_driver.c -- TEST INFRASTRUCTURE: runs every routine of conv_oracle.c on heap buffers of
 * exactly the size the routines are entitled to touch, so that a build with
 * -fsanitize=address,undefined turns any read or write outside them, any signed overflow and
 * any misaligned or invalid access into a failure.  A few results are compared with
 * hand-expanded sums as well (the same ones the Python pins use), so that the sanitized build is
 * known to compute and not only to run.
 *
 *   gcc -std=c99 -g -O1 -fopenmp -fsanitize=address,undefined -fno-sanitize-recover=all \
 *       -static-libasan oracle/conv_oracle.c oracle/san_driver.c -o san_driver && ./san_driver
 *
 * Exit status 0 = clean.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_conv1d(const float *x, size_t n, const float *w, int k, double *y, int nthreads);
int oracle_absdot1d(const float *x, size_t n, const float *w, int k, double *s, int nthreads);
int oracle_conv1d_strided(const float *x, size_t n, const float *w, int k, int stride, double *y, int nthreads);
int oracle_absdot1d_strided(const float *x, size_t n, const float *w, int k, int stride, double *s, int nthreads);
int oracle_conv2d(const float *x, int h, int w_img, size_t x_pitch, const float *f, int kh, int kw,
                  double *y, size_t y_pitch, int nthreads);
int oracle_absdot2d(const float *x, int h, int w_img, size_t x_pitch, const float *f, int kh, int kw,
                    double *s, size_t s_pitch, int nthreads);
int oracle_conv2d_strided(const float *x, int h, int w_img, size_t x_pitch, const float *f, int kh, int kw, int stride,
                          double *y, size_t y_pitch, int nthreads);
int oracle_absdot2d_strided(const float *x, int h, int w_img, size_t x_pitch, const float *f, int kh, int kw,
                            int stride, double *s, size_t s_pitch, int nthreads);
int oracle_threads(int nthreads);

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

static float *ramp(size_t n, float scale)
{
    float *p = (float *)malloc(n * sizeof(float));
    for (size_t i = 0; i < n; ++i) p[i] = scale * (float)((int)(i % 17) - 8);
    return p;
}

static void run_1d(size_t n, int k, int stride, int threads)
{
    float *x = ramp(n, 0.25f), *w = ramp((size_t)k, 0.5f);
    const size_t m = (n - (size_t)k) / (size_t)stride + 1;
    double *y = (double *)malloc(m * sizeof(double)), *s = (double *)malloc(m * sizeof(double));
    if (stride == 1) {
        CHECK(oracle_conv1d(x, n, w, k, y, threads) == 0);
        CHECK(oracle_absdot1d(x, n, w, k, s, threads) == 0);
    }
    CHECK(oracle_conv1d_strided(x, n, w, k, stride, y, threads) == 0);
    CHECK(oracle_absdot1d_strided(x, n, w, k, stride, s, threads) == 0);
    for (size_t c = 0; c < m; ++c) CHECK(fabs(y[c]) <= s[c]);               /* |sum| <= sum of magnitudes */
    free(x); free(w); free(y); free(s);
}

static void run_2d(int h, int w_img, size_t xp, int kh, int kw, int stride, size_t ypad, int threads)
{
    float *x = ramp((size_t)(h - 1) * xp + (size_t)w_img, 0.125f);          /* the last row ends at its last element */
    float *f = ramp((size_t)kh * kw, 0.5f);
    const int oh = (h - kh) / stride + 1, ow = (w_img - kw) / stride + 1;
    const size_t yp = (size_t)ow + ypad;
    const size_t ylen = (size_t)(oh - 1) * yp + (size_t)ow;
    double *y = (double *)malloc(ylen * sizeof(double)), *s = (double *)malloc(ylen * sizeof(double));
    if (stride == 1) {
        CHECK(oracle_conv2d(x, h, w_img, xp, f, kh, kw, y, yp, threads) == 0);
        CHECK(oracle_absdot2d(x, h, w_img, xp, f, kh, kw, s, yp, threads) == 0);
    }
    CHECK(oracle_conv2d_strided(x, h, w_img, xp, f, kh, kw, stride, y, yp, threads) == 0);
    CHECK(oracle_absdot2d_strided(x, h, w_img, xp, f, kh, kw, stride, s, yp, threads) == 0);
    for (int r = 0; r < oh; ++r)
        for (int c = 0; c < ow; ++c) CHECK(fabs(y[(size_t)r * yp + c]) <= s[(size_t)r * yp + c]);
    free(x); free(f); free(y); free(s);
}

int main(void)
{
    /* hand-expanded sums: Eq. 2 with asymmetric taps, Eq. 3 with an asymmetric 2 x 2 filter, the scale of a 2 x 3 filter */
    {
        const float x[5] = {1, 2, 4, 8, 16}, w[3] = {3, 0, -1};
        double y[3];
        CHECK(oracle_conv1d(x, 5, w, 3, y, 1) == 0);
        CHECK(y[0] == -1 && y[1] == -2 && y[2] == -4);
        const float img[9] = {1, 2, 3, 4, 5, 6, 7, 8, 9}, f[4] = {1, 2, 3, 4};
        double z[4];
        CHECK(oracle_conv2d(img, 3, 3, 3, f, 2, 2, z, 2, 1) == 0);
        CHECK(z[0] == 37 && z[1] == 47 && z[2] == 67 && z[3] == 77);
        const float im2[12] = {1, -2, 3, -4, -5, 6, -7, 8, 9, -10, 11, -12}, f2[6] = {1, -2, 3, -4, 5, -6};
        double a[4];
        CHECK(oracle_absdot2d(im2, 3, 4, 4, f2, 2, 3, a, 2, 1) == 0);
        CHECK(a[0] == 106 && a[1] == 127 && a[2] == 190 && a[3] == 211);
    }
    /* sizes around the edges of the definition: one output, k == n, strides that leave a ragged rest */
    const int threads[2] = {1, 3};
    for (int t = 0; t < 2; ++t) {
        run_1d(1, 1, 1, threads[t]);
        run_1d(64, 64, 1, threads[t]);
        run_1d(1000, 5, 1, threads[t]);
        run_1d(1001, 16, 2, threads[t]);
        run_1d(1002, 7, 3, threads[t]);
        run_1d(9, 9, 2, threads[t]);
        run_2d(1, 1, 1, 1, 1, 1, 0, threads[t]);
        run_2d(15, 15, 15, 15, 15, 1, 0, threads[t]);
        run_2d(37, 53, 53, 5, 5, 1, 0, threads[t]);
        run_2d(37, 53, 61, 3, 11, 1, 7, threads[t]);                        /* pitches wider than the rows */
        run_2d(40, 41, 41, 11, 11, 2, 0, threads[t]);
        run_2d(23, 31, 40, 4, 6, 2, 3, threads[t]);
        run_2d(13, 19, 19, 3, 5, 3, 1, threads[t]);
    }
    /* argument errors are statuses, not accesses */
    {
        float x[4] = {0, 0, 0, 0}, w[5] = {0, 0, 0, 0, 0};
        double y[4];
        CHECK(oracle_conv1d(x, 4, w, 5, y, 1) != 0);
        CHECK(oracle_conv1d(NULL, 4, w, 1, y, 1) != 0);
        CHECK(oracle_conv1d_strided(x, 4, w, 2, 0, y, 1) != 0);
        CHECK(oracle_conv2d(x, 2, 2, 1, w, 1, 1, y, 2, 1) != 0);             /* pitch narrower than the image */
        CHECK(oracle_conv2d(x, 2, 2, 2, w, 3, 1, y, 2, 1) != 0);
        CHECK(oracle_conv2d(x, 2, 2, 2, w, 1, 1, y, 1, 1) != 0);
        CHECK(oracle_threads(0) == 1);
    }
    printf(failures ? "FAILED (%d)\n" : "clean\n", failures);
    return failures ? 1 : 0;
}
