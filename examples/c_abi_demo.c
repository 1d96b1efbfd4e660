/*
 * Plain-C use of libsysconv through include/sysconv.h: no Python, no torch.
 *
 *   gcc -std=c99 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -I include examples/c_abi_demo.c \
 *       -L paper_2010_15884_amd -lsysconv -L/opt/rocm/lib -lamdhip64 -lm \
 *       -Wl,-rpath,$PWD/paper_2010_15884_amd -Wl,-rpath,/opt/rocm/lib -o c_abi_demo && ./c_abi_demo
 *
 * Runs y = conv1d(x, w) in every projection, at stride 2, and through the generic
 * space-time-transform kernel with a design written down as data; a 5x5 conv2d in every
 * projection; checks everything against sums computed here, and shows the error paths.
 * Exit status 0 = all good.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include <hip/hip_runtime_api.h>

#include "sysconv.h"

#define CHECK_HIP(e) do { hipError_t r_ = (e); if (r_ != hipSuccess) { \
    fprintf(stderr, "HIP error %d at line %d\n", (int)r_, __LINE__); return 2; } } while (0)

/* The library's stated accuracy: every output within 1e-5 of the fp64 sum, measured against the
 * size of the terms that went into it, sum_q |w[q]| |x[stride*c + q]|. */
#define TOL 1e-5

static double worst_rel_err(const float *y, const float *x, size_t n, const float *w, int k, int stride)
{
    double worst = 0;
    for (size_t c = 0; (size_t)stride * c + (size_t)k <= n; ++c) {
        double ref = 0, scale = 0;
        for (int q = 0; q < k; ++q) {
            const double t = (double)w[q] * (double)x[(size_t)stride * c + q];
            ref += t;
            scale += fabs(t);
        }
        const double e = fabs((double)y[c] - ref);
        if (scale == 0) { if (e != 0) return INFINITY; continue; }
        if (e / scale > worst) worst = e / scale;
    }
    return worst;
}

int main(void)
{
    const size_t n = 100003;
    const int k = 7;
    const float w[7] = {0.5f, -1.0f, 2.0f, 0.25f, -0.75f, 1.5f, 3.0f};

    float *hx = (float *)malloc(n * sizeof(float)), *hy = (float *)malloc(n * sizeof(float));
    for (size_t i = 0; i < n; ++i) hx[i] = (float)(i % 1000);      /* sawtooth: exact in fp32 */
    float *dx, *dy;
    CHECK_HIP(hipMalloc((void **)&dx, n * sizeof(float)));
    CHECK_HIP(hipMalloc((void **)&dy, n * sizeof(float)));
    CHECK_HIP(hipMemcpy(dx, hx, n * sizeof(float), hipMemcpyHostToDevice));

    int failures = 0;
    for (int proj = SYS_PROJ_AUTO; proj <= SYS_PROJ_FFS; ++proj) {
        if (!sys_conv1d_has(proj, k)) continue;
        int st = sys_conv1d(dx, n, w, k, dy, proj, 0);
        if (st != SYS_OK) { fprintf(stderr, "conv1d %s: %s\n", sys_projection_name(proj), sys_status_string(st)); return 3; }
        CHECK_HIP(hipDeviceSynchronize());
        CHECK_HIP(hipMemcpy(hy, dy, (n - k + 1) * sizeof(float), hipMemcpyDeviceToHost));
        double worst = worst_rel_err(hy, hx, n, w, k, 1);
        printf("conv1d %-4s n=%zu k=%d: max err / sum|w||x| = %.3g\n", sys_projection_name(proj), n, k, worst);
        if (!(worst <= TOL)) ++failures;
    }

    /* stride 2 (FBS only), and a design given as data to the generic kernel: SBM whose
     * partial sums move every second step (PE = c + q, time = c + 2q), which no table lists */
    {
        const size_t m2 = (n - k) / 2 + 1;
        int st = sys_conv1d_strided(dx, n, w, k, 2, dy, SYS_PROJ_FBS, 0);
        if (st != SYS_OK) { fprintf(stderr, "stride 2: %s\n", sys_status_string(st)); return 3; }
        CHECK_HIP(hipDeviceSynchronize());
        CHECK_HIP(hipMemcpy(hy, dy, m2 * sizeof(float), hipMemcpyDeviceToHost));
        double worst = worst_rel_err(hy, hx, n, w, k, 2);
        printf("conv1d FBS stride 2, %zu outputs: max err / sum|w||x| = %.3g\n", m2, worst);
        if (!(worst <= TOL)) ++failures;

        const sys_stt_design_t half_speed_sbm = {{1, 1}, {1, 2}, 1, {-1, 1}, 0, {0, 0}, {0, 1}};
        const sys_stt_design_t singular = {{1, 1}, {1, 1}, 0, {0, 0}, 0, {0, 0}, {0, 1}};
        printf("half-speed SBM  -> %s\n", sys_status_string(sys_stt_check(&half_speed_sbm, k)));
        printf("singular design -> %s\n", sys_status_string(sys_stt_check(&singular, k)));
        failures += sys_stt_check(&singular, k) != SYS_ERR_DESIGN;
        st = sys_conv1d_stt(dx, n, w, k, dy, &half_speed_sbm, 0);
        if (st != SYS_OK) { fprintf(stderr, "generic kernel: %s\n", sys_status_string(st)); return 3; }
        CHECK_HIP(hipDeviceSynchronize());
        CHECK_HIP(hipMemcpy(hy, dy, (n - k + 1) * sizeof(float), hipMemcpyDeviceToHost));
        worst = worst_rel_err(hy, hx, n, w, k, 1);
        printf("conv1d generic kernel, half-speed SBM: max err / sum|w||x| = %.3g\n", worst);
        if (!(worst <= TOL)) ++failures;
    }

    /* 2-D: 300 x 500 image x[r][c] = r + 2c, 5x5 box filter => y = 25*(r + 2c) + sum(p + 2q) = ... + 150 */
    const int h = 300, wd = 500, kh = 5, kw = 5;
    float f[25];
    for (int i = 0; i < 25; ++i) f[i] = 1.0f;
    float *himg = (float *)malloc((size_t)h * wd * sizeof(float)), *hout = (float *)malloc((size_t)h * wd * sizeof(float));
    for (int r = 0; r < h; ++r) for (int c = 0; c < wd; ++c) himg[r * wd + c] = (float)(r + 2 * c);
    float *dimg, *dout;
    CHECK_HIP(hipMalloc((void **)&dimg, (size_t)h * wd * sizeof(float)));
    CHECK_HIP(hipMalloc((void **)&dout, (size_t)h * wd * sizeof(float)));
    CHECK_HIP(hipMemcpy(dimg, himg, (size_t)h * wd * sizeof(float), hipMemcpyHostToDevice));
    const int oh = h - kh + 1, ow = wd - kw + 1;
    for (int proj = SYS_PROJ_AUTO; proj <= SYS_PROJ_SBM; ++proj) {
        if (!sys_conv2d_has(proj, kh, kw)) continue;
        int st = sys_conv2d(dimg, h, wd, wd, f, kh, kw, dout, ow, proj, 0);
        if (st != SYS_OK) { fprintf(stderr, "conv2d %s: %s\n", sys_projection_name(proj), sys_status_string(st)); return 3; }
        CHECK_HIP(hipDeviceSynchronize());
        CHECK_HIP(hipMemcpy(hout, dout, (size_t)oh * ow * sizeof(float), hipMemcpyDeviceToHost));
        int bad = 0;
        for (int r = 0; r < oh; ++r) for (int c = 0; c < ow; ++c)
            if (hout[r * ow + c] != 25.0f * (r + 2 * c) + 150.0f) ++bad;     /* small integers: exact */
        printf("conv2d %-4s %dx%d 5x5: %d wrong outputs\n", sys_projection_name(proj), h, wd, bad);
        failures += bad != 0;
    }

    /* error paths: nothing is launched, a status comes back */
    printf("k > n           -> %s\n", sys_status_string(sys_conv1d(dx, 3, w, k, dy, SYS_PROJ_FBS, 0)));
    printf("aliasing        -> %s\n", sys_status_string(sys_conv1d(dx, n, w, k, dx + 10, SYS_PROJ_FBS, 0)));
    printf("65 taps         -> %s\n", sys_status_string(sys_conv1d(dx, n, w, 65, dy, SYS_PROJ_FBS, 0)));
    failures += sys_conv1d(dx, 3, w, k, dy, SYS_PROJ_FBS, 0) != SYS_ERR_SIZE;
    failures += sys_conv1d(dx, n, w, k, dx + 10, SYS_PROJ_FBS, 0) != SYS_ERR_ALIAS;

    hipFree(dx); hipFree(dy); hipFree(dimg); hipFree(dout);
    free(hx); free(hy); free(himg); free(hout);
    printf(failures ? "FAILED\n" : "all good\n");
    return failures ? 1 : 0;
}
