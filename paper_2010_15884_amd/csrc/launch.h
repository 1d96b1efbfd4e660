// Internal launch interface between the C-ABI layer (api.hip) and the kernel
// translation units.  Arguments are already validated; every function only
// enqueues work on `stream` and returns the launch status.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>

namespace sysconv {

constexpr int kMaxK1D = 64;
constexpr int kMaxK2D = 15;

// Tap blocks travel by value in the kernel-argument segment (uniform scalar
// loads, no device allocation).  Padded so that a block of four taps can
// always be fetched.
constexpr int kTaps1DLen = kMaxK1D + 12;      // room for a 3-tap lead-in and a 7-wide fetch at the end
struct Taps1D { float w[kTaps1DLen]; };
constexpr int kTaps2DLen = kMaxK2D * kMaxK2D + 7;
struct Taps2D { float f[kTaps2DLen]; };


hipError_t launch_conv1d_fbs(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s);
hipError_t launch_conv1d_sbm(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s);
hipError_t launch_conv1d_bsm(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s);
hipError_t launch_conv1d_fsm(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s);
hipError_t launch_conv1d_ffs(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s);
hipError_t launch_conv1d_fbs_stride2(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s);
bool has_conv1d_bfs(int k);
hipError_t launch_conv1d_bfs(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s);

// Generic space-time-transform kernel (conv1d_stt.hip).  A plan is what the host derives
// from a design: the transform, its inverse's sign, the chunk of outputs one wavefront
// takes, the lowest PE / time coordinates, and per passed variable its dependence and
// the space (dl = P.e) and time (dt = s.e) distance it travels.
constexpr int kSttDepth = 3;                  // longest time distance a passed value may travel
struct SttPlan {
    int p0, p1, s0, s1, det;
    int chunk, pe_min, time_min, steps;
    int x_on, x_ec, x_eq, x_dl, x_dt;
    int w_on, w_ec, w_dl, w_dt;
    int z_eq, z_dl, z_dt;
};
enum SttVerdict {
    kSttOk = 0,
    kSttBadDependence,        // a dependence vector does not fit the convolution recurrences
    kSttSingular,             // det(P; s) = 0: two iteration points on one PE at one time
    kSttNotCausal,            // s.e < 1 for a passed variable
    kSttTooLarge              // valid, but outside what the kernel is built for
};
SttVerdict plan_stt(const int alloc[2], const int sched[2], bool x_on, const int ex[2], bool w_on, const int ew[2],
                    const int ez[2], int k, SttPlan* out);
hipError_t launch_conv1d_stt(const float* x, size_t n, const float* w, int k, float* y, const SttPlan& plan,
                             hipStream_t s);

hipError_t launch_conv2d_fbs(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw,
                             float* y, size_t yp, hipStream_t s);
hipError_t launch_conv2d_fbs_stride2(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw,
                                     float* y, size_t yp, hipStream_t s);
bool has_conv2d_fbs_static(int kh, int kw);      // sizes the FBS tile kernel is specialised for
bool has_conv2d_bfs(int kh, int kw);
hipError_t launch_conv2d_bfs(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw,
                             float* y, size_t yp, hipStream_t s);
bool has_conv2d_sbm(int kh, int kw);
hipError_t launch_conv2d_sbm(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw,
                             float* y, size_t yp, hipStream_t s);

// Matrix-core path (conv2d_mfma.hip): any filter up to 13 x 13.
bool has_conv2d_mfma(int kh, int kw);
bool conv2d_mfma_taps_in_range(const float* f, int n);      // largest |f| is 0 or within [1e-30, 1e30]
hipError_t launch_conv2d_mfma(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw,
                              float* y, size_t yp, hipStream_t s);

hipError_t launch_copy_f32(const float* src, float* dst, size_t n, hipStream_t s);
hipError_t launch_alu_yardstick(float* out, int workgroups, int trips, hipStream_t s);
long long alu_yardstick_fmas(int workgroups, int trips);

}  // namespace sysconv
