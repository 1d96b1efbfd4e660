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

hipError_t launch_conv2d_fbs(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw,
                             float* y, size_t yp, hipStream_t s);
bool has_conv2d_bfs(int kh, int kw);
hipError_t launch_conv2d_bfs(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw,
                             float* y, size_t yp, hipStream_t s);
bool has_conv2d_sbm(int kh, int kw);
hipError_t launch_conv2d_sbm(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw,
                             float* y, size_t yp, hipStream_t s);

hipError_t launch_copy_f32(const float* src, float* dst, size_t n, hipStream_t s);

}  // namespace sysconv
