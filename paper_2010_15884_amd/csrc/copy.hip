// Plain streaming copy with dwordx4 accesses: the memory-system yard-stick the
// benchmark prints beside every convolution, and the kernel of known traffic
// that hardware byte counters are calibrated against.
#include "launch.h"
#include "systolic.h"

namespace sysconv {
namespace {

constexpr int kCopyGroups = 4;

__global__ __launch_bounds__(kBlock) void copy_f32_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                          long long n)
{
    const int lane = threadIdx.x & (kWave - 1);
    const long long wave = (long long)blockIdx.x * (kBlock / kWave) + wave_in_block();
    const long long base = wave * kCopyGroups * kWave * kTile + kTile * lane;
    float v[kCopyGroups][4];
#pragma unroll
    for (int r = 0; r < kCopyGroups; ++r) load4_guarded(src, base + (long long)r * kWave * kTile, n, v[r]);
#pragma unroll
    for (int r = 0; r < kCopyGroups; ++r) store4_guarded(dst, base + (long long)r * kWave * kTile, n, v[r]);
}

// Register-only multiply-add loop: what the vector ALUs sustain when nothing else is in the
// way (taps in SGPRs as in the convolution kernels, eight independent partial sums per lane,
// 32 taps per trip).  Every lane stores one value so that the arithmetic cannot be dropped.
constexpr int kAluAcc = 8, kAluTaps = 32;
struct AluTaps { float w[kAluTaps]; };

__global__ __launch_bounds__(kBlock) void alu_yardstick_kernel(float* __restrict__ out, int trips, AluTaps taps)
{
    float acc[kAluAcc], x[8];
#pragma unroll
    for (int i = 0; i < kAluAcc; ++i) acc[i] = threadIdx.x * 0.001f + i;
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = threadIdx.x * 0.5f + i;
    for (int it = 0; it < trips; ++it) {
#pragma unroll
        for (int t = 0; t < kAluTaps; ++t)
#pragma unroll
            for (int i = 0; i < kAluAcc; ++i) acc[i] = __builtin_fmaf(taps.w[t], x[(t + i) & 7], acc[i]);
    }
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < kAluAcc; ++i) sum += acc[i];
    out[(size_t)blockIdx.x * kBlock + threadIdx.x] = sum;
}

}  // namespace

hipError_t launch_alu_yardstick(float* out, int workgroups, int trips, hipStream_t s)
{
    AluTaps taps;
    for (int i = 0; i < kAluTaps; ++i) taps.w[i] = 1.0f + i * 1e-7f;
    hipLaunchKernelGGL(alu_yardstick_kernel, dim3((unsigned)workgroups), dim3(kBlock), 0, s, out, trips, taps);
    return hipGetLastError();
}

long long alu_yardstick_fmas(int workgroups, int trips)
{
    return (long long)workgroups * kBlock * trips * kAluTaps * kAluAcc;
}

hipError_t launch_copy_f32(const float* src, float* dst, size_t n, hipStream_t s)
{
    const long long per_block = (long long)kCopyGroups * kBlock * kTile;
    const long long blocks = ((long long)n + per_block - 1) / per_block;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(copy_f32_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, s, src, dst, (long long)n);
    return hipGetLastError();
}

}  // namespace sysconv
