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

}  // namespace

hipError_t launch_copy_f32(const float* src, float* dst, size_t n, hipStream_t s)
{
    const long long per_block = (long long)kCopyGroups * kBlock * kTile;
    const long long blocks = ((long long)n + per_block - 1) / per_block;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(copy_f32_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, s, src, dst, (long long)n);
    return hipGetLastError();
}

}  // namespace sysconv
