// 1-D valid convolution with stride 2,  y[c] = sum_q x[2c+q] * w[q],  as the FBS
// design of the paper's Table 2, row 3 right: PE = c, time = q, partial sums and
// weights stay, and an input is handed one PE down every TWO steps,
// X(c,q) = X(c+1,q-2).  (The table prints x(c+q) as the loaded element; only
// x(2c+q) agrees with that hand-over, so that is what is computed.)
//
// The hand-over rule splits the inputs of a PE into two chains that never mix: the
// even taps see x(2c), x(2c+2), ... and the odd taps x(2c+1), x(2c+3), ...  Each is an
// ordinary stride-1 FBS array over the de-interleaved signal, E(c) = x(2c) resp.
// O(c) = x(2c+1), both adding into the same partial sums.  A lane loads eight
// consecutive inputs (two dwordx4), which are E and O of its four PEs, and the two
// chains then run the stride-1 time steps with the even resp. the odd taps.  The
// chains are independent, so they are issued one after the other (all even steps,
// then all odd steps) rather than alternating.
#include "launch.h"
#include "systolic.h"

namespace sysconv {
namespace {

typedef const float __attribute__((address_space(4)))* kernarg_floats;

constexpr int kGroups = 4;                      // register groups per wavefront
constexpr int kChainLen = kMaxK1D / 2 + 8;      // taps of one chain, zero-padded so a block of four can always be read
struct TapsStride2 { float even[kChainLen]; float odd[kChainLen]; };

template <int NT, bool MORE>
__device__ __forceinline__ void chain_groups(float (&e)[kGroups][4], float (&acc)[kGroups][4], const float (&w)[4])
{
#pragma unroll
    for (int r = 0; r < kGroups; ++r) fbs_steps<NT, MORE>(e[r], acc[r], w);
}

// All kc >= 1 time steps of one chain (KC > 0: count known at compile time).
template <int KC>
__device__ __forceinline__ void run_chain(float (&e)[kGroups][4], float (&acc)[kGroups][4], kernarg_floats w, int kc_rt)
{
    const int kc = KC ? KC : kc_rt;
    int j = 0;
    if (KC) {
#pragma unroll
        for (; j + 4 < kc; j += 4) {
            const float wb[4] = {w[j], w[j + 1], w[j + 2], w[j + 3]};
            chain_groups<4, true>(e, acc, wb);
        }
    } else {
#pragma nounroll
        for (; j + 4 < kc; j += 4) {
            const float wb[4] = {w[j], w[j + 1], w[j + 2], w[j + 3]};
            chain_groups<4, true>(e, acc, wb);
        }
    }
    const float wb[4] = {w[j], w[j + 1], w[j + 2], w[j + 3]};
    switch (kc - j) {                           // uniform across the wavefront
    case 4: chain_groups<4, false>(e, acc, wb); break;
    case 3: chain_groups<3, false>(e, acc, wb); break;
    case 2: chain_groups<2, false>(e, acc, wb); break;
    default: chain_groups<1, false>(e, acc, wb); break;
    }
}

// The taps are the first kernel argument (offset 0 of the kernel-argument segment).
template <int KT>
__global__ __launch_bounds__(kBlock) void conv1d_fbs_stride2_kernel(TapsStride2 taps, const float* __restrict__ x,
                                                                    float* __restrict__ y, long long n, long long m,
                                                                    int k_rt, int valid_lanes)
{
    (void)taps;
    kernarg_floats tw = (kernarg_floats)__builtin_amdgcn_kernarg_segment_ptr();
    const int k = KT ? KT : k_rt;
    const int lane = threadIdx.x & (kWave - 1);
    const long long per_group = (long long)kTile * valid_lanes;            // outputs a group yields
    const long long wave = (long long)blockIdx.x * (kBlock / kWave) + wave_in_block();
    const long long base = wave * kGroups * per_group;                     // first output of the wavefront
    if (base >= m) return;                                                 // uniform per wavefront

    float ev[kGroups][4], od[kGroups][4], acc[kGroups][4];
#pragma unroll
    for (int r = 0; r < kGroups; ++r) {
        const long long c0 = base + r * per_group + kTile * lane;          // this lane's first PE
        float lo[4], hi[4];
        // The two loads of a lane split every 64 bytes of x between them, so each cache line
        // is asked for twice in a row: the loads stay cacheable, and the second one hits
        // (n = 2^27, k = 5: 145 us against 214 us with the non-temporal hint).
        load4_guarded<false>(x, 2 * c0, n, lo);
        load4_guarded<false>(x, 2 * c0 + 4, n, hi);
        ev[r][0] = lo[0]; od[r][0] = lo[1]; ev[r][1] = lo[2]; od[r][1] = lo[3];
        ev[r][2] = hi[0]; od[r][2] = hi[1]; ev[r][3] = hi[2]; od[r][3] = hi[3];
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[r][i] = 0.0f;
    }

    run_chain<(KT + 1) / 2>(ev, acc, tw, (k + 1) / 2);                     // q = 0, 2, 4, ...
    if (k > 1) run_chain<KT / 2>(od, acc, tw + kChainLen, k / 2);          // q = 1, 3, 5, ...

    if (lane < valid_lanes) {
#pragma unroll
        for (int r = 0; r < kGroups; ++r)
            store4_guarded(y, base + r * per_group + kTile * lane, m, acc[r]);
    }
}

template <int KT>
hipError_t launch_stride2(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s)
{
    TapsStride2 taps;
    for (int j = 0; j < kChainLen; ++j) {
        taps.even[j] = 2 * j < k ? w[2 * j] : 0.0f;
        taps.odd[j] = 2 * j + 1 < k ? w[2 * j + 1] : 0.0f;
    }
    const long long m = ((long long)n - k) / 2 + 1;
    // The longer (even) chain reaches (k+1)/2 - 1 PEs up: that many PEs at the top of a
    // group compute values that are never stored.  Whole lanes, and a multiple of four
    // of them, so that every group starts on a 64-byte boundary of x and of y.
    const int v = kWave - halo_lanes((k + 1) / 2);
    const int valid_lanes = v - v % 4;
    const long long per_wave = (long long)kGroups * kTile * valid_lanes;
    const long long waves = (m + per_wave - 1) / per_wave;
    const long long blocks = (waves + (kBlock / kWave) - 1) / (kBlock / kWave);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((conv1d_fbs_stride2_kernel<KT>), dim3((unsigned)blocks), dim3(kBlock), 0, s,
                       taps, x, y, (long long)n, m, k, valid_lanes);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_conv1d_fbs_stride2(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s)
{
    switch (k) {                                // the paper's filter sizes (Section 6) and the headline's are unrolled
    case 2: return launch_stride2<2>(x, n, w, k, y, s);
    case 5: return launch_stride2<5>(x, n, w, k, y, s);
    case 16: return launch_stride2<16>(x, n, w, k, y, s);
    default: return launch_stride2<0>(x, n, w, k, y, s);
    }
}

}  // namespace sysconv
