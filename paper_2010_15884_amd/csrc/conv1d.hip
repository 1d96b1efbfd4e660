// 1-D valid convolution  y[c] = sum_q x[c+q] * w[q]  (paper Eq. 2) as software
// systolic arrays inside a wavefront.  One wavefront streams R register groups
// of 256 consecutive inputs; a group is a linear array of 256 PEs (4 per lane).
//
// Neighbouring groups overlap by 4*halo_lanes(k) inputs, the way neighbouring
// threads of the paper's designs each load their CCC+Q-1 inputs (Section 3.1):
// the PEs whose taps would reach past the group compute values that are never
// stored, so no step needs a bounds or time check.
#include "launch.h"
#include "systolic.h"

#include <cstdlib>

namespace sysconv {
namespace {

#ifndef SYSCONV_1D_GROUPS
#define SYSCONV_1D_GROUPS 4
#endif
constexpr int kGroups = SYSCONV_1D_GROUPS;     // register groups per wavefront (R)

// ---------------------------------------------------------------- FBS ------
// Table 2, row 3 left: PE = c, time = q.  Partial sums and weights never move;
// the inputs travel one PE towards lower c per step.  KT > 0 fixes the tap
// count at compile time (taps live in SGPRs, the time loop is unrolled);
// KT == 0 runs the same steps in blocks of four with a run-time count.
template <int NT, bool MORE>
__device__ __forceinline__ void fbs_groups(float (&e)[kGroups][4], float (&acc)[kGroups][4], const float (&w)[4])
{
#pragma unroll
    for (int r = 0; r < kGroups; ++r) fbs_steps<NT, MORE>(e[r], acc[r], w);
}

// the last 1..4 taps (nt is uniform across the wavefront)
__device__ __forceinline__ void fbs_groups_last(int nt, float (&e)[kGroups][4], float (&acc)[kGroups][4],
                                                const float (&w)[4])
{
    switch (nt) {
    case 4: fbs_groups<4, false>(e, acc, w); break;
    case 3: fbs_groups<3, false>(e, acc, w); break;
    case 2: fbs_groups<2, false>(e, acc, w); break;
    default: fbs_groups<1, false>(e, acc, w); break;
    }
}

template <int KT>
__global__ __launch_bounds__(kBlock) void conv1d_fbs_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                            long long n, long long m, int k_rt, int valid_lanes,
                                                            Taps1D taps)
{
    const int k = KT ? KT : k_rt;
    const int lane = threadIdx.x & (kWave - 1);
    const long long per_group = (long long)kTile * valid_lanes;            // outputs a group yields
    const long long wave = (long long)blockIdx.x * (kBlock / kWave) + wave_in_block();
    const long long base = wave * kGroups * per_group;
    if (base >= m) return;                                                 // uniform per wavefront

    float e[kGroups][4], acc[kGroups][4];
#pragma unroll
    for (int r = 0; r < kGroups; ++r) {
        load4_guarded(x, base + r * per_group + kTile * lane, n, e[r]);
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[r][i] = 0.0f;
    }

    int q = 0;
    if (KT) {
#pragma unroll
        for (; q + 4 < k; q += 4) {
            const float w[4] = {taps.w[q], taps.w[q + 1], taps.w[q + 2], taps.w[q + 3]};
            fbs_groups<4, true>(e, acc, w);
        }
    } else {
#pragma nounroll
        for (; q + 4 < k; q += 4) {
            const float w[4] = {taps.w[q], taps.w[q + 1], taps.w[q + 2], taps.w[q + 3]};
            fbs_groups<4, true>(e, acc, w);
        }
    }
    {
        const float w[4] = {taps.w[q], taps.w[q + 1], taps.w[q + 2], taps.w[q + 3]};
        fbs_groups_last(k - q, e, acc, w);
    }

    if (lane < valid_lanes) {
#pragma unroll
        for (int r = 0; r < kGroups; ++r)
            store4_guarded(y, base + r * per_group + kTile * lane, m, acc[r]);
    }
}

// ---------------------------------------------------------------- SBM ------
// Section 3.1: PE s = c + q, time = q.  Inputs stay where they were loaded;
// before every step but the first the whole partial-sum vector moves one PE
// up, Z(s) <- Z(s-1), then Z(s) += x(s) * w(q).  After k steps PE s holds
// output c = s - (k-1): the first k-1 PEs of a group hold garbage (the paper's
// register vectors of length Q+CCC-1 with results read from lane Q-1 on).
// Steps are taken up to four at a time so that the register rotation inside a
// lane is a compile-time rename.
template <int NT, bool FIRST>
__device__ __forceinline__ void sbm_steps(const float (&x)[4], float (&z)[4], const float (&w)[4])
{
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if (!(FIRST && t == 0)) {
            const float below = from_lane_below(z[3]);
            z[3] = z[2]; z[2] = z[1]; z[1] = z[0]; z[0] = below;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) z[i] = __builtin_fmaf(w[t], x[i], z[i]);
    }
}

template <int NT, bool FIRST>
__device__ __forceinline__ void sbm_groups(const float (&x)[kGroups][4], float (&z)[kGroups][4], const float (&w)[4])
{
#pragma unroll
    for (int r = 0; r < kGroups; ++r) sbm_steps<NT, FIRST>(x[r], z[r], w);
}

template <bool FIRST>
__device__ __forceinline__ void sbm_groups_n(int nt, const float (&x)[kGroups][4], float (&z)[kGroups][4],
                                             const float (&w)[4])
{
    switch (nt) {
    case 4: sbm_groups<4, FIRST>(x, z, w); break;
    case 3: sbm_groups<3, FIRST>(x, z, w); break;
    case 2: sbm_groups<2, FIRST>(x, z, w); break;
    default: sbm_groups<1, FIRST>(x, z, w); break;
    }
}

template <int KT>
__global__ __launch_bounds__(kBlock) void conv1d_sbm_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                            long long n, long long m, int k_rt, int valid_lanes,
                                                            Taps1D taps)
{
    const int k = KT ? KT : k_rt;
    const int lane = threadIdx.x & (kWave - 1);
    const long long per_group = (long long)kTile * valid_lanes;            // <= 257 - k
    const long long wave = (long long)blockIdx.x * (kBlock / kWave) + wave_in_block();
    const long long base = wave * kGroups * per_group;
    if (base >= m) return;

    float xs[kGroups][4], z[kGroups][4];
#pragma unroll
    for (int r = 0; r < kGroups; ++r) {
        load4_guarded(x, base + r * per_group + kTile * lane, n, xs[r]);
#pragma unroll
        for (int i = 0; i < 4; ++i) z[r][i] = 0.0f;
    }

    {
        const float w[4] = {taps.w[0], taps.w[1], taps.w[2], taps.w[3]};
        sbm_groups_n<true>(k < 4 ? k : 4, xs, z, w);
    }
    int q = 4;
    if (KT) {
#pragma unroll
        for (; q + 4 <= k; q += 4) {
            const float w[4] = {taps.w[q], taps.w[q + 1], taps.w[q + 2], taps.w[q + 3]};
            sbm_groups<4, false>(xs, z, w);
        }
    } else {
#pragma nounroll
        for (; q + 4 <= k; q += 4) {
            const float w[4] = {taps.w[q], taps.w[q + 1], taps.w[q + 2], taps.w[q + 3]};
            sbm_groups<4, false>(xs, z, w);
        }
    }
    if (q < k) {
        const float w[4] = {taps.w[q], taps.w[q + 1], taps.w[q + 2], taps.w[q + 3]};
        sbm_groups_n<false>(k - q, xs, z, w);                              // 1..3 taps left
    }

    // PE s = 4*lane + i of group r holds output  base + r*per_group + s - (k-1)
    // provided 0 <= s - (k-1) < per_group.
    const long long o0 = (long long)kTile * lane - (k - 1);
#pragma unroll
    for (int r = 0; r < kGroups; ++r) {
        const long long gbase = base + r * per_group;
        if (o0 >= 0 && o0 + 4 <= per_group) {
            store4_guarded(y, gbase + o0, m, z[r]);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const long long o = o0 + i;
                if (o >= 0 && o < per_group && gbase + o < m) y[gbase + o] = z[r][i];
            }
        }
    }
}

// Lanes of a group that keep their results.  At most 64 - halo_lanes(k) can; the
// count is rounded down to a multiple of kLaneAlign so that consecutive groups
// start on a 16*kLaneAlign-byte boundary (measured: groups that straddle 64-byte
// lines cost ~6 % of the streaming rate).
#ifndef SYSCONV_1D_LANE_ALIGN
#define SYSCONV_1D_LANE_ALIGN 4
#endif
int group_valid_lanes(int k)
{
    int v = kWave - halo_lanes(k);
    static const int forced = [] { const char* e = std::getenv("SYSCONV_1D_VALID"); return e ? std::atoi(e) : 0; }();
    if (forced > 0 && forced <= v) return forced;
    return v - v % SYSCONV_1D_LANE_ALIGN;
}

template <int KT, bool SBM>
hipError_t launch_1d(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s)
{
    Taps1D taps;
    for (int q = 0; q < kMaxK1D + 4; ++q) taps.w[q] = q < k ? w[q] : 0.0f;
    const long long m = (long long)n - k + 1;
    const int valid_lanes = group_valid_lanes(k);
    const long long per_wave = (long long)kGroups * kTile * valid_lanes;
    const long long waves = (m + per_wave - 1) / per_wave;
    const long long blocks = (waves + (kBlock / kWave) - 1) / (kBlock / kWave);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    if (SBM)
        hipLaunchKernelGGL((conv1d_sbm_kernel<KT>), dim3((unsigned)blocks), dim3(kBlock), 0, s,
                           x, y, (long long)n, m, k, valid_lanes, taps);
    else
        hipLaunchKernelGGL((conv1d_fbs_kernel<KT>), dim3((unsigned)blocks), dim3(kBlock), 0, s,
                           x, y, (long long)n, m, k, valid_lanes, taps);
    return hipGetLastError();
}

template <bool SBM>
hipError_t launch_by_k(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s)
{
    switch (k) {
    case 3: return launch_1d<3, SBM>(x, n, w, k, y, s);
    case 5: return launch_1d<5, SBM>(x, n, w, k, y, s);
    case 7: return launch_1d<7, SBM>(x, n, w, k, y, s);
    case 9: return launch_1d<9, SBM>(x, n, w, k, y, s);
    case 16: return launch_1d<16, SBM>(x, n, w, k, y, s);
    case 32: return launch_1d<32, SBM>(x, n, w, k, y, s);
    default: return launch_1d<0, SBM>(x, n, w, k, y, s);
    }
}

}  // namespace

hipError_t launch_conv1d_fbs(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s)
{
    return launch_by_k<false>(x, n, w, k, y, s);
}

hipError_t launch_conv1d_sbm(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s)
{
    return launch_by_k<true>(x, n, w, k, y, s);
}

bool has_conv1d_bfs(int) { return false; }

hipError_t launch_conv1d_bfs(const float*, size_t, const float*, int, float*, hipStream_t)
{
    return hipErrorNotSupported;
}

}  // namespace sysconv
