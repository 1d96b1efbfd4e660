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

__device__ __forceinline__ void sbm_readout_lane(float (&z)[kGroups][4])
{
#pragma unroll
    for (int r = 0; r < kGroups; ++r)
#pragma unroll
        for (int i = 0; i < 4; ++i) z[r][i] = from_lane_above(z[r][i]);
}

template <int N>
__device__ __forceinline__ void sbm_readout_pe(float (&z)[kGroups][4])
{
#pragma unroll
    for (int r = 0; r < kGroups; ++r)
#pragma unroll
        for (int t = 0; t < N; ++t) {
            const float above = from_lane_above(z[r][0]);
            z[r][0] = z[r][1]; z[r][1] = z[r][2]; z[r][2] = z[r][3]; z[r][3] = above;
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

    // PE s = 4*lane + i of group r now holds output  base + r*per_group + s - (k-1).
    // Read the result vector out k-1 PEs further down (Section 3.1: the results of an
    // SBM array are taken from PE Q-1 on): a whole lane at a time while four or more PEs
    // remain, then PE by PE.  After that PE s holds output s and the stores line up
    // with the loads.
    int left = k - 1;
    if (KT) {
#pragma unroll
        for (; left >= 4; left -= 4) sbm_readout_lane(z);
    } else {
#pragma nounroll
        for (; left >= 4; left -= 4) sbm_readout_lane(z);
    }
    switch (left) {                                                        // uniform
    case 3: sbm_readout_pe<3>(z); break;
    case 2: sbm_readout_pe<2>(z); break;
    case 1: sbm_readout_pe<1>(z); break;
    default: break;
    }
    if (lane < valid_lanes) {
#pragma unroll
        for (int r = 0; r < kGroups; ++r)
            store4_guarded(y, base + r * per_group + kTile * lane, m, z[r]);
    }
}

// ---------------------------------------------------------------- BFS ------
// Table 2, row 2 left: PE = c, time = c + q.  At time t the input x(t) is
// broadcast to every PE, PE c applies the weight w(t-c) that has just been
// forwarded to it, partial sums never move.  Across 64 lanes that array would
// idle most PEs (k of k+63 steps), so the arrays are laid along the registers:
// every lane is an independent 4-PE array (its four consecutive outputs), the
// inputs x(4*lane + m), m = 0..k+2, arrive one aligned float4 at a time, and
// each arriving input is applied to the up-to-four PEs whose weight window
// covers it.  Idle PE-steps of the paper's model cost nothing here because the
// PEs of a lane are time-multiplexed on one ALU.  The broadcast medium is LDS:
// a wavefront stages its 4 register groups plus a (k-1)-element halo once and
// every lane then reads its own overlapping window with aligned ds_read_b128.
// No lane computes garbage, and no value moves between lanes through DPP.
//
// One block = the four inputs m = 4b..4b+3.  wv[i] = w(4b-3+i), i = 0..6, are
// the weights that can meet them; pair (input u, PE j) uses wv[u-j+3].  LO/HI
// bound the valid part of wv (head block: indices below 3 are taps < 0; tail
// blocks: indices above k+2-4b are taps >= k).
template <int LO, int HI>
__device__ __forceinline__ void bfs_block(float (&acc)[4], const float (&xa)[4], const float (&wv)[7])
{
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = u - j + 3;
            if (i >= LO && i <= HI) acc[j] = __builtin_fmaf(wv[i], xa[u], acc[j]);
        }
}

template <int LO>
__device__ __forceinline__ void bfs_block_hi(int hi, float (&acc)[4], const float (&xa)[4], const float (&wv)[7])
{
    switch (hi) {                                                          // uniform
    case 0: bfs_block<LO, 0>(acc, xa, wv); break;
    case 1: bfs_block<LO, 1>(acc, xa, wv); break;
    case 2: bfs_block<LO, 2>(acc, xa, wv); break;
    case 3: bfs_block<LO, 3>(acc, xa, wv); break;
    case 4: bfs_block<LO, 4>(acc, xa, wv); break;
    case 5: bfs_block<LO, 5>(acc, xa, wv); break;
    default: bfs_block<LO, 6>(acc, xa, wv); break;
    }
}

constexpr int kBfsLdsFloats = (kGroups + 1) * kWave * kTile;               // per wavefront: groups + halo group

template <int KT>
__global__ __launch_bounds__(kBlock) void conv1d_bfs_kernel(Taps1D taps, const float* __restrict__ x,
                                                            float* __restrict__ y, long long n, long long m,
                                                            int k_rt)
{
    __shared__ __attribute__((aligned(16))) float stage[(kBlock / kWave) * kBfsLdsFloats];
    // taps through the kernel-argument segment (first argument = offset 0), padded in
    // front by 3 so that w(4b-3+i) can be fetched for b = 0
    typedef const float __attribute__((address_space(4)))* kernarg_floats;
    kernarg_floats tw = (kernarg_floats)__builtin_amdgcn_kernarg_segment_ptr();
    (void)taps;

    const int k = KT ? KT : k_rt;
    const int lane = threadIdx.x & (kWave - 1);
    const int wv_id = wave_in_block();
    const long long wave = (long long)blockIdx.x * (kBlock / kWave) + wv_id;
    const long long base = wave * kGroups * kWave * kTile;                 // first output (= first input) of this wavefront
    float* lds = stage + wv_id * kBfsLdsFloats;

    // stage: kGroups full groups and the first k-1 (rounded up to 4) floats of the next one
    if (base < m) {
#pragma unroll
        for (int r = 0; r <= kGroups; ++r) {
            if (r < kGroups || lane < halo_lanes(k)) {
                float v[4];
                load4_guarded(x, base + (long long)r * kWave * kTile + kTile * lane, n, v);
                f4 t;
                t.x = v[0]; t.y = v[1]; t.z = v[2]; t.w = v[3];
                *reinterpret_cast<f4*>(lds + r * kWave * kTile + kTile * lane) = t;
            }
        }
    }
    __syncthreads();                                                       // every wavefront reaches this
    if (base >= m) return;

    float acc[kGroups][4];
#pragma unroll
    for (int r = 0; r < kGroups; ++r) acc[r][0] = acc[r][1] = acc[r][2] = acc[r][3] = 0.0f;

    auto window = [&](int r, int b, float (&xa)[4]) {
        const f4 t = *reinterpret_cast<const f4*>(lds + r * kWave * kTile + kTile * lane + 4 * b);
        xa[0] = t.x; xa[1] = t.y; xa[2] = t.z; xa[3] = t.w;
    };
    auto weights = [&](int b, float (&wv)[7]) {
#pragma unroll
        for (int i = 0; i < 7; ++i) wv[i] = tw[4 * b + i];               // tw[j] = w(j-3)
    };

    // head block b = 0: taps below 0 do not exist
    {
        float wv[7];
        weights(0, wv);
        const int hi = k + 2 < 6 ? k + 2 : 6;
#pragma unroll
        for (int r = 0; r < kGroups; ++r) {
            float xa[4];
            window(r, 0, xa);
            bfs_block_hi<3>(hi, acc[r], xa, wv);
        }
    }
    int b = 1;
    // interior blocks: all sixteen (input, PE) pairs are valid
    if (KT) {
#pragma unroll
        for (; 4 * b + 3 <= k - 1; ++b) {
            float wv[7];
            weights(b, wv);
#pragma unroll
            for (int r = 0; r < kGroups; ++r) {
                float xa[4];
                window(r, b, xa);
                bfs_block<0, 6>(acc[r], xa, wv);
            }
        }
    } else {
#pragma nounroll
        for (; 4 * b + 3 <= k - 1; ++b) {
            float wv[7];
            weights(b, wv);
#pragma unroll
            for (int r = 0; r < kGroups; ++r) {
                float xa[4];
                window(r, b, xa);
                bfs_block<0, 6>(acc[r], xa, wv);
            }
        }
    }
    // tail blocks (at most two): taps >= k do not exist
#pragma unroll 2
    for (; 4 * b <= k + 2; ++b) {
        float wv[7];
        weights(b, wv);
        const int hi = k + 2 - 4 * b;                                      // 0..5
#pragma unroll
        for (int r = 0; r < kGroups; ++r) {
            float xa[4];
            window(r, b, xa);
            bfs_block_hi<0>(hi, acc[r], xa, wv);
        }
    }

#pragma unroll
    for (int r = 0; r < kGroups; ++r)
        store4_guarded(y, base + (long long)r * kWave * kTile + kTile * lane, m, acc[r]);
}

template <int KT>
hipError_t launch_1d_bfs(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s)
{
    Taps1D taps;
    for (int q = 0; q < kTaps1DLen; ++q) taps.w[q] = 0.0f;
    for (int q = 0; q < k; ++q) taps.w[q + 3] = w[q];                      // three leading zeros: w(-3..-1), never multiplied
    const long long m = (long long)n - k + 1;
    const long long per_wave = (long long)kGroups * kWave * kTile;
    const long long waves = (m + per_wave - 1) / per_wave;
    const long long blocks = (waves + (kBlock / kWave) - 1) / (kBlock / kWave);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((conv1d_bfs_kernel<KT>), dim3((unsigned)blocks), dim3(kBlock), 0, s,
                       taps, x, y, (long long)n, m, k);
    return hipGetLastError();
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
    const int v = kWave - halo_lanes(k);
    return v - v % SYSCONV_1D_LANE_ALIGN;
}

template <int KT, bool SBM>
hipError_t launch_1d(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s)
{
    Taps1D taps;
    for (int q = 0; q < kTaps1DLen; ++q) taps.w[q] = q < k ? w[q] : 0.0f;
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

bool has_conv1d_bfs(int k) { return k >= 1 && k <= kMaxK1D; }

hipError_t launch_conv1d_bfs(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s)
{
    switch (k) {
    case 5: return launch_1d_bfs<5>(x, n, w, k, y, s);
    case 16: return launch_1d_bfs<16>(x, n, w, k, y, s);
    default: return launch_1d_bfs<0>(x, n, w, k, y, s);
    }
}

}  // namespace sysconv
