// A miniature of the paper's generator (Section 2.2, Section 4.1): one kernel that runs
// the 1-D convolution recurrences
//
//     X(c,q) = inside(z - ex) ? X(z - ex) : x(c+q)        (or always x(c+q): "broadcast")
//     W(c,q) = inside(z - ew) ? W(z - ew) : w(q)          (or always w(q))
//     Z(c,q) = (inside(z - ez) ? Z(z - ez) : 0) + X(c,q) * W(c,q)
//
// under ANY space-time transform  PE = P.z, time = s.z  that passes the checks of
// plan_stt() below -- the six designs of Section 3.1 / Table 2 are six argument sets, and
// transforms the paper does not list run just as well.  It follows the general code shape
// of Section 4.1: every PE keeps a short history of each variable (as deep as the
// variable's time distance s.e), and at every time step it inverts the transform to find
// its iteration point, guards it against the domain, takes each operand from the
// neighbour P.e PEs away and s.e steps back (or from memory at the domain's edge), and
// shifts its histories.  One PE per lane, one array per wavefront; nothing is specialised,
// so this is the slow, general end of the library (the hand-laid kernels are the fast one).
#include "launch.h"
#include "systolic.h"

namespace sysconv {
namespace {

typedef const float __attribute__((address_space(4)))* kernarg_floats;

constexpr int kSttIn = 2 * kWave;               // a chunk reads C + k - 1 <= 127 inputs

// Value of `h` as it was `dt` steps ago, seen from `dl` PEs further up (dl = P.e).
// Both lane moves execute in every lane (a DPP read from a masked-off lane returns 0);
// the choice is made afterwards and is uniform.
__device__ __forceinline__ float passed(const float (&h)[kSttDepth], int dl, int dt)
{
    const float v = dt == 1 ? h[0] : (dt == 2 ? h[1] : h[2]);
    const float from_up = from_lane_above(v), from_down = from_lane_below(v);
    return dl == 0 ? v : (dl > 0 ? from_down : from_up);
}

__device__ __forceinline__ void remember(float (&h)[kSttDepth], float v)
{
#pragma unroll
    for (int i = kSttDepth - 1; i > 0; --i) h[i] = h[i - 1];
    h[0] = v;
}

// The taps are the first kernel argument (offset 0 of the kernel-argument segment).
__global__ __launch_bounds__(kBlock) void conv1d_stt_kernel(Taps1D taps, const float* __restrict__ x,
                                                            float* __restrict__ y, long long n, long long m, int k,
                                                            SttPlan pl)
{
    __shared__ float lds_in[kBlock / kWave][kSttIn];
    __shared__ float lds_w[kMaxK1D];
    (void)taps;
    kernarg_floats tw = (kernarg_floats)__builtin_amdgcn_kernarg_segment_ptr();

    const int lane = threadIdx.x & (kWave - 1);
    const int wv = wave_in_block();
    const long long base = ((long long)blockIdx.x * (kBlock / kWave) + wv) * pl.chunk;   // first output of the wavefront
    const bool live = base < m;                                                          // uniform per wavefront
    float* in = lds_in[wv];

    if (threadIdx.x < kMaxK1D) lds_w[threadIdx.x] = (int)threadIdx.x < k ? tw[threadIdx.x] : 0.0f;
    if (live)
        for (int i = lane; i < pl.chunk + k - 1; i += kWave) in[i] = base + i < n ? x[base + i] : 0.0f;
    __syncthreads();
    if (!live) return;

    const int cv = (int)(m - base < pl.chunk ? m - base : pl.chunk);      // outputs that exist in this chunk
    const int pe = lane + pl.pe_min;
    float hx[kSttDepth] = {}, hw[kSttDepth] = {}, hz[kSttDepth] = {};

    for (int t = 0; t < pl.steps; ++t) {
        // z = T^-1 (PE, time); the transform is unimodular, so the inverse is integral
        const int tp = t + pl.time_min;
        const int c = pl.det * (pl.s1 * pe - pl.p1 * tp);
        const int q = pl.det * (pl.p0 * tp - pl.s0 * pe);
        const bool valid = c >= 0 && c < cv && q >= 0 && q < k;
        const int cq = c + q;
        const float x_mem = in[cq < 0 ? 0 : (cq > kSttIn - 1 ? kSttIn - 1 : cq)];
        const float w_mem = lds_w[q < 0 ? 0 : (q > k - 1 ? k - 1 : q)];

        float xv = x_mem, wv_ = w_mem;
        if (pl.x_on) {                                                    // uniform
            const float nb = passed(hx, pl.x_dl, pl.x_dt);
            const int pc = c - pl.x_ec, pq = q - pl.x_eq;
            xv = (pc >= 0 && pc < cv && pq >= 0 && pq < k) ? nb : x_mem;
        }
        if (pl.w_on) {
            const float nb = passed(hw, pl.w_dl, pl.w_dt);
            const int pc = c - pl.w_ec;
            wv_ = (pc >= 0 && pc < cv) ? nb : w_mem;
        }
        const float zn = passed(hz, pl.z_dl, pl.z_dt);
        const int zq = q - pl.z_eq;
        const float zv = __builtin_fmaf(xv, wv_, (zq >= 0 && zq < k) ? zn : 0.0f);

        remember(hx, xv);
        remember(hw, wv_);
        remember(hz, zv);

        const int nq = q + pl.z_eq;                                       // the sum is complete when its chain ends
        if (valid && (nq < 0 || nq >= k)) y[base + c] = zv;
    }
}

// |v| > limit without negating v (INT_MIN has no negative)
bool beyond(int v, int limit) { return v > limit || v < -limit; }

int iabs(int v) { return v < 0 ? -v : v; }                               // for values already known to be small

}  // namespace

// Section 2.2's conditions on a design, then the limits of this kernel.
SttVerdict plan_stt(const int alloc[2], const int sched[2], bool x_on, const int ex[2], bool w_on, const int ew[2],
                    const int ez[2], int k, SttPlan* out)
{
    const int p0 = alloc[0], p1 = alloc[1], s0 = sched[0], s1 = sched[1];
    for (int v : {p0, p1, s0, s1})
        if (beyond(v, kWave)) return kSttTooLarge;
    // the recurrences themselves: X must be handed on between points that read the same
    // input (c+q constant), W between points with the same tap, Z along the taps
    if (x_on && ((long long)ex[0] + ex[1] != 0 || ex[0] == 0)) return kSttBadDependence;
    if (w_on && (ew[1] != 0 || ew[0] == 0)) return kSttBadDependence;
    if (ez[0] != 0 || (ez[1] != 1 && ez[1] != -1)) return kSttBadDependence;
    // two points on one PE must differ in time
    const int det = p0 * s1 - p1 * s0;
    if (det == 0) return kSttSingular;

    SttPlan pl = {};
    pl.p0 = p0; pl.p1 = p1; pl.s0 = s0; pl.s1 = s1; pl.det = det;
    struct Dep { bool on; const int* e; int* dl; int* dt; };
    const Dep deps[3] = {{x_on, ex, &pl.x_dl, &pl.x_dt}, {w_on, ew, &pl.w_dl, &pl.w_dt}, {true, ez, &pl.z_dl, &pl.z_dt}};
    bool far = false;
    for (const Dep& d : deps) {
        if (!d.on) continue;
        if (beyond(d.e[0], kWave) || beyond(d.e[1], kWave)) return kSttTooLarge;
        *d.dl = p0 * d.e[0] + p1 * d.e[1];                                 // space distance P.e
        *d.dt = s0 * d.e[0] + s1 * d.e[1];                                 // time distance s.e
        if (*d.dt < 1) return kSttNotCausal;                               // a value would be read before it exists
        if (beyond(*d.dl, 1) || *d.dt > kSttDepth) far = true;
    }
    if (det != 1 && det != -1) return kSttTooLarge;                        // idle holes in the PE-time grid: not built
    if (far) return kSttTooLarge;                                          // only nearest-neighbour moves, short histories
    // outputs per wavefront: as many as keep the PE vector within 64 lanes
    int chunk = kWave;
    if (p0 != 0) {
        const int room = kWave - 1 - iabs(p1) * (k - 1);
        if (room < 0) return kSttTooLarge;
        chunk = room / iabs(p0) + 1;
        if (chunk > kWave) chunk = kWave;
    } else if (iabs(p1) * (k - 1) + 1 > kWave) {
        return kSttTooLarge;
    }
    pl.chunk = chunk;
    pl.pe_min = (p0 < 0 ? p0 * (chunk - 1) : 0) + (p1 < 0 ? p1 * (k - 1) : 0);
    pl.time_min = (s0 < 0 ? s0 * (chunk - 1) : 0) + (s1 < 0 ? s1 * (k - 1) : 0);
    pl.steps = iabs(s0) * (chunk - 1) + iabs(s1) * (k - 1) + 1;
    pl.x_on = x_on; pl.w_on = w_on;
    if (x_on) { pl.x_ec = ex[0]; pl.x_eq = ex[1]; }
    if (w_on) { pl.w_ec = ew[0]; }
    pl.z_eq = ez[1];
    if (out) *out = pl;
    return kSttOk;
}

hipError_t launch_conv1d_stt(const float* x, size_t n, const float* w, int k, float* y, const SttPlan& pl,
                             hipStream_t s)
{
    Taps1D taps;
    for (int q = 0; q < kTaps1DLen; ++q) taps.w[q] = q < k ? w[q] : 0.0f;
    const long long m = (long long)n - k + 1;
    const long long waves = (m + pl.chunk - 1) / pl.chunk;
    const long long blocks = (waves + (kBlock / kWave) - 1) / (kBlock / kWave);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(conv1d_stt_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, s,
                       taps, x, y, (long long)n, m, k, pl);
    return hipGetLastError();
}

}  // namespace sysconv
