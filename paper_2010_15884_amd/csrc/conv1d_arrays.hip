// 1-D valid convolution with the three remaining designs of the paper's Table 2,
// each realised with one PE per LANE, as the table draws them:
//
//   BSM  (row 1 left)   PE = tap q, time = c + q.  Weights stay, the input x(t) is
//        broadcast to the K PEs of an array, partial sums move one PE up per step.
//   FSM  (row 1 right)  PE = tap q, time = c - q.  Weights stay, inputs move towards
//        lower q at half speed (two steps per PE), partial sums move towards lower q.
//   FFS  (row 2 right)  PE = output c, time = 2c + q.  Inputs move up one PE per step,
//        weights one PE per two steps, partial sums stay.
//
// BSM and FSM arrays are K lanes long, so a wavefront holds 64/K of them side by side,
// each streaming through its own segment of the signal without refilling (one fill and
// one drain of K-1 steps per segment).  FFS arrays are 16 PEs long, the size the paper
// analyses (Table 4): 4 per wavefront, 30+K steps for 16 outputs each.  These are the
// designs the paper measures as inferior -- every step costs a lane move and a select
// per multiply-add, and FFS idles most PEs -- and they are here to reproduce that
// ranking on this machine, not to compete with FBS / SBM / BFS.
//
// Inputs and results pass through LDS (per wavefront: staged with coalesced 16-byte
// accesses, read by the PEs one element per step; an array's K lanes read the same
// address, which LDS serves as a broadcast).
#include "launch.h"
#include "systolic.h"

namespace sysconv {
namespace {

typedef const float __attribute__((address_space(4)))* kernarg_floats;

constexpr int kChunk = 1024;                                  // outputs per wavefront (at most)
constexpr int kInFloats = kChunk + kMaxK1D + 4;               // chunk + k - 1, rounded up to float4s
constexpr int kFfsWidth = 16;                                 // PEs of an FFS array

enum ArrayDesign { kBsm, kFsm, kFfs };

__device__ __forceinline__ void stage_in(const float* __restrict__ x, long long base, long long n, int count,
                                         float* lds, int lane)
{
    for (int i = kTile * lane; i < count; i += kWave * kTile) {
        float v[4];
        load4_guarded(x, base + i, n, v);
        f4 t;
        t.x = v[0]; t.y = v[1]; t.z = v[2]; t.w = v[3];
        *reinterpret_cast<f4*>(lds + i) = t;
    }
}

__device__ __forceinline__ void stage_out(float* __restrict__ y, long long base, long long m, int count,
                                          const float* lds, int lane)
{
    for (int i = kTile * lane; i < count; i += kWave * kTile) {
        const f4 t = *reinterpret_cast<const f4*>(lds + i);
        const float v[4] = {t.x, t.y, t.z, t.w};
        store4_guarded(y, base + i, m, v);
    }
}

// The taps are the first kernel argument (offset 0 of the kernel-argument segment).
template <int DESIGN>
__global__ __launch_bounds__(kBlock) void conv1d_array_kernel(Taps1D taps, const float* __restrict__ x,
                                                              float* __restrict__ y, long long n, long long m,
                                                              int k, int seg, int chunk)
{
    __shared__ __attribute__((aligned(16))) float lds_in[(kBlock / kWave) * kInFloats];
    __shared__ __attribute__((aligned(16))) float lds_out[(kBlock / kWave) * kChunk];
    (void)taps;
    kernarg_floats tw = (kernarg_floats)__builtin_amdgcn_kernarg_segment_ptr();

    const int lane = threadIdx.x & (kWave - 1);
    const int wv = wave_in_block();
    const long long base = ((long long)blockIdx.x * (kBlock / kWave) + wv) * chunk;   // first output of the wavefront
    float* in = lds_in + wv * kInFloats;
    float* out = lds_out + wv * kChunk;
    const bool live = base < m;                                            // uniform per wavefront

    if (live) stage_in(x, base, n, chunk + k - 1, in, lane);
    __syncthreads();

    if (live) {
        if (DESIGN == kBsm || DESIGN == kFsm) {
            const int arrays = kWave / k;
            const int a_raw = lane / k, q = lane - a_raw * k;
            const bool active = a_raw < arrays;
            const int a = active ? a_raw : 0;                              // idle lanes shadow array 0, store nothing
            const float wq = tw[q];
            const float* seg_in = in + a * seg;
            float* seg_out = out + a * seg;
            float z = 0.0f;
            if (DESIGN == kBsm) {
                const bool first = q == 0, last = active && q == k - 1;
                for (int t = 0; t < seg + k - 1; ++t) {
                    const float xin = seg_in[t];                           // broadcast to the array's K PEs
                    // Z(c,q) <- Z(c,q-1) from PE q-1.  The lane move runs in ALL lanes and the
                    // select comes after it: a DPP read from a lane that is masked off returns 0.
                    const float zdown = from_lane_below(z);
                    const float zprev = first ? 0.0f : zdown;
                    z = __builtin_fmaf(xin, wq, zprev);
                    if (last && t >= k - 1) seg_out[t - (k - 1)] = z;     // output c = t-(K-1) leaves PE K-1
                }
            } else {
                const bool top = q == k - 1, bottom = active && q == 0;
                float x1 = 0.0f, x2 = 0.0f;                                // X of one and of two steps ago
                for (int t = -(k - 1); t < seg; ++t) {
                    int idx = t + 2 * q;                                   // = c + q for c = t + q
                    idx = idx < 0 ? 0 : (idx > seg + k - 2 ? seg + k - 2 : idx);
                    const float xload = seg_in[idx];
                    const float xup = from_lane_above(x2);                 // X(c,q) <- X(c-1,q+1), two steps old
                    const float xt = (top || t + q == 0) ? xload : xup;
                    const float zup = from_lane_above(z);                  // Z(c,q) <- Z(c,q+1) from PE q+1
                    const float zprev = top ? 0.0f : zup;
                    z = __builtin_fmaf(xt, wq, zprev);
                    x2 = x1;
                    x1 = xt;
                    if (bottom && t >= 0) seg_out[t] = z;                  // output c = t leaves PE 0
                }
            }
        } else {
            const int c = lane & (kFfsWidth - 1);
            const int a0 = lane - c;                                       // first output of this lane's array in a pass
            const bool first = c == 0;
            for (int pass = 0; pass < chunk / kWave; ++pass) {
                const float* arr_in = in + pass * kWave + a0;
                float z = 0.0f, xt = 0.0f, w1 = 0.0f, w2 = 0.0f;
                for (int t = 0; t < 2 * (kFfsWidth - 1) + k; ++t) {
                    const int q = t - 2 * c;
                    int idx = t - c;                                       // = c + q
                    idx = idx < 0 ? 0 : (idx > kFfsWidth + k - 2 ? kFfsWidth + k - 2 : idx);
                    const float xload = arr_in[idx];
                    const float xdown = from_lane_below(xt);               // X(c,q) <- X(c-1,q+1), one step old
                    xt = (first || q == k - 1) ? xload : xdown;
                    const float wdown = from_lane_below(w2);               // W(c,q) <- W(c-1,q), two steps old
                    const float wt = first ? tw[t < k ? t : k] : wdown;     // w(q) for q = t < K, else the zero behind the taps
                    if (q >= 0 && q < k) z = __builtin_fmaf(xt, wt, z);
                    w2 = w1;
                    w1 = wt;
                }
                out[pass * kWave + lane] = z;
            }
        }
    }
    __syncthreads();
    if (live) stage_out(y, base, m, chunk, out, lane);
}

template <int DESIGN>
hipError_t launch_array(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s)
{
    Taps1D taps;
    for (int q = 0; q < kTaps1DLen; ++q) taps.w[q] = q < k ? w[q] : 0.0f;
    const long long m = (long long)n - k + 1;
    int seg = 0, chunk = kChunk;
    if (DESIGN != kFfs) {
        const int arrays = kWave / k;
        seg = (kChunk / arrays) & ~3;                                      // segments start on float4 boundaries
        chunk = arrays * seg;
    }
    const long long waves = (m + chunk - 1) / chunk;
    const long long blocks = (waves + (kBlock / kWave) - 1) / (kBlock / kWave);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((conv1d_array_kernel<DESIGN>), dim3((unsigned)blocks), dim3(kBlock), 0, s,
                       taps, x, y, (long long)n, m, k, seg, chunk);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_conv1d_bsm(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s)
{
    return launch_array<kBsm>(x, n, w, k, y, s);
}
hipError_t launch_conv1d_fsm(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s)
{
    return launch_array<kFsm>(x, n, w, k, y, s);
}
hipError_t launch_conv1d_ffs(const float* x, size_t n, const float* w, int k, float* y, hipStream_t s)
{
    return launch_array<kFfs>(x, n, w, k, y, s);
}

}  // namespace sysconv
