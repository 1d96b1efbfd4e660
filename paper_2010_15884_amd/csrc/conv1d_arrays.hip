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
constexpr int kStepBlock = 4;                                 // time steps per loop trip (BSM, FSM)
constexpr int kInFloats = kChunk + kMaxK1D + 2 * kStepBlock;  // chunk + k - 1 inputs, plus the look-ahead of BSM's reads
constexpr int kFfsWidth = 16;                                 // PEs of an FFS array
constexpr int kFfsPasses = kChunk / kWave;                    // 64 outputs (four arrays) per pass

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

__device__ __forceinline__ int clamp_index(int i, int hi) { return i < 0 ? 0 : (i > hi ? hi : i); }

// One PE of an FSM array and kStepBlock of its time steps.  PE q works on output c = t + q
// at step t and needs x(c + q) = x(t + 2q).  EDGE trips clamp that index into the array's
// window (the PEs it is clamped for are filling or draining), let a PE load its own input
// for its first output, and store only steps 0 <= t < seg.
struct FsmArray {
    bool top, bottom;
    int q, seg, hi;
    float wq;
    float z = 0.0f, x1 = 0.0f, x2 = 0.0f;                                  // X of one and of two steps ago

    template <bool EDGE>
    __device__ __forceinline__ void steps(int t0, const float* seg_in, float* seg_out)
    {
        float xl[kStepBlock], zs[kStepBlock];
#pragma unroll
        for (int j = 0; j < kStepBlock; ++j) {
            const int idx = t0 + j + 2 * q;
            xl[j] = seg_in[EDGE ? clamp_index(idx, hi) : idx];
        }
#pragma unroll
        for (int j = 0; j < kStepBlock; ++j) {
            const int t = t0 + j;
            const float xup = from_lane_above(x2);                         // X(c,q) <- X(c-1,q+1), two steps old
            const float xt = (top || (EDGE && t + q == 0)) ? xl[j] : xup;
            const float zup = from_lane_above(z);                          // Z(c,q) <- Z(c,q+1) from PE q+1
            z = __builtin_fmaf(xt, wq, top ? 0.0f : zup);
            x2 = x1;
            x1 = xt;
            zs[j] = z;
        }
        if (bottom) {                                                      // output c = t leaves PE 0
#pragma unroll
            for (int j = 0; j < kStepBlock; ++j)
                if (!EDGE || (t0 + j >= 0 && t0 + j < seg)) seg_out[t0 + j] = zs[j];
        }
    }
};

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
                // Four time steps per trip: their inputs are one aligned 16-byte LDS read, issued
                // one trip ahead.  Steps past the segment's end (t >= seg + k - 1) read staged or
                // stale LDS words inside this wavefront's buffer and store nothing.
                f4 xv = *reinterpret_cast<const f4*>(seg_in);
                for (int t0 = 0; t0 < seg + k - 1; t0 += kStepBlock) {
                    const f4 xnext = *reinterpret_cast<const f4*>(seg_in + t0 + kStepBlock);
                    const float xin[kStepBlock] = {xv.x, xv.y, xv.z, xv.w};   // x(t) goes to the array's K PEs
                    float zs[kStepBlock];
#pragma unroll
                    for (int j = 0; j < kStepBlock; ++j) {
                        // Z(c,q) <- Z(c,q-1) from PE q-1.  The lane move runs in ALL lanes and the
                        // select comes after it: a DPP read from a lane that is masked off returns 0.
                        const float zdown = from_lane_below(z);
                        z = __builtin_fmaf(xin[j], wq, first ? 0.0f : zdown);
                        zs[j] = z;
                    }
                    // Output c leaves PE K-1 at t = c + K - 1.
                    const int c0 = t0 - (k - 1);
                    if (c0 >= 0 && c0 + kStepBlock <= seg) {               // the usual trip: all four are outputs
                        if (last) {
#pragma unroll
                            for (int j = 0; j < kStepBlock; ++j) seg_out[c0 + j] = zs[j];
                        }
                    } else if (last) {
#pragma unroll
                        for (int j = 0; j < kStepBlock; ++j)
                            if (c0 + j >= 0 && c0 + j < seg) seg_out[c0 + j] = zs[j];
                    }
                    xv = xnext;
                }
            } else {
                FsmArray pe;
                pe.top = q == k - 1;
                pe.bottom = active && q == 0;
                pe.q = q;
                pe.wq = wq;
                pe.seg = seg;
                pe.hi = seg + k - 2;
                // Trips whose steps all lie in 1 <= t, t + 2(K-1) <= hi, t < seg need no index
                // clamp, no test for a PE's first output and no test before a store.
                const int t_plain_end = (seg < pe.hi - 2 * (k - 1) + 1 ? seg : pe.hi - 2 * (k - 1) + 1) - kStepBlock;
                for (int t0 = -(k - 1); t0 < seg; t0 += kStepBlock) {
                    if (t0 >= 1 && t0 <= t_plain_end) pe.template steps<false>(t0, seg_in, seg_out);
                    else                              pe.template steps<true>(t0, seg_in, seg_out);
                }
            }
        } else {
            // All chunk / 64 passes of the wavefront advance together, one time step at a time:
            // the weights' journey through the PEs is the same in every pass, so it is made once,
            // and the passes' independent X and Z chains overlap each other's LDS latency.
            const int c = lane & (kFfsWidth - 1);
            const int a0 = lane - c;                                       // first output of this lane's array in a pass
            const bool first = c == 0;
            const int hi = kFfsWidth + k - 2;
            float z[kFfsPasses], xt[kFfsPasses];
#pragma unroll
            for (int p = 0; p < kFfsPasses; ++p) z[p] = xt[p] = 0.0f;
            float w1 = 0.0f, w2 = 0.0f;
            for (int t = 0; t < 2 * (kFfsWidth - 1) + k; ++t) {
                const int q = t - 2 * c;
                const float* arr_in = in + a0 + clamp_index(t - c, hi);    // x(c + q), c + q = t - c
                const float wdown = from_lane_below(w2);                   // W(c,q) <- W(c-1,q), two steps old
                const float wt = first ? tw[t < k ? t : k] : wdown;        // w(q) for q = t < K, else the zero behind the taps
                const bool fresh = first || q == k - 1;                    // this PE is the first to use x(c + q)
                const bool busy = q >= 0 && q < k;
#pragma unroll
                for (int p = 0; p < kFfsPasses; ++p) {
                    const float xload = arr_in[p * kWave];
                    const float xdown = from_lane_below(xt[p]);            // X(c,q) <- X(c-1,q+1), one step old
                    xt[p] = fresh ? xload : xdown;
                    z[p] = busy ? __builtin_fmaf(xt[p], wt, z[p]) : z[p];
                }
                w2 = w1;
                w1 = wt;
            }
#pragma unroll
            for (int p = 0; p < kFfsPasses; ++p) out[p * kWave + lane] = z[p];
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
        // Segments start on float4 boundaries, and their length is 4 (mod 8) floats, so that
        // the arrays of a wavefront, which read in + a * seg + t at the same step, start in
        // different LDS banks instead of all in one.
        seg = (((kChunk / arrays) - 4) & ~7) + 4;
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
