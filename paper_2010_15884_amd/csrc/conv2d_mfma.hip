// 2-D valid convolution (paper Eq. 3) for filters whose kh*kw multiply-adds per output
// exceed what the vector ALUs deliver per byte of HBM traffic: the sums are taken by the
// matrix cores (the hardware systolic arrays of the CU) instead of the software array.
//
// One v_mfma_f32_16x16x32_f16 multiplies a 16 x 32 by a 32 x 16 matrix.  A single-channel
// filter has no channel dimension to contract over, so the contraction is made from the
// filter's own extent in BOTH directions (a doubly blocked Toeplitz form):
//
//   N (16)  "bases": 16 output positions (r, c0 + 4 i), i = 0..15, of one output row
//   M (16)  "offsets": the 4 x 4 outputs (r + jr, c + jc) next to a base, j = 4 jr + jc
//   K       input offsets (dr, dc), dr < kh + 3 rows, dc < 16 columns, taken 2 rows
//           (= 32 values) per instruction: NS = ceil((kh + 3) / 2) instructions
//
//   A[j][(dr, dc)] = f[dr - jr][dc - jc]      (0 outside the filter)   -- constant, in registers
//   B[(dr, dc)][i] = x[r + dr][c0 + 4 i + dc]                          -- 8 consecutive inputs per lane
//   D[j][i]        = y[r + jr][c0 + 4 i + jc]                          -- 4 consecutive outputs per lane
//
// so NS instructions produce a 4-row x 64-column block of outputs; kh*kw of the
// 2*16*NS products per output are non-zero (11x11: 121 of 224).
//
// Precision.  The matrix cores multiply fp16.  Inputs and taps are therefore split,
// v = hi + lo with hi = fp16(v) and lo = fp16(v - hi) (kept 2^11 times larger, so that it
// is a normal fp16 number like hi), which keeps 22 significant bits, and three products
// are accumulated in fp32: hi*hi, and hi*lo + lo*hi in accumulators of their own that
// enter the result times 2^-11 (the lo*lo term is below 2^-22 of the product).  Both
// operands are scaled by a power of two first: taps by a factor the host derives from
// their largest magnitude, inputs by a fixed 2^13.  That fixes the admissible input range:
// |x| < 8 (larger values become infinite in fp16), and inputs below 2^-27 count as zero.
//
// Data path of a wavefront (strip of 64 output columns, block of up to 64 rows walked 4 at a
// time).  Input travels in "units" of 2 rows x 80 columns (40 float4).  Interior strips:
// global_load_lds_dwordx4 (40 lanes) puts a unit straight into a 16-slot queue in LDS, so that
// the 14 units in flight per wavefront cost no registers; when a unit has arrived every lane
// reads its 8-input window (the B operand), scales, splits and packs it into a ring of NS (+1)
// operand pairs in registers -- each 2-row unit serves NS consecutive instruction slots as the
// block moves down -- then MFMA and global_store_dwordx4.  Strips that reach past the right
// edge of the image fetch through registers with bounds checks instead.
// Measured on MI355X, 8192^2: 11x11 138 us, 13x13 151 us (the vector-ALU kernels: 243 us and
// 397 us); the vector ALUs (scaling and splitting, 44 % busy) and the matrix cores (26 %) still
// take turns rather than overlap, and that, not HBM, bounds it.
#include "launch.h"
#include "systolic.h"
#include "tiling.h"

#include <math.h>
#include <type_traits>

namespace sysconv {
namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));

constexpr int kMOutCols = 64;              // output columns of a wavefront's strip: 16 bases x 4
constexpr int kMInCols = 80;               // staged input columns: 64 + 12 are read, 20 float4 are fetched
constexpr int kMUnitLanes = 40;            // lanes that fetch a unit: 2 rows x 20 float4
constexpr int kMWaves = kBlock / kWave;
constexpr float kMXScale = 8192.0f;        // 2^13: inputs up to 8 stay finite in fp16
constexpr float kMLoScale = 2048.0f;       // 2^11: the lo parts are kept this much larger

typedef const float __attribute__((address_space(4)))* kernarg_floats;

template <int NS>
struct MfmaShape {
    static_assert(NS >= 2 && NS <= 8, "2 <= NS <= 8 covers filters of 1 .. 13 rows");
    static constexpr int RS = NS <= 4 ? 4 : 8;     // ring slots (a power of two >= NS, >= 4)
    static constexpr int PERIOD = RS / 2;          // steps after which the ring indices repeat
    static constexpr int TROWS = 2 * NS + 3;       // rows of the tap tables: dr - jr + 3 = 0 .. 2 NS + 2
};

// Where a lane fetches its share of a unit (two consecutive input rows, 80 columns = 40 float4;
// lanes 40 .. 63 repeat the work of lanes 0 .. 23, so that no lane is switched off and the
// fetches need no branch).  Units are fetched in order; everything but the lane's two offsets
// is uniform across the wavefront and advances with scalar arithmetic.
struct MfmaFetcher {
    const float* __restrict__ rowp;  // first row of the next unit (uniform)
    long long xp;
    int w_img;
    int rows_left;            // rows of the block that lie beyond the next unit's first row (uniform)
    int fcol;                 // first of the lane's four input columns
    long long off_two;        // lane's offset from the unit's first row when the unit has both rows
    long long off_one;        // ... when its second row lies beyond the block (it repeats the first)

    // Fetch the next unit.  Past the block's last row the last row is read again: an unconditional
    // load keeps the control flow straight, and what it brings in only feeds rows that are not stored.
    // Address of the lane's part of the next unit; moves on to the unit after it.
    __device__ __forceinline__ const float* next_address()
    {
        const float* p = rowp + (rows_left > 0 ? off_two : off_one);
        rowp += rows_left >= 2 ? 2 * xp : rows_left == 1 ? xp : 0;
        rows_left -= min(rows_left, 2);
        return p;
    }

    template <bool EDGE>
    __device__ __forceinline__ void next(float (&v)[4])
    {
        const float* p = next_address();
        if (EDGE) {
            load4_guarded<false>(p - fcol, fcol, w_img, v);
        } else {
            const f4u t = *reinterpret_cast<const f4u*>(p);
            v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
        }
    }
};

// Interior strips do not stage through registers at all: the unit travels from global memory
// straight into a queue slot in LDS (global_load_lds_dwordx4: lane l's 16 bytes land at
// M0 + 16 l; lanes switched off write nothing), so the data in flight costs no registers and
// the queue can be deep enough to cover the memory latency with two or three wavefronts per
// SIMD.  The compiler does not see these loads; the waits are written by hand (mfma_wait_loads).
constexpr int kMQueue = 16;                // queue slots per wavefront
constexpr int kMAhead = kMQueue - 2;       // loads in flight behind the unit being taken (at most kMAhead + 2 slots are in use)
constexpr int kMSlotBytes = 2 * kMInCols * (int)sizeof(float);

__device__ __forceinline__ void mfma_dma_unit(const float* p, unsigned lds_byte_address, unsigned long long lanes)
{
    unsigned long long saved;
    asm volatile("s_mov_b64 %0, exec\n\t"
                 "s_mov_b32 m0, %2\n\t"
                 "s_mov_b64 exec, %3\n\t"
                 "global_load_lds_dwordx4 %1, off\n\t"
                 "s_mov_b64 exec, %0"
                 : "=&s"(saved)
                 : "v"(p), "s"(lds_byte_address), "s"(lanes)
                 : "memory");
}

// Wait until at most `kMAhead` of the wavefront's vector-memory operations are outstanding.
// Loads complete in the order they were issued, so a unit that kMAhead younger loads have
// followed has arrived by then -- whatever stores are outstanding besides (they only make the
// wait stricter).
__device__ __forceinline__ void mfma_wait_loads()
{
    static_assert(kMAhead == 14, "the wait below is written for 14 loads in flight");
    asm volatile("s_waitcnt vmcnt(14)" ::: "memory");
}

// Eight consecutive inputs, scaled and split as in mfma_split.
__device__ __forceinline__ void mfma_split8(const f4& a, const f4& b, h8& hi, h8& lo)
{
    const f4 sa = a * kMXScale, sb = b * kMXScale;
    const h4 ha = __builtin_convertvector(sa, h4), hb = __builtin_convertvector(sb, h4);
    const h4 la = __builtin_convertvector((sa - __builtin_convertvector(ha, f4)) * kMLoScale, h4);
    const h4 lb = __builtin_convertvector((sb - __builtin_convertvector(hb, f4)) * kMLoScale, h4);
    hi = __builtin_shufflevector(ha, hb, 0, 1, 2, 3, 4, 5, 6, 7);
    lo = __builtin_shufflevector(la, lb, 0, 1, 2, 3, 4, 5, 6, 7);
}

// v * 2^13 = hi + lo * 2^-11 in fp16 (both rounded to nearest): the remainder v*2^13 - hi is
// exact in fp32 and at most half an fp16 ulp of hi; stored 2^11 times larger it has the
// magnitude of hi at most and stays a normal fp16 number whenever hi is one (the matrix
// cores treat subnormal fp16 inputs as zero).  A value of 8 or more becomes infinite here
// and shows up as inf / NaN in the results it feeds.
__device__ __forceinline__ void mfma_split(const float (&v)[4], h4& hi, h4& lo)
{
    f4 s;
#pragma unroll
    for (int i = 0; i < 4; ++i) s[i] = v[i] * kMXScale;
    hi = __builtin_convertvector(s, h4);
    lo = __builtin_convertvector((s - __builtin_convertvector(hi, f4)) * kMLoScale, h4);
}

template <int NS>
__global__ __launch_bounds__(kBlock) void conv2d_mfma_kernel(Taps2D taps, const float* __restrict__ x,
                                                             float* __restrict__ y, int w_img, long long xp,
                                                             int oh, int ow, long long yp, int kh, int kw,
                                                             int rows, int row_blocks, int col_groups, int per_xcd,
                                                             float tap_scale, float inv_scale)
{
    (void)taps;
    using S = MfmaShape<NS>;
    constexpr int RS = S::RS, PERIOD = S::PERIOD, TROWS = S::TROWS;

    // wtab[plane][jc][dr - jr + 3][dc] = hi / lo part of f[dr - jr][dc - jc] * tap_scale
    __shared__ __attribute__((aligned(16))) _Float16 wtab[2][4][TROWS][16];
    // per wavefront: two unit buffers x (hi, lo) x 2 rows x 80 columns
    __shared__ __attribute__((aligned(16))) _Float16 stage[kMWaves][2][2][2][kMInCols];
    // per wavefront: queue of units as they come from memory, 2 rows x 80 columns of fp32 each
    __shared__ __attribute__((aligned(16))) float queue[kMWaves][kMQueue][2][kMInCols];

    kernarg_floats taps_f = (kernarg_floats)__builtin_amdgcn_kernarg_segment_ptr();
    for (int e = threadIdx.x; e < 4 * TROWS * 16; e += kBlock) {
        const int dc = e & 15, tr = (e >> 4) % TROWS, jc = e / (16 * TROWS);
        const int p = tr - 3, q = dc - jc;
        float v = 0.0f;
        if (p >= 0 && p < kh && q >= 0 && q < kw) v = taps_f[p * kw + q] * tap_scale;
        const _Float16 hi = (_Float16)v;
        wtab[0][jc][tr][dc] = hi;
        wtab[1][jc][tr][dc] = (_Float16)((v - (float)hi) * kMLoScale);
    }
    __syncthreads();

    const int g = xcd_contiguous(blockIdx.x, per_xcd);
    if (g >= row_blocks * col_groups) return;
    const int rb = g / col_groups, cg = g - rb * col_groups;               // workgroups walk along the rows of the image
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_in_block();
    const int c0 = (cg * kMWaves + wave) * kMOutCols;
    if (c0 >= ow) return;
    const int r0 = rb * rows;
    const int rows_out = min(rows, oh - r0);
    const int steps = (rows_out + 3) >> 2;

    const int i16 = lane & 15, kb = lane >> 4;                             // MFMA operand coordinates of the lane

    // A operands: the Toeplitz form of the taps, constant for the whole kernel
    h8 ah[NS], al[NS];
    {
        const int jr = i16 >> 2, jc = i16 & 3;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int tr = 2 * s + (kb >> 1) - jr + 3;
            ah[s] = *reinterpret_cast<const h8*>(&wtab[0][jc][tr][8 * (kb & 1)]);
            al[s] = *reinterpret_cast<const h8*>(&wtab[1][jc][tr][8 * (kb & 1)]);
        }
    }

    MfmaFetcher fetch;
    fetch.rowp = x + (long long)r0 * xp;
    fetch.xp = xp; fetch.w_img = w_img;
    fetch.rows_left = rows_out + kh - 2;                                    // the block reads rows r0 .. r0 + rows_left
    const int flane = lane < kMUnitLanes ? lane : lane - kMUnitLanes;     // lanes 40 .. 63 shadow lanes 0 .. 23
    const int frow = flane >= 20 ? 1 : 0;
    fetch.fcol = c0 + kTile * (flane - 20 * frow);
    fetch.off_one = fetch.fcol;
    fetch.off_two = fetch.fcol + (frow ? xp : 0);
    const bool edge = c0 + kMInCols > w_img;

    _Float16* const st_w = &stage[wave][0][0][frow][kTile * (flane - 20 * frow)];          // where the lane stages
    const _Float16* const st_r = &stage[wave][0][0][kb >> 1][kTile * i16 + 8 * (kb & 1)];  // where its window starts
    constexpr int kPlane = 2 * kMInCols, kBuf = 2 * kPlane;

    h8 bh[RS], bl[RS];                     // ring: unit u lives in slot u % RS

    // ------------------------------------------------------------------- edge strips
    // Strips that reach past the right edge of the image fetch through registers with per-lane
    // bounds checks (columns outside the image read as 0), split in the 40 fetching lanes and hand
    // the fp16 values to the other lanes through a wave-private staging buffer.  They are a small
    // part of any large image, so nothing is kept in flight beyond the step at hand.
    auto run_edge = [&]() {
        float pre[2][4];
        // stage the unit in pre[k] and read the lane's windows of it into ring slot `slot`
        auto consume = [&](int k, int slot) {
            {
                h4 hi, lo;
                mfma_split(pre[k], hi, lo);
                *reinterpret_cast<h4*>(st_w + k * kBuf) = hi;              // (shadow lanes write the same values again)
                *reinterpret_cast<h4*>(st_w + k * kBuf + kPlane) = lo;
            }
            // Other lanes of this wavefront read what was just written.  The hardware serves a
            // wavefront's LDS accesses in order; all that is needed is that the compiler keeps
            // the reads behind the writes.
            asm volatile("" ::: "memory");
            const h4 h0 = *reinterpret_cast<const h4*>(st_r + k * kBuf);
            const h4 h1 = *reinterpret_cast<const h4*>(st_r + k * kBuf + 4);
            const h4 l0 = *reinterpret_cast<const h4*>(st_r + k * kBuf + kPlane);
            const h4 l1 = *reinterpret_cast<const h4*>(st_r + k * kBuf + kPlane + 4);
            bh[slot] = __builtin_shufflevector(h0, h1, 0, 1, 2, 3, 4, 5, 6, 7);
            bl[slot] = __builtin_shufflevector(l0, l1, 0, 1, 2, 3, 4, 5, 6, 7);
        };
#pragma unroll
        for (int u = 0; u < NS; ++u) {
            fetch.template next<true>(pre[u & 1]);
            consume(u & 1, u % RS);
        }
        const int col = c0 + kTile * i16;
        for (int t0 = 0; t0 < steps; t0 += PERIOD) {
#pragma unroll
            for (int ph = 0; ph < PERIOD; ++ph) {
                const int t = t0 + ph;
                if (t >= steps) break;
                fetch.template next<true>(pre[0]);
                fetch.template next<true>(pre[1]);
                f4 acc_hh = {0.0f, 0.0f, 0.0f, 0.0f}, acc_x = acc_hh;
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    const int slot = (2 * ph + s) % RS;
                    acc_x = __builtin_amdgcn_mfma_f32_16x16x32_f16(al[s], bh[slot], acc_x, 0, 0, 0);
                    acc_hh = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah[s], bh[slot], acc_hh, 0, 0, 0);
                    acc_x = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah[s], bl[slot], acc_x, 0, 0, 0);
                }
                // lane (i16, kb) holds outputs (row 4 t + kb, columns c0 + 4 i16 .. + 3)
                if (4 * t + kb < rows_out) {
                    float o[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        o[v] = __builtin_fmaf(acc_x[v], inv_scale * (1.0f / kMLoScale), acc_hh[v] * inv_scale);
                    store4_guarded(y + (long long)(r0 + 4 * t + kb) * yp, col, ow, o);
                }
                consume(0, (2 * ph + NS) % RS);
                consume(1, (2 * ph + NS + 1) % RS);
            }
        }
    };

    // ---------------------------------------------------------------- interior strips
    auto run_queued = [&]() {
        const unsigned long long fetch_lanes = (1ull << kMUnitLanes) - 1;  // lanes 0 .. 39 fetch
        const unsigned q_base = (unsigned)(size_t)&queue[wave][0][0][0];   // LDS byte address of slot 0
        const float* const win = &queue[wave][0][kb >> 1][kTile * i16 + 8 * (kb & 1)];   // the lane's window in slot 0
        int q_in = 0, q_out = 0;                                           // slots of the next unit in / out (uniform)

        auto issue = [&]() {
            mfma_dma_unit(fetch.next_address(), q_base + q_in * kMSlotBytes, fetch_lanes);
            q_in = q_in + 1 == kMQueue ? 0 : q_in + 1;
        };
        // the lane's 8-input window of the oldest queued unit -> ring slot
        auto take = [&](int slot) {
            const float* w8 = win + q_out * (kMSlotBytes / (int)sizeof(float));
            const f4 a = *reinterpret_cast<const f4*>(w8);
            const f4 b = *reinterpret_cast<const f4*>(w8 + 4);
            mfma_split8(a, b, bh[slot], bl[slot]);
            q_out = q_out + 1 == kMQueue ? 0 : q_out + 1;
        };

        // Units 0 .. NS-3 go into the ring before the first step; every step then starts by sending
        // two more units on their way and taking in the two newest units it needs (2t+NS-2 and
        // 2t+NS-1), which its last six instructions use -- their split overlaps the instructions
        // that work on the older units.  kMAhead younger loads are in flight at every wait.
#pragma unroll 1
        for (int u = 0; u < kMAhead; ++u) issue();
#pragma unroll
        for (int u = 0; u < NS - 2; ++u) {
            issue();                                                       // unit u now has kMAhead younger loads behind it
            mfma_wait_loads();
            take(u % RS);
        }

        const int col = c0 + kTile * i16;
        const long long yoff = (long long)kb * yp + col;

        auto step = [&](int t, int ph, auto whole_tag) {
            constexpr bool WHOLE = decltype(whole_tag)::value;
            // nothing moves across a step's start (the scheduler would otherwise pull the first
            // instructions of later steps' splits up to here, in front of their waits)
            __builtin_amdgcn_sched_barrier(0);
            issue();
            issue();
            mfma_wait_loads();
            take((2 * ph + NS - 2) % RS);
            take((2 * ph + NS - 1) % RS);
            f4 acc_hh = {0.0f, 0.0f, 0.0f, 0.0f}, acc_lh = acc_hh, acc_hl = acc_hh;
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const int slot = (2 * ph + s) % RS;
                acc_hh = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah[s], bh[slot], acc_hh, 0, 0, 0);
                acc_lh = __builtin_amdgcn_mfma_f32_16x16x32_f16(al[s], bh[slot], acc_lh, 0, 0, 0);
                acc_hl = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah[s], bl[slot], acc_hl, 0, 0, 0);
            }
            if (WHOLE || 4 * t + kb < rows_out) {
                f4u o4;
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    o4[v] = __builtin_fmaf(acc_lh[v] + acc_hl[v], inv_scale * (1.0f / kMLoScale), acc_hh[v] * inv_scale);
                float* yr = y + (long long)(r0 + 4 * t) * yp;              // uniform; the lane's part is yoff
                if (SYSCONV_NONTEMPORAL_STORE) __builtin_nontemporal_store(o4, reinterpret_cast<f4u*>(yr + yoff));
                else *reinterpret_cast<f4u*>(yr + yoff) = o4;
            }
        };

        const int whole_steps = rows_out >> 2;
        int t0 = 0;
        for (; t0 + PERIOD <= whole_steps; t0 += PERIOD) {
#pragma unroll
            for (int ph = 0; ph < PERIOD; ++ph) step(t0 + ph, ph, std::true_type{});
        }
#pragma unroll
        for (int ph = 0; ph < PERIOD; ++ph) {
            if (t0 + ph >= steps) break;
            step(t0 + ph, ph, std::false_type{});
        }
        // nothing may still be on its way into this workgroup's LDS when the wavefront ends
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };

    if (edge) run_edge();
    else run_queued();
}

float largest_finite_magnitude(const float* f, int n)
{
    float amax = 0.0f;
    for (int i = 0; i < n; ++i) {
        const float a = fabsf(f[i]);
        if (a > amax && a <= 3.0e38f) amax = a;                    // NaN and inf fail the comparisons
    }
    return amax;
}

template <int NS>
hipError_t launch_mfma(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw, float* y,
                       size_t yp, hipStream_t s)
{
    Taps2D taps;
    for (int i = 0; i < kTaps2DLen; ++i) taps.f[i] = i < kh * kw ? f[i] : 0.0f;
    // power of two that brings the largest tap into [2^13, 2^14): its fp16 parts are then
    // as far from the subnormal range as they can be
    const float amax = largest_finite_magnitude(f, kh * kw);
    int e = 0;
    if (amax > 0.0f) (void)frexpf(amax, &e);                      // amax = m * 2^e, 0.5 <= m < 1
    const float tap_scale = amax > 0.0f ? ldexpf(1.0f, 14 - e) : 1.0f;
    const float inv_scale = 1.0f / (tap_scale * kMXScale);

    const int oh = h - kh + 1, ow = w - kw + 1;
    const int col_groups = (ow + kMWaves * kMOutCols - 1) / (kMWaves * kMOutCols);
    int rows = 64;
    while (rows > 8 && (long long)((oh + rows - 1) / rows) * col_groups < 2048) rows >>= 1;
    const int row_blocks = (oh + rows - 1) / rows;
    const long long groups = (long long)row_blocks * col_groups;
    const long long per_xcd = (groups + kXcds - 1) / kXcds;
    const long long blocks = per_xcd * kXcds;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(conv2d_mfma_kernel<NS>, dim3((unsigned)blocks), dim3(kBlock), 0, s, taps, x, y, w,
                       (long long)xp, oh, ow, (long long)yp, kh, kw, rows, row_blocks, col_groups, (int)per_xcd,
                       tap_scale, inv_scale);
    return hipGetLastError();
}

}  // namespace

bool has_conv2d_mfma(int kh, int kw) { return kh >= 1 && kw >= 1 && kh <= 13 && kw <= 13; }

// Both the scale 2^(14-e) and its reciprocal times 2^-13 must be normal fp32 numbers.
bool conv2d_mfma_taps_in_range(const float* f, int n)
{
    const float amax = largest_finite_magnitude(f, n);
    return amax == 0.0f || (amax >= 1.0e-30f && amax <= 1.0e30f);
}

hipError_t launch_conv2d_mfma(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw,
                              float* y, size_t yp, hipStream_t s)
{
    if (!has_conv2d_mfma(kh, kw)) return hipErrorInvalidValue;
    switch ((kh + 4) / 2) {                                    // NS = ceil((kh + 3) / 2)
    case 2: return launch_mfma<2>(x, h, w, xp, f, kh, kw, y, yp, s);
    case 3: return launch_mfma<3>(x, h, w, xp, f, kh, kw, y, yp, s);
    case 4: return launch_mfma<4>(x, h, w, xp, f, kh, kw, y, yp, s);
    case 5: return launch_mfma<5>(x, h, w, xp, f, kh, kw, y, yp, s);
    case 6: return launch_mfma<6>(x, h, w, xp, f, kh, kw, y, yp, s);
    case 7: return launch_mfma<7>(x, h, w, xp, f, kh, kw, y, yp, s);
    case 8: return launch_mfma<8>(x, h, w, xp, f, kh, kw, y, yp, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace sysconv
