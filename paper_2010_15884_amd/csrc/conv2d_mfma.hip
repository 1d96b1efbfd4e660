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
// Data path.  A column group is 256 output columns, computed by 4 wavefronts (a strip of 64
// columns each) that walk a block of rows 4 rows at a time.  Input travels in "units" of 2 rows
// x 272 columns.  The four wavefronts take turns fetching units with global_load_lds_dwordx4:
// whole-wavefront loads of 1 KB per row straight into a 16-slot queue in LDS that all four read,
// so that the 12 units in flight cost no registers.  When a unit has arrived (a wait on the
// fetching wavefront's own loads, then a workgroup barrier) every lane reads its 8-input window
// (the B operand), scales, splits and packs it into a ring of NS (+1) operand pairs in registers
// -- each 2-row unit serves NS consecutive instruction slots as the block moves down -- then
// MFMA and global_store_dwordx4.  The column group at the right edge of the image runs the same
// code with the lanes beyond the image switched off in the loads (their queue entries stay 0)
// and column checks in the stores.
//
// Launch shape.  Measured on MI355X: workgroups that share a CU do not advance at the same rate
// (of three 4-wavefront workgroups started together the first ends after 77 us, the last after
// 113 us, on an 8192^2 image), and the stragglers run with too few wavefronts to keep HBM busy.
// So a workgroup is three column groups wide (12 wavefronts, the whole CU) and its barrier keeps
// them in step; the row blocks are sized so that the grid is one round of resident workgroups:
// set-up and pipeline fill are paid once, nothing starts late.  8192^2: 11x11 114 - 125 us,
// 13x13 119 - 126 us, 3x3 106 us (a copy of the same bytes: 86 us; the vector-ALU kernels take
// 243 us for 11x11); with 4-wavefront workgroups of 64 rows, many rounds: 138 us and 151 us.
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
constexpr int kMWaves = kBlock / kWave;
constexpr int kMGroupCols = kMWaves * kMOutCols;   // output columns of a workgroup
constexpr float kMXScale = 8192.0f;        // 2^13: inputs up to 8 stay finite in fp16
constexpr float kMLoScale = 2048.0f;       // 2^11: the lo parts are kept this much larger
constexpr int kMaxDevices = 64;            // devices whose occupancy answer is remembered

typedef const float __attribute__((address_space(4)))* kernarg_floats;

template <int NS>
struct MfmaShape {
    static_assert(NS >= 2 && NS <= 8, "2 <= NS <= 8 covers filters of 1 .. 13 rows");
    static constexpr int RS = NS <= 4 ? 4 : 8;     // ring slots (a power of two >= NS, >= 4)
    static constexpr int PERIOD = RS / 2;          // steps after which the ring indices repeat
    static constexpr int TROWS = 2 * NS + 3;       // rows of the tap tables: dr - jr + 3 = 0 .. 2 NS + 2
};

// The queue of units in LDS.  A slot, in floats: [0, 256) first row, [256, 512) second row,
// [512, 528) and [528, 544) the 16 halo columns of the two rows, [544, 548) a pad that takes
// the loads issued only to keep the count of loads per unit fixed.
constexpr int kSQueue = 16;                // slots
constexpr int kSAhead = 12;                // units in flight behind the two being taken; every wavefront owns a quarter
constexpr int kSCols = kMGroupCols + 16;   // input columns of a unit (a filter is at most 13 wide: 256 + 12 are read)
constexpr int kSPad = 2 * kSCols;          // float offset of the pad
constexpr int kSSlotFloats = 2 * kSCols + 4;
constexpr unsigned kSSlotBytes = kSSlotFloats * sizeof(float);
static_assert(kSQueue >= kSAhead + 4, "a slot is written again only after the barrier that follows its last reader");

__device__ __forceinline__ int shared_slot_offset(int row, int col)
{
    return col < kMGroupCols ? row * kMGroupCols + col : 2 * kMGroupCols + row * 16 + (col - kMGroupCols);
}

// Loads from global memory straight into LDS: lane l's 16 (4) bytes land at M0 + 16 l (M0 + 4 l);
// lanes switched off load nothing and write nothing.  The compiler does not see these loads as
// such; the waits for them are written by hand.
__device__ __forceinline__ void dma_b128(const float* p, unsigned lds_byte_address, unsigned long long lanes)
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

__device__ __forceinline__ void dma_b32(const float* p, unsigned lds_byte_address, unsigned long long lanes)
{
    unsigned long long saved;
    asm volatile("s_mov_b64 %0, exec\n\t"
                 "s_mov_b32 m0, %2\n\t"
                 "s_mov_b64 exec, %3\n\t"
                 "global_load_lds_dword %1, off\n\t"
                 "s_mov_b64 exec, %0"
                 : "=&s"(saved)
                 : "v"(p), "s"(lds_byte_address), "s"(lanes)
                 : "memory");
}

// A wavefront fetches every fourth unit, with kLoads loads; kSAhead = 12 younger units follow
// the one that must have arrived, three of them its own.  Vector-memory operations complete in
// the order they were issued, so "at most 3 kLoads outstanding" says that unit has landed,
// whatever stores are outstanding besides (they only make the wait stricter).
template <int kLoads>
__device__ __forceinline__ void wait_own_units()
{
    static_assert(kSAhead == 12 && (kLoads == 3 || kLoads == 5), "the waits below are written for three own units in flight");
    if (kLoads == 3) asm volatile("s_waitcnt vmcnt(9)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(15)" ::: "memory");
}

// Workgroup barrier and nothing else (no wait for outstanding memory operations: the loads in
// flight must stay in flight).
__device__ __forceinline__ void barrier_only()
{
    asm volatile("s_barrier" ::: "memory");
}

// Eight consecutive inputs times 2^13, split into fp16 hi and lo parts: v * 2^13 = hi + lo * 2^-11
// (both rounded to nearest).  The remainder v * 2^13 - hi is exact in fp32 and at most half an
// fp16 ulp of hi; stored 2^11 times larger it has the magnitude of hi at most and stays a normal
// fp16 number whenever hi is one (the matrix cores treat subnormal fp16 inputs as zero).  A value
// of 8 or more becomes infinite here and shows up as inf / NaN in the results it feeds.
__device__ __forceinline__ void mfma_split8(const f4& a, const f4& b, h8& hi, h8& lo)
{
    // Three instructions per element, spelled out (the compiler's own selection takes four):
    // v_fma_mixlo/mixhi_f16 scale in fp32 and round once to fp16 into one half of a register,
    // v_fma_mix_f32 takes v * 2^13 - hi with hi read as fp16 from either half (exact).
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    const float xs = kMXScale, ls = kMLoScale;
    u4 hp, lp;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float v0 = i < 2 ? a[2 * i] : b[2 * i - 4], v1 = i < 2 ? a[2 * i + 1] : b[2 * i - 3];
        unsigned h, l;
        float r0, r1;
        asm("v_fma_mixlo_f16 %0, %1, %2, 0" : "=v"(h) : "v"(v0), "s"(xs));
        asm("v_fma_mixhi_f16 %0, %1, %2, 0" : "+v"(h) : "v"(v1), "s"(xs));
        asm("v_fma_mix_f32 %0, %1, %2, -%3 op_sel_hi:[0,0,1]" : "=v"(r0) : "v"(v0), "s"(xs), "v"(h));
        asm("v_fma_mix_f32 %0, %1, %2, -%3 op_sel:[0,0,1] op_sel_hi:[0,0,1]" : "=v"(r1) : "v"(v1), "s"(xs), "v"(h));
        asm("v_fma_mixlo_f16 %0, %1, %2, 0" : "=v"(l) : "v"(r0), "s"(ls));
        asm("v_fma_mixhi_f16 %0, %1, %2, 0" : "+v"(l) : "v"(r1), "s"(ls));
        hp[i] = h; lp[i] = l;
    }
    hi = __builtin_bit_cast(h8, hp);
    lo = __builtin_bit_cast(h8, lp);
}

template <int NS, int G>
__global__ __launch_bounds__(G * kBlock) void conv2d_mfma_kernel(Taps2D taps, const float* __restrict__ x,
                                                             float* __restrict__ y, int w_img, long long xp,
                                                             int oh, int ow, long long yp, int kh, int kw,
                                                             int rows, int row_blocks, int col_sets, int per_xcd,
                                                             float tap_scale, float inv_scale)
{
    (void)taps;
    using S = MfmaShape<NS>;
    constexpr int RS = S::RS, PERIOD = S::PERIOD, TROWS = S::TROWS;

    // wtab[plane][jc][dr - jr + 3][dc] = hi / lo part of f[dr - jr][dc - jc] * tap_scale
    __shared__ __attribute__((aligned(16))) _Float16 wtab[2][4][TROWS][16];
    __shared__ __attribute__((aligned(16))) float squeues[G][kSQueue][kSSlotFloats];

    const int g = xcd_contiguous(blockIdx.x, per_xcd);
    if (g >= row_blocks * col_sets) return;                                // (the whole workgroup)
    const int rb = g / col_sets, cs = g - rb * col_sets;                   // workgroups walk along the rows of the image
    const int wave_wg = wave_in_block();
    const int grp = wave_wg / kMWaves, wave = wave_wg - grp * kMWaves;     // column group within the workgroup, wavefront within the group
    const int c0g = (cs * G + grp) * kMGroupCols;
    const bool beyond = c0g >= ow;                                         // uniform: a group of the last workgroup with no outputs
    float (*squeue)[kSSlotFloats] = squeues[grp];
    // Columns of the unit that lie inside the image: whole groups of four go with the 16-byte
    // loads, up to three more ("fringe") one by one; the rest is never loaded and reads as 0.
    const int in_cols = beyond ? 0 : min(w_img - c0g, kSCols);
    const bool ragged = in_cols < kSCols;                                  // uniform: the column group at the right edge
    if (ragged) {
        f4* q4 = reinterpret_cast<f4*>(&squeue[0][0]);
        for (int e = threadIdx.x & (kBlock - 1); e < kSQueue * kSSlotFloats / 4; e += kBlock) q4[e] = f4{0.0f, 0.0f, 0.0f, 0.0f};
    }

    kernarg_floats taps_f = (kernarg_floats)__builtin_amdgcn_kernarg_segment_ptr();
    for (int e = threadIdx.x; e < 4 * TROWS * 16; e += G * kBlock) {
        const int dc = e & 15, tr = (e >> 4) % TROWS, jc = e / (16 * TROWS);
        const int p = tr - 3, q = dc - jc;
        float v = 0.0f;
        if (p >= 0 && p < kh && q >= 0 && q < kw) v = taps_f[p * kw + q] * tap_scale;
        const _Float16 hi = (_Float16)v;
        wtab[0][jc][tr][dc] = hi;
        wtab[1][jc][tr][dc] = (_Float16)((v - (float)hi) * kMLoScale);
    }
    __syncthreads();

    const int lane = threadIdx.x & (kWave - 1);
    const int c0 = c0g + wave * kMOutCols;                                 // may lie beyond the image: such a strip stores nothing
    const int r0 = rb * rows;
    const int rows_out = min(rows, oh - r0);
    const int steps = (rows_out + 3) >> 2;
    const int last_row = r0 + rows_out + kh - 2;                           // last input row the block needs

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

    h8 bh[RS], bl[RS];                     // ring: unit u lives in slot u % RS

    // ------------------------------------------------------------------ fetching a unit
    // Unit u = rows r0 + 2u and r0 + 2u + 1 (past the block's last row the last row is read
    // again: that keeps the count of loads fixed, and what it brings in only feeds rows that are
    // not stored).  Whole column groups: a 1 KB load per row and one of 8 lanes for the halo
    // columns of both rows.  The ragged group: the same with the lanes beyond the image off,
    // and two 4-byte loads for the fringes; a load that would have no lane left is replaced by
    // a 4-byte load of an element inside the image into the slot's pad.
    const unsigned q_base = (unsigned)(size_t)&squeue[0][0];               // LDS byte address of slot 0
    const int full4 = in_cols >> 2;                                        // whole groups of four columns (0 .. 68)
    const int fringe = in_cols & 3;                                        // (0 when the unit is whole: 272 = 4 * 68)
    const int main4 = min(full4, kMGroupCols / 4), tail4 = full4 - main4;  // groups in the main part and in the halo part
    const unsigned long long mask_main = main4 >= 64 ? ~0ull : (1ull << main4) - 1;
    const unsigned long long mask_tail = ((1ull << tail4) - 1) * 0x11ull;  // lanes 0 .. 3: first row, 4 .. 7: second row
    const unsigned long long mask_fringe = (1ull << fringe) - 1;
    const unsigned fringe_at = (unsigned)shared_slot_offset(0, 4 * full4 < kSCols ? 4 * full4 : 0) * (unsigned)sizeof(float);
    const unsigned fringe_row = (4 * full4 < kMGroupCols ? kMGroupCols : 16) * (unsigned)sizeof(float);   // first row -> second row
    const long long off_main = c0g + kTile * lane;
    const int tail_row = (lane >> 2) & 1;
    const long long off_tail = c0g + kMGroupCols + kTile * (lane & 3);
    const long long off_fringe = c0g + 4 * full4 + (lane & 3);

    auto issue = [&](int u, auto ragged_tag) {                             // u is uniform
        constexpr bool RAGGED = decltype(ragged_tag)::value;
        if ((u & (kMWaves - 1)) != wave) return;
        const int ra = min(r0 + 2 * u, last_row), rb2 = min(r0 + 2 * u + 1, last_row);
        const float* pa = x + (long long)ra * xp;
        const float* pb = x + (long long)rb2 * xp;
        const unsigned slot = q_base + (unsigned)(u & (kSQueue - 1)) * kSSlotBytes;
        if (!RAGGED) {
            dma_b128(pa + off_main, slot, ~0ull);
            dma_b128(pb + off_main, slot + kMGroupCols * (unsigned)sizeof(float), ~0ull);
            dma_b128((tail_row ? pb : pa) + off_tail, slot + 2 * kMGroupCols * (unsigned)sizeof(float), 0xffull);
        } else {
            const unsigned pad = slot + kSPad * (unsigned)sizeof(float);
            if (main4 > 0) {
                dma_b128(pa + off_main, slot, mask_main);
                dma_b128(pb + off_main, slot + kMGroupCols * (unsigned)sizeof(float), mask_main);
            } else {
                dma_b32(pa + c0g, pad, 1ull);
                dma_b32(pb + c0g, pad, 1ull);
            }
            if (tail4 > 0) dma_b128((tail_row ? pb : pa) + off_tail, slot + 2 * kMGroupCols * (unsigned)sizeof(float), mask_tail);
            else dma_b32(pa + c0g, pad, 1ull);
            if (fringe > 0) {
                dma_b32(pa + off_fringe, slot + fringe_at, mask_fringe);
                dma_b32(pb + off_fringe, slot + fringe_at + fringe_row, mask_fringe);
            } else {
                dma_b32(pa + c0g, pad, 1ull);
                dma_b32(pb + c0g, pad, 1ull);
            }
        }
    };

    // --------------------------------------------------------- taking a unit into the ring
    const int col_w = wave * kMOutCols + kTile * i16 + 8 * (kb & 1);       // the lane's window starts here (workgroup columns)
    const float* const win_a = &squeue[0][0] + shared_slot_offset(kb >> 1, col_w);
    const float* const win_b = &squeue[0][0] + shared_slot_offset(kb >> 1, col_w + 4);
    int q_out = 0;                                                         // float offset of the oldest unit not taken yet
    auto take = [&](int slot) {
        const f4 a = *reinterpret_cast<const f4*>(win_a + q_out);
        const f4 b = *reinterpret_cast<const f4*>(win_b + q_out);
        mfma_split8(a, b, bh[slot], bl[slot]);
        q_out = q_out + kSSlotFloats == kSQueue * kSSlotFloats ? 0 : q_out + kSSlotFloats;
    };

    const int col = c0 + kTile * i16;
    const long long yoff = (long long)kb * yp + col;

    // Every step: the owners send units 2t + NS + 10 and 2t + NS + 11 on their way, every wavefront
    // waits for its own loads of units <= 2t + NS - 1, a barrier makes them visible to all, and
    // each lane takes its windows of units 2t + NS - 2 and 2t + NS - 1 into the ring.  The slot a
    // unit goes to was last read two steps earlier, before the previous step's barrier.
    auto run = [&](auto ragged_tag) {
        constexpr bool RAGGED = decltype(ragged_tag)::value;
        constexpr int kLoads = RAGGED ? 5 : 3;
#pragma unroll 1
        for (int u = 0; u < kSAhead; ++u) issue(u, ragged_tag);
#pragma unroll
        for (int u = 0; u < NS - 2; ++u) {
            issue(kSAhead + u, ragged_tag);                                // unit u now has kSAhead younger units behind it
            wait_own_units<kLoads>();
            barrier_only();
            take(u % RS);
        }

        auto step = [&](int t, int ph, auto whole_tag) {
            constexpr bool WHOLE = decltype(whole_tag)::value;
            // nothing moves across a step's start (the scheduler would otherwise pull the first
            // instructions of later steps' splits up to here, in front of their waits)
            __builtin_amdgcn_sched_barrier(0);
            issue(2 * t + NS - 2 + kSAhead, ragged_tag);
            issue(2 * t + NS - 1 + kSAhead, ragged_tag);
            wait_own_units<kLoads>();
            barrier_only();
            take((2 * ph + NS - 2) % RS);
            take((2 * ph + NS - 1) % RS);
            // hi*hi in one accumulator, the two cross terms (both 2^11 too large) in another
            f4 acc_hh = {0.0f, 0.0f, 0.0f, 0.0f}, acc_x = acc_hh;
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const int slot = (2 * ph + s) % RS;
                acc_x = __builtin_amdgcn_mfma_f32_16x16x32_f16(al[s], bh[slot], acc_x, 0, 0, 0);
                acc_hh = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah[s], bh[slot], acc_hh, 0, 0, 0);
                acc_x = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah[s], bl[slot], acc_x, 0, 0, 0);
            }
            // lane (i16, kb) holds outputs (row 4 t + kb, columns c0 + 4 i16 .. + 3)
            if (WHOLE || 4 * t + kb < rows_out) {
                float* yr = y + (long long)(r0 + 4 * t) * yp;              // uniform; the lane's part is yoff
                if (!RAGGED) {
                    f4u o4;
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        o4[v] = __builtin_fmaf(acc_x[v], inv_scale * (1.0f / kMLoScale), acc_hh[v] * inv_scale);
                    if (SYSCONV_NONTEMPORAL_STORE) __builtin_nontemporal_store(o4, reinterpret_cast<f4u*>(yr + yoff));
                    else *reinterpret_cast<f4u*>(yr + yoff) = o4;
                } else {
                    float o[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        o[v] = __builtin_fmaf(acc_x[v], inv_scale * (1.0f / kMLoScale), acc_hh[v] * inv_scale);
                    store4_guarded(yr + (long long)kb * yp, col, ow, o);
                }
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

    if (beyond) {
        // no outputs, no loads: only the barriers the other groups of the workgroup count on
        for (int b = 0; b < NS - 2 + steps; ++b) barrier_only();
    } else if (ragged) {
        run(std::true_type{});
    } else {
        run(std::false_type{});
    }
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

// How many workgroups of the kernel the device the calling thread has current holds at once
// (asked once per filter height class and device).
template <int NS, int G>
int resident_workgroups()
{
    static int cached[kMaxDevices];                                // 0: not asked yet
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    if (cached[dev] == 0) {
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, conv2d_mfma_kernel<NS, G>, G * kBlock, 0) != hipSuccess) return 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cached[dev] = per_cu * cus;
    }
    return cached[dev];
}

template <int NS, int G>
hipError_t launch_mfma_g(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw, float* y,
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
    const int col_sets = (ow + G * kMGroupCols - 1) / (G * kMGroupCols);
    // Row blocks sized so that the grid is one round of resident workgroups (or, when there are
    // more column groups than places, one block per column group): every column group is cut
    // into as many blocks as its share of the places allows, at least 8 rows each.
    const int places = resident_workgroups<NS, G>();
    if (places <= 0) return hipErrorInvalidConfiguration;
    const int cuts = places / col_sets > 1 ? places / col_sets : 1;
    const int quads = (oh + 3) / 4;
    int rows = 4 * ((quads + cuts - 1) / cuts);
    if (rows < 8) rows = 8;
    const int row_blocks = (oh + rows - 1) / rows;
    const long long groups = (long long)row_blocks * col_sets;
    const long long per_xcd = (groups + kXcds - 1) / kXcds;
    const long long blocks = per_xcd * kXcds;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((conv2d_mfma_kernel<NS, G>), dim3((unsigned)blocks), dim3(G * kBlock), 0, s, taps, x, y, w,
                       (long long)xp, oh, ow, (long long)yp, kh, kw, rows, row_blocks, col_sets, (int)per_xcd,
                       tap_scale, inv_scale);
    return hipGetLastError();
}

constexpr int kMGroups = 3;                // column groups per workgroup: 12 wavefronts, one workgroup per CU

template <int NS>
hipError_t launch_mfma(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw, float* y,
                       size_t yp, hipStream_t s)
{
    return launch_mfma_g<NS, kMGroups>(x, h, w, xp, f, kh, kw, y, yp, s);
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
