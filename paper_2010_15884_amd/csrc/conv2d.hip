// 2-D valid convolution  y[r][c] = sum_p sum_q x[r+p][c+q] * f[p][q]  (paper
// Eq. 3; the paper's systolic axis c,q is the image column) as software
// systolic arrays.  A wavefront always works on a strip of 256 consecutive
// input columns held four per lane.  In the FBS and SBM kernels neighbouring
// strips overlap by 4*halo_lanes(kw) columns and the PEs whose taps reach past
// the strip compute values that are never stored; the BFS kernels' strips do
// not overlap and fetch the kw-1 columns to their right separately.
//
//   conv2d_fbs_kernel<RPW>            any kh, kw <= 15: LDS tile, one 1-D FBS pass per filter row
//   conv2d_fbs_static_kernel<KH,KW,R> kh, kw <= 11 with min(kh, kw) <= 7: the same array with the sizes known
//                                     at compile time and each staged row's window shared by the rows it feeds
//   conv2d_bfs_block_kernel<K,K,ROWS> 2x2 .. 7x7: short row block, all loads up front
//   conv2d_bfs_kernel<K,K,PD>         8x8 .. 11x11: strip walk with rows in flight
//   conv2d_sbm_block_kernel<K,K,ROWS> 2x2 .. 7x7
//   conv2d_sbm_kernel<K,K,PD>         8x8 .. 11x11
#include "launch.h"
#include "systolic.h"
#include "tiling.h"

#include <stdlib.h>

namespace sysconv {
namespace {

// ------------------------------------------------------------- FBS 2-D -----
// Section 6.2 describes the 2-D FBS design as a set of 1-D FBS convolutions, one per
// filter row, that add into the same partial sums.  A workgroup stages a (4*RPW + kh - 1) x 256 input tile in LDS
// once; each of its four wavefronts then owns RPW output rows (RPW independent
// partial-sum vectors; RPW = 3, or 2 for tall filters) and, for every filter row p,
// re-reads the input rows r+p from LDS and runs the 1-D FBS time loop over q on them.
// Filter sizes are run-time values.

template <int NT, bool MORE, int RPW>
__device__ __forceinline__ void fbs_rows(float (&e)[RPW][4], float (&acc)[RPW][4], const float (&w)[4])
{
#pragma unroll
    for (int j = 0; j < RPW; ++j) fbs_steps<NT, MORE>(e[j], acc[j], w);
}

template <int RPW>
__global__ __launch_bounds__(kBlock) void conv2d_fbs_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                            int h, int w_img, long long xp, int oh, int ow,
                                                            long long yp, int kh, int kw, int tiles_y, int n_tiles,
                                                            int side, int per_xcd, Taps2D taps)
{
    extern __shared__ __attribute__((aligned(16))) float tile[];           // (kFbsTileRows + kh - 1) x kStrip
    constexpr int kFbsRowsPerWave = RPW;
    constexpr int kFbsTileRows = RPW * (kBlock / kWave);                   // output rows per workgroup

    const int t = xcd_contiguous(blockIdx.x, per_xcd);
    if (t >= n_tiles) return;                                              // whole workgroup leaves together
    int tile_y, tile_x;
    band_order(t, tiles_y, n_tiles / tiles_y, side, tile_y, tile_x);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_in_block();
    const int valid_lanes = kWave - halo_lanes(kw);
    const int col0 = tile_x * kTile * valid_lanes;
    const int row0 = tile_y * kFbsTileRows;

    // stage: wavefront v copies input rows v, v+4, ... of the tile (1 KB each, coalesced)
    const int in_rows = min(kFbsTileRows + kh - 1, h - row0);
    for (int rr = wave; rr < in_rows; rr += kBlock / kWave) {
        float v[4];
        load4_guarded<false>(x + (long long)(row0 + rr) * xp, col0 + kTile * lane, w_img, v);
        f4 t4;
        t4.x = v[0]; t4.y = v[1]; t4.z = v[2]; t4.w = v[3];
        *reinterpret_cast<f4*>(tile + rr * kStrip + kTile * lane) = t4;
    }
    __syncthreads();

    float acc[kFbsRowsPerWave][4];
#pragma unroll
    for (int j = 0; j < kFbsRowsPerWave; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[j][i] = 0.0f;

    const int lrow0 = wave * kFbsRowsPerWave;
#pragma nounroll
    for (int p = 0; p < kh; ++p) {
        float e[kFbsRowsPerWave][4];
#pragma unroll
        for (int j = 0; j < kFbsRowsPerWave; ++j) {
            // rows below the staged part of the tile hold stale LDS; they only feed
            // output rows >= oh, which are not stored
            const f4 t4 = *reinterpret_cast<const f4*>(tile + (lrow0 + j + p) * kStrip + kTile * lane);
            e[j][0] = t4.x; e[j][1] = t4.y; e[j][2] = t4.z; e[j][3] = t4.w;
        }
        const float* fp = taps.f + p * kw;
        int q = 0;
#pragma nounroll
        for (; q + 4 < kw; q += 4) {
            const float w[4] = {fp[q], fp[q + 1], fp[q + 2], fp[q + 3]};
            fbs_rows<4, true, RPW>(e, acc, w);
        }
        const float w[4] = {fp[q], fp[q + 1], fp[q + 2], fp[q + 3]};
        switch (kw - q) {
        case 4: fbs_rows<4, false, RPW>(e, acc, w); break;
        case 3: fbs_rows<3, false, RPW>(e, acc, w); break;
        case 2: fbs_rows<2, false, RPW>(e, acc, w); break;
        default: fbs_rows<1, false, RPW>(e, acc, w); break;
        }
    }

    if (lane < valid_lanes) {
#pragma unroll
        for (int j = 0; j < kFbsRowsPerWave; ++j) {
            const int r = row0 + lrow0 + j;
            if (r < oh) store4_guarded(y + (long long)r * yp, col0 + kTile * lane, ow, acc[j]);
        }
    }
}

// Pointer into the kernel-argument segment (constant address space: uniform
// reads become scalar loads).
typedef const float __attribute__((address_space(4)))* kernarg_floats;

// The same design with the filter size known at compile time (has_conv2d_fbs_static): every loop
// below is unrolled, the taps sit in SGPRs for the whole kernel, and the 1-D passes are taken
// input row by input row -- the array hands a staged row's inputs on from PE to PE once
// (KW-1 DPP moves) and each of the up to min(RPW, KH) output rows that the input row feeds
// takes its KW products from that one window, so the hand-overs are shared between the 1-D
// convolutions instead of repeated per filter row.
// Lanes of a strip that keep their results.  Single-row filters move as many bytes as a copy, and
// there strips that start on 64-byte boundaries measure faster (8192^2, 1x5: 98.8 -> 91.5 us), as in
// the 1-D kernels; with taller filters the rounding does not pay.
__host__ __device__ constexpr int fbs_static_valid_lanes(int kh, int kw)
{
    return kh == 1 ? ((kWave - halo_lanes(kw)) & ~3) : kWave - halo_lanes(kw);
}

template <int KH, int KW, int RPW>
__global__ __launch_bounds__(kBlock) void conv2d_fbs_static_kernel(Taps2D taps, const float* __restrict__ x,
                                                                   float* __restrict__ y, int h, int w_img,
                                                                   long long xp, int oh, int ow, long long yp,
                                                                   int tiles_y, int n_tiles, int side, int per_xcd)
{
    (void)taps;
    constexpr int kTileRows = RPW * (kBlock / kWave);                      // output rows per workgroup
    constexpr int kInRows = kTileRows + KH - 1;
    __shared__ __attribute__((aligned(16))) float tile[kInRows * kStrip];
    kernarg_floats taps_f = (kernarg_floats)__builtin_amdgcn_kernarg_segment_ptr();

    const int t = xcd_contiguous(blockIdx.x, per_xcd);
    if (t >= n_tiles) return;                                              // whole workgroup leaves together
    int tile_y, tile_x;
    band_order(t, tiles_y, n_tiles / tiles_y, side, tile_y, tile_x);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_in_block();
    constexpr int valid_lanes = fbs_static_valid_lanes(KH, KW);
    const int col0 = tile_x * kTile * valid_lanes;
    const int row0 = tile_y * kTileRows;

    // stage: wavefront v copies input rows v, v+4, ... of the tile; all its loads go out first
    const int last_row = h - 1 - row0;                                     // rows past the image repeat its last row
    constexpr int kPerWave = (kInRows + 3) / 4;
    float stage[kPerWave][4];
#pragma unroll
    for (int k = 0; k < kPerWave; ++k)
        load4_guarded<false>(x + (long long)(row0 + min(wave + 4 * k, last_row)) * xp, col0 + kTile * lane, w_img,
                             stage[k]);
#pragma unroll
    for (int k = 0; k < kPerWave; ++k) {
        const int rr = wave + 4 * k;
        if (rr < kInRows) {
            f4 t4;
            t4.x = stage[k][0]; t4.y = stage[k][1]; t4.z = stage[k][2]; t4.w = stage[k][3];
            *reinterpret_cast<f4*>(tile + rr * kStrip + kTile * lane) = t4;
        }
    }
    __syncthreads();

    float acc[RPW][4];
    const int lrow0 = wave * RPW;
#pragma unroll
    for (int rho = 0; rho < RPW + KH - 1; ++rho) {
        float win[KW + 3];
        const f4 t4 = *reinterpret_cast<const f4*>(tile + (lrow0 + rho) * kStrip + kTile * lane);
        win[0] = t4.x; win[1] = t4.y; win[2] = t4.z; win[3] = t4.w;
#pragma unroll
        for (int m = 4; m < KW + 3; ++m) win[m] = from_lane_above(win[m - 4]);   // X(c) <- X(c+1), once per row
#pragma unroll
        for (int j = 0; j < RPW; ++j) {
            const int p = rho - j;                                         // compile-time
            if (p < 0 || p >= KH) continue;
#pragma unroll
            for (int q = 0; q < KW; ++q) {
                const float wv = taps_f[p * KW + q];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (p == 0 && q == 0) acc[j][i] = wv * win[i];
                    else acc[j][i] = __builtin_fmaf(wv, win[q + i], acc[j][i]);
                }
            }
        }
    }

    if (lane < valid_lanes) {
#pragma unroll
        for (int j = 0; j < RPW; ++j) {
            const int r = row0 + lrow0 + j;
            if (r < oh) store4_guarded(y + (long long)r * yp, col0 + kTile * lane, ow, acc[j]);
        }
    }
}

// A zero the optimiser cannot see through (one SALU move).
__device__ __forceinline__ int opaque_zero()
{
    int z;
    asm volatile("s_mov_b32 %0, 0" : "=s"(z));
    return z;
}

// ------------------------------------------------------------- BFS 2-D -----
// Along the rows the array is the BFS design of Table 2 (row 2 left) with
// (c, q) read as (r, p): PE = output row, time = input row rho = r + p.  The
// PEs are the KH live partial-sum vectors of a lane; at step rho the input row
// rho is broadcast to all of them, PE r applies filter row p = rho - r (the
// weights move one PE per step while the partial sums stay), and the PE whose
// last filter row was just applied retires its output row.  Along a row the
// KW-wide window of every PE is built once by KW-1 FBS hand-overs and reused
// by all KH filter rows, so lane traffic is amortised KH times.  Everything
// streams from global memory through registers: no LDS.
//
// A wavefront walks `rows` output rows of one strip; PD input rows are in
// flight ahead of the one being consumed (PD divides KH so that the slot of a
// row in the prefetch ring is a compile-time constant of the unrolled loop).
// EDGE = the strip reaches past the right edge of the image: only then are
// loads and stores bounds-checked per lane.
enum BfsMode { kBfsFirst, kBfsMiddle, kBfsLast, kBfsChecked };

template <int KH, int KW, int PD, bool EDGE>
struct BfsStrip {
    static_assert(KH % PD == 0, "prefetch depth must divide the filter height");
    static constexpr bool kReloadTaps = KH * KW > 25;
    static constexpr int NH = (KW + 2) / 4;                                // halo float4s: ceil((KW-1)/4)

    const float* __restrict__ xrow;
    float* __restrict__ yrow;
    int col, w_img, ow, rows_out, rows_in;
    long long xp, yp;
    bool last_lane;                        // lane 63: the lane the halo enters through
    float ring[PD][4];
    float halo[PD][NH][4];                 // meaningful in lane 63 only
    float acc[KH][4];

    __device__ __forceinline__ void load_row(int row, float (&v)[4], float (&h)[NH][4]) const
    {
        // past the end of the strip the last row is read again: an unconditional load
        // keeps the control flow straight and the wait counts exact
        const float* p = xrow + (long long)min(row, rows_in - 1) * xp;
        // Halo: the KW-1 columns right of the strip, fetched by lane 63 alone (one
        // 16-byte access per float4) into the registers that the window hand-overs
        // leave untouched in that lane.
        if (last_lane) {
#pragma unroll
            for (int j = 0; j < NH; ++j) {
                if (EDGE) {
                    load4_guarded<false>(p, col + 4 * (j + 1), w_img, h[j]);
                } else {
                    const f4u t = *reinterpret_cast<const f4u*>(p + col + 4 * (j + 1));
                    h[j][0] = t.x; h[j][1] = t.y; h[j][2] = t.z; h[j][3] = t.w;
                }
            }
        }
        if (EDGE) {
            load4_guarded<false>(p, col, w_img, v);
        } else {
            // plain (cacheable) loads: the KH-1 halo rows are read again by the wavefront
            // working on the next row block and should then come from L2 / the memory-side
            // cache, not from HBM (measured on 4096^2, 5x5: 33 us against 43 us with the
            // non-temporal hint)
            const f4u t = *reinterpret_cast<const f4u*>(p + col);
            v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
        }
    }

    // KH consecutive input rows rho0 .. rho0+KH-1 (rho0 a multiple of KH, so every slot
    // index below is a compile-time constant).
    //   kBfsFirst    rho0 == 0: output rows r = rho - p < 0 do not exist (decided statically)
    //   kBfsMiddle   every (rho, p) pair is valid, no checks
    //   kBfsLast     the block that holds the last input row: run-time checks
    //   kBfsChecked  all checks at run time (one loop body for filters whose code is large)
    template <BfsMode MODE>
    __device__ __forceinline__ void block(int rho0, kernarg_floats taps_f)
    {
#pragma unroll
        for (int ph = 0; ph < KH; ++ph) {
            const int rho = rho0 + ph;
            if ((MODE == kBfsLast || MODE == kBfsChecked) && rho >= rows_in) break;

            // window of input row rho: win[m] = x[rho][col + m], m < KW + 3
            float win[KW + 3];
            float hin[NH][4];
#pragma unroll
            for (int i = 0; i < 4; ++i) win[i] = ring[ph % PD][i];
#pragma unroll
            for (int j = 0; j < NH; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) hin[j][i] = halo[ph % PD][j][i];
            load_row(rho + PD, ring[ph % PD], halo[ph % PD]);
            // X(c) <- X(c+1): lanes 0..62 take the value of the lane above, lane 63 takes
            // the next halo element
#pragma unroll
            for (int m = 4; m < KW + 3; ++m) win[m] = from_lane_above_or(win[m - 4], hin[(m - 4) / 4][(m - 4) % 4]);

            // broadcast the row to the KH partial-sum vectors it feeds
#pragma unroll
            for (int p = 0; p < KH; ++p) {
                const int slot = (ph - p + KH) % KH;                       // compile-time after unrolling
                const int r = rho - p;
                if (MODE == kBfsFirst && p > ph) continue;
                if (MODE == kBfsChecked && r < 0) continue;
                if ((MODE == kBfsLast || MODE == kBfsChecked) && r >= rows_out) continue;
                // Small filters keep all taps in SGPRs for the whole kernel.  Larger ones
                // would spill them, so each filter row is re-fetched here with scalar
                // loads; the offset is made opaque to keep the loads in the loop.
                kernarg_floats fp = taps_f + p * KW + (kReloadTaps ? opaque_zero() : 0);
#pragma unroll
                for (int q = 0; q < KW; ++q) {
                    const float wv = fp[q];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        // the first tap of the first filter row opens a fresh partial sum
                        if (p == 0 && q == 0) acc[slot][i] = wv * win[i];
                        else acc[slot][i] = __builtin_fmaf(wv, win[q + i], acc[slot][i]);
                    }
                }
            }

            // output row rho-(KH-1) has now seen all its filter rows
            const int done = rho - (KH - 1);
            constexpr int kh1 = KH - 1;
            const int dslot = (ph - kh1 + KH) % KH;
            if (MODE == kBfsFirst && ph < KH - 1) continue;
            if (done >= 0 && done < rows_out) {
                float* yr = yrow + (long long)done * yp;
                if (EDGE) {
                    store4_guarded(yr, col, ow, acc[dslot]);
                } else {
                    f4u t;
                    t.x = acc[dslot][0]; t.y = acc[dslot][1]; t.z = acc[dslot][2]; t.w = acc[dslot][3];
                    if (SYSCONV_NONTEMPORAL_STORE) __builtin_nontemporal_store(t, reinterpret_cast<f4u*>(yr + col));
                    else *reinterpret_cast<f4u*>(yr + col) = t;
                }
            }
        }
    }

    __device__ __forceinline__ void run(kernarg_floats taps_f)
    {
#pragma unroll
        for (int d = 0; d < PD; ++d) load_row(d, ring[d], halo[d]);
#pragma unroll
        for (int s = 0; s < KH; ++s) acc[s][0] = acc[s][1] = acc[s][2] = acc[s][3] = 0.0f;

        if (kReloadTaps) {
            for (int rho0 = 0; rho0 < rows_in; rho0 += KH) block<kBfsChecked>(rho0, taps_f);
        } else {
            // rows_in >= KH always; the last block is the one that contains row rows_in-1
            const int last0 = ((rows_in - 1) / KH) * KH;
            if (last0 == 0) {
                block<kBfsChecked>(0, taps_f);
            } else {
                block<kBfsFirst>(0, taps_f);
                for (int rho0 = KH; rho0 < last0; rho0 += KH) block<kBfsMiddle>(rho0, taps_f);
                block<kBfsLast>(last0, taps_f);
            }
        }
    }
};

// The taps are the FIRST kernel argument, i.e. they sit at offset 0 of the
// kernel-argument segment; reading them through that segment's pointer keeps
// run-time-indexed taps on the scalar load path (indexing the by-value struct
// itself can make the compiler copy it to scratch).
template <int KH, int KW, int PD>
__global__ __launch_bounds__(kBlock) void conv2d_bfs_kernel(Taps2D taps, const float* __restrict__ x,
                                                            float* __restrict__ y, int w_img, long long xp, int oh,
                                                            int ow, long long yp, int rows, int row_blocks,
                                                            int strips, int side, int per_xcd, int valid_lanes)
{
    (void)taps;
    (void)valid_lanes;
    kernarg_floats taps_f = (kernarg_floats)__builtin_amdgcn_kernarg_segment_ptr();
    int rb, strip;
    if (!wave_tile(per_xcd, row_blocks, strips, side, rb, strip)) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int col0 = strip * kStrip;                                       // strips are 256 outputs wide
    const int r0 = rb * rows;
    const int rows_out = min(rows, oh - r0);
    const int rows_in = rows_out + KH - 1;
    const float* xrow = x + (long long)r0 * xp;
    float* yrow = y + (long long)r0 * yp;
    const bool last_lane = lane == kWave - 1;
    constexpr int halo_cols = kTile * ((KW + 2) / 4);
    if (col0 + kStrip + halo_cols <= w_img) {
        BfsStrip<KH, KW, PD, false> st{xrow, yrow, col0 + kTile * lane, w_img, ow, rows_out, rows_in,
                                       xp, yp, last_lane, {}, {}, {}};
        st.run(taps_f);
    } else {
        BfsStrip<KH, KW, PD, true> st{xrow, yrow, col0 + kTile * lane, w_img, ow, rows_out, rows_in,
                                      xp, yp, last_lane, {}, {}, {}};
        st.run(taps_f);
    }
}

// ------------------------------------------------------------- SBM 2-D -----
// Section 5 (two projections): PE = c + q, time = p + P*q, the row loop r stays
// outside.  Every PE keeps a KH-tall column of inputs x(r..r+KH-1, s); the
// partial sum of output (r, c) starts at PE c, takes the KH products of filter
// column q there, and moves one PE up each time q advances, so after KH*KW steps
// PE c + KW - 1 holds it.  A wavefront owns a strip of 256 PEs (image columns)
// and walks down the rows with a ring of KH + PD input rows in registers (KH in
// use, PD in flight); the ring is indexed by row mod (KH+PD) and the row loop is
// unrolled that many times so that all indices are compile-time constants.
// Before storing, the result vector is read out KW-1 PEs further down (the
// results of an SBM array start at PE Q-1, Section 3.1), which lines the stores up
// with the loads.  Taps arrive transposed (filter column q contiguous).
template <int KH, int KW, int PD, bool EDGE>
struct SbmStrip {
    static constexpr int RS = KH + PD;                                     // ring size
    static constexpr bool kReloadTaps = KH * KW > 25;

    const float* __restrict__ xrow;
    float* __restrict__ yrow;
    int col, w_img, ow, rows_out, rows_in;
    long long xp, yp;
    bool lane_valid;
    float ring[RS][4];

    __device__ __forceinline__ void load_row(int row, float (&v)[4]) const
    {
        const float* p = xrow + (long long)min(row, rows_in - 1) * xp;
        if (EDGE) {
            load4_guarded<false>(p, col, w_img, v);
        } else {
            const f4u t = *reinterpret_cast<const f4u*>(p + col);
            v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
        }
    }

    __device__ __forceinline__ void run(kernarg_floats taps_t)
    {
#pragma unroll
        for (int d = 0; d < RS - 1; ++d) load_row(d, ring[d]);

        for (int r0 = 0; r0 < rows_out; r0 += RS) {
#pragma unroll
            for (int ph = 0; ph < RS; ++ph) {
                const int r = r0 + ph;
                if (r >= rows_out) break;
                // the slot of row r-1 is free now: fetch row r+KH+PD-1 into it
                load_row(r + RS - 1, ring[(ph + RS - 1) % RS]);

                float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int q = 0; q < KW; ++q) {
                    if (q > 0) {                                           // Z(s) <- Z(s-1)
                        const float below = from_lane_below(z[3]);
                        z[3] = z[2]; z[2] = z[1]; z[1] = z[0]; z[0] = below;
                    }
                    kernarg_floats ft = taps_t + q * KH + (kReloadTaps ? opaque_zero() : 0);
#pragma unroll
                    for (int p = 0; p < KH; ++p) {
                        const float wv = ft[p];
#pragma unroll
                        for (int i = 0; i < 4; ++i) z[i] = __builtin_fmaf(wv, ring[(ph + p) % RS][i], z[i]);
                    }
                }
                // read the results out KW-1 PEs further down: PE s gets output column s
#pragma unroll
                for (int t = 0; t < KW - 1; ++t) {
                    const float above = from_lane_above(z[0]);
                    z[0] = z[1]; z[1] = z[2]; z[2] = z[3]; z[3] = above;
                }
                if (lane_valid) {
                    float* yr = yrow + (long long)r * yp;
                    if (EDGE) {
                        store4_guarded(yr, col, ow, z);
                    } else {
                        f4u t;
                        t.x = z[0]; t.y = z[1]; t.z = z[2]; t.w = z[3];
                        if (SYSCONV_NONTEMPORAL_STORE) __builtin_nontemporal_store(t, reinterpret_cast<f4u*>(yr + col));
                        else *reinterpret_cast<f4u*>(yr + col) = t;
                    }
                }
            }
        }
    }
};

template <int KH, int KW, int PD>
__global__ __launch_bounds__(kBlock) void conv2d_sbm_kernel(Taps2D taps_t, const float* __restrict__ x,
                                                            float* __restrict__ y, int w_img, long long xp, int oh,
                                                            int ow, long long yp, int rows, int row_blocks,
                                                            int strips, int side, int per_xcd, int valid_lanes)
{
    (void)taps_t;
    kernarg_floats tf = (kernarg_floats)__builtin_amdgcn_kernarg_segment_ptr();
    int rb, strip;
    if (!wave_tile(per_xcd, row_blocks, strips, side, rb, strip)) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int col0 = strip * kTile * valid_lanes;
    const int r0 = rb * rows;
    const int rows_out = min(rows, oh - r0);
    const int rows_in = rows_out + KH - 1;
    const float* xrow = x + (long long)r0 * xp;
    float* yrow = y + (long long)r0 * yp;
    const bool lane_valid = lane < valid_lanes;
    if (col0 + kStrip <= w_img) {
        SbmStrip<KH, KW, PD, false> st{xrow, yrow, col0 + kTile * lane, w_img, ow, rows_out, rows_in,
                                       xp, yp, lane_valid, {}};
        st.run(tf);
    } else {
        SbmStrip<KH, KW, PD, true> st{xrow, yrow, col0 + kTile * lane, w_img, ow, rows_out, rows_in,
                                      xp, yp, lane_valid, {}};
        st.run(tf);
    }
}

// ----------------------------------------------------- BFS 2-D, block form ---
// The same BFS-along-rows x FBS-along-columns array as BfsStrip, for filters
// small enough to be bound by memory: a wavefront takes a block of ROWS output
// rows of one 256-column strip, issues the loads of ALL ROWS+KH-1 input rows up
// front, and then runs in straight-line code (no row loop, every validity test
// decided at compile time).  With every load in flight at once a wavefront pays
// one memory latency per block, and the compiler's wait counts are exact.
// The KW-1 halo columns right of the strip are the same for all lanes, so they
// are fetched with uniform (scalar) loads and enter the array in lane 63.
template <int KH, int KW, int ROWS, bool EDGE>
__device__ __forceinline__ void bfs_block_rows(kernarg_floats taps_f, const float* __restrict__ xrow,
                                               float* __restrict__ yrow, int col0, int lane, int w_img,
                                               long long xp, int ow, long long yp, int rows_out)
{
    constexpr int NIN = ROWS + KH - 1;
    constexpr int NH = (KW + 2) / 4;                                       // halo float4s
    const int col = col0 + kTile * lane;
    const int rows_in = rows_out + KH - 1;

    float v[NIN][4];
    float h[NIN][NH][4];
#pragma unroll
    for (int rho = 0; rho < NIN; ++rho) {
        // rows past the end of the block repeat its last row; they only feed output rows
        // that are not stored
        const float* p = xrow + (long long)min(rho, rows_in - 1) * xp;
        if (EDGE) {
            load4_guarded<false>(p, col, w_img, v[rho]);
#pragma unroll
            for (int j = 0; j < NH; ++j) load4_guarded<false>(p, col0 + kStrip + 4 * j, w_img, h[rho][j]);
        } else {
            const f4u t = *reinterpret_cast<const f4u*>(p + col);
            v[rho][0] = t.x; v[rho][1] = t.y; v[rho][2] = t.z; v[rho][3] = t.w;
            const float* hp = p + col0 + kStrip;                           // wave-uniform address
#pragma unroll
            for (int j = 0; j < NH; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) h[rho][j][i] = hp[4 * j + i];
        }
    }

    float acc[ROWS][4];
#pragma unroll
    for (int rho = 0; rho < NIN; ++rho) {
        float win[KW + 3];
#pragma unroll
        for (int i = 0; i < 4; ++i) win[i] = v[rho][i];
#pragma unroll
        for (int m = 4; m < KW + 3; ++m)
            win[m] = from_lane_above_or(win[m - 4], h[rho][(m - 4) / 4][(m - 4) % 4]);
#pragma unroll
        for (int p = 0; p < KH; ++p) {
            const int r = rho - p;                                         // compile-time
            if (r < 0 || r >= ROWS) continue;
#pragma unroll
            for (int q = 0; q < KW; ++q) {
                const float wv = taps_f[p * KW + q];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (p == 0 && q == 0) acc[r][i] = wv * win[i];
                    else acc[r][i] = __builtin_fmaf(wv, win[q + i], acc[r][i]);
                }
            }
        }
        const int done = rho - (KH - 1);
        if (done >= 0 && done < rows_out) {
            float* yr = yrow + (long long)done * yp;
            if (EDGE) {
                store4_guarded(yr, col, ow, acc[done]);
            } else {
                f4u t;
                t.x = acc[done][0]; t.y = acc[done][1]; t.z = acc[done][2]; t.w = acc[done][3];
                if (SYSCONV_NONTEMPORAL_STORE) __builtin_nontemporal_store(t, reinterpret_cast<f4u*>(yr + col));
                else *reinterpret_cast<f4u*>(yr + col) = t;
            }
        }
    }
}

template <int KH, int KW, int ROWS>
__global__ __launch_bounds__(kBlock) void conv2d_bfs_block_kernel(Taps2D taps, const float* __restrict__ x,
                                                                  float* __restrict__ y, int w_img, long long xp,
                                                                  int oh, int ow, long long yp, int row_blocks,
                                                                  int strips, int side, int per_xcd, int wide)
{
    (void)taps;
    kernarg_floats taps_f = (kernarg_floats)__builtin_amdgcn_kernarg_segment_ptr();
    int rb, strip;
    if (wide) {
        if (!wave_tile_wide(per_xcd, row_blocks, strips, rb, strip)) return;
    } else {
        if (!wave_tile(per_xcd, row_blocks, strips, side, rb, strip)) return;
    }
    const int lane = threadIdx.x & (kWave - 1);
    const int col0 = strip * kStrip;
    const int r0 = rb * ROWS;
    const int rows_out = min(ROWS, oh - r0);
    const float* xrow = x + (long long)r0 * xp;
    float* yrow = y + (long long)r0 * yp;
    constexpr int halo_cols = kTile * ((KW + 2) / 4);
    if (col0 + kStrip + halo_cols <= w_img)
        bfs_block_rows<KH, KW, ROWS, false>(taps_f, xrow, yrow, col0, lane, w_img, xp, ow, yp, rows_out);
    else
        bfs_block_rows<KH, KW, ROWS, true>(taps_f, xrow, yrow, col0, lane, w_img, xp, ow, yp, rows_out);
}

// ----------------------------------------------------- SBM 2-D, block form ---
// The SBM array of SbmStrip (PE = c + q, time = p + P*q) in the block form of
// bfs_block_rows: the ROWS+KH-1 input rows of a block of ROWS output rows are all
// requested up front and the output rows are then computed one after the other in
// straight-line code.  Taps arrive transposed (filter column q contiguous).
template <int KH, int KW, int ROWS, bool EDGE>
__device__ __forceinline__ void sbm_block_rows(kernarg_floats taps_t, const float* __restrict__ xrow,
                                               float* __restrict__ yrow, int col, int w_img, long long xp, int ow,
                                               long long yp, int rows_out, bool lane_valid)
{
    constexpr int NIN = ROWS + KH - 1;
    constexpr bool kReloadTaps = KH * KW > 25;
    const int rows_in = rows_out + KH - 1;

    float v[NIN][4];
#pragma unroll
    for (int rho = 0; rho < NIN; ++rho) {
        // rows past the end of the block repeat its last row; they only feed output rows
        // that are not stored
        const float* p = xrow + (long long)min(rho, rows_in - 1) * xp;
        if (EDGE) {
            load4_guarded<false>(p, col, w_img, v[rho]);
        } else {
            const f4u t = *reinterpret_cast<const f4u*>(p + col);
            v[rho][0] = t.x; v[rho][1] = t.y; v[rho][2] = t.z; v[rho][3] = t.w;
        }
    }

#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        float z[4];
#pragma unroll
        for (int q = 0; q < KW; ++q) {
            if (q > 0) {                                                   // Z(s) <- Z(s-1)
                const float below = from_lane_below(z[3]);
                z[3] = z[2]; z[2] = z[1]; z[1] = z[0]; z[0] = below;
            }
            kernarg_floats ft = taps_t + q * KH + (kReloadTaps ? opaque_zero() : 0);
#pragma unroll
            for (int p = 0; p < KH; ++p) {
                const float wv = ft[p];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (p == 0 && q == 0) z[i] = wv * v[r][i];
                    else z[i] = __builtin_fmaf(wv, v[r + p][i], z[i]);
                }
            }
        }
        // read the results out KW-1 PEs further down: PE s gets output column s
#pragma unroll
        for (int t = 0; t < KW - 1; ++t) {
            const float above = from_lane_above(z[0]);
            z[0] = z[1]; z[1] = z[2]; z[2] = z[3]; z[3] = above;
        }
        if (r < rows_out && lane_valid) {
            float* yr = yrow + (long long)r * yp;
            if (EDGE) {
                store4_guarded(yr, col, ow, z);
            } else {
                f4u t;
                t.x = z[0]; t.y = z[1]; t.z = z[2]; t.w = z[3];
                if (SYSCONV_NONTEMPORAL_STORE) __builtin_nontemporal_store(t, reinterpret_cast<f4u*>(yr + col));
                else *reinterpret_cast<f4u*>(yr + col) = t;
            }
        }
    }
}

template <int KH, int KW, int ROWS>
__global__ __launch_bounds__(kBlock) void conv2d_sbm_block_kernel(Taps2D taps_t, const float* __restrict__ x,
                                                                  float* __restrict__ y, int w_img, long long xp,
                                                                  int oh, int ow, long long yp, int row_blocks,
                                                                  int strips, int side, int per_xcd, int valid_lanes)
{
    (void)taps_t;
    kernarg_floats tf = (kernarg_floats)__builtin_amdgcn_kernarg_segment_ptr();
    int rb, strip;
    if (!wave_tile(per_xcd, row_blocks, strips, side, rb, strip)) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int col0 = strip * kTile * valid_lanes;
    const int r0 = rb * ROWS;
    const int rows_out = min(ROWS, oh - r0);
    const float* xrow = x + (long long)r0 * xp;
    float* yrow = y + (long long)r0 * yp;
    const bool lane_valid = lane < valid_lanes;
    if (col0 + kStrip <= w_img)
        sbm_block_rows<KH, KW, ROWS, false>(tf, xrow, yrow, col0 + kTile * lane, w_img, xp, ow, yp, rows_out, lane_valid);
    else
        sbm_block_rows<KH, KW, ROWS, true>(tf, xrow, yrow, col0 + kTile * lane, w_img, xp, ow, yp, rows_out, lane_valid);
}

// Lanes of an SBM strip that keep their results: 64 - halo_lanes(kw).  (Rounding the
// strip width down to whole cache lines was measured and does not pay in 2-D:
// 4096^2, 5x5: 28.1 us with 63 lanes, 29.0 with 60, 29.3 with 56.)
int strip_valid_lanes(int kw) { return kWave - halo_lanes(kw); }

void fill_taps(Taps2D& taps, const float* f, int n)
{
    for (int i = 0; i < kMaxK2D * kMaxK2D + 7; ++i) taps.f[i] = i < n ? f[i] : 0.0f;
}

// Shared launcher of the two strip-walking kernels (BFS and SBM).
template <int KH, int KW, int PD, bool SBM>
hipError_t launch_strip(const float* x, int h, int w, size_t xp, const float* f, float* y, size_t yp, hipStream_t s)
{
    // BFS reads its taps row by row, SBM column by column (transposed)
    Taps2D taps;
    float ft[KH * KW];
    for (int p = 0; p < KH; ++p)
        for (int q = 0; q < KW; ++q) ft[SBM ? q * KH + p : p * KW + q] = f[p * KW + q];
    fill_taps(taps, ft, KH * KW);
    const int oh = h - KH + 1, ow = w - KW + 1;
    // SBM strips overlap (the partial sums of the first KW-1 PEs come from the strip to
    // the left, so those lanes are redundant); BFS strips are exactly 256 outputs wide and
    // fetch the KW-1 halo columns separately
    const int valid_lanes = SBM ? strip_valid_lanes(KW) : kWave;
    const int strips = (ow + kTile * valid_lanes - 1) / (kTile * valid_lanes);
    // Rows per wavefront.  Measured on MI355X (in-process A/B sweeps): short items win
    // everywhere -- small filters are bound by memory latency and need > 8 K wavefronts
    // in flight (4096^2, 5x5, SBM: 27 us with 4 rows, 30 us with 16), large ones are
    // bound by the VALUs and lose to the tail of a coarse decomposition (8192^2, 11x11,
    // SBM: 246 us with 8 rows, 266 us with 24, 317 us with 64).  BFS pays KH(KH-1)/2
    // skipped filter-row blocks per item, so its items are a little taller.  The price
    // is halo traffic: an item re-reads KH-1 input rows; most of those re-reads hit in
    // cache (HBM reads 1.12x the image for 5x5, 1.6x for 11x11, which is bound by the
    // VALUs anyway).
    int rows = SBM ? (KH <= 5 ? 4 : 8) : (KH <= 5 ? 6 : 16);
    // Images too small to give the machine 4096 items of that height get shorter ones
    // (1024^2, 11x11: SBM 18.4 -> 12.4 us, BFS 43.9 -> 16.4 us; 2048^2, 11x11: 31 -> 25 us,
    // 44 -> 32 us; asking for 8192 or 16384 items instead costs up to 28 % elsewhere).
    while (rows > 2 && (long long)((oh + rows - 1) / rows) * strips < 4096) rows = (rows + 1) / 2;
    if (rows > oh) rows = oh;
    const int row_blocks = (oh + rows - 1) / rows;
    long long per_xcd;
    const long long blocks = tile_workgroups(row_blocks, strips, per_xcd);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    if constexpr (SBM)
        hipLaunchKernelGGL((conv2d_sbm_kernel<KH, KW, PD>), dim3((unsigned)blocks), dim3(kBlock), 0, s,
                           taps, x, y, w, (long long)xp, oh, ow, (long long)yp, rows, row_blocks, strips, band_width(xp),
                           (int)per_xcd, valid_lanes);
    else
        hipLaunchKernelGGL((conv2d_bfs_kernel<KH, KW, PD>), dim3((unsigned)blocks), dim3(kBlock), 0, s,
                           taps, x, y, w, (long long)xp, oh, ow, (long long)yp, rows, row_blocks, strips, band_width(xp),
                           (int)per_xcd, valid_lanes);
    return hipGetLastError();
}

}  // namespace

namespace {
template <int RPW>
hipError_t launch_fbs_tiles(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw, float* y,
                            size_t yp, hipStream_t s)
{
    constexpr int tile_rows = RPW * (kBlock / kWave);
    Taps2D taps;
    fill_taps(taps, f, kh * kw);
    const int oh = h - kh + 1, ow = w - kw + 1;
    const int cols = kTile * (kWave - halo_lanes(kw));
    const int tiles_x = (ow + cols - 1) / cols;
    const int tiles_y = (oh + tile_rows - 1) / tile_rows;
    const long long n_tiles = (long long)tiles_x * tiles_y;
    const long long per_xcd = (n_tiles + kXcds - 1) / kXcds;
    const long long blocks = per_xcd * kXcds;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const size_t lds = (size_t)(tile_rows + kh - 1) * kStrip * sizeof(float);
    hipLaunchKernelGGL(conv2d_fbs_kernel<RPW>, dim3((unsigned)blocks), dim3(kBlock), lds, s,
                       x, y, h, w, (long long)xp, oh, ow, (long long)yp, kh, kw, tiles_y, (int)n_tiles,
                       band_width(xp), (int)per_xcd, taps);
    return hipGetLastError();
}
}  // namespace

namespace {
template <int KH, int KW, int RPW>
hipError_t launch_fbs_static(const float* x, int h, int w, size_t xp, const float* f, float* y, size_t yp,
                             hipStream_t s)
{
    constexpr int tile_rows = RPW * (kBlock / kWave);
    Taps2D taps;
    fill_taps(taps, f, KH * KW);
    const int oh = h - KH + 1, ow = w - KW + 1;
    const int cols = kTile * fbs_static_valid_lanes(KH, KW);
    const int tiles_x = (ow + cols - 1) / cols;
    const int tiles_y = (oh + tile_rows - 1) / tile_rows;
    const long long n_tiles = (long long)tiles_x * tiles_y;
    const long long per_xcd = (n_tiles + kXcds - 1) / kXcds;
    const long long blocks = per_xcd * kXcds;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((conv2d_fbs_static_kernel<KH, KW, RPW>), dim3((unsigned)blocks), dim3(kBlock), 0, s,
                       taps, x, y, h, w, (long long)xp, oh, ow, (long long)yp, tiles_y, (int)n_tiles,
                       band_width(xp), (int)per_xcd);
    return hipGetLastError();
}

}  // namespace

// Filters whose size is known at compile time: every kh x kw with 2 <= kh, kw <= 11 of which at
// least one is at most 7 (4096^2, us, this kernel / the run-time-sized one: 9x3 29.9 / 40.4, 3x9 27.5 / 32.7,
// 11x5 41.2 / 51.0, 5x11 43.7 / 45.2, 10x4 36.3 / 48.5, 7x11 56.5 / 57.0), single rows 1 x 2..11 and
// single columns 2..11 x 1 (the two passes of a separable filter).  From 8x8 on the taps no longer
// fit the scalar registers and the unrolled form loses to the run-time-sized kernel (11x11 on
// 8192^2: 353 us with 4 rows per wavefront, 423 us with 2, against 313 us).  Output rows per wavefront
// from a sweep on MI355X (us with 1 / 2 / 3 / 4 rows): 4096^2 3x3 27.1 / 26.4 / 28.0 / 28.2,
// 5x5 32.3 / 27.7 / 28.1 / 29.6, 7x7 51.7 / 41.2 / 42.1 / 39.6; 8192^2 5x5 115.5 / 95.3 / 96.8 / 102.2.
bool has_conv2d_fbs_static(int kh, int kw)
{
    if (kh >= 2 && kh <= 11 && kw >= 2 && kw <= 11 && (kh <= 7 || kw <= 7)) return true;
    return (kh == 1 && kw >= 2 && kw <= 11) || (kw == 1 && kh >= 2 && kh <= 11);
}

namespace {
#define SYSCONV_FBS_STATIC(KH, KW, RPW) \
    if (kh == KH && kw == KW) return launch_fbs_static<KH, KW, RPW>(x, h, w, xp, f, y, yp, s)

hipError_t launch_fbs_static_any(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw, float* y,
                                 size_t yp, hipStream_t s)
{
    // two output rows per wavefront up to 5 filter rows, four from 6 on (the sweep above)
#define SYSCONV_FBS_STATIC_ROW(KH, RPW)                                                                     \
    SYSCONV_FBS_STATIC(KH, 2, RPW); SYSCONV_FBS_STATIC(KH, 3, RPW); SYSCONV_FBS_STATIC(KH, 4, RPW);       \
    SYSCONV_FBS_STATIC(KH, 5, RPW); SYSCONV_FBS_STATIC(KH, 6, RPW); SYSCONV_FBS_STATIC(KH, 7, RPW)
    SYSCONV_FBS_STATIC_ROW(2, 2); SYSCONV_FBS_STATIC_ROW(3, 2); SYSCONV_FBS_STATIC_ROW(4, 2);
    SYSCONV_FBS_STATIC_ROW(5, 2); SYSCONV_FBS_STATIC_ROW(6, 4); SYSCONV_FBS_STATIC_ROW(7, 4);
    SYSCONV_FBS_STATIC_ROW(8, 4); SYSCONV_FBS_STATIC_ROW(9, 4); SYSCONV_FBS_STATIC_ROW(10, 4); SYSCONV_FBS_STATIC_ROW(11, 4);
#undef SYSCONV_FBS_STATIC_ROW
#define SYSCONV_FBS_STATIC_WIDE(KH, RPW)                                                                    \
    SYSCONV_FBS_STATIC(KH, 8, RPW); SYSCONV_FBS_STATIC(KH, 9, RPW); SYSCONV_FBS_STATIC(KH, 10, RPW);      \
    SYSCONV_FBS_STATIC(KH, 11, RPW)
    SYSCONV_FBS_STATIC_WIDE(2, 2); SYSCONV_FBS_STATIC_WIDE(3, 2); SYSCONV_FBS_STATIC_WIDE(4, 2);
    SYSCONV_FBS_STATIC_WIDE(5, 2); SYSCONV_FBS_STATIC_WIDE(6, 4); SYSCONV_FBS_STATIC_WIDE(7, 4);
#undef SYSCONV_FBS_STATIC_WIDE
    SYSCONV_FBS_STATIC(1, 2, 4); SYSCONV_FBS_STATIC(1, 3, 4); SYSCONV_FBS_STATIC(1, 4, 4); SYSCONV_FBS_STATIC(1, 5, 4);
    SYSCONV_FBS_STATIC(1, 6, 4); SYSCONV_FBS_STATIC(1, 7, 4); SYSCONV_FBS_STATIC(1, 8, 4); SYSCONV_FBS_STATIC(1, 9, 4);
    SYSCONV_FBS_STATIC(1, 10, 4); SYSCONV_FBS_STATIC(1, 11, 4);
    SYSCONV_FBS_STATIC(2, 1, 4); SYSCONV_FBS_STATIC(3, 1, 4); SYSCONV_FBS_STATIC(4, 1, 4); SYSCONV_FBS_STATIC(5, 1, 4);
    SYSCONV_FBS_STATIC(6, 1, 4); SYSCONV_FBS_STATIC(7, 1, 4); SYSCONV_FBS_STATIC(8, 1, 4); SYSCONV_FBS_STATIC(9, 1, 4);
    SYSCONV_FBS_STATIC(10, 1, 4); SYSCONV_FBS_STATIC(11, 1, 4);
    return hipErrorInvalidValue;
}
#undef SYSCONV_FBS_STATIC
}  // namespace

hipError_t launch_conv2d_fbs(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw,
                             float* y, size_t yp, hipStream_t s)
{
    if (has_conv2d_fbs_static(kh, kw)) return launch_fbs_static_any(x, h, w, xp, f, kh, kw, y, yp, s);
    // Output rows per wavefront, measured on MI355X with 1, 2, 3, 4, 6 and 8 (us):
    //   4096^2 5x5   50.7  38.6  34.9  36.9  39.8  43.5      8192^2 5x5    178  127  122  121  125  134
    //   4096^2 7x7   63.3  50.1  48.6  49.9  53.3   -        8192^2 11x11  374  313  313  313  334  349
    //   8000^2 15x15  565   532   540   541   580  603       4096^2 3x3   38.6 33.6 33.2 34.0 33.6   -
    // Short tiles keep the LDS footprint small (more workgroups per CU); below two rows
    // the halo rows staged per tile dominate.
    if (kh <= 8) return launch_fbs_tiles<3>(x, h, w, xp, f, kh, kw, y, yp, s);
    return launch_fbs_tiles<2>(x, h, w, xp, f, kh, kw, y, yp, s);
}

// SYSCONV_TILE_WIDE=1 in the environment (read once) makes the block-form BFS kernels use the
// arrangement of wave_tile_wide().  It is a tuning aid, not a default: on 4096^2, 5x5 it cuts
// the HBM reads from 1.118 to 1.043 times the image (the cache line that holds a strip's halo
// columns is no longer fetched twice) without changing the time (26.2 -> 27.4 us); it is 6 %
// faster on 8192^2 and 5 % slower on 16384^2.
bool tile_wide_requested()
{
    static const bool wide = [] {
        const char* v = getenv("SYSCONV_TILE_WIDE");
        return v && v[0] == '1';
    }();
    return wide;
}

template <int KH, int KW, int ROWS>
hipError_t launch_bfs_block(const float* x, int h, int w, size_t xp, const float* f, float* y, size_t yp,
                            hipStream_t s)
{
    Taps2D taps;
    fill_taps(taps, f, KH * KW);
    const int oh = h - KH + 1, ow = w - KW + 1;
    const int strips = (ow + kStrip - 1) / kStrip;
    const int row_blocks = (oh + ROWS - 1) / ROWS;
    const int wide = tile_wide_requested() ? 1 : 0;
    long long per_xcd;
    const long long blocks = wide ? tile_workgroups_wide(row_blocks, strips, per_xcd)
                                  : tile_workgroups(row_blocks, strips, per_xcd);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((conv2d_bfs_block_kernel<KH, KW, ROWS>), dim3((unsigned)blocks), dim3(kBlock), 0, s,
                       taps, x, y, w, (long long)xp, oh, ow, (long long)yp, row_blocks, strips, band_width(xp),
                       (int)per_xcd, wide);
    return hipGetLastError();
}

template <int KH, int KW, int ROWS>
hipError_t launch_sbm_block(const float* x, int h, int w, size_t xp, const float* f, float* y, size_t yp,
                            hipStream_t s)
{
    Taps2D taps;
    float ft[KH * KW];
    for (int p = 0; p < KH; ++p)
        for (int q = 0; q < KW; ++q) ft[q * KH + p] = f[p * KW + q];      // filter column q contiguous
    fill_taps(taps, ft, KH * KW);
    const int oh = h - KH + 1, ow = w - KW + 1;
    const int valid_lanes = strip_valid_lanes(KW);
    const int strips = (ow + kTile * valid_lanes - 1) / (kTile * valid_lanes);
    const int row_blocks = (oh + ROWS - 1) / ROWS;
    long long per_xcd;
    const long long blocks = tile_workgroups(row_blocks, strips, per_xcd);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((conv2d_sbm_block_kernel<KH, KW, ROWS>), dim3((unsigned)blocks), dim3(kBlock), 0, s,
                       taps, x, y, w, (long long)xp, oh, ow, (long long)yp, row_blocks, strips, band_width(xp),
                       (int)per_xcd, valid_lanes);
    return hipGetLastError();
}

bool has_conv2d_bfs(int kh, int kw)
{
    return kh == kw && kh >= 2 && kh <= 11;
}

hipError_t launch_conv2d_bfs(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw,
                             float* y, size_t yp, hipStream_t s)
{
    if (kh != kw) return hipErrorInvalidValue;
    switch (kh) {
    // Filters up to 7x7 are bound by memory on large images and run the block form (block
    // heights from a sweep on 4096^2, cold data: 2x2..5x5: 29 us with 2 rows against 31-35 us
    // for taller blocks or the strip walk; 6x6: 35 us with 3; 7x7: 38 us with 4); from 8x8 on
    // the VALUs bound the kernel and the strip walk with its register ring is faster.
    case 2: return launch_bfs_block<2, 2, 2>(x, h, w, xp, f, y, yp, s);
    case 3: return launch_bfs_block<3, 3, 2>(x, h, w, xp, f, y, yp, s);
    case 4: return launch_bfs_block<4, 4, 2>(x, h, w, xp, f, y, yp, s);
    case 5: return launch_bfs_block<5, 5, 2>(x, h, w, xp, f, y, yp, s);
    case 6: return launch_bfs_block<6, 6, 3>(x, h, w, xp, f, y, yp, s);
    case 7: return launch_bfs_block<7, 7, 4>(x, h, w, xp, f, y, yp, s);
    case 8: return launch_strip<8, 8, 2, false>(x, h, w, xp, f, y, yp, s);
    case 9: return launch_strip<9, 9, 1, false>(x, h, w, xp, f, y, yp, s);
    case 10: return launch_strip<10, 10, 1, false>(x, h, w, xp, f, y, yp, s);
    case 11: return launch_strip<11, 11, 1, false>(x, h, w, xp, f, y, yp, s);
    default: return hipErrorInvalidValue;
    }
}

bool has_conv2d_sbm(int kh, int kw) { return has_conv2d_bfs(kh, kw); }

hipError_t launch_conv2d_sbm(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw,
                             float* y, size_t yp, hipStream_t s)
{
    if (kh != kw) return hipErrorInvalidValue;
    switch (kh) {
    // Up to 7x7 the block form (all loads of a short row block up front) beats the strip walk
    // (4096^2: 2x2 33.8 -> 30.3 us, 3x3 32.1 -> 28.6, 5x5 34.2 -> 31.4, 7x7 39.2 -> 37.9;
    // 16384 x 40960, 5x5: 1191 -> 1119 us); block heights from a sweep over 1, 2, 3, 4, 6 rows.
    case 2: return launch_sbm_block<2, 2, 2>(x, h, w, xp, f, y, yp, s);
    case 3: return launch_sbm_block<3, 3, 2>(x, h, w, xp, f, y, yp, s);
    case 4: return launch_sbm_block<4, 4, 2>(x, h, w, xp, f, y, yp, s);
    case 5: return launch_sbm_block<5, 5, 4>(x, h, w, xp, f, y, yp, s);
    case 6: return launch_sbm_block<6, 6, 4>(x, h, w, xp, f, y, yp, s);
    case 7: return launch_sbm_block<7, 7, 4>(x, h, w, xp, f, y, yp, s);
    case 8: return launch_strip<8, 8, 2, true>(x, h, w, xp, f, y, yp, s);
    case 9: return launch_strip<9, 9, 2, true>(x, h, w, xp, f, y, yp, s);
    case 10: return launch_strip<10, 10, 1, true>(x, h, w, xp, f, y, yp, s);
    case 11: return launch_strip<11, 11, 1, true>(x, h, w, xp, f, y, yp, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace sysconv
