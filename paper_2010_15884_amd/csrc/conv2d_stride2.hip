// 2-D valid convolution with stride 2 on both axes,
//     y[r][c] = sum_p sum_q x[2r+p][2c+q] * f[p][q],
// as the FBS design: the stride-2 FBS array of Table 2 (row 3 right) along the image
// columns, one 1-D pass per filter row as in the stride-1 2-D FBS kernel (Section 6.2),
// all passes adding into the same partial sums.
//
// A workgroup stages a (2*(4*RPW-1) + kh) x 512 input tile in LDS; each of its four
// wavefronts owns RPW output rows.  For filter row p a lane reads eight consecutive
// inputs of image row 2r+p -- x(2c) and x(2c+1) of its four PEs -- and the even and the
// odd taps of that filter row then run as two stride-1 FBS chains over the
// de-interleaved values (the hand-over X(c,q) = X(c+1,q-2) never mixes the two).
#include "launch.h"
#include "systolic.h"
#include "tiling.h"

namespace sysconv {
namespace {

typedef const float __attribute__((address_space(4)))* kernarg_floats;

constexpr int kCols = 2 * kStrip;                        // input columns of a tile (eight per lane)
constexpr int kRowTaps = 20;                             // per filter row: 8 even taps, 8 odd taps, 4 of slack
struct TapsStride2D { float f[kMaxK2D * kRowTaps]; };

template <int NT, bool MORE, int RPW>
__device__ __forceinline__ void chain_rows(float (&e)[RPW][4], float (&acc)[RPW][4], const float (&w)[4])
{
#pragma unroll
    for (int j = 0; j < RPW; ++j) fbs_steps<NT, MORE>(e[j], acc[j], w);
}

// All kc >= 1 time steps of one chain of one filter row, for the RPW rows of a wavefront.
template <int RPW>
__device__ __forceinline__ void run_chain(float (&e)[RPW][4], float (&acc)[RPW][4], kernarg_floats w, int kc)
{
    int j = 0;
#pragma nounroll
    for (; j + 4 < kc; j += 4) {
        const float wb[4] = {w[j], w[j + 1], w[j + 2], w[j + 3]};
        chain_rows<4, true, RPW>(e, acc, wb);
    }
    const float wb[4] = {w[j], w[j + 1], w[j + 2], w[j + 3]};
    switch (kc - j) {                                    // uniform across the wavefront
    case 4: chain_rows<4, false, RPW>(e, acc, wb); break;
    case 3: chain_rows<3, false, RPW>(e, acc, wb); break;
    case 2: chain_rows<2, false, RPW>(e, acc, wb); break;
    default: chain_rows<1, false, RPW>(e, acc, wb); break;
    }
}

// The taps are the first kernel argument (offset 0 of the kernel-argument segment).
template <int RPW>
__global__ __launch_bounds__(kBlock) void conv2d_fbs_stride2_kernel(TapsStride2D taps, const float* __restrict__ x,
                                                                    float* __restrict__ y, int h, int w_img,
                                                                    long long xp, int oh, int ow, long long yp,
                                                                    int kh, int kw, int tiles_y, int n_tiles, int side,
                                                                    int per_xcd)
{
    extern __shared__ __attribute__((aligned(16))) float tile[];           // (2*(kTileRows-1) + kh) x kCols
    constexpr int kTileRows = RPW * (kBlock / kWave);                      // output rows per workgroup
    (void)taps;
    kernarg_floats tw = (kernarg_floats)__builtin_amdgcn_kernarg_segment_ptr();

    const int t = xcd_contiguous(blockIdx.x, per_xcd);
    if (t >= n_tiles) return;                                              // whole workgroup leaves together
    int tile_y, tile_x;
    band_order(t, tiles_y, n_tiles / tiles_y, side, tile_y, tile_x);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_in_block();
    const int ke = (kw + 1) / 2, ko = kw / 2;                              // even taps q = 0, 2, ..; odd taps q = 1, 3, ..
    const int valid_lanes = kWave - halo_lanes(ke);
    const int out_col0 = tile_x * kTile * valid_lanes;
    const int out_row0 = tile_y * kTileRows;
    const int in_col0 = 2 * out_col0, in_row0 = 2 * out_row0;

    // stage: wavefront v copies input rows v, v+4, ... of the tile (2 KB each, coalesced)
    const int in_rows = min(2 * (kTileRows - 1) + kh, h - in_row0);
    for (int rr = wave; rr < in_rows; rr += kBlock / kWave) {
        const float* src = x + (long long)(in_row0 + rr) * xp;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            float v[4];
            load4_guarded<false>(src, in_col0 + half * kStrip + kTile * lane, w_img, v);
            f4 t4;
            t4.x = v[0]; t4.y = v[1]; t4.z = v[2]; t4.w = v[3];
            *reinterpret_cast<f4*>(tile + rr * kCols + half * kStrip + kTile * lane) = t4;
        }
    }
    __syncthreads();

    float acc[RPW][4];
#pragma unroll
    for (int j = 0; j < RPW; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[j][i] = 0.0f;

    const int lrow0 = wave * RPW;
#pragma nounroll
    for (int p = 0; p < kh; ++p) {
        float ev[RPW][4], od[RPW][4];
#pragma unroll
        for (int j = 0; j < RPW; ++j) {
            // rows below the staged part of the tile hold stale LDS; they only feed
            // output rows >= oh, which are not stored
            const float* row = tile + (2 * (lrow0 + j) + p) * kCols + 2 * kTile * lane;
            const f4 lo = *reinterpret_cast<const f4*>(row), hi = *reinterpret_cast<const f4*>(row + 4);
            ev[j][0] = lo.x; od[j][0] = lo.y; ev[j][1] = lo.z; od[j][1] = lo.w;
            ev[j][2] = hi.x; od[j][2] = hi.y; ev[j][3] = hi.z; od[j][3] = hi.w;
        }
        kernarg_floats fp = tw + p * kRowTaps;
        run_chain<RPW>(ev, acc, fp, ke);
        if (ko > 0) run_chain<RPW>(od, acc, fp + 8, ko);
    }

    if (lane < valid_lanes) {
#pragma unroll
        for (int j = 0; j < RPW; ++j) {
            const int r = out_row0 + lrow0 + j;
            if (r < oh) store4_guarded(y + (long long)r * yp, out_col0 + kTile * lane, ow, acc[j]);
        }
    }
}

// ------------------------------------------------------------ block form ----
// For the small square filters of the paper's experiment (Section 6) the same array
// without LDS: a wavefront takes ROWS output rows of a strip of 512 input columns,
// requests all 2*(ROWS-1)+KH input rows up front (eight consecutive inputs per lane and
// row) and then, input row by input row, builds the shifted windows of the even and of
// the odd chain once and applies them to every output row whose filter covers that input
// row (p = rho - 2r).  Strips overlap like the tiles above: the PEs whose even chain
// would reach past lane 63 compute values that are never stored.
template <int KH, int KW, int ROWS, bool EDGE>
__device__ __forceinline__ void stride2_block_rows(kernarg_floats taps_f, const float* __restrict__ xrow,
                                                   float* __restrict__ yrow, int in_col, int out_col, int w_img,
                                                   long long xp, int ow, long long yp, int rows_out, bool lane_valid)
{
    constexpr int NIN = 2 * (ROWS - 1) + KH;
    constexpr int KE = (KW + 1) / 2, KO = KW / 2;
    const int rows_in = 2 * (rows_out - 1) + KH;

    float v[NIN][8];
#pragma unroll
    for (int rho = 0; rho < NIN; ++rho) {
        // rows past the end of the block repeat its last row; they only feed output rows
        // that are not stored
        const float* p = xrow + (long long)min(rho, rows_in - 1) * xp;
        if (EDGE) {
            float lo[4], hi[4];
            load4_guarded<false>(p, in_col, w_img, lo);
            load4_guarded<false>(p, in_col + 4, w_img, hi);
#pragma unroll
            for (int i = 0; i < 4; ++i) { v[rho][i] = lo[i]; v[rho][4 + i] = hi[i]; }
        } else {
            const f4u lo = *reinterpret_cast<const f4u*>(p + in_col), hi = *reinterpret_cast<const f4u*>(p + in_col + 4);
            v[rho][0] = lo.x; v[rho][1] = lo.y; v[rho][2] = lo.z; v[rho][3] = lo.w;
            v[rho][4] = hi.x; v[rho][5] = hi.y; v[rho][6] = hi.z; v[rho][7] = hi.w;
        }
    }

    float acc[ROWS][4];
#pragma unroll
    for (int rho = 0; rho < NIN; ++rho) {
        float ev[KE + 3], od[KO + 3];
#pragma unroll
        for (int i = 0; i < 4; ++i) { ev[i] = v[rho][2 * i]; od[i] = v[rho][2 * i + 1]; }
#pragma unroll
        for (int m = 4; m < KE + 3; ++m) ev[m] = from_lane_above(ev[m - 4]);
#pragma unroll
        for (int m = 4; m < KO + 3; ++m) od[m] = from_lane_above(od[m - 4]);
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            const int p = rho - 2 * r;                                     // compile-time
            if (p < 0 || p >= KH) continue;
#pragma unroll
            for (int q = 0; q < KW; ++q) {
                const float wv = taps_f[p * KW + q];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float xv = (q & 1) ? od[q / 2 + i] : ev[q / 2 + i];
                    if (p == 0 && q == 0) acc[r][i] = wv * xv;
                    else acc[r][i] = __builtin_fmaf(wv, xv, acc[r][i]);
                }
            }
            if (p == KH - 1 && r < rows_out && lane_valid) {
                float* yr = yrow + (long long)r * yp;
                if (EDGE) {
                    store4_guarded(yr, out_col, ow, acc[r]);
                } else {
                    f4u t;
                    t.x = acc[r][0]; t.y = acc[r][1]; t.z = acc[r][2]; t.w = acc[r][3];
                    if (SYSCONV_NONTEMPORAL_STORE) __builtin_nontemporal_store(t, reinterpret_cast<f4u*>(yr + out_col));
                    else *reinterpret_cast<f4u*>(yr + out_col) = t;
                }
            }
        }
    }
}

// The taps (row-major, as the caller gave them) are the first kernel argument.
template <int KH, int KW, int ROWS>
__global__ __launch_bounds__(kBlock) void conv2d_fbs_stride2_block_kernel(Taps2D taps, const float* __restrict__ x,
                                                                          float* __restrict__ y, int w_img,
                                                                          long long xp, int oh, int ow, long long yp,
                                                                          int row_blocks, int strips, int side,
                                                                          int per_xcd)
{
    (void)taps;
    kernarg_floats tf = (kernarg_floats)__builtin_amdgcn_kernarg_segment_ptr();
    int rb, strip;
    if (!wave_tile(per_xcd, row_blocks, strips, side, rb, strip)) return;
    constexpr int valid_lanes = kWave - halo_lanes((KW + 1) / 2);
    const int lane = threadIdx.x & (kWave - 1);
    const int out_col0 = strip * kTile * valid_lanes;
    const int r0 = rb * ROWS;
    const int rows_out = min(ROWS, oh - r0);
    const float* xrow = x + (long long)(2 * r0) * xp;
    float* yrow = y + (long long)r0 * yp;
    const bool lane_valid = lane < valid_lanes;
    const int in_col = 2 * out_col0 + 2 * kTile * lane, out_col = out_col0 + kTile * lane;
    // interior strips: all 512 input columns exist, and then so do the valid lanes' outputs
    if (2 * out_col0 + kCols <= w_img)
        stride2_block_rows<KH, KW, ROWS, false>(tf, xrow, yrow, in_col, out_col, w_img, xp, ow, yp, rows_out, lane_valid);
    else
        stride2_block_rows<KH, KW, ROWS, true>(tf, xrow, yrow, in_col, out_col, w_img, xp, ow, yp, rows_out, lane_valid);
}

template <int KH, int KW, int ROWS>
hipError_t launch_block(const float* x, int h, int w, size_t xp, const float* f, float* y, size_t yp, hipStream_t s)
{
    Taps2D taps;
    for (int i = 0; i < kTaps2DLen; ++i) taps.f[i] = i < KH * KW ? f[i] : 0.0f;
    const int oh = (h - KH) / 2 + 1, ow = (w - KW) / 2 + 1;
    const int cols = kTile * (kWave - halo_lanes((KW + 1) / 2));
    const int strips = (ow + cols - 1) / cols;
    const int row_blocks = (oh + ROWS - 1) / ROWS;
    long long per_xcd;
    const long long blocks = tile_workgroups(row_blocks, strips, per_xcd);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((conv2d_fbs_stride2_block_kernel<KH, KW, ROWS>), dim3((unsigned)blocks), dim3(kBlock), 0, s,
                       taps, x, y, w, (long long)xp, oh, ow, (long long)yp, row_blocks, strips, band_width(xp),
                       (int)per_xcd);
    return hipGetLastError();
}

template <int RPW>
hipError_t launch_tiles(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw, float* y, size_t yp,
                        hipStream_t s)
{
    constexpr int tile_rows = RPW * (kBlock / kWave);
    TapsStride2D taps;
    for (int i = 0; i < kMaxK2D * kRowTaps; ++i) taps.f[i] = 0.0f;
    for (int p = 0; p < kh; ++p)
        for (int q = 0; q < kw; ++q) taps.f[p * kRowTaps + (q & 1) * 8 + q / 2] = f[p * kw + q];
    const int oh = (h - kh) / 2 + 1, ow = (w - kw) / 2 + 1;
    const int cols = kTile * (kWave - halo_lanes((kw + 1) / 2));
    const int tiles_x = (ow + cols - 1) / cols;
    const int tiles_y = (oh + tile_rows - 1) / tile_rows;
    const long long n_tiles = (long long)tiles_x * tiles_y;
    const long long per_xcd = (n_tiles + kXcds - 1) / kXcds;
    const long long blocks = per_xcd * kXcds;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const size_t lds = (size_t)(2 * (tile_rows - 1) + kh) * kCols * sizeof(float);
    hipLaunchKernelGGL(conv2d_fbs_stride2_kernel<RPW>, dim3((unsigned)blocks), dim3(kBlock), lds, s,
                       taps, x, y, h, w, (long long)xp, oh, ow, (long long)yp, kh, kw, tiles_y, (int)n_tiles,
                       band_width(xp), (int)per_xcd);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_conv2d_fbs_stride2(const float* x, int h, int w, size_t xp, const float* f, int kh, int kw,
                                     float* y, size_t yp, hipStream_t s)
{
    // Square filters up to 5x5 run the block form, two output rows per wavefront (8192^2, 5x5: 70 us
    // against 88 us for the LDS tiles and 56 us for a copy of the same bytes; 1, 3 and 4 rows: 83, 68, 74 us;
    // 2x2: 58.6 against 64.8 us); everything else the tiles.
    if (kh == kw) {
        switch (kh) {
        case 2: return launch_block<2, 2, 2>(x, h, w, xp, f, y, yp, s);
        case 3: return launch_block<3, 3, 2>(x, h, w, xp, f, y, yp, s);
        case 4: return launch_block<4, 4, 2>(x, h, w, xp, f, y, yp, s);
        case 5: return launch_block<5, 5, 2>(x, h, w, xp, f, y, yp, s);
        default: break;
        }
    }
    return launch_tiles<2>(x, h, w, xp, f, kh, kw, y, yp, s);
}

}  // namespace sysconv
