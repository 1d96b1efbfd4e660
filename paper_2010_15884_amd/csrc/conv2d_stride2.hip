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
    return launch_tiles<2>(x, h, w, xp, f, kh, kw, y, yp, s);
}

}  // namespace sysconv
