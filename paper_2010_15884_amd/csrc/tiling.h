// Work order of the 2-D kernels: which workgroup / wavefront takes which tile of the
// image (gfx950: 8 XCDs with one L2 each, workgroups dealt to them round-robin).
#pragma once

#include "systolic.h"

namespace sysconv {

constexpr int kStrip = kWave * kTile;                                      // 256 input columns per register group
constexpr int kXcds = 8;       // L2 caches (one per XCD); workgroups are dealt to them round-robin

// Workgroup b runs on XCD b % 8.  Give every XCD one contiguous run of work
// items, so that items that share halo rows meet in the same L2.
__device__ __forceinline__ int xcd_contiguous(int b, int per_xcd)
{
    return (b % kXcds) * per_xcd + (b / kXcds);
}

// Wavefront -> (row block, strip) for the kernels whose wavefronts each take one
// block of rows of one 256-column strip.
//   - The four wavefronts of a workgroup take four vertically adjacent row blocks of
//     one strip: the halo rows they share are fetched by one CU at about the same time.
//   - Workgroups are ordered strip after strip across a band of `side` strips, then one
//     step down, and on to the next band when the bottom is reached.  side = 1 walks
//     down single strips, which puts the pitch between all concurrent requests;
//     side = 16 keeps long contiguous pieces of image rows in flight, side >= strips is plain
//     row-major order (band_width()).
//   - Every XCD owns one contiguous run of workgroups in that order, so row blocks that
//     share halo rows meet in one L2.
// Returns false for a wavefront without work (uniform per wavefront).
__device__ __forceinline__ void band_order(int g, int steps_down, int strips, int side, int& down, int& strip)
{
    side = min(side, strips);                                              // (whole rows: one band)
    const int per_band = side * steps_down;
    const int full = strips / side;                                        // bands of `side` strips
    const int band = min(g / per_band, full);
    const int width = band < full ? side : strips - full * side;           // the last band takes what is left (> 0 here)
    const int within = g - band * per_band;
    down = within / width;
    strip = band * side + (within - down * width);
}

__device__ __forceinline__ bool wave_tile(int per_xcd, int row_blocks, int strips, int side, int& rb, int& strip)
{
    constexpr int kWaves = kBlock / kWave;
    const int g = xcd_contiguous(blockIdx.x, per_xcd);
    const int rb_groups = (row_blocks + kWaves - 1) / kWaves;
    if (g >= rb_groups * strips) return false;
    int rbg;
    band_order(g, rb_groups, strips, side, rbg, strip);
    rb = rbg * kWaves + wave_in_block();
    return rb < row_blocks;
}

// The other arrangement: the four wavefronts of a workgroup take four horizontally adjacent
// strips of ONE row block (a 1024-column piece of ROWS rows), and workgroups walk down such a
// column of pieces before moving to the next.  The halo columns of a strip are the first
// columns of its right neighbour; here three of four such neighbours are in the same workgroup,
// so the cache line they share is fetched from memory once.
__device__ __forceinline__ bool wave_tile_wide(int per_xcd, int row_blocks, int strips, int& rb, int& strip)
{
    constexpr int kWaves = kBlock / kWave;
    const int g = xcd_contiguous(blockIdx.x, per_xcd);
    const int strip_groups = (strips + kWaves - 1) / kWaves;
    if (g >= row_blocks * strip_groups) return false;
    const int sg = g / row_blocks;
    rb = g - sg * row_blocks;
    strip = sg * kWaves + wave_in_block();
    return strip < strips;
}

inline long long tile_workgroups_wide(int row_blocks, int strips, long long& per_xcd)
{
    const long long groups = (long long)row_blocks * ((strips + (kBlock / kWave) - 1) / (kBlock / kWave));
    per_xcd = (groups + kXcds - 1) / kXcds;
    return per_xcd * kXcds;
}

// Strips per band, from in-process A/B runs on MI355X (block-form BFS, 5x5 unless noted;
// us with 1 / 16 strips per band / whole rows):
//   pitch 16 KB (4096^2) 26.0 / 29.8 / 29.5, (8192 x 4096) 50 / 57 / 58, pitch 8 KB (16384 x 2048) 54 / 61 / 61,
//   pitch 32 KB (8192^2) 130 / 101 / 98.5 (SBM 150 / 116; 7x7 156 / 130), (4096 x 8192) 65 / 53 / 58,
//   pitch 64 KB (2048 x 16384) 78 / 52 / 60, (16384^2) 657 / 397 / 421, (40960 x 16384) 1275 / 971,
//   pitch 18 KB (4608^2) 39.1 / 36.4 / 33.9, 20 KB 44.4 / 45.3 / 41.9, 28 KB 89.5 / 83.1 / 80.5, 40 KB 184 / 174 / 167,
//   48 KB 260 / 241 / 236, 160 KB (16384 x 40960) 1381 / 1096 / 1085, 14 KB 24.8 / 22.7 / 22.7, 12 KB level;
//   4 and 8 strips lie between.  Whole rows (plain row-major order) are best or level at every pitch
//   tried that is not a power of two; at power-of-two pitches single strips win while the rows are
//   short, bands of 16 from 32 KB on.
constexpr int kWholeRows = 1 << 30;                                        // band_order() clamps to the strips there are
inline int band_width(size_t x_pitch)
{
    const size_t bytes = x_pitch * sizeof(float);
    if ((bytes & (bytes - 1)) != 0) return kWholeRows;
    return bytes >= 32768 ? 16 : 1;
}

// Workgroups a launch of such a kernel needs (a multiple of the XCD count) and the
// length of an XCD's run.
inline long long tile_workgroups(int row_blocks, int strips, long long& per_xcd)
{
    const long long groups = (long long)((row_blocks + (kBlock / kWave) - 1) / (kBlock / kWave)) * strips;
    per_xcd = (groups + kXcds - 1) / kXcds;
    return per_xcd * kXcds;
}

}  // namespace sysconv
