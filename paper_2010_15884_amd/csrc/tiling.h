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
//     side = 16 keeps long contiguous pieces of image rows in flight (band_width()).
//   - Every XCD owns one contiguous run of workgroups in that order, so row blocks that
//     share halo rows meet in one L2.
// Returns false for a wavefront without work (uniform per wavefront).
__device__ __forceinline__ void band_order(int g, int steps_down, int strips, int side, int& down, int& strip)
{
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
// us with 1 / 16 strips per band):
//   pitch 16 KB (4096^2) 28.6 / 33.2, 20 KB 46 / 48, 24 KB and 28 KB level,
//   pitch 32 KB (8192^2) 133 / 104 (SBM 150 / 116; 7x7 156 / 130), 48 KB level,
//   pitch 64 KB (2048 x 16384) 59 / 46, (40960 x 16384) 1275 / 971,
//   pitch 160 KB (16384 x 40960) 1320 / 1016 (2x2: 1289 / 969), pitch 2.5 MB 1117 / 1084;
//   4 and 8 strips lie between.  Single strips win while the rows are short, bands as
//   soon as walking down a strip strides over 32 KB or more.
inline int band_width(size_t x_pitch) { return x_pitch * sizeof(float) >= 32768 ? 16 : 1; }

// Workgroups a launch of such a kernel needs (a multiple of the XCD count) and the
// length of an XCD's run.
inline long long tile_workgroups(int row_blocks, int strips, long long& per_xcd)
{
    const long long groups = (long long)((row_blocks + (kBlock / kWave) - 1) / (kBlock / kWave)) * strips;
    per_xcd = (groups + kXcds - 1) / kXcds;
    return per_xcd * kXcds;
}

}  // namespace sysconv
