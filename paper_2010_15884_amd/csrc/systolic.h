// Device-side building blocks shared by the 1-D and 2-D kernels (gfx950 only).
//
// Layout of a "register group": lane l of a wavefront holds four consecutive
// fp32 elements (one dwordx4), so a group is a virtual vector of 256 processing
// elements, PE index s = 4*l + i.  Moving a value from PE s+1 to PE s is a
// register rename for i = 0..2 and a one-lane DPP move for i = 3; moving it the
// other way is the mirror image.  Those two moves are the only cross-PE traffic
// the systolic designs of the paper (Section 3.1, Table 2) need.
#pragma once

#include <hip/hip_runtime.h>

namespace sysconv {

constexpr int kWave = 64;          // lanes of a gfx950 wavefront
constexpr int kTile = 4;           // consecutive elements per lane in a register group
constexpr int kBlock = 256;        // threads per workgroup: 4 wavefronts

// A dwordx4 access that is only promised dword alignment.  Global memory
// instructions of gfx9 need no more; the compiler still emits one
// global_load_dwordx4 / global_store_dwordx4.
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
typedef float f4 __attribute__((ext_vector_type(4)));

// DPP controls (GFX9 encoding): whole-wavefront shifts by one lane.
constexpr int kDppWaveShl1 = 0x130;   // lane l reads lane l+1; lane 63 reads nothing
constexpr int kDppWaveShr1 = 0x138;   // lane l reads lane l-1; lane 0 reads nothing

// Index of this wavefront inside its workgroup, as a scalar (the compiler cannot
// see by itself that threadIdx.x / 64 is uniform across a wavefront).
__device__ __forceinline__ int wave_in_block()
{
    return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
}

// Value of the next-higher lane (lane 63 gets 0): the input hand-over of the
// FBS design, X(c) <- X(c+1).
__device__ __forceinline__ float from_lane_above(float v)
{
    return __builtin_bit_cast(float,
        __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kDppWaveShl1, 0xf, 0xf, true));
}

// Same hand-over, but lane 63 keeps `edge` (the element that enters the array from
// outside the register group).  bound_ctrl off: a lane without a source keeps the
// destination's old value, which is `edge`.
__device__ __forceinline__ float from_lane_above_or(float v, float edge)
{
    return __builtin_bit_cast(float,
        __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, edge), __builtin_bit_cast(int, v), kDppWaveShl1,
                                    0xf, 0xf, false));
}

// Value of the next-lower lane (lane 0 gets 0): the partial-sum migration of
// the SBM design, Z(s) <- Z(s-1).
__device__ __forceinline__ float from_lane_below(float v)
{
    return __builtin_bit_cast(float,
        __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kDppWaveShr1, 0xf, 0xf, true));
}

// Streamed data is touched once, so by default the 16-byte accesses carry the
// non-temporal hint (measured on MI355X: a copy moves ~6.0 TB/s with it and
// ~5.4-5.9 TB/s without).
#ifndef SYSCONV_NONTEMPORAL
#define SYSCONV_NONTEMPORAL 1
#endif
#ifndef SYSCONV_NONTEMPORAL_STORE
#define SYSCONV_NONTEMPORAL_STORE SYSCONV_NONTEMPORAL
#endif

// Load elements [idx, idx+4) of a row of `len` floats; elements past the end
// read as 0 and are never dereferenced.
template <bool NT = (SYSCONV_NONTEMPORAL != 0)>
__device__ __forceinline__ void load4_guarded(const float* __restrict__ row, long long idx, long long len,
                                              float (&v)[4])
{
    if (idx + 4 <= len) {
        const f4u* p = reinterpret_cast<const f4u*>(row + idx);
        const f4u t = NT ? __builtin_nontemporal_load(p) : *p;
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = (idx + i < len) ? row[idx + i] : 0.0f;
    }
}

// Store elements [idx, idx+4) of a row of `len` floats, clipped at the end.
template <bool NT = (SYSCONV_NONTEMPORAL_STORE != 0)>
__device__ __forceinline__ void store4_guarded(float* __restrict__ row, long long idx, long long len,
                                               const float (&v)[4])
{
    if (idx + 4 <= len) {
        f4u t;
        t.x = v[0]; t.y = v[1]; t.z = v[2]; t.w = v[3];
        f4u* p = reinterpret_cast<f4u*>(row + idx);
        if (NT) __builtin_nontemporal_store(t, p);
        else *p = t;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (idx + i < len) row[idx + i] = v[i];
    }
}

// FBS time steps (Table 2, row 3 left: PE = c, time = q) for NT <= 4 taps.
// Every step does  acc(c) += X(c) * w(q)  and then hands X one PE down,
// X(c) <- X(c+1).  e[0..3] are the lane's four X registers; x[4..7] are the
// values arriving from the lane above.  MORE tells whether a further block of
// taps follows (then all four registers must be handed over).
template <int NT, bool MORE>
__device__ __forceinline__ void fbs_steps(float (&e)[4], float (&acc)[4], const float (&w)[4])
{
    static_assert(NT >= 1 && NT <= 4, "a block holds 1..4 taps");
    float x[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = e[i];
    constexpr int touched = MORE ? 8 : NT + 3;
#pragma unroll
    for (int m = 4; m < touched; ++m) x[m] = from_lane_above(x[m - 4]);
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_fmaf(w[t], x[t + i], acc[i]);
    if (MORE) {
#pragma unroll
        for (int i = 0; i < 4; ++i) e[i] = x[4 + i];
    }
}

// Lanes of a group whose window of `k` taps reaches into the next group: they
// compute garbage that is never stored (the paper's transforms run every PE at
// every step without a time check, Section 4.1.1).
__host__ __device__ constexpr int halo_lanes(int k) { return (k + 2) >> 2; }   // ceil((k-1)/4)

}  // namespace sysconv
