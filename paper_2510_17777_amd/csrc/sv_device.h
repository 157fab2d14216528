// Device-side helpers shared by the gfx950 kernels: 128-bit row-chunk loads,
// wavefront (64 lanes) reductions through DPP, and the order-preserving integer
// image of a float score.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sv {

constexpr int kWave = 64;

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));

// One 16-byte chunk of a K/V/q row, widened to fp32 on use.
template <typename T> struct Chunk;
template <> struct Chunk<_Float16> {
    static constexpr int kElems = 8;
    half8_t v;
    __device__ __forceinline__ float at(int i) const { return (float)v[i]; }
};
template <> struct Chunk<float> {
    static constexpr int kElems = 4;
    float4_t v;
    __device__ __forceinline__ float at(int i) const { return v[i]; }
};

template <typename T>
__device__ __forceinline__ Chunk<T> load_chunk(const T* p) {
    Chunk<T> c;
    c.v = *reinterpret_cast<const decltype(c.v)*>(p);
    return c;
}

// Streaming variant: the row is used once, so it should not displace reusable lines.
template <typename T>
__device__ __forceinline__ Chunk<T> load_chunk_stream(const T* p) {
    Chunk<T> c;
    c.v = __builtin_nontemporal_load(reinterpret_cast<const decltype(c.v)*>(p));
    return c;
}

template <typename T>
__device__ __forceinline__ Chunk<T> zero_chunk() {
    Chunk<T> c;
    c.v = 0;
    return c;
}

// ---- DPP lane exchange (all controls stay inside one row of 16 lanes) ----
template <int kCtrl>
__device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), kCtrl, 0xF, 0xF, true));
}

constexpr int kDppQuadXor1 = 0xB1;       // quad_perm [1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;       // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141; // lane i <-> 7-i inside 8 lanes
constexpr int kDppRowMirror = 0x140;     // lane i <-> 15-i inside 16 lanes

// Sum over each aligned group of kLanes consecutive lanes; every lane of the group
// ends with the total.  kLanes in {8, 16, 32}.
template <int kLanes>
__device__ __forceinline__ float group_sum(float x) {
    static_assert(kLanes == 8 || kLanes == 16 || kLanes == 32, "unsupported group width");
    x += dpp_move<kDppQuadXor1>(x);
    x += dpp_move<kDppQuadXor2>(x);
    x += dpp_move<kDppRowHalfMirror>(x);
    if (kLanes >= 16) x += dpp_move<kDppRowMirror>(x);
    if (kLanes >= 32) x += __shfl_xor(x, 16, kWave);
    return x;
}

// Cross-row steps of the 64-lane reductions read one lane of each 16-lane row into a scalar
// register (v_readlane) instead of going through the LDS crossbar (ds_bpermute): measured on
// the selection kernel, a bpermute step costs over a hundred cycles when 16 wavefronts share a
// compute unit.
__device__ __forceinline__ float lane_value(float x, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), lane));
}

__device__ __forceinline__ float wave_max(float x) {
    x = fmaxf(x, dpp_move<kDppQuadXor1>(x));
    x = fmaxf(x, dpp_move<kDppQuadXor2>(x));
    x = fmaxf(x, dpp_move<kDppRowHalfMirror>(x));
    x = fmaxf(x, dpp_move<kDppRowMirror>(x));
    return fmaxf(fmaxf(lane_value(x, 0), lane_value(x, 16)), fmaxf(lane_value(x, 32), lane_value(x, 48)));
}

__device__ __forceinline__ float wave_sum(float x) {
    x = group_sum<16>(x);
    return (lane_value(x, 0) + lane_value(x, 16)) + (lane_value(x, 32) + lane_value(x, 48));
}

// Inclusive prefix sum over the 64 lanes: shifts inside each 16-lane row (lanes shifted in from
// outside the row read 0), then the totals of the rows below.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x, int lane) {
    constexpr int kRowShr = 0x110;   // row_shr:n is 0x110 + n
#define SV_SCAN_STEP(n) x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, kRowShr + n, 0xF, 0xF, true)
    SV_SCAN_STEP(1);
    SV_SCAN_STEP(2);
    SV_SCAN_STEP(4);
    SV_SCAN_STEP(8);
#undef SV_SCAN_STEP
    const uint32_t t0 = (uint32_t)__builtin_amdgcn_readlane((int)x, 15);
    const uint32_t t1 = (uint32_t)__builtin_amdgcn_readlane((int)x, 31);
    const uint32_t t2 = (uint32_t)__builtin_amdgcn_readlane((int)x, 47);
    const int r = lane >> 4;
    return x + (r > 0 ? t0 : 0u) + (r > 1 ? t1 : 0u) + (r > 2 ? t2 : 0u);
}

// Monotone map float -> uint32: a < b  <=>  key(a) < key(b); +0 and -0 share a key.
__device__ __forceinline__ uint32_t score_key(float s) {
    uint32_t u = __float_as_uint(s);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

}  // namespace sv
