// Device-side helpers shared by the kernel translation units (wave64 cross-lane sums, bf16).
#pragma once

#include "fs_common.h"

namespace fs {

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// x + (x of the lane 32 away) in every lane: one cross-half swap per 32-bit word, no LDS traffic
__device__ __forceinline__ double add_xor32(double x) {
    const unsigned lo = (unsigned)__double2loint(x), hi = (unsigned)__double2hiint(x);
    const u32x2 a = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const u32x2 b = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    return __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
}

// x + (x of the lane 16 away) in every lane
__device__ __forceinline__ double add_xor16(double x) {
    const unsigned lo = (unsigned)__double2loint(x), hi = (unsigned)__double2hiint(x);
    const u32x2 a = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    const u32x2 b = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
    return __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
}

// sum over the 64/LPR groups of a wavefront, result in every lane; fixed order
template <int LPR>
__device__ __forceinline__ double across_groups(double x) {
    if (LPR == 32) return add_xor32(x);
    if (LPR == 16) return add_xor32(add_xor16(x));
#pragma unroll
    for (int m = LPR; m < kWave; m <<= 1) x += __shfl_xor(x, m, kWave);
    return x;
}

// sum over the LPR lanes of one group, result in every lane of the group; fixed order
template <int LPR>
__device__ __forceinline__ double group_sum(double x) {
#pragma unroll
    for (int m = LPR / 2; m >= 1; m >>= 1) x += __shfl_xor(x, m, kWave);
    return x;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// round to nearest even; NaN stays NaN
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

}  // namespace fs
