// Helpers shared by the kernels that give one wavefront one row at a time: 4-element vector access
// for float and bf16 rows, and the choice of how many such chunks a lane holds.
#pragma once
#include "common.h"

namespace rev {

// ---- 4-element vector access for float and bf16 -------------------------------
struct f4 { float x, y, z, w; };

__device__ __forceinline__ f4 load4(const float* p) {
    float4 v = *reinterpret_cast<const float4*>(p);
    return {v.x, v.y, v.z, v.w};
}
__device__ __forceinline__ f4 load4(const bf16* p) {
    uint2 u = *reinterpret_cast<const uint2*>(p);
    f4 r;
    r.x = __uint_as_float(u.x << 16);
    r.y = __uint_as_float(u.x & 0xFFFF0000u);
    r.z = __uint_as_float(u.y << 16);
    r.w = __uint_as_float(u.y & 0xFFFF0000u);
    return r;
}
__device__ __forceinline__ void store4(float* p, f4 v) {
    *reinterpret_cast<float4*>(p) = make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    bf16 a = __float2bfloat16(lo), b = __float2bfloat16(hi);
    uint16_t ua = *reinterpret_cast<uint16_t*>(&a), ub = *reinterpret_cast<uint16_t*>(&b);
    return (uint32_t)ua | ((uint32_t)ub << 16);
}
__device__ __forceinline__ void store4(bf16* p, f4 v) {
    uint2 u;
    u.x = pack_bf16x2(v.x, v.y);
    u.y = pack_bf16x2(v.z, v.w);
    *reinterpret_cast<uint2*>(p) = u;
}

// Register chunks (of 4 floats) each lane holds of a row: the smallest instantiated count that covers
// D / 4 / 64.  Intermediate sizes matter: the kernels keep several row-long arrays in registers, so a
// width of 768 (3 chunks) or 1280 (5) should not pay for 4 or 8.
inline int pick_maxj(int D) {
    const int nch = D / 4, need = (nch + 63) / 64;
    static const int sizes[] = {2, 3, 4, 5, 6, 8, 12, 16, 24, 32};
    for (int j : sizes)
        if (j >= need) return j;
    return 64;   // D > 8192: no instantiation
}

}  // namespace rev
