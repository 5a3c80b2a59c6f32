// Row helpers shared by the kernels that gather K / V rows (attend.hip, step_small.hip): a row of
// 128 elements is read by 16 (bfloat16) or 32 (binary32) adjacent lanes, 16 bytes per lane.
#pragma once
#include "internal.h"

namespace spotlight {
namespace rows {

struct bf16_raw { uint16_t v; };

template <typename T> struct RowTraits;
template <> struct RowTraits<bf16_raw> { static constexpr int kLanesPerRow = 16, kElems = 8; };
template <> struct RowTraits<float> { static constexpr int kLanesPerRow = 32, kElems = 4; };

template <typename T>
__device__ __forceinline__ void unpack(const uint4& u, float (&o)[RowTraits<T>::kElems])
{
    if constexpr (sizeof(T) == 2) {
        o[0] = __uint_as_float(u.x << 16); o[1] = __uint_as_float(u.x & 0xffff0000u);
        o[2] = __uint_as_float(u.y << 16); o[3] = __uint_as_float(u.y & 0xffff0000u);
        o[4] = __uint_as_float(u.z << 16); o[5] = __uint_as_float(u.z & 0xffff0000u);
        o[6] = __uint_as_float(u.w << 16); o[7] = __uint_as_float(u.w & 0xffff0000u);
    } else {
        o[0] = __uint_as_float(u.x); o[1] = __uint_as_float(u.y);
        o[2] = __uint_as_float(u.z); o[3] = __uint_as_float(u.w);
    }
}

// 16 bytes of a gathered row.  A row is used once per decode step and the rows of a step do not fit
// in any cache: non-temporal loads (measured 11 % faster than plain ones on a cold random gather).
__device__ __forceinline__ uint4 load_row16(const void* p)
{
    const uint4* s = reinterpret_cast<const uint4*>(p);
    uint4 r;
    r.x = __builtin_nontemporal_load(&s->x);
    r.y = __builtin_nontemporal_load(&s->y);
    r.z = __builtin_nontemporal_load(&s->z);
    r.w = __builtin_nontemporal_load(&s->w);
    return r;
}

// Sum of x over the LPR (16 or 32) adjacent lanes that share a row, the same bits in every lane:
// rotations within a row of 16 lanes (data-parallel-primitive moves, no LDS traffic), then one
// exchange between the two rows of a 32-lane group.
template <int LPR>
__device__ __forceinline__ float add_across_row(float x)
{
    static_assert(LPR == 16 || LPR == 32, "a row spans 16 or 32 lanes");
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x128, 0xf, 0xf, true));  // row_ror:8
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x124, 0xf, 0xf, true));  // row_ror:4
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x122, 0xf, 0xf, true));  // row_ror:2
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x121, 0xf, 0xf, true));  // row_ror:1
    if constexpr (LPR == 32) x += __shfl_xor(x, 16);
    return x;
}

}  // namespace rows
}  // namespace spotlight
