// Cross-lane sums on the vector ALU (DPP modifiers and lane reads: no trip through the LDS crossbar).
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

namespace climber {

// sum over the 16 lanes of a DPP row, in every lane of the row
__device__ __forceinline__ float row_sum16(float x)
{
    auto dpp = [](float v, auto ctrl) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value, 0xf, 0xf, false));
    };
    x += dpp(x, std::integral_constant<int, 0xB1>{});   // quad_perm [1,0,3,2]
    x += dpp(x, std::integral_constant<int, 0x4E>{});   // quad_perm [2,3,0,1]
    x += dpp(x, std::integral_constant<int, 0x141>{});  // row_half_mirror
    x += dpp(x, std::integral_constant<int, 0x140>{});  // row_mirror
    return x;
}

// sum over the 64 lanes of a wavefront, in every lane (all lanes must be active)
__device__ __forceinline__ float wave_sum64(float x)
{
    const int r = __float_as_int(row_sum16(x));
    const float a = __int_as_float(__builtin_amdgcn_readlane(r, 0)), b = __int_as_float(__builtin_amdgcn_readlane(r, 16));
    const float c = __int_as_float(__builtin_amdgcn_readlane(r, 32)), d = __int_as_float(__builtin_amdgcn_readlane(r, 48));
    return (a + b) + (c + d);
}

}  // namespace climber
