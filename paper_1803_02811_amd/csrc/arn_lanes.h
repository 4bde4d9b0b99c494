// Cross-lane reductions on the vector ALU (DPP and permlane-swap operands) instead of LDS permutes.
// All of them are butterflies: every lane ends with the same bits, in an order of additions that is fixed.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace arn {

// the value of another lane of the same row of 16, chosen by a DPP control word:
// 0xB1 quad_perm [1,0,3,2], 0x4E quad_perm [2,3,0,1], 0x141 mirror within 8 lanes, 0x140 mirror within 16
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}

// over the 16 lanes of a row (lanes 16r .. 16r+15); all lanes of the wavefront must be active
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_f<0xB1>(v);
    v += dpp_f<0x4E>(v);
    v += dpp_f<0x141>(v);
    v += dpp_f<0x140>(v);
    return v;
}
__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, dpp_f<0xB1>(v));
    v = fmaxf(v, dpp_f<0x4E>(v));
    v = fmaxf(v, dpp_f<0x141>(v));
    v = fmaxf(v, dpp_f<0x140>(v));
    return v;
}
__device__ __forceinline__ int row16_min(int v) {
    v = min(v, dpp_i<0xB1>(v));
    v = min(v, dpp_i<0x4E>(v));
    v = min(v, dpp_i<0x141>(v));
    v = min(v, dpp_i<0x140>(v));
    return v;
}

// the values of the lanes 16 and 32 away (v_permlane16_swap / v_permlane32_swap with both operands equal
// return the lane's own value and the other lane's, in an order that depends on the row)
__device__ __forceinline__ void swap16(float v, float &a, float &b) {
    const uint32_t u = __builtin_bit_cast(uint32_t, v);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    a = __builtin_bit_cast(float, (uint32_t)r[0]);
    b = __builtin_bit_cast(float, (uint32_t)r[1]);
}
__device__ __forceinline__ void swap32(float v, float &a, float &b) {
    const uint32_t u = __builtin_bit_cast(uint32_t, v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    a = __builtin_bit_cast(float, (uint32_t)r[0]);
    b = __builtin_bit_cast(float, (uint32_t)r[1]);
}

// over all 64 lanes
__device__ __forceinline__ float wave_sum(float v) {
    float a, b;
    v = row16_sum(v);
    swap16(v, a, b);
    v = a + b;
    swap32(v, a, b);
    return a + b;
}
__device__ __forceinline__ float wave_max(float v) {
    float a, b;
    v = row16_max(v);
    swap16(v, a, b);
    v = fmaxf(a, b);
    swap32(v, a, b);
    return fmaxf(a, b);
}
// lane j's value in every lane (j uniform over the wavefront)
__device__ __forceinline__ float lane_value(float v, int j) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), j));
}

}  // namespace arn
