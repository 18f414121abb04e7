// Device-side helpers: bf16 bit handling and reductions inside a 64-lane wavefront.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tpq {

__device__ __forceinline__ float bf16_lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// round-to-nearest-even on the 16 discarded bits (finite inputs)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// the same rounding, result kept as a float whose low 16 bits are zero
__device__ __forceinline__ float round_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return __uint_as_float(u & 0xFFFF0000u);
}

// ---- DPP lane exchange ---------------------------------------------------------
// dpp_ctrl encodings: quad_perm [1,0,3,2] = 0xB1, [2,3,0,1] = 0x4E,
// row_ror:n = 0x120 + n (rotate within a row of 16 lanes), row_half_mirror = 0x141
// (lane i <-> 7 - i within each 8 lanes).
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    int x = __float_as_int(v);
    return __int_as_float(__builtin_amdgcn_update_dpp(x, x, CTRL, 0xF, 0xF, false));
}

// min and max over aligned groups of LPG lanes (LPG in {4, 8, 16, 32}); every lane
// of the group ends up with the group's result.
template <int LPG>
__device__ __forceinline__ void group_minmax(float &mn, float &mx)
{
    static_assert(LPG == 4 || LPG == 8 || LPG == 16 || LPG == 32, "lanes per group");
    mn = fminf(mn, dpp_f32<0xB1>(mn));
    mx = fmaxf(mx, dpp_f32<0xB1>(mx));
    mn = fminf(mn, dpp_f32<0x4E>(mn));
    mx = fmaxf(mx, dpp_f32<0x4E>(mx));
    if (LPG == 8) {
        mn = fminf(mn, dpp_f32<0x141>(mn));
        mx = fmaxf(mx, dpp_f32<0x141>(mx));
    }
    if (LPG >= 16) {
        mn = fminf(mn, dpp_f32<0x124>(mn));
        mx = fmaxf(mx, dpp_f32<0x124>(mx));
        mn = fminf(mn, dpp_f32<0x128>(mn));
        mx = fmaxf(mx, dpp_f32<0x128>(mx));
    }
    if (LPG == 32) {
        mn = fminf(mn, __shfl_xor(mn, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    }
}

}  // namespace tpq
