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

// 128-bit vector that the compiler may load / store as one instruction
// Workgroups are handed to the chip's 8 XCDs in turn by linear id, and every XCD has an
// L2 of its own.  For a grid whose x extent n is a multiple of 8 this turns the hardware
// id into a logical index such that each XCD works through one contiguous range of
// logical indices in order: neighbours in the index space then share an L2, close in
// time (lines that two of them touch are fetched once and written whole).
__device__ __forceinline__ uint32_t xcd_contiguous_index(uint32_t id, uint32_t n)
{
    return (id & 7u) * (n >> 3) + (id >> 3);
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
// ... also at 2-byte alignment (gfx9 global memory accepts unaligned accesses in
// the HSA configuration; the hardware splits an access that crosses a cache line)
typedef u32x4 u32x4_a2 __attribute__((aligned(2)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));

// scalars at byte alignment (code widths other than 4 bits put a chunk's codes at any byte)
typedef uint16_t u16_a1 __attribute__((aligned(1)));
typedef uint32_t u32_a1 __attribute__((aligned(1)));
typedef uint32_t u32_a2 __attribute__((aligned(2)));
typedef uint64_t u64_a1 __attribute__((aligned(1)));

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// two floats rounded to bf16 (nearest even, one hardware instruction), packed
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// A float rounded to bf16 (nearest even) and returned as a float again: the hardware's
// pair conversion with a zero in the low half leaves exactly that in the register --
// one instruction per value, against one and a half for converting pairs and taking
// them apart again.
__device__ __forceinline__ float round_via_bf16(float x)
{
    return __uint_as_float(pack_bf16x2(0.0f, x));
}

// Orders one wavefront's LDS traffic: writes by any lane before this point are
// seen by reads of any lane after it.  LDS operations of a wave execute in issue
// order, so only the compiler has to be held back.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- DPP lane exchange ---------------------------------------------------------
// dpp_ctrl encodings: quad_perm [1,0,3,2] = 0xB1, [2,3,0,1] = 0x4E,
// row_ror:n = 0x120 + n (rotate within a row of 16 lanes), row_half_mirror = 0x141
// (lane i <-> 7 - i within each 8 lanes).
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    // every lane has a source under these controls, so the "old" operand is never used
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// min and max over aligned groups of LPG lanes (LPG in {2, 4, 8, 16, 32}); every lane
// of the group ends up with the group's result.
template <int LPG>
__device__ __forceinline__ void group_minmax(float &mn, float &mx)
{
    static_assert(LPG == 2 || LPG == 4 || LPG == 8 || LPG == 16 || LPG == 32, "lanes per group");
    mn = fminf(mn, dpp_f32<0xB1>(mn));
    mx = fmaxf(mx, dpp_f32<0xB1>(mx));
    if (LPG >= 4) {
        mn = fminf(mn, dpp_f32<0x4E>(mn));
        mx = fmaxf(mx, dpp_f32<0x4E>(mx));
    }
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

// The same reduction for N independent (min, max) pairs at once, stage by stage, so
// that consecutive DPP instructions never depend on each other.
template <int LPG, int N>
__device__ __forceinline__ void group_minmax_n(float (&mn)[N], float (&mx)[N])
{
    static_assert(LPG == 4 || LPG == 8 || LPG == 16 || LPG == 32, "lanes per group");
#define TPQ_STAGE(CTRL)                                                  \
    _Pragma("unroll") for (int i = 0; i < N; ++i)                        \
    {                                                                    \
        mn[i] = fminf(mn[i], dpp_f32<CTRL>(mn[i]));                      \
        mx[i] = fmaxf(mx[i], dpp_f32<CTRL>(mx[i]));                      \
    }
    TPQ_STAGE(0xB1)
    TPQ_STAGE(0x4E)
    if (LPG == 8) { TPQ_STAGE(0x141) }
    if (LPG >= 16) { TPQ_STAGE(0x124) TPQ_STAGE(0x128) }
#undef TPQ_STAGE
    if (LPG == 32) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            mn[i] = fminf(mn[i], __shfl_xor(mn[i], 16, 64));
            mx[i] = fmaxf(mx[i], __shfl_xor(mx[i], 16, 64));
        }
    }
}

// x / 15, correctly rounded: the product with fl(1/15) is off by at most an ulp, the
// remainder x - 15 q is exact in a fused multiply-add, and one more of them lands on the
// rounded quotient (checked against the division for every positive float).
__device__ __forceinline__ float div_by_15(float x)
{
    const float y = 0x1.111112p-4f;
    const float q = x * y;
    const float r = __builtin_fmaf(-15.0f, q, x);
    return __builtin_fmaf(r, y, q);
}

// 1 / s for a bf16-valued scale s: hardware reciprocal (1 ulp) and one Newton step.
// Equal to the IEEE quotient for every bf16 s with a normal reciprocal.
__device__ __forceinline__ float reciprocal_of_scale(float s)
{
    const float y = __builtin_amdgcn_rcpf(s);
    const float e = __builtin_fmaf(-s, y, 1.0f);
    return __builtin_fmaf(e, y, y);
}

}  // namespace tpq
