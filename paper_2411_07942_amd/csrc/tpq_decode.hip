// tpq_decode_reduce kernels: dequantise the N devices' messages and add them
// (paper Sec. 2, decompression D^(i) and the sum over devices; Fig. 2 caption),
// selected features scattered back to their original columns.
#include "tpq_device.h"
#include "tpq_internal.h"

namespace tpq {

template <int ACC>
__device__ __forceinline__ float acc_first(float x)
{
    return ACC == TPQ_ACC_BF16 ? round_to_bf16(x) : x;
}

template <int ACC>
__device__ __forceinline__ float acc_next(float acc, float x)
{
    if (ACC == TPQ_ACC_BF16) return round_to_bf16(acc + round_to_bf16(x));
    return acc + x;
}

// ---------------------------------------------------------------------------
// Row-per-wavefront kernel with the output row staged in LDS.
//
// One 64-lane workgroup produces one output row.  Per pass of 64 chunks each
// lane reads one 32-bit word of codes (8 features) from every rank together with
// the group's scale and zero, accumulates the 8 sums in registers in ascending
// rank order, and drops them into an LDS row at their original feature positions
// (the plan's src_of table).  The selected features' bf16 values are summed the
// same way and written to their columns.  The finished row leaves with 128-bit
// coalesced stores.
// ---------------------------------------------------------------------------
template <int LPG, int ACC, int OUT>
__global__ __launch_bounds__(64) void k_decode_row(DecodeArgs a, RankPtrs codesp, RankPtrs scalep,
                                                   RankPtrs zerop, RankPtrs outlp)
{
    const PlanHeader *ph = reinterpret_cast<const PlanHeader *>(a.plan);
    if (ph->magic != kPlanMagic || ph->status != kPlanOk || ph->E != a.E || ph->k != a.k ||
        ph->G != a.G)
        return;
    const int32_t *idx = reinterpret_cast<const int32_t *>(a.plan + ph->idx_offset);
    const uint4 *src_of = reinterpret_cast<const uint4 *>(a.plan + ph->src_offset);

    const int lane = threadIdx.x;
    const int64_t t = blockIdx.x;

    extern __shared__ uint4 smem[];
    uint16_t *lout16 = reinterpret_cast<uint16_t *>(smem);
    float *lout32 = reinterpret_cast<float *>(smem);

    for (int base = 0; base < a.chunks; base += 64) {
        const int chunk = base + lane;
        if (chunk < a.chunks) {
            const int g = chunk / LPG;
            float acc[8];
            for (int i = 0; i < a.n_ranks; ++i) {
                const uint32_t w = reinterpret_cast<const uint32_t *>(
                    static_cast<const uint8_t *>(codesp.p[i]) + t * a.pitch_codes)[chunk];
                const float s = bf16_bits_to_f32(reinterpret_cast<const uint16_t *>(
                    static_cast<const uint8_t *>(scalep.p[i]) + t * a.pitch_meta)[g]);
                const float z = bf16_bits_to_f32(reinterpret_cast<const uint16_t *>(
                    static_cast<const uint8_t *>(zerop.p[i]) + t * a.pitch_meta)[g]);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float q = static_cast<float>((w >> (4 * e)) & 15u);
                    const float x = __builtin_fmaf(q, s, z);  // q*s is exact
                    acc[e] = i == 0 ? acc_first<ACC>(x) : acc_next<ACC>(acc[e], x);
                }
            }
            const uint4 tab = src_of[chunk];
            const uint32_t tw[4] = {tab.x, tab.y, tab.z, tab.w};
            const int n_valid = a.r - 8 * chunk;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (e < n_valid) {
                    const uint32_t j = (e & 1) ? (tw[e >> 1] >> 16) : (tw[e >> 1] & 0xFFFFu);
                    if (OUT == TPQ_OUT_FP32)
                        lout32[j] = acc[e];
                    else
                        lout16[j] = static_cast<uint16_t>(f32_to_bf16_bits(acc[e]));
                }
            }
        }
    }

    for (int p = lane; p < a.k; p += 64) {
        float acc = 0.f;
        for (int i = 0; i < a.n_ranks; ++i) {
            const float x = bf16_bits_to_f32(reinterpret_cast<const uint16_t *>(
                static_cast<const uint8_t *>(outlp.p[i]) + t * a.pitch_outl)[p]);
            acc = i == 0 ? acc_first<ACC>(x) : acc_next<ACC>(acc, x);
        }
        const int j = idx[p];
        if (OUT == TPQ_OUT_FP32)
            lout32[j] = acc;
        else
            lout16[j] = static_cast<uint16_t>(f32_to_bf16_bits(acc));
    }
    __syncthreads();

    const int out_bytes = OUT == TPQ_OUT_FP32 ? 4 : 2;
    uint4 *dst = reinterpret_cast<uint4 *>(static_cast<uint8_t *>(a.out) + t * a.ldOut * out_bytes);
    const int n16 = a.E * out_bytes / 16;
    for (int c = lane; c < n16; c += 64) dst[c] = smem[c];
}

int launch_decode(const DecodeArgs &a, const RankPtrs &codes, const RankPtrs &scale,
                  const RankPtrs &zero, const RankPtrs &outl, int accum, int out_dtype,
                  hipStream_t s)
{
    const int lpg = a.G / 8;
    const dim3 grid(static_cast<unsigned>(a.T));
    const size_t lds = static_cast<size_t>(a.E) * (out_dtype == TPQ_OUT_FP32 ? 4 : 2);
    hipError_t e = hipSuccess;
#define TPQ_LAUNCH3(LPG, ACC, OUT)                                                           \
    do {                                                                                     \
        if (lds > 65536)                                                                     \
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_decode_row<LPG, ACC, OUT>), \
                                    hipFuncAttributeMaxDynamicSharedMemorySize,              \
                                    static_cast<int>(lds));                                  \
        if (e == hipSuccess)                                                                 \
            k_decode_row<LPG, ACC, OUT><<<grid, 64, lds, s>>>(a, codes, scale, zero, outl);  \
    } while (0)
#define TPQ_LAUNCH2(LPG)                                                                     \
    do {                                                                                     \
        if (accum == TPQ_ACC_FP32 && out_dtype == TPQ_OUT_BF16)                              \
            TPQ_LAUNCH3(LPG, TPQ_ACC_FP32, TPQ_OUT_BF16);                                    \
        else if (accum == TPQ_ACC_FP32)                                                      \
            TPQ_LAUNCH3(LPG, TPQ_ACC_FP32, TPQ_OUT_FP32);                                    \
        else if (out_dtype == TPQ_OUT_BF16)                                                  \
            TPQ_LAUNCH3(LPG, TPQ_ACC_BF16, TPQ_OUT_BF16);                                    \
        else                                                                                 \
            TPQ_LAUNCH3(LPG, TPQ_ACC_BF16, TPQ_OUT_FP32);                                    \
    } while (0)
    switch (lpg) {
    case 4: TPQ_LAUNCH2(4); break;
    case 8: TPQ_LAUNCH2(8); break;
    case 16: TPQ_LAUNCH2(16); break;
    case 32: TPQ_LAUNCH2(32); break;
    default: return TPQ_ERR_UNSUPPORTED;
    }
#undef TPQ_LAUNCH2
#undef TPQ_LAUNCH3
    if (e != hipSuccess) return hip_result(e);
    return hip_result(hipGetLastError());
}

}  // namespace tpq
