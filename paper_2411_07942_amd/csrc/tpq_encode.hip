// tpq_encode kernels: the compression function C^(i) (paper Sec. 2) in the hybrid
// form of Fig. 2 -- selected features verbatim in BF16, the rest as packed 4-bit
// codes with a per-group bf16 scale and zero.
#include "tpq_device.h"
#include "tpq_internal.h"

namespace tpq {

// ---------------------------------------------------------------------------
// Row-per-wavefront kernel with the row staged in LDS.
//
// One 64-lane workgroup encodes one row of one rank:
//   0. 128-bit coalesced loads of the bf16 row into LDS;
//   1. per pass of 64 chunks (8 compacted features per lane, gathered from the
//      LDS row through the plan's src_of table): lane-local min / max, then a
//      DPP reduction over the lanes of a group; group leaders park (min, max)
//      in LDS;
//   2. lanes 0..ng-1 turn (min, max) into zero, bf16 scale and its reciprocal --
//      the two IEEE divisions happen once per group, not once per lane -- and
//      store scale / zero as contiguous bf16 runs;
//   3. per pass: quantise 8 features, pack 8 nibbles into one 32-bit word,
//      coalesced store.
// ---------------------------------------------------------------------------
template <int LPG>
__global__ __launch_bounds__(64) void k_encode_row(EncodeArgs a, RankPtrs Yp, RankPtrs codesp,
                                                   RankPtrs scalep, RankPtrs zerop,
                                                   RankPtrs outlp)
{
    const PlanHeader *ph = reinterpret_cast<const PlanHeader *>(a.plan);
    if (ph->magic != kPlanMagic || ph->status != kPlanOk || ph->E != a.E || ph->k != a.k ||
        ph->G != a.G)
        return;
    const int32_t *idx = reinterpret_cast<const int32_t *>(a.plan + ph->idx_offset);
    const uint4 *src_of = reinterpret_cast<const uint4 *>(a.plan + ph->src_offset);

    const int lane = threadIdx.x;
    const int64_t row = blockIdx.x;
    const int rank = static_cast<int>(row / a.T);
    const int64_t t = row - static_cast<int64_t>(rank) * a.T;

    extern __shared__ uint4 smem[];
    uint4 *lrow = smem;
    const uint16_t *lrow16 = reinterpret_cast<const uint16_t *>(smem);
    float2 *lmeta = reinterpret_cast<float2 *>(smem + a.E / 8);

    const uint4 *y = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(Yp.p[rank]) +
                                                     t * a.ldY);
    for (int c = lane; c < a.E / 8; c += 64) lrow[c] = y[c];
    __syncthreads();

    if (a.k > 0) {
        uint16_t *outl = reinterpret_cast<uint16_t *>(
            static_cast<uint8_t *>(const_cast<void *>(outlp.p[rank])) + t * a.pitch_outl);
        for (int p = lane; p < a.k; p += 64) outl[p] = lrow16[idx[p]];
    }
    if (a.r == 0) return;

    // phase 1: group min / max
    for (int base = 0; base < a.chunks_padded; base += 64) {
        const int chunk = base + lane;
        const uint4 tab = src_of[chunk];
        const uint32_t tw[4] = {tab.x, tab.y, tab.z, tab.w};
        float mn = 0.f, mx = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float v0 = bf16_bits_to_f32(lrow16[tw[e] & 0xFFFFu]);
            const float v1 = bf16_bits_to_f32(lrow16[tw[e] >> 16]);
            if (e == 0) {
                mn = fminf(v0, v1);
                mx = fmaxf(v0, v1);
            } else {
                mn = fminf(mn, fminf(v0, v1));
                mx = fmaxf(mx, fmaxf(v0, v1));
            }
        }
        group_minmax<LPG>(mn, mx);
        if ((lane % LPG) == 0) lmeta[chunk / LPG] = make_float2(mn, mx);
    }
    __syncthreads();

    // phase 2: zero, scale, reciprocal
    {
        uint16_t *scale = reinterpret_cast<uint16_t *>(
            static_cast<uint8_t *>(const_cast<void *>(scalep.p[rank])) + t * a.pitch_meta);
        uint16_t *zero = reinterpret_cast<uint16_t *>(
            static_cast<uint8_t *>(const_cast<void *>(zerop.p[rank])) + t * a.pitch_meta);
        for (int g = lane; g < a.ng; g += 64) {
            const float2 mm = lmeta[g];
            const float mn = mm.x + 0.0f;  // a zero minimum is stored as +0
            const float span = mm.y - mn;
            const float s32 = span / 15.0f;
            const uint32_t sb = f32_to_bf16_bits(s32);
            const float s = bf16_bits_to_f32(sb);
            const bool constant = s < 1e-30f;
            const float inv = constant ? 0.0f : 1.0f / s;
            scale[g] = constant ? uint16_t(0) : static_cast<uint16_t>(sb);
            zero[g] = static_cast<uint16_t>(__float_as_uint(mn) >> 16);
            lmeta[g] = make_float2(mn, inv);
        }
    }
    __syncthreads();

    // phase 3: quantise and pack
    uint32_t *codes = reinterpret_cast<uint32_t *>(
        static_cast<uint8_t *>(const_cast<void *>(codesp.p[rank])) + t * a.pitch_codes);
    for (int base = 0; base < a.chunks_padded; base += 64) {
        const int chunk = base + lane;
        const uint4 tab = src_of[chunk];
        const uint32_t tw[4] = {tab.x, tab.y, tab.z, tab.w};
        const float2 mi = lmeta[chunk / LPG];
        uint32_t w = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float v0 = bf16_bits_to_f32(lrow16[tw[e] & 0xFFFFu]);
            const float v1 = bf16_bits_to_f32(lrow16[tw[e] >> 16]);
            const float d0 = v0 - mi.x, d1 = v1 - mi.x;
            const float p0 = d0 * mi.y, p1 = d1 * mi.y;
            const float q0 = fminf(fmaxf(rintf(p0), 0.0f), 15.0f);
            const float q1 = fminf(fmaxf(rintf(p1), 0.0f), 15.0f);
            w |= static_cast<uint32_t>(q0) << (8 * e);
            w |= static_cast<uint32_t>(q1) << (8 * e + 4);
        }
        const int n_valid = a.r - 8 * chunk;  // features of this chunk that exist
        if (n_valid < 8) w &= n_valid > 0 ? ((1u << (4 * n_valid)) - 1u) : 0u;
        if (chunk < a.chunks) codes[chunk] = w;
    }
}

static size_t encode_row_lds(const EncodeArgs &a, int lpg)
{
    const size_t groups_padded = static_cast<size_t>(a.chunks_padded) / lpg;
    const size_t meta = (groups_padded > static_cast<size_t>(a.ng) ? groups_padded : a.ng) * 8;
    return static_cast<size_t>(a.E) * 2 + (meta + 15) / 16 * 16;
}

int launch_encode(const EncodeArgs &a, const RankPtrs &Y, const RankPtrs &codes,
                  const RankPtrs &scale, const RankPtrs &zero, const RankPtrs &outl,
                  hipStream_t s)
{
    const int lpg = a.G / 8;
    const dim3 grid(static_cast<unsigned>(a.T * a.n_ranks));
    const size_t lds = encode_row_lds(a, lpg);
    hipError_t e = hipSuccess;
#define TPQ_LAUNCH(LPG)                                                                      \
    do {                                                                                     \
        if (lds > 65536)                                                                     \
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_encode_row<LPG>),      \
                                    hipFuncAttributeMaxDynamicSharedMemorySize,              \
                                    static_cast<int>(lds));                                  \
        if (e == hipSuccess)                                                                 \
            k_encode_row<LPG><<<grid, 64, lds, s>>>(a, Y, codes, scale, zero, outl);         \
    } while (0)
    switch (lpg) {
    case 4: TPQ_LAUNCH(4); break;
    case 8: TPQ_LAUNCH(8); break;
    case 16: TPQ_LAUNCH(16); break;
    case 32: TPQ_LAUNCH(32); break;
    default: return TPQ_ERR_UNSUPPORTED;
    }
#undef TPQ_LAUNCH
    if (e != hipSuccess) return hip_result(e);
    return hip_result(hipGetLastError());
}

}  // namespace tpq
