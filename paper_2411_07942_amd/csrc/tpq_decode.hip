// tpq_decode_reduce kernel: dequantise the N devices' messages and add them
// (paper Sec. 2, decompression D^(i) and the sum over devices; Fig. 2 caption),
// selected features scattered back to their original columns.
#include "tpq_device.h"
#include "tpq_internal.h"

namespace tpq {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// two floats rounded to bf16 (nearest even, one hardware instruction), packed
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// round a pair of floats to bf16 and return them as floats again
__device__ __forceinline__ void round_pair_to_bf16(float &x, float &y)
{
    const uint32_t pk = pack_bf16x2(x, y);
    x = bf16_lo_to_f32(pk);
    y = bf16_hi_to_f32(pk);
}

// acc <- acc (+) x for 8 features at once, in the requested arithmetic
template <int ACC>
__device__ __forceinline__ void accumulate8(float (&acc)[8], float (&x)[8], bool first)
{
    if (ACC == TPQ_ACC_BF16) {
#pragma unroll
        for (int e = 0; e < 8; e += 2) round_pair_to_bf16(x[e], x[e + 1]);
    }
    if (first) {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = x[e];
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = acc[e] + x[e];
        if (ACC == TPQ_ACC_BF16) {
#pragma unroll
            for (int e = 0; e < 8; e += 2) round_pair_to_bf16(acc[e], acc[e + 1]);
        }
    }
}

#define TPQ_LDS(T) __attribute__((address_space(3))) T
template <typename T>
__device__ __forceinline__ TPQ_LDS(T) * lds_at(uint32_t addr)
{
    return reinterpret_cast<TPQ_LDS(T) *>(static_cast<uintptr_t>(addr));
}

// ---------------------------------------------------------------------------
// One wavefront produces one output row (4 rows per workgroup, no workgroup
// barrier: all LDS use is private to a wave).
//
//   1. the row's scales and zeros of all ranks (contiguous bf16 runs) are loaded
//      once and parked in LDS as float pairs;
//   2. the selected features: lane p adds the ranks' bf16 values of outlier p and
//      drops the sum at its column in the LDS output row;
//   3. per pass of 64 chunks a lane reads one 32-bit word of codes (8 features) per
//      rank -- the loads of the next batch of 8 ranks are in flight while the
//      current batch is dequantised (code * scale + zero, one FMA, the product is
//      exact) and accumulated in ascending rank order.  The 8 sums go to the LDS
//      output row at the chunk's start column with one 128-bit write (2-byte
//      aligned: removing the selected columns shifted the compacted stream); a
//      chunk that an outlier splits parks its sums in a patch slot instead;
//   4. as many lanes as there are split chunks move the parked sums to their
//      columns half-word by half-word;
//   5. the finished row leaves LDS with aligned 128-bit reads and coalesced
//      128-bit stores.
// ---------------------------------------------------------------------------
template <int LPG, int ACC, int OUT>
__global__ __launch_bounds__(256) void k_decode_stream(DecodeArgs a, RankPtrs codesp,
                                                       RankPtrs scalep, RankPtrs zerop,
                                                       RankPtrs outlp)
{
    const PlanHeader *ph = reinterpret_cast<const PlanHeader *>(a.plan);
    if (ph->magic != kPlanMagic || ph->status != kPlanOk || ph->E != a.E || ph->k != a.k ||
        ph->G != a.G)
        return;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t t = blockIdx.x * a.waves_per_block + wave;
    if (wave >= static_cast<uint32_t>(a.waves_per_block) || t >= static_cast<uint32_t>(a.T)) return;

    const int32_t *idx = reinterpret_cast<const int32_t *>(a.plan + ph->idx_offset);
    const uint32_t *cpos = reinterpret_cast<const uint32_t *>(a.plan + ph->pos_offset);
    const uint16_t *irr = reinterpret_cast<const uint16_t *>(a.plan + ph->irr_offset);
    const uint16_t *irr_src = reinterpret_cast<const uint16_t *>(a.plan + ph->irr_src_offset);
    const uint16_t *pass_irr = reinterpret_cast<const uint16_t *>(a.plan + ph->pass_irr_offset);

    constexpr uint32_t OB = OUT == TPQ_OUT_FP32 ? 4u : 2u;  // bytes per output value
    const uint32_t N = static_cast<uint32_t>(a.n_ranks);
    const uint32_t ng = static_cast<uint32_t>(a.ng);
    const uint32_t chunks = static_cast<uint32_t>(a.chunks);
    const uint32_t passes = static_cast<uint32_t>(a.chunks_padded) >> 6;
    const uint32_t n_irr = passes ? pass_irr[passes] : 0u;

    // LDS map of this wave: output row | (scale, zero) float pairs [N][ng] | patch
    extern __shared__ u32x4 smem_dec[];
    const uint32_t lds0 =
        static_cast<uint32_t>(reinterpret_cast<uintptr_t>((TPQ_LDS(u32x4) *)smem_dec));
    const uint32_t row = lds0 + wave * a.lds_per_wave;
    const uint32_t meta = row + ((static_cast<uint32_t>(a.E) * OB + 15u) & ~15u);
    const uint32_t patch = meta + (a.meta_in_lds ? ((N * ng * 8u + 15u) & ~15u) : 0u);

    const int64_t off_meta = static_cast<int64_t>(t) * a.pitch_meta;
    const int64_t off_codes = static_cast<int64_t>(t) * a.pitch_codes;
    const int64_t off_outl = static_cast<int64_t>(t) * a.pitch_outl;

    // 1. scales and zeros -> LDS (unless the table would not fit)
    for (uint32_t i = 0; a.meta_in_lds && i < N; ++i) {
        const uint16_t *sc = reinterpret_cast<const uint16_t *>(
            static_cast<const uint8_t *>(scalep.p[i]) + off_meta);
        const uint16_t *ze = reinterpret_cast<const uint16_t *>(
            static_cast<const uint8_t *>(zerop.p[i]) + off_meta);
        for (uint32_t g = lane; g < ng; g += 64)
            *lds_at<f32x2>(meta + 8u * (i * ng + g)) =
                f32x2{bf16_bits_to_f32(sc[g]), bf16_bits_to_f32(ze[g])};
    }

    // 2. selected features
    for (uint32_t p = lane; p < static_cast<uint32_t>(a.k); p += 64) {
        float acc = 0.f;
        for (uint32_t i = 0; i < N; ++i) {
            float x = bf16_bits_to_f32(reinterpret_cast<const uint16_t *>(
                static_cast<const uint8_t *>(outlp.p[i]) + off_outl)[p]);
            if (i == 0) {
                acc = x;
            } else {
                acc = acc + x;
                if (ACC == TPQ_ACC_BF16) acc = bf16_lo_to_f32(pack_bf16x2(acc, acc));
            }
        }
        const uint32_t j = static_cast<uint32_t>(idx[p]);
        if (OUT == TPQ_OUT_FP32)
            *lds_at<float>(row + 4u * j) = acc;
        else
            *lds_at<uint16_t>(row + 2u * j) = static_cast<uint16_t>(pack_bf16x2(acc, acc));
    }
    wave_lds_fence();

    // 3. quantised features: batches of 8 ranks, the next batch's codes in flight
    if (passes > 0) {
        const uint32_t rb = (N + 7u) >> 3;        // batches per pass
        const uint32_t n_batches = passes * rb;
        uint32_t wnext[8], cp_next;
        auto issue = [&](uint32_t b) {
            const uint32_t pass = b / rb, i0 = (b - pass * rb) * 8u;
            const uint32_t chunk = min(pass * 64u + lane, chunks - 1u);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t i = min(i0 + j, N - 1u);
                wnext[j] = __builtin_nontemporal_load(
                    reinterpret_cast<const uint32_t *>(static_cast<const uint8_t *>(codesp.p[i]) +
                                                       off_codes) + chunk);
            }
            if (i0 == 0) cp_next = cpos[pass * 64u + lane];
        };
        issue(0);
        float acc[8];
        uint32_t cp = 0;
        for (uint32_t b = 0; b < n_batches; ++b) {
            uint32_t w[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) w[j] = wnext[j];
            const uint32_t pass = b / rb, i0 = (b - pass * rb) * 8u;
            if (i0 == 0) cp = cp_next;
            if (b + 1 < n_batches) issue(b + 1);

            const uint32_t chunk = pass * 64u + lane;
            const uint32_t g = min(chunk / LPG, ng - 1u);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (i0 + j < N) {  // uniform
                    f32x2 sz;
                    if (a.meta_in_lds) {
                        sz = *lds_at<f32x2>(meta + 8u * ((i0 + j) * ng + g));
                    } else {
                        sz.x = bf16_bits_to_f32(reinterpret_cast<const uint16_t *>(
                            static_cast<const uint8_t *>(scalep.p[i0 + j]) + off_meta)[g]);
                        sz.y = bf16_bits_to_f32(reinterpret_cast<const uint16_t *>(
                            static_cast<const uint8_t *>(zerop.p[i0 + j]) + off_meta)[g]);
                    }
                    const uint32_t lo = w[j] & 0x0F0F0F0Fu, hi = (w[j] >> 4) & 0x0F0F0F0Fu;
                    float x[8];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        x[2 * e] = __builtin_fmaf(static_cast<float>((lo >> (8 * e)) & 0xFFu), sz.x, sz.y);
                        x[2 * e + 1] = __builtin_fmaf(static_cast<float>((hi >> (8 * e)) & 0xFFu), sz.x, sz.y);
                    }
                    accumulate8<ACC>(acc, x, i0 + j == 0);
                }
            }
            if (i0 + 8 >= N && chunk < chunks) {
                // the 8 sums of this chunk are complete
                const bool patched = (cp & kNotRegular) != 0;  // a slot exists for every such chunk
                if (OUT == TPQ_OUT_FP32) {
                    const u32x4 lo4 = {__float_as_uint(acc[0]), __float_as_uint(acc[1]),
                                       __float_as_uint(acc[2]), __float_as_uint(acc[3])};
                    const u32x4 hi4 = {__float_as_uint(acc[4]), __float_as_uint(acc[5]),
                                       __float_as_uint(acc[6]), __float_as_uint(acc[7])};
                    const uint32_t dst = patched ? patch + 32u * ((cp >> 16) & 0x7FFFu)
                                                 : row + 4u * (cp & 0xFFFFu);
                    *lds_at<u32x4_a4>(dst) = lo4;
                    *lds_at<u32x4_a4>(dst + 16u) = hi4;
                } else {
                    const u32x4 pk = {pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]),
                                      pack_bf16x2(acc[4], acc[5]), pack_bf16x2(acc[6], acc[7])};
                    const uint32_t dst = patched ? patch + 16u * ((cp >> 16) & 0x7FFFu)
                                                 : row + 2u * (cp & 0xFFFFu);
                    *lds_at<u32x4_a2>(dst) = pk;
                }
            }
        }
        wave_lds_fence();

        // 4. split chunks: parked sums -> their columns
        for (uint32_t q = lane; q < n_irr; q += 64) {
            const uint32_t c = irr[q];
            if (c < chunks) {
                const int n_valid = a.r - 8 * static_cast<int>(c);
                const u32x4 tab = *reinterpret_cast<const u32x4 *>(irr_src + 8u * q);
                const uint32_t col[8] = {tab.x & 0xFFFFu, tab.x >> 16, tab.y & 0xFFFFu, tab.y >> 16,
                                         tab.z & 0xFFFFu, tab.z >> 16, tab.w & 0xFFFFu, tab.w >> 16};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    if (e < n_valid) {
                        if (OUT == TPQ_OUT_FP32)
                            *lds_at<float>(row + 4u * col[e]) = *lds_at<float>(patch + 32u * q + 4u * e);
                        else
                            *lds_at<uint16_t>(row + 2u * col[e]) =
                                *lds_at<uint16_t>(patch + 16u * q + 2u * e);
                    }
                }
            }
        }
        wave_lds_fence();
    }

    // 5. LDS row -> global
    {
        u32x4 *dst = reinterpret_cast<u32x4 *>(static_cast<uint8_t *>(a.out) +
                                               static_cast<int64_t>(t) * a.ldOut * OB);
        const uint32_t n16 = static_cast<uint32_t>(a.E) * OB / 16u;
        for (uint32_t c = lane; c < n16; c += 64)
            __builtin_nontemporal_store(*lds_at<u32x4>(row + 16u * c), dst + c);
    }
}

int launch_decode(const DecodeArgs &a_in, const RankPtrs &codes, const RankPtrs &scale,
                  const RankPtrs &zero, const RankPtrs &outl, int accum, int out_dtype,
                  hipStream_t s)
{
    DecodeArgs a = a_in;
    const int lpg = a.G / 8;
    const size_t ob = out_dtype == TPQ_OUT_FP32 ? 4 : 2;
    const size_t slots = a.r > 0 ? static_cast<size_t>(irr_slots_of(a.k, a.r, a.G)) : 0;
    const size_t row_bytes = (static_cast<size_t>(a.E) * ob + 15) & ~static_cast<size_t>(15);
    const size_t meta_bytes = (static_cast<size_t>(a.n_ranks) * a.ng * 8 + 15) & ~static_cast<size_t>(15);
    a.meta_in_lds = meta_bytes <= 16 * 1024;
    const size_t per_wave = row_bytes + (a.meta_in_lds ? meta_bytes : 0) + slots * 8 * ob;
    if (per_wave > 160 * 1024) return TPQ_ERR_UNSUPPORTED;  // cannot happen for E <= 32768, k + 1 slots <= ...
    // as many waves per workgroup (at most 4) as keep two workgroups on a CU
    int wpb = static_cast<int>((80 * 1024) / per_wave);
    if (wpb > 4) wpb = 4;
    if (wpb < 1) wpb = 1;
    a.lds_per_wave = static_cast<int32_t>(per_wave);
    a.waves_per_block = wpb;
    const size_t lds = per_wave * wpb;
    const dim3 grid(static_cast<unsigned>((a.T + wpb - 1) / wpb));
    hipError_t e = hipSuccess;
#define TPQ_LAUNCH3(LPG, ACC, OUT)                                                           \
    do {                                                                                     \
        if (lds > 65536)                                                                     \
            e = hipFuncSetAttribute(                                                         \
                reinterpret_cast<const void *>(&k_decode_stream<LPG, ACC, OUT>),             \
                hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));          \
        if (e == hipSuccess)                                                                 \
            k_decode_stream<LPG, ACC, OUT><<<grid, 256, lds, s>>>(a, codes, scale, zero, outl); \
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
