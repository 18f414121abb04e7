// tpq_decode_reduce, row kernel: dequantise the N devices' messages and add them
// (paper Sec. 2, decompression D^(i) and the sum over devices; Fig. 2 caption), the
// selected features put back at their original columns ("post-sync concatenation",
// Sec. 3 "Selecting High Precision Features").
//
// One persistent workgroup per output row at a time: wave p of the workgroup owns pass p
// of the row (64 chunks of 8 compacted features, one chunk per lane) for as long as the
// kernel runs, so everything a lane needs from the plan (the 8 columns its sums go to)
// is read once and kept in registers.  Per row:
//   - every lane loads its chunk's code word of each device (one 32-bit load per device;
//     the loads of the next row are issued before this row's arithmetic);
//   - the row's scales, zeros and selected features of all devices (a few hundred bytes)
//     come in as 16-byte pieces spread over the workgroup's threads and are parked in LDS,
//     scales and zeros already widened to (scale, zero) float pairs;
//   - sums are written to a row buffer in LDS at their original columns, 16 bits (or 32)
//     at a time; lanes take their 8 features in a rotated order so that the 32 lanes that
//     write together hit 32 different banks;
//   - after the workgroup's one barrier per row the finished row leaves as aligned
//     128-bit stores, whole cache lines, while the next row is being computed.
// HBM traffic per row is exactly the messages in and the row out.
#include <stdlib.h>

#include "tpq_device.h"
#include "tpq_internal.h"

namespace tpq {

struct RowsGeom {
    uint32_t lds_out;    // bytes of one row buffer: E * OB + 16 (dump slot), multiple of 16
    uint32_t lds_small;  // bytes of one stage of scales / zeros / selected features
    uint32_t srb;        // bytes per device in that stage: 64 * pm + 16 * po
    uint32_t pm, po;     // 16-byte pieces per device and row of scale (= of zero), of outl
    uint32_t pieces;     // n_ranks * (2 * pm + po)
    uint32_t lpg;        // lanes (chunks) per group
    uint32_t off_src;    // byte offset of the plan's src_of table
};

template <int ACC, int OUT, int MS>
__global__ __launch_bounds__(1024) void k_decode_rows(DecodeArgs a, RowsGeom gm, RankPtrs codesp, RankPtrs scalep,
                                                      RankPtrs zerop, RankPtrs outlp)
{
    extern __shared__ u32x4 smem_rows[];
    uint8_t *const lds = reinterpret_cast<uint8_t *>(smem_rows);
    // nothing is stored unless the plan is good (tables are read inside the plan buffer only)
    const bool bad = plan_header_bad(a.plan, a.E, a.k, a.G);
    constexpr uint32_t OB = OUT == TPQ_OUT_FP32 ? 4u : 2u;
    const uint32_t tid = threadIdx.x, ln = tid & 63u, threads = blockDim.x;
    const uint32_t N = static_cast<uint32_t>(a.n_ranks), nb = (N + 7u) >> 3;
    const uint32_t T = static_cast<uint32_t>(a.T), G = gridDim.x;
    const uint32_t chunks = static_cast<uint32_t>(a.chunks);
    const uint32_t cc = min(tid, chunks - 1u);  // this lane's chunk (lanes past the row repeat the last)
    const bool has_chunk = tid < chunks;
    uint8_t *const outbuf = lds;
    uint8_t *const small = lds + 2u * gm.lds_out;

    // ---- once per kernel: this lane's columns, rotated ---------------------------------
    // rot: how far the lane's features are rotated (acc[e] belongs to feature (e + rot) % 8):
    // chosen so that lanes whose chunks lie a multiple of 128 bytes apart in the row buffer
    // write different banks
    const uint32_t rot = OB == 2u ? 2u * ((ln >> 3) & 3u) : ((ln >> 2) & 7u);
    uint32_t waddr[8];  // LDS byte offset inside a row buffer of acc[e]'s column
    {
        const u32x4 t4 = *reinterpret_cast<const u32x4 *>(a.plan + gm.off_src + 16u * cc);
        const uint32_t tw[4] = {t4.x, t4.y, t4.z, t4.w};
        const uint32_t r = static_cast<uint32_t>(a.r);
#pragma unroll
        for (uint32_t e = 0; e < 8; ++e) {
            const uint32_t f = (e + rot) & 7u;  // feature of the chunk
            uint32_t col = 0;
#pragma unroll
            for (uint32_t q = 0; q < 8; ++q)
                if (f == q) col = (q & 1u) ? (tw[q >> 1] >> 16) : (tw[q >> 1] & 0xFFFFu);
            const bool valid = has_chunk && 8u * cc + f < r && col < static_cast<uint32_t>(a.E);
            waddr[e] = (valid ? col : static_cast<uint32_t>(a.E)) * OB;  // (E: the dump slot)
        }
    }
    const uint32_t g = min(cc / gm.lpg, static_cast<uint32_t>(a.ng) - 1u);

    // ---- once per kernel: the 16-byte pieces of the small sections this thread brings in ----
    const uint32_t ppr = 2u * gm.pm + gm.po;  // pieces per device
    const uint8_t *pbase[MS];
    uint32_t ppitch[MS], pdst[MS], pkind[MS];  // kind: 0 scale, 1 zero, 2 selected features, 3 none
#pragma unroll
    for (int m = 0; m < MS; ++m) {
        const uint32_t p = tid + static_cast<uint32_t>(m) * threads;
        const bool on = p < gm.pieces;
        const uint32_t pr = on ? p / ppr : 0u, q = on ? p - pr * ppr : 0u;
        const uint32_t kind = !on ? 3u : q < gm.pm ? 0u : q < 2u * gm.pm ? 1u : 2u;
        const uint32_t qi = kind == 0u ? q : kind == 1u ? q - gm.pm : q - 2u * gm.pm;
        pkind[m] = kind;
        ppitch[m] = static_cast<uint32_t>(kind == 2u ? a.pitch_outl : a.pitch_meta);
        pdst[m] = pr * gm.srb + (kind == 2u ? 64u * gm.pm + 16u * qi : 64u * qi + (kind == 1u ? 4u : 0u));
        const uint8_t *base = nullptr;
        for (uint32_t i = 0; i < N; ++i) {  // (pointer tables are kernel arguments: uniform reads, selected per lane)
            const uint8_t *cand = static_cast<const uint8_t *>(kind == 2u ? outlp.p[i] : kind == 1u ? zerop.p[i] : scalep.p[i]);
            if (pr == i) base = cand;
        }
        pbase[m] = base + 16u * qi;
    }

    uint32_t row = blockIdx.x;
    if (row >= T) return;
    u32x4 S[MS];
    uint32_t A[8];
#pragma unroll
    for (int m = 0; m < MS; ++m)
        if (pkind[m] != 3u)
            S[m] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(pbase[m] + static_cast<uint64_t>(row) * ppitch[m]));
#pragma unroll
    for (uint32_t j = 0; j < 8; ++j)
        A[j] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(
            static_cast<const uint8_t *>(codesp.p[min(j, N - 1u)]) + static_cast<uint64_t>(row) * a.pitch_codes + 4u * cc));

    auto store_row = [&](const uint8_t *ob, uint32_t t) {
        uint8_t *dst = static_cast<uint8_t *>(a.out) + static_cast<uint64_t>(t) * a.ldOut * OB;
        const uint32_t np = static_cast<uint32_t>(a.E) * OB / 16u;
        for (uint32_t q = tid; q < np; q += threads)
            __builtin_nontemporal_store(reinterpret_cast<const u32x4 *>(ob)[q], reinterpret_cast<u32x4 *>(dst) + q);
    };

#ifdef TPQ_PROF
    uint64_t pf[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    uint64_t pt = __builtin_amdgcn_s_memtime();
    const uint64_t pstart = pt;
#define TPQ_STAMP(i) { const uint64_t n_ = __builtin_amdgcn_s_memtime(); pf[i] += n_ - pt; pt = n_; }
#else
#define TPQ_STAMP(i)
#endif
    uint32_t it = 0;
    for (;; ++it) {
        uint8_t *const sm = small + (it & 1u) * gm.lds_small;
        uint8_t *const ob = outbuf + (it & 1u) * gm.lds_out;
        // 1. this row's small sections -> LDS
#pragma unroll
        for (int m = 0; m < MS; ++m) {
            if (pkind[m] == 2u) {
                *reinterpret_cast<u32x4 *>(sm + pdst[m]) = S[m];
            } else if (pkind[m] != 3u) {
                const uint32_t sw[4] = {S[m].x, S[m].y, S[m].z, S[m].w};
#pragma unroll
                for (uint32_t e = 0; e < 4; ++e) {
                    *reinterpret_cast<uint32_t *>(sm + pdst[m] + 16u * e) = sw[e] << 16;
                    *reinterpret_cast<uint32_t *>(sm + pdst[m] + 16u * e + 8u) = sw[e] & 0xFFFF0000u;
                }
            }
        }
        // 2. the next row's small sections (a workgroup's last row fetches itself again)
        const bool more = row + G < T;
        const uint32_t nrow = more ? row + G : row;
#pragma unroll
        for (int m = 0; m < MS; ++m)
            if (pkind[m] != 3u)
                S[m] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x4 *>(pbase[m] + static_cast<uint64_t>(nrow) * ppitch[m]));
        TPQ_STAMP(0)
        __syncthreads();
        TPQ_STAMP(1)
        // 3. the previous row leaves while this one is computed
        if (it > 0 && !bad) store_row(outbuf + ((it - 1u) & 1u) * gm.lds_out, row - G);

        TPQ_STAMP(2)
        // 4. the devices, 8 at a time; the next batch's code words are fetched first
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        float zs = 0.f;
        for (uint32_t b = 0; b < nb; ++b) {
            uint32_t nA[8];
            {
                // (after a workgroup's last batch nothing follows: every lane then reads the row's
                // first word again, one cached line, so that the loop's loads stay unconditional)
                const bool same = b + 1u < nb;
                const uint32_t r2 = same ? row : nrow, i0 = same ? 8u * (b + 1u) : 0u;
                const uint32_t off = (same || more) ? 4u * cc : 0u;
#pragma unroll
                for (uint32_t j = 0; j < 8; ++j)
                    nA[j] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(
                        static_cast<const uint8_t *>(codesp.p[min(i0 + j, N - 1u)]) +
                        static_cast<uint64_t>(r2) * a.pitch_codes + off));
            }
#pragma unroll
            for (uint32_t j = 0; j < 8; ++j) {
                const uint32_t i = 8u * b + j;
                if (i < N) {  // uniform
                    const float2 sz = *reinterpret_cast<const float2 *>(sm + i * gm.srb + 8u * g);
                    const float sc = sz.x, ze = sz.y;
                    // the chunk's 8 nibbles, rotated; read as FP8 (E4M3) a byte 0..15 is the code
                    // times 2^-9, so the scaled pair conversion makes two floats at once
                    const uint32_t w = __builtin_amdgcn_alignbit(A[j], A[j], 4u * rot);
                    const uint32_t lo = w & 0x0F0F0F0Fu, hi = (w >> 4) & 0x0F0F0F0Fu;
                    const f32x2 c02 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(lo, 512.0f, false);
                    const f32x2 c46 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(lo, 512.0f, true);
                    const f32x2 c13 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(hi, 512.0f, false);
                    const f32x2 c57 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(hi, 512.0f, true);
                    const float c[8] = {c02.x, c13.x, c02.y, c13.y, c46.x, c57.x, c46.y, c57.y};
                    if (ACC == TPQ_ACC_FAST) {
                        // sum of code * scale by fused multiply-add, the zeros summed apart
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf(c[e], sc, acc[e]);
                        zs += ze;
                    } else {
                        float x[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) x[e] = __builtin_fmaf(c[e], sc, ze);  // product exact
                        if (ACC == TPQ_ACC_BF16) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) x[e] = round_via_bf16(x[e]);
                        }
                        if (i == 0) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) acc[e] = x[e];
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e) acc[e] = acc[e] + x[e];
                            if (ACC == TPQ_ACC_BF16) {
#pragma unroll
                                for (int e = 0; e < 8; ++e) acc[e] = round_via_bf16(acc[e]);
                            }
                        }
                    }
                }
            }
            TPQ_STAMP(3)
#pragma unroll
            for (uint32_t j = 0; j < 8; ++j) A[j] = nA[j];
#ifdef TPQ_PROF
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
            TPQ_STAMP(4)
        }
        if (ACC == TPQ_ACC_FAST) {
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += zs;
        }

        // 5. selected features: the devices' bf16 values added in the same arithmetic
        for (uint32_t p = tid; p < static_cast<uint32_t>(a.k); p += threads) {
            const uint32_t col = static_cast<uint32_t>(reinterpret_cast<const int32_t *>(a.plan + a.off_idx)[p]);
            float s = 0.f;
            for (uint32_t i = 0; i < N; ++i) {
                const float x = bf16_bits_to_f32(*reinterpret_cast<const uint16_t *>(sm + i * gm.srb + 64u * gm.pm + 2u * p));
                if (i == 0) {
                    s = x;
                } else {
                    s = s + x;
                    if (ACC == TPQ_ACC_BF16) s = round_via_bf16(s);
                }
            }
            const uint32_t at = min(col, static_cast<uint32_t>(a.E)) * OB;
            if (OUT == TPQ_OUT_FP32)
                *reinterpret_cast<float *>(ob + at) = s;
            else
                *reinterpret_cast<uint16_t *>(ob + at) = static_cast<uint16_t>(pack_bf16x2(s, s));
        }
        TPQ_STAMP(5)
        // 6. the chunk's sums to their columns
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (OUT == TPQ_OUT_FP32)
                *reinterpret_cast<float *>(ob + waddr[e]) = acc[e];
            else
                *reinterpret_cast<uint16_t *>(ob + waddr[e]) = static_cast<uint16_t>(pack_bf16x2(acc[e], acc[e]));
        }
        TPQ_STAMP(6)
        if (!more) break;
        row += G;
    }
    __syncthreads();
    if (!bad) store_row(outbuf + (it & 1u) * gm.lds_out, row);
#ifdef TPQ_PROF
    if (a.bias && (tid & 63u) == 0 && blockIdx.x < 64) {
        uint64_t *dbg = reinterpret_cast<uint64_t *>(const_cast<uint8_t *>(a.bias)) + (blockIdx.x * 16u + (tid >> 6)) * 12u;
        for (int i = 0; i < 7; ++i) dbg[i] = pf[i];
        dbg[7] = __builtin_amdgcn_s_memtime() - pstart;
        dbg[8] = it + 1;
    }
#endif
}

// Workgroups per compute unit the persistent grid is sized for, given how many fit.
static int tuned_wg_per_cu(int fit)
{
#ifdef TPQ_TUNE
    if (const char *v = getenv("TPQ_DEC_WG_PER_CU")) {
        const int n = atoi(v);
        if (n >= 1 && n <= fit) return n;
    }
#endif
    return fit;
}

// TPQ_OK: launched; TPQ_ERR_UNSUPPORTED: this shape is not for the row kernel (nothing done)
int launch_decode_rows(const DecodeArgs &a_in, const RankPtrs &codes, const RankPtrs &scale,
                       const RankPtrs &zero, const RankPtrs &outl, int accum, int out_dtype, hipStream_t s)
{
    const DecodeArgs &a = a_in;
#ifdef TPQ_PROF
    if (a.bits != 4 || a.step_c || a.addend || a.r <= 0) return TPQ_ERR_UNSUPPORTED;
#else
    if (a.bits != 4 || a.step_c || a.addend || a.bias || a.r <= 0) return TPQ_ERR_UNSUPPORTED;
#endif
    const int passes = a.chunks_padded / 64;
    if (passes > 16) return TPQ_ERR_UNSUPPORTED;
    const uint32_t ob = out_dtype == TPQ_OUT_FP32 ? 4u : 2u;
    if ((static_cast<uint32_t>(a.E) * ob) % 16u) return TPQ_ERR_UNSUPPORTED;
    // 32-bit row offsets inside the kernel's small-section reads; rows numbered in 32 bits
    if (a.T > 0x7FFFFFFFLL) return TPQ_ERR_UNSUPPORTED;
    RowsGeom gm;
    gm.lds_out = (static_cast<uint32_t>(a.E) * ob + 16u + 15u) / 16u * 16u;
    gm.pm = (2u * static_cast<uint32_t>(a.ng) + 15u) / 16u;
    gm.po = (2u * static_cast<uint32_t>(a.k) + 15u) / 16u;
    gm.srb = 64u * gm.pm + 16u * gm.po;
    gm.lds_small = gm.srb * static_cast<uint32_t>(a.n_ranks);
    gm.pieces = static_cast<uint32_t>(a.n_ranks) * (2u * gm.pm + gm.po);
    gm.lpg = static_cast<uint32_t>(a.G) / 8u;
    const PlanOffsets o = plan_offsets(a.k, a.r, a.G);
    gm.off_src = static_cast<uint32_t>(o.src);
    const uint32_t threads = 64u * static_cast<uint32_t>(passes);
    const int ms = static_cast<int>((gm.pieces + threads - 1u) / threads);
    if (ms > 4) return TPQ_ERR_UNSUPPORTED;
    const size_t lds = 2u * (static_cast<size_t>(gm.lds_out) + gm.lds_small);
    if (lds > 160u * 1024u) return TPQ_ERR_UNSUPPORTED;
    if (static_cast<int64_t>(gm.pm) * 16 > a.pitch_meta || static_cast<int64_t>(gm.po) * 16 > a.pitch_outl)
        return TPQ_ERR_UNSUPPORTED;  // (whole pieces must lie inside a row's pitch)

    DecodeArgs b = a;
    b.off_idx = o.idx;
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return hip_result(e);
    int per_cu = 0;
    int64_t grid = 0;

#define TPQ_ROWS3(ACC, OUT, MS)                                                                        \
    do {                                                                                               \
        auto kern = k_decode_rows<ACC, OUT, MS>;                                                       \
        if (lds > 65536)                                                                               \
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                              \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)); \
        if (e == hipSuccess)                                                                           \
            e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, static_cast<int>(threads), lds); \
        if (e == hipSuccess && per_cu < 1) e = hipErrorLaunchOutOfResources;                           \
        if (e == hipSuccess) {                                                                         \
            per_cu = tuned_wg_per_cu(per_cu);                                                          \
            grid = static_cast<int64_t>(cus) * per_cu;                                                 \
            if (grid > a.T) grid = a.T;                                                                \
            launch_kernel(kern, dim3(static_cast<unsigned>(grid)), dim3(threads), lds, s, b, gm, codes, scale, zero, outl); \
        }                                                                                              \
    } while (0)
#define TPQ_ROWS2(ACC, OUT)                   \
    do {                                      \
        if (ms <= 1) TPQ_ROWS3(ACC, OUT, 1);  \
        else if (ms == 2) TPQ_ROWS3(ACC, OUT, 2); \
        else TPQ_ROWS3(ACC, OUT, 4);          \
    } while (0)
    if (out_dtype == TPQ_OUT_FP32) {
        if (accum == TPQ_ACC_FP32) TPQ_ROWS2(TPQ_ACC_FP32, TPQ_OUT_FP32);
        else if (accum == TPQ_ACC_BF16) TPQ_ROWS2(TPQ_ACC_BF16, TPQ_OUT_FP32);
        else TPQ_ROWS2(TPQ_ACC_FAST, TPQ_OUT_FP32);
    } else {
        if (accum == TPQ_ACC_FP32) TPQ_ROWS2(TPQ_ACC_FP32, TPQ_OUT_BF16);
        else if (accum == TPQ_ACC_BF16) TPQ_ROWS2(TPQ_ACC_BF16, TPQ_OUT_BF16);
        else TPQ_ROWS2(TPQ_ACC_FAST, TPQ_OUT_BF16);
    }
#undef TPQ_ROWS2
#undef TPQ_ROWS3
    if (e == hipSuccess) e = hipGetLastError();
    return hip_result(e);
}

}  // namespace tpq
