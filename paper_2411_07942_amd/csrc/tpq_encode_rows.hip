// tpq_encode, row kernel: the compression function C^(i) (paper Sec. 2) in the hybrid form
// of Fig. 2 -- the selected features of a row verbatim in BF16 ("pre-sync BF16 feature
// selection", Sec. 3), the rest as packed 4-bit codes with a bf16 scale and zero per group.
//
// One persistent workgroup per (device, row) at a time; wave p of the workgroup owns pass p
// of the row (64 chunks of 8 compacted features, one chunk per lane) for as long as the
// kernel runs, so what a lane needs from the plan (the 8 columns of its features) is read
// once and kept in registers.  Per row:
//   - the bf16 row comes in as aligned 128-bit loads, one 16-byte piece per thread, whole
//     cache lines; the next row's loads are issued as soon as this row is in LDS;
//   - every lane gathers its 8 features from the LDS row, 16 bits at a time, in a rotated
//     order so that the 32 lanes that read together hit 32 different banks;
//   - group minimum / maximum by DPP over the group's lanes; zero, bf16 scale, reciprocal;
//     codes from registers; the 8 codes of a lane packed into one word;
//   - codes, scales, zeros and the selected features are collected in LDS and leave, after
//     the workgroup's one barrier per row, as 128-bit stores (section tails as narrower
//     ones: nothing outside a section's logical bytes is written).
// HBM traffic per row is exactly the row in and the message out.
#include <stdlib.h>

#include "tpq_device.h"
#include "tpq_internal.h"

namespace tpq {

struct EncRowsGeom {
    uint32_t lds_row;    // bytes of one row buffer (E * 2)
    uint32_t lds_stage;  // bytes of one message stage
    uint32_t st_scale, st_zero, st_outl;  // byte offsets of the sections in a stage (codes: 0)
    uint32_t nb_codes, nb_meta, nb_outl;  // logical bytes per row: 4 * chunks, 2 * ng, 2 * k
    uint32_t pc, pm, po;                  // 16-byte pieces per section (rounded up)
    uint32_t row_pieces;                  // E / 8
    uint32_t off_src;                     // byte offset of the plan's src_of table
};

// One row's message from its LDS stage to memory: 128-bit stores, the tail of a section as
// narrower ones, so that nothing outside a section's logical bytes is written.  The four
// pointers are the row's sections (device and row already applied).
__device__ __forceinline__ void store_message(const EncRowsGeom &gm, const uint8_t *st, uint8_t *d_codes,
                                              uint8_t *d_scale, uint8_t *d_zero, uint8_t *d_outl,
                                              uint32_t tid, uint32_t threads)
{
    const uint32_t P = gm.pc + 2u * gm.pm + gm.po;
    for (uint32_t q = tid; q < P; q += threads) {
        const uint32_t sec = q < gm.pc ? 0u : q < gm.pc + gm.pm ? 1u : q < gm.pc + 2u * gm.pm ? 2u : 3u;
        const uint32_t qi = sec == 0u ? q : sec == 1u ? q - gm.pc : sec == 2u ? q - gm.pc - gm.pm : q - gm.pc - 2u * gm.pm;
        const uint32_t so = sec == 0u ? 0u : sec == 1u ? gm.st_scale : sec == 2u ? gm.st_zero : gm.st_outl;
        const uint32_t nbytes = sec == 0u ? gm.nb_codes : sec == 3u ? gm.nb_outl : gm.nb_meta;
        uint8_t *dst = (sec == 0u ? d_codes : sec == 1u ? d_scale : sec == 2u ? d_zero : d_outl) + 16u * qi;
        const uint8_t *src = st + so + 16u * qi;
        if (16u * qi + 16u <= nbytes) {
            __builtin_nontemporal_store(*reinterpret_cast<const u32x4 *>(src), reinterpret_cast<u32x4 *>(dst));
        } else if (sec == 0u) {
            for (uint32_t o = 0; 16u * qi + o < nbytes; o += 4u)
                *reinterpret_cast<uint32_t *>(dst + o) = *reinterpret_cast<const uint32_t *>(src + o);
        } else {
            for (uint32_t o = 0; 16u * qi + o < nbytes; o += 2u)
                *reinterpret_cast<uint16_t *>(dst + o) = *reinterpret_cast<const uint16_t *>(src + o);
        }
    }
}

template <int LPG, int MR>
__global__ __launch_bounds__(1024) void k_encode_rows(EncodeArgs a, EncRowsGeom gm, RankPtrs Yp, RankPtrs codesp,
                                                      RankPtrs scalep, RankPtrs zerop, RankPtrs outlp)
{
    extern __shared__ u32x4 smem_er[];
    uint8_t *const lds = reinterpret_cast<uint8_t *>(smem_er);
    const bool bad = plan_header_bad(a.plan, a.E, a.k, a.G);  // nothing is stored unless the plan is good
    const uint32_t tid = threadIdx.x, ln = tid & 63u, threads = blockDim.x;
    const uint32_t T = static_cast<uint32_t>(a.T), G = gridDim.x;
    const uint32_t total = T * static_cast<uint32_t>(a.n_ranks);
    const uint32_t chunks = static_cast<uint32_t>(a.chunks);
    const uint32_t cc = min(tid, chunks - 1u);  // this lane's chunk (lanes past the row repeat the last)
    const bool has_chunk = tid < chunks;
    uint8_t *const rowbuf = lds;
    uint8_t *const stage = lds + 2u * gm.lds_row;

    // ---- once per kernel: where this lane's features sit in the row, rotated by pairs -----
    // (word b of the lane holds the chunk's feature pair (b + rot) % 4: lanes whose chunks lie a
    // multiple of 128 bytes apart then read different banks)
    const uint32_t rot = (ln >> 3) & 3u;
    uint32_t raddr[8];
    {
        const u32x4 t4 = *reinterpret_cast<const u32x4 *>(a.plan + gm.off_src + 16u * cc);
        const uint32_t tw[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
        for (uint32_t b = 0; b < 4; ++b) {
            uint32_t word = 0;
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q)
                if (((b + rot) & 3u) == q) word = tw[q];
            // (columns of a bad plan are kept inside the row)
            raddr[2 * b] = 2u * min(word & 0xFFFFu, static_cast<uint32_t>(a.E) - 1u);
            raddr[2 * b + 1] = 2u * min(word >> 16, static_cast<uint32_t>(a.E) - 1u);
        }
    }
    const uint32_t g = tid / LPG;  // the lane's group (meaningful where has_chunk)
    const int32_t *idx = reinterpret_cast<const int32_t *>(a.plan + a.off_idx);
    const uint32_t ocol = tid < static_cast<uint32_t>(a.k) ? min(static_cast<uint32_t>(idx[tid]), static_cast<uint32_t>(a.E) - 1u) : 0u;

    uint32_t u = blockIdx.x;
    if (u >= total) return;
    uint32_t rank = u / T, t = u - rank * T;
    u32x4 R[MR];
#pragma unroll
    for (int m = 0; m < MR; ++m) {
        const uint32_t piece = tid + static_cast<uint32_t>(m) * threads;
        if (piece < gm.row_pieces)
            R[m] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(
                static_cast<const uint8_t *>(Yp.p[rank]) + static_cast<uint64_t>(t) * a.ldY * 2) + piece);
    }

    uint32_t it = 0;
    for (;; ++it) {
        uint8_t *const rb = rowbuf + (it & 1u) * gm.lds_row;
        uint8_t *const st = stage + (it & 1u) * gm.lds_stage;
        // 1. this row -> LDS
#pragma unroll
        for (int m = 0; m < MR; ++m) {
            const uint32_t piece = tid + static_cast<uint32_t>(m) * threads;
            if (piece < gm.row_pieces) reinterpret_cast<u32x4 *>(rb)[piece] = R[m];
        }
        __syncthreads();
        // 2. the next row's loads (after a workgroup's last row every thread re-reads one cached
        // piece, so that the loop's loads stay unconditional)
        const bool more = u + G < total;
        const uint32_t nu = more ? u + G : u;
        const uint32_t nrank = nu / T, nt = nu - nrank * T;
#pragma unroll
        for (int m = 0; m < MR; ++m) {
            const uint32_t piece = tid + static_cast<uint32_t>(m) * threads;
            if (piece < gm.row_pieces)
                R[m] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(
                    static_cast<const uint8_t *>(Yp.p[nrank]) + static_cast<uint64_t>(nt) * a.ldY * 2) + (more ? piece : 0u));
        }
        // 3. the previous row's message leaves while this one is computed
        if (it > 0 && !bad) {
            const uint32_t pu = u - G, pr = pu / T;
            const uint64_t pt = pu - pr * T;
            store_message(gm, stage + ((it - 1u) & 1u) * gm.lds_stage,
                          static_cast<uint8_t *>(const_cast<void *>(codesp.p[pr])) + pt * a.pitch_codes,
                          static_cast<uint8_t *>(const_cast<void *>(scalep.p[pr])) + pt * a.pitch_meta,
                          static_cast<uint8_t *>(const_cast<void *>(zerop.p[pr])) + pt * a.pitch_meta,
                          static_cast<uint8_t *>(const_cast<void *>(outlp.p[pr])) + pt * a.pitch_outl, tid, threads);
        }

        // 4. the chunk's 8 features, as four words of two
        u32x4 v;
        {
#define TPQ_HW(e) static_cast<uint32_t>(*reinterpret_cast<const uint16_t *>(rb + raddr[e]))
            v.x = TPQ_HW(0) | (TPQ_HW(1) << 16);
            v.y = TPQ_HW(2) | (TPQ_HW(3) << 16);
            v.z = TPQ_HW(4) | (TPQ_HW(5) << 16);
            v.w = TPQ_HW(6) | (TPQ_HW(7) << 16);
#undef TPQ_HW
        }
        // selected features: a copy
        {
            uint16_t *so = reinterpret_cast<uint16_t *>(st + gm.st_outl);
            if (tid < static_cast<uint32_t>(a.k)) so[tid] = *reinterpret_cast<const uint16_t *>(rb + 2u * ocol);
            for (uint32_t p = tid + threads; p < static_cast<uint32_t>(a.k); p += threads)
                so[p] = *reinterpret_cast<const uint16_t *>(
                    rb + 2u * min(static_cast<uint32_t>(idx[p]), static_cast<uint32_t>(a.E) - 1u));
        }

        // 5. group minimum / maximum.  The upper feature of a word is compared as the whole
        // word: as a float the word lies between that feature and its successor in magnitude,
        // so it wins exactly where the feature would, and masking the winner's low half gives
        // the feature itself.  (Positions past the row repeat the row's last feature.)
        float mn, mx;
        {
            const float l0 = bf16_lo_to_f32(v.x), l1 = bf16_lo_to_f32(v.y);
            const float l2 = bf16_lo_to_f32(v.z), l3 = bf16_lo_to_f32(v.w);
            const float h0 = __uint_as_float(v.x), h1 = __uint_as_float(v.y);
            const float h2 = __uint_as_float(v.z), h3 = __uint_as_float(v.w);
            const float lo = fminf(fminf(fminf(l0, l1), fminf(l2, l3)), fminf(fminf(h0, h1), fminf(h2, h3)));
            const float hi = fmaxf(fmaxf(fmaxf(l0, l1), fmaxf(l2, l3)), fmaxf(fmaxf(h0, h1), fmaxf(h2, h3)));
            mn = __uint_as_float(__float_as_uint(lo) & 0xFFFF0000u);
            mx = __uint_as_float(__float_as_uint(hi) & 0xFFFF0000u);
        }
        group_minmax<LPG>(mn, mx);

        // 6. zero, bf16 scale and its reciprocal (both divisions are exact replacements of the
        // IEEE ones, see div_by_15 / reciprocal_of_scale)
        mn = mn + 0.0f;  // a zero minimum is stored as +0
        const float span = mx - mn;
        const float s32 = div_by_15(span);
        const uint32_t sb = pack_bf16x2(s32, s32) & 0xFFFFu;
        const float s = bf16_bits_to_f32(sb);
        const bool constant = s < 1e-30f;
        const float inv = constant ? 0.0f : reciprocal_of_scale(s);
        if ((ln % LPG) == 0 && has_chunk) {
            reinterpret_cast<uint16_t *>(st + gm.st_scale)[g] = static_cast<uint16_t>(constant ? 0u : sb);
            reinterpret_cast<uint16_t *>(st + gm.st_zero)[g] = static_cast<uint16_t>(__float_as_uint(mn) >> 16);
        }

        // 7. quantise and pack: (x - zero) * inv lies in [0, 15.06], so the rounded value is a
        // 4-bit code without a clamp; the float -> byte conversion rounds to nearest even
        uint32_t w;
        {
            const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
            uint32_t h[2];
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                float pr[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t word = wv[half * 2 + (e >> 1)];
                    const float x = (e & 1) ? bf16_hi_to_f32(word) : bf16_lo_to_f32(word);
                    const float df = x - mn;
                    pr[e] = df * inv;
                }
                uint32_t b = __builtin_amdgcn_cvt_pk_u8_f32(pr[1], 0u, 0u);
                b = __builtin_amdgcn_cvt_pk_u8_f32(pr[0], 1u, b);
                b = __builtin_amdgcn_cvt_pk_u8_f32(pr[3], 2u, b);
                b = __builtin_amdgcn_cvt_pk_u8_f32(pr[2], 3u, b);
                h[half] = (b << 12) | b;
            }
            w = __builtin_amdgcn_perm(h[1], h[0], 0x07050301u);
            // byte b holds the codes of pair (b + rot) % 4: back to feature order
            w = __builtin_amdgcn_alignbit(w, w, (32u - 8u * rot) & 31u);
            const int n_valid = a.r - 8 * static_cast<int>(cc);
            if (n_valid < 8) w &= (1u << (4 * (n_valid & 7))) - 1u;
        }
        if (has_chunk) reinterpret_cast<uint32_t *>(st)[cc] = w;

        if (!more) break;
        u = nu;
        rank = nrank;
        t = nt;
    }
    __syncthreads();
    if (!bad) {
        const uint64_t pt = t;
        store_message(gm, stage + (it & 1u) * gm.lds_stage,
                      static_cast<uint8_t *>(const_cast<void *>(codesp.p[rank])) + pt * a.pitch_codes,
                      static_cast<uint8_t *>(const_cast<void *>(scalep.p[rank])) + pt * a.pitch_meta,
                      static_cast<uint8_t *>(const_cast<void *>(zerop.p[rank])) + pt * a.pitch_meta,
                      static_cast<uint8_t *>(const_cast<void *>(outlp.p[rank])) + pt * a.pitch_outl, tid, threads);
    }
}

static int tuned_enc_wg_per_cu(int fit)
{
#ifdef TPQ_TUNE
    if (const char *v = getenv("TPQ_ENC_WG_PER_CU")) {
        const int n = atoi(v);
        if (n >= 1 && n <= fit) return n;
    }
#endif
    return fit;
}

// TPQ_OK: launched; TPQ_ERR_UNSUPPORTED: this shape is not for the row kernel (nothing done)
int launch_encode_rows(const EncodeArgs &a, const RankPtrs &Y, const RankPtrs &codes, const RankPtrs &scale,
                       const RankPtrs &zero, const RankPtrs &outl, hipStream_t s)
{
    if (a.bits != 4 || a.inv_c || a.r <= 0) return TPQ_ERR_UNSUPPORTED;
    const int passes = a.chunks_padded / 64;
    if (passes > 16) return TPQ_ERR_UNSUPPORTED;
    const uint32_t threads = 64u * static_cast<uint32_t>(passes);
    EncRowsGeom gm;
    gm.row_pieces = static_cast<uint32_t>(a.E) / 8u;
    const int mr = static_cast<int>((gm.row_pieces + threads - 1u) / threads);
    if (mr > 2) return TPQ_ERR_UNSUPPORTED;
    gm.lds_row = static_cast<uint32_t>(a.E) * 2u;
    gm.nb_codes = 4u * static_cast<uint32_t>(a.chunks);
    gm.nb_meta = 2u * static_cast<uint32_t>(a.ng);
    gm.nb_outl = 2u * static_cast<uint32_t>(a.k);
    gm.pc = (gm.nb_codes + 15u) / 16u;
    gm.pm = (gm.nb_meta + 15u) / 16u;
    gm.po = (gm.nb_outl + 15u) / 16u;
    gm.st_scale = 16u * gm.pc;
    gm.st_zero = gm.st_scale + 16u * gm.pm;
    gm.st_outl = gm.st_zero + 16u * gm.pm;
    gm.lds_stage = gm.st_outl + 16u * gm.po;
    const PlanOffsets o = plan_offsets(a.k, a.r, a.G);
    gm.off_src = static_cast<uint32_t>(o.src);
    const size_t lds = 2u * (static_cast<size_t>(gm.lds_row) + gm.lds_stage);
    if (lds > 160u * 1024u) return TPQ_ERR_UNSUPPORTED;
    if (a.T * a.n_ranks > 0x7FFFFFFFLL) return TPQ_ERR_UNSUPPORTED;

    EncodeArgs b = a;
    b.off_idx = o.idx;
    int dev = 0, cus = 0, per_cu = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return hip_result(e);
    const int64_t total = a.T * a.n_ranks;

#define TPQ_EROWS2(LPG, MR)                                                                            \
    do {                                                                                               \
        auto kern = k_encode_rows<LPG, MR>;                                                            \
        if (lds > 65536)                                                                               \
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                              \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)); \
        if (e == hipSuccess)                                                                           \
            e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, static_cast<int>(threads), lds); \
        if (e == hipSuccess && per_cu < 1) e = hipErrorLaunchOutOfResources;                           \
        if (e == hipSuccess) {                                                                         \
            int64_t grid = static_cast<int64_t>(cus) * tuned_enc_wg_per_cu(per_cu);                    \
            if (grid > total) grid = total;                                                            \
            launch_kernel(kern, dim3(static_cast<unsigned>(grid)), dim3(threads), lds, s, b, gm, Y, codes, scale, zero, outl); \
        }                                                                                              \
    } while (0)
#define TPQ_EROWS(LPG)                 \
    do {                               \
        if (mr <= 1) TPQ_EROWS2(LPG, 1); \
        else TPQ_EROWS2(LPG, 2);       \
    } while (0)
    switch (a.G / 8) {
    case 4: TPQ_EROWS(4); break;
    case 8: TPQ_EROWS(8); break;
    case 16: TPQ_EROWS(16); break;
    case 32: TPQ_EROWS(32); break;
    default: return TPQ_ERR_UNSUPPORTED;
    }
#undef TPQ_EROWS
#undef TPQ_EROWS2
    if (e == hipSuccess) e = hipGetLastError();
    return hip_result(e);
}

}  // namespace tpq
