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

// ---------------------------------------------------------------------------
// Streaming kernel (the fast path).
//
// Work unit: one segment (P passes of 64 chunks) of one row of one rank.  Groups
// never straddle a pass (64 chunks = 512 features, a multiple of every G), so
// segments are independent.  The grid is persistent: blockIdx.y = rank,
// blockIdx.z = segment, and the 4 wavefronts of each of the gridDim.x workgroups
// walk over the rows t = 4*blockIdx.x + wave, + 4*gridDim.x, ...  Each wave keeps
// the next row's loads in flight while it works on the current one.
//
// LDS stage of a wave.  The row slice is kept as 32-bit words in blocks of
// 32 words (8 aligned 16-byte chunks) that occupy 37 words each: the 32 words,
// a copy of the next block's first 4 words, and one pad word.  A lane reads the
// 5 words that hold its 8 consecutive compacted features starting at any word;
// the copy keeps those 5 words contiguous and the odd block stride spreads the
// 64 lanes (16 bytes apart) over all banks.  Every LDS access is word aligned:
// removing the selected columns shifts the compacted stream by their count, so a
// chunk starts at any 2-byte boundary, and the remaining half-word shift is one
// funnel shift per word in registers.
//
// Once per workgroup: per-chunk stage addresses go to registers; the stage
// addresses of the split chunks' sources and of the selected columns go to LDS.
// Per row:
//   A. the row slice arrives through aligned, coalesced 128-bit loads issued one
//      row ahead, is written to the stage, and the next row's loads are issued;
//   B. the few chunks that an outlier splits (at most k + 1 per row, plus the
//      absent tail of the last group) are gathered half-word by half-word from the
//      stage by as many lanes into a patch area; the selected columns are copied
//      from the stage to the outlier section;
//   C. every lane fetches its 8 features (5 words + funnel shift); owners of
//      split chunks take theirs from the patch area;
//   D. lane-local min / max, DPP reduction over the group's lanes, leaders park
//      (min, max) in LDS;
//   E. one lane per group derives zero, bf16 scale and reciprocal (two IEEE
//      divisions per group instead of per lane) and stores scale / zero;
//   F. quantise from registers, pack 8 nibbles per lane, coalesced store.
// No workgroup barrier inside the row loop: stage, patch and meta are private to
// a wave.
// ---------------------------------------------------------------------------
constexpr uint32_t kStageBlockBytes = 37 * 4;

// byte offset in the stage of the half-word at relative column c
__device__ __forceinline__ uint32_t stage_addr(uint32_t c)
{
    const uint32_t word = c >> 1;
    return 4u * (word + 5u * (word >> 5)) + 2u * (c & 1u);
}

template <int LPG, int P>
__global__ __launch_bounds__(256) void k_encode_stream(EncodeArgs a, RankPtrs Yp, RankPtrs codesp,
                                                       RankPtrs scalep, RankPtrs zerop,
                                                       RankPtrs outlp)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t rank = blockIdx.y;
    const uint32_t seg = blockIdx.z;

    const uint32_t pass0 = seg * P;
    const uint32_t passes_total = static_cast<uint32_t>(a.chunks_padded) >> 6;
    const uint32_t n_pass = passes_total - pass0 < P ? passes_total - pass0 : P;
    const bool last_seg = pass0 + n_pass == passes_total;

    // Columns [col_lo, col_hi) of the row are staged; both are multiples of 8.  The
    // first compacted feature of pass p sits at column 512*p + (selected columns
    // before it), so the segment lies inside [512*pass0, 512*(pass0 + n_pass) + k]:
    // bounds that need nothing from the plan, so the first row's loads can leave
    // before any table has arrived.
    const uint32_t col_lo = 512u * pass0;
    const uint32_t col_hi =
        last_seg ? static_cast<uint32_t>(a.E)
                 : min(static_cast<uint32_t>(a.E), (512u * (pass0 + n_pass) + a.k + 7u) & ~7u);
    const uint32_t n16 = (col_hi - col_lo) >> 3;

    const uint32_t t0 = blockIdx.x * 4u + wave, t_step = gridDim.x * 4u;
    const uint32_t T = static_cast<uint32_t>(a.T);
    const uint16_t *ybase = static_cast<const uint16_t *>(Yp.p[rank]) + col_lo;
    constexpr int S = P + 1;  // staging loads per lane; 64*S >= n16 (checked by the host)
    u32x4 rbuf[S];
    if (t0 < T) {
        const u32x4 *yrow = reinterpret_cast<const u32x4 *>(ybase + static_cast<int64_t>(t0) * a.ldY);
#pragma unroll
        for (int j = 0; j < S; ++j)
            rbuf[j] = __builtin_nontemporal_load(yrow + min(j * 64u + lane, n16 - 1u));
    }

    const PlanHeader *ph = reinterpret_cast<const PlanHeader *>(a.plan);
    if (ph->magic != kPlanMagic || ph->status != kPlanOk || ph->E != a.E || ph->k != a.k ||
        ph->G != a.G)
        return;  // the whole grid takes this branch together
    const int32_t *idx = reinterpret_cast<const int32_t *>(a.plan + ph->idx_offset);
    const uint32_t *cpos = reinterpret_cast<const uint32_t *>(a.plan + ph->pos_offset);
    const uint16_t *pass_irr = reinterpret_cast<const uint16_t *>(a.plan + ph->pass_irr_offset);
    const uint16_t *pass_col = reinterpret_cast<const uint16_t *>(a.plan + ph->pass_col_offset);
    const uint16_t *irr_src = reinterpret_cast<const uint16_t *>(a.plan + ph->irr_src_offset);

    // selected columns and split chunks owned by this segment: the selected columns
    // below the next segment's first feature that no earlier segment owns
    const uint32_t c_first = pass_col[pass0], c_next = pass_col[pass0 + n_pass];
    const uint32_t p_lo = seg == 0 ? 0u : c_first - 512u * pass0;
    const uint32_t p_hi = last_seg ? static_cast<uint32_t>(a.k) : c_next - 512u * (pass0 + n_pass);
    const uint32_t q_lo = pass_irr[pass0], q_hi = pass_irr[pass0 + n_pass];
    const uint32_t n_q = q_hi - q_lo, n_sel = p_hi - p_lo;

    constexpr int GPS = 64 * P / LPG;  // groups per segment
    constexpr uint32_t STAGE_BYTES = (8u * S * kStageBlockBytes + 15u) / 16u * 16u;
    constexpr uint32_t META_BYTES = (GPS * 8u + 15u) / 16u * 16u;
    extern __shared__ u32x4 smem_stream[];
    uint8_t *lds = reinterpret_cast<uint8_t *>(smem_stream);
    // workgroup-wide tables, then one (stage | patch | meta) region per wave
    uint16_t *l_irr = reinterpret_cast<uint16_t *>(lds);                       // [patch_slots][8]
    uint16_t *l_sel = reinterpret_cast<uint16_t *>(lds + 16u * a.patch_slots);  // [k]
    const uint32_t tables_bytes = 16u * a.patch_slots + ((2u * a.k + 15u) & ~15u);
    const uint32_t wave_bytes = STAGE_BYTES + 16u * a.patch_slots + META_BYTES;
    uint8_t *stage = lds + tables_bytes + wave * wave_bytes;
    u32x4 *patch = reinterpret_cast<u32x4 *>(stage + STAGE_BYTES);
    float2 *meta = reinterpret_cast<float2 *>(stage + STAGE_BYTES + 16u * a.patch_slots);

    // tables -> LDS as stage byte offsets
    for (uint32_t i = threadIdx.x; i < 8u * n_q; i += 256)
        l_irr[i] = static_cast<uint16_t>(stage_addr(irr_src[8u * q_lo + i] - col_lo));
    for (uint32_t i = threadIdx.x; i < n_sel; i += 256)
        l_sel[i] = static_cast<uint16_t>(stage_addr(static_cast<uint32_t>(idx[p_lo + i]) - col_lo));
    // per chunk: bits 15..0 = stage byte offset of the word holding its first feature,
    // bits 20..16 = funnel shift (16 if that feature is the word's upper half),
    // bits 30..21 = patch slot within the segment (kSlotNone: none), bit 31 = take
    // the features from the patch area
    constexpr uint32_t kSlotNone = 0x3FFu;
    uint32_t cp[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const uint32_t c = static_cast<uint32_t>(p) < n_pass
                               ? cpos[(pass0 + p) * 64u + lane]
                               : (kNotRegular | (kNoSlot << 16) | (col_hi - 8u));
        const uint32_t col = (c & 0xFFFFu) - col_lo;
        const uint32_t slot = (c >> 16) & 0x7FFFu;
        const bool patched = (c & kNotRegular) && slot != kNoSlot;
        cp[p] = (stage_addr(col) & ~3u) | ((col & 1u) << 20) |
                ((patched ? slot - q_lo : kSlotNone) << 21) | (patched ? kNotRegular : 0u);
    }
    __syncthreads();

    for (uint32_t t = t0; t < T; t += t_step) {
        // Re-derive every per-lane address inside the iteration: hoisted out of the
        // loop they would cost more registers than the few instructions they save.
        uint32_t ln = lane;
        asm volatile("" : "+v"(ln));
#pragma unroll
        for (int p = 0; p < P; ++p) asm volatile("" : "+v"(cp[p]));

        // A: current row -> stage (chunk 64*j + ln: block 8*j + ln/8, slot ln%8; the
        // first chunk of a block is also copied behind the previous block), then the
        // next row's loads -> flight
        {
            uint8_t *w = stage + kStageBlockBytes * (ln >> 3) + 16u * (ln & 7u);
            const bool first_of_block = (ln & 7u) == 0;
#pragma unroll
            for (int j = 0; j < S; ++j) {
                *reinterpret_cast<u32x4_a4 *>(w + j * 8 * kStageBlockBytes) = rbuf[j];
                if (first_of_block && (j > 0 || ln >= 8))
                    *reinterpret_cast<u32x4_a4 *>(w + j * 8 * kStageBlockBytes - 20) = rbuf[j];
            }
        }
        if (t + t_step < T) {
            const u32x4 *yrow = reinterpret_cast<const u32x4 *>(
                ybase + static_cast<int64_t>(t + t_step) * a.ldY);
#pragma unroll
            for (int j = 0; j < S; ++j)
                rbuf[j] = __builtin_nontemporal_load(yrow + min(j * 64u + ln, n16 - 1u));
        }
        wave_lds_fence();

        // B: split chunks -> patch area; selected columns -> outlier section
        for (uint32_t q = ln; q < n_q; q += 64) {
            const u32x4 tab = *reinterpret_cast<const u32x4 *>(l_irr + 8u * q);
            u32x4 g;
#define TPQ_HW(off) static_cast<uint32_t>(*reinterpret_cast<const uint16_t *>(stage + (off)))
            g.x = TPQ_HW(tab.x & 0xFFFFu) | (TPQ_HW(tab.x >> 16) << 16);
            g.y = TPQ_HW(tab.y & 0xFFFFu) | (TPQ_HW(tab.y >> 16) << 16);
            g.z = TPQ_HW(tab.z & 0xFFFFu) | (TPQ_HW(tab.z >> 16) << 16);
            g.w = TPQ_HW(tab.w & 0xFFFFu) | (TPQ_HW(tab.w >> 16) << 16);
            patch[q] = g;
        }
        if (n_sel > 0) {
            uint16_t *outl = reinterpret_cast<uint16_t *>(
                                 static_cast<uint8_t *>(const_cast<void *>(outlp.p[rank])) +
                                 static_cast<int64_t>(t) * a.pitch_outl) + p_lo;
            for (uint32_t p = ln; p < n_sel; p += 64) outl[p] = static_cast<uint16_t>(TPQ_HW(l_sel[p]));
        }
#undef TPQ_HW

        // C: 8 consecutive compacted features per lane and pass
        u32x4 v[P];
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const uint32_t *src = reinterpret_cast<const uint32_t *>(stage + (cp[p] & 0xFFFFu));
            const uint32_t d0 = src[0], d1 = src[1], d2 = src[2], d3 = src[3], d4 = src[4];
            const uint32_t sh = (cp[p] >> 16) & 31u;
            v[p].x = __builtin_amdgcn_alignbit(d1, d0, sh);
            v[p].y = __builtin_amdgcn_alignbit(d2, d1, sh);
            v[p].z = __builtin_amdgcn_alignbit(d3, d2, sh);
            v[p].w = __builtin_amdgcn_alignbit(d4, d3, sh);
        }
        wave_lds_fence();
#pragma unroll
        for (int p = 0; p < P; ++p)
            if (cp[p] & kNotRegular) v[p] = patch[(cp[p] >> 21) & 0x3FFu];

        // D: group min / max.  The upper feature of a word is compared as the whole
        // word: as a float the word lies between that feature and its successor in
        // magnitude, so it wins exactly where the feature would, and masking the
        // winner's low half gives the feature itself.
        {
            float mn[P], mx[P];
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const float l0 = bf16_lo_to_f32(v[p].x), l1 = bf16_lo_to_f32(v[p].y);
                const float l2 = bf16_lo_to_f32(v[p].z), l3 = bf16_lo_to_f32(v[p].w);
                const float h0 = __uint_as_float(v[p].x), h1 = __uint_as_float(v[p].y);
                const float h2 = __uint_as_float(v[p].z), h3 = __uint_as_float(v[p].w);
                const float lo = fminf(fminf(fminf(l0, l1), fminf(l2, l3)),
                                       fminf(fminf(h0, h1), fminf(h2, h3)));
                const float hi = fmaxf(fmaxf(fmaxf(l0, l1), fmaxf(l2, l3)),
                                       fmaxf(fmaxf(h0, h1), fmaxf(h2, h3)));
                mn[p] = __uint_as_float(__float_as_uint(lo) & 0xFFFF0000u);
                mx[p] = __uint_as_float(__float_as_uint(hi) & 0xFFFF0000u);
            }
            group_minmax_n<LPG, P>(mn, mx);
            if ((ln % LPG) == 0) {
#pragma unroll
                for (int p = 0; p < P; ++p) meta[(p * 64 + ln) / LPG] = make_float2(mn[p], mx[p]);
            }
        }
        wave_lds_fence();

        // E: zero, scale, reciprocal -- one lane per group
        {
            uint16_t *scale = reinterpret_cast<uint16_t *>(
                static_cast<uint8_t *>(const_cast<void *>(scalep.p[rank])) +
                static_cast<int64_t>(t) * a.pitch_meta);
            uint16_t *zero = reinterpret_cast<uint16_t *>(
                static_cast<uint8_t *>(const_cast<void *>(zerop.p[rank])) +
                static_cast<int64_t>(t) * a.pitch_meta);
            const uint32_t g0 = pass0 * (64 / LPG);
            for (uint32_t gl = ln; gl < static_cast<uint32_t>(GPS); gl += 64) {
                const uint32_t g = g0 + gl;
                if (g < static_cast<uint32_t>(a.ng)) {
                    const float2 mm = meta[gl];
                    const float mn = mm.x + 0.0f;  // a zero minimum is stored as +0
                    const float span = mm.y - mn;
                    const float s32 = div_by_15(span);
                    const uint32_t sb = pack_bf16x2(s32, s32) & 0xFFFFu;
                    const float s = bf16_bits_to_f32(sb);
                    const bool constant = s < 1e-30f;
                    const float inv = constant ? 0.0f : reciprocal_of_scale(s);
                    scale[g] = constant ? uint16_t(0) : static_cast<uint16_t>(sb);
                    zero[g] = static_cast<uint16_t>(__float_as_uint(mn) >> 16);
                    meta[gl] = make_float2(mn, inv);
                }
            }
        }
        wave_lds_fence();

        // F: quantise and pack.  (x - zero) * inv lies in [0, 15.06] for finite input
        // (scale is (max - min) / 15 rounded to 8 significant bits), so the rounded
        // value needs no clamp to stay a 4-bit code.
        uint32_t *codes = reinterpret_cast<uint32_t *>(
            static_cast<uint8_t *>(const_cast<void *>(codesp.p[rank])) +
            static_cast<int64_t>(t) * a.pitch_codes);
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const uint32_t chunk = (pass0 + p) * 64u + ln;
            const float2 mi = meta[(p * 64 + ln) / LPG];
            const uint32_t wv[4] = {v[p].x, v[p].y, v[p].z, v[p].w};
            uint32_t h[2];
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                float pr[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t word = wv[half * 2 + (e >> 1)];
                    const float x = (e & 1) ? bf16_hi_to_f32(word) : bf16_lo_to_f32(word);
                    const float d = x - mi.x;
                    pr[e] = d * mi.y;
                }
                // float -> byte conversion (nearest even) into swapped neighbouring bytes;
                // (b << 12) | b then joins each pair of codes into one byte
                uint32_t b = __builtin_amdgcn_cvt_pk_u8_f32(pr[1], 0u, 0u);
                b = __builtin_amdgcn_cvt_pk_u8_f32(pr[0], 1u, b);
                b = __builtin_amdgcn_cvt_pk_u8_f32(pr[3], 2u, b);
                b = __builtin_amdgcn_cvt_pk_u8_f32(pr[2], 3u, b);
                h[half] = (b << 12) | b;
            }
            uint32_t w = __builtin_amdgcn_perm(h[1], h[0], 0x07050301u);
            const int n_valid = a.r - 8 * static_cast<int>(chunk);
            if (n_valid < 8) w &= (1u << (4 * (n_valid & 7))) - 1u;
            if (chunk < static_cast<uint32_t>(a.chunks)) __builtin_nontemporal_store(w, codes + chunk);
        }
        wave_lds_fence();  // the next row overwrites stage / patch / meta
    }
}

// ---------------------------------------------------------------------------
// Direct kernel (the fast path).
//
// Work unit ("task"): one segment (P passes of 64 chunks) of one row of one rank,
// handled by one wavefront from start to end; blockIdx.y = rank and the four waves
// of workgroup blockIdx.x take tasks 4*blockIdx.x .. +3 of that rank (task =
// t * segs + seg).  Waves are independent (no barrier, no shared tables) and short,
// so the hardware scheduler staggers them and a CU always holds waves in every phase.
// No stage of the row in LDS: lane l of pass p loads the 16 bytes ("window") that
// hold its chunk's 8 features straight from the row, at the even column at or below
// the chunk's first feature -- a 4-byte aligned 128-bit load.  Where that feature is
// the upper half of the first word, the 8th feature is the first half-word of the
// next lane's window: one DPP move and a funnel shift per word put the features in
// place.
//
// A chunk that cannot be had that way (an outlier splits it, it is ragged, the next
// lane's window is not adjacent) has a "slot": 32 bytes of LDS private to the wave.
// Its lane writes its window to the slot's first half; lane q of the wave loads the
// second window (the next 8 columns) of the segment's q-th slot into the other half,
// picks the slot's 8 features half-word by half-word at the positions the plan lists
// and writes them back to the first half, where the owner reads them.  The selected
// features themselves are read from the slots too (each lies in the windows of the
// chunk it splits or follows) and copied to the outlier section.  A feature or
// selected column out of a slot's reach (eight or more selected columns in a row) is
// read from memory instead.
//
// Then: min / max per lane, DPP reduction over the group's lanes; zero, bf16 scale
// and reciprocal in every lane; quantise from registers, pack 8 codes per lane,
// coalesced store.
//
// The address unit of a CU takes about as long for a vector memory instruction with
// four active lanes as for a full one, and it is the unit this kernel keeps busiest:
// hence one 128-bit load for a lane's plan entries of all passes, one load of second
// windows per 64 slots instead of one per pass, and scale / zero of all the task's
// groups collected through LDS into one store each.
// ---------------------------------------------------------------------------
template <int P>
struct DirectOcc {  // waves per SIMD the register budget is set for
    static constexpr int value = 8;
};

template <int LPG, int P>
__global__ __launch_bounds__(256, DirectOcc<P>::value) void k_encode_direct(
    EncodeArgs a, RankPtrs Yp, RankPtrs codesp, RankPtrs scalep, RankPtrs zerop, RankPtrs outlp)
{
    const uint32_t ln = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    const uint32_t passes = static_cast<uint32_t>(a.chunks_padded) >> 6;
    const uint32_t segs = static_cast<uint32_t>(a.segs);
    const uint32_t rank = blockIdx.y;
    const uint32_t task = blockIdx.x * 4u + wave;
    if (task >= static_cast<uint32_t>(a.n_tasks)) return;
    // t = task / segs by multiplication (exact below 2^32 / segs, which the host keeps)
    const uint32_t t = segs == 1 ? task : __umulhi(task, a.segs_magic);
    const uint32_t seg = task - t * segs;
    const uint32_t pass0 = seg * P, pass1 = min(pass0 + P, passes);
    const bool last_seg = pass1 == passes;

    // The tables sit at offsets the host knows, so the first plan reads leave together
    // with the header's (they stay inside the plan buffer whatever it holds); nothing
    // is done with them unless the header says that the plan is good.
    const int32_t *idx = reinterpret_cast<const int32_t *>(a.plan + a.off_idx);
    const u32x4 *dirr = reinterpret_cast<const u32x4 *>(a.plan + a.off_dirr);
    const uint32_t *dsel = reinterpret_cast<const uint32_t *>(a.plan + a.off_dsel);
    const uint2 *dslot8 = reinterpret_cast<const uint2 *>(a.plan + a.off_dslot8);
    const uint2 *dseg = reinterpret_cast<const uint2 *>(a.plan + a.off_dseg);
    const u32x4 *drec = reinterpret_cast<const u32x4 *>(a.plan + a.off_drec);
    const u32x4 dp8 = drec[(seg * 64u + ln) * 2u];
    const u32x4 rec1 = drec[(seg * 64u + ln) * 2u + 1u];
    const uint2 sg = dseg[seg];
    const PlanHeader *ph = reinterpret_cast<const PlanHeader *>(a.plan);
    if (ph->magic != kPlanMagic || ph->status != kPlanOk || ph->E != a.E || ph->k != a.k ||
        ph->G != a.G || ph->dir_P != P)
        return;  // the whole grid takes this branch together

    // slots and selected columns of this segment
    const uint32_t q_lo = sg.x & 0xFFFFu, n_q = sg.x >> 16;
    const uint32_t s_lo = sg.y & 0xFFFFu, n_sel = sg.y >> 16;

    // the segment's ln-th slot and selected feature (zero where there is none)
    const uint2 slot8 = make_uint2(rec1.x, rec1.y);
    const uint32_t sel0 = rec1.z;
    uint32_t d[P];
    {
        const uint32_t w4[4] = {dp8.x, dp8.y, dp8.z, dp8.w};
#pragma unroll
        for (int p = 0; p < P; ++p) d[p] = (p & 1) ? (w4[p >> 1] >> 16) : (w4[p >> 1] & 0xFFFFu);
    }

    // windows: every lane its chunk's; lane q the second window of slot q
    const uint8_t *yrow = static_cast<const uint8_t *>(Yp.p[rank]) + static_cast<int64_t>(t) * a.ldY * 2;
    u32x4 raw[P];
#pragma unroll
    for (int p = 0; p < P; ++p)
        raw[p] = __builtin_nontemporal_load(
            reinterpret_cast<const u32x4_a4 *>(yrow + 4u * (d[p] & 0x3FFFu)));
    u32x4 win_b = {0u, 0u, 0u, 0u};
    if (ln < n_q) win_b = *reinterpret_cast<const u32x4_a4 *>(yrow + (slot8.y & 0x1FFFFu));

    constexpr int GPS = 64 * P / LPG;  // groups per segment
    extern __shared__ u32x4 smem_direct[];
    uint8_t *slots = reinterpret_cast<uint8_t *>(smem_direct) + wave * (32u * a.patch_slots + 4u * GPS);
    uint32_t *l_meta = reinterpret_cast<uint32_t *>(slots + 32u * a.patch_slots);

    // A: windows -> slots (lanes that have one) and -> features (the others).  A lane's
    // slot number within the segment: the flagged chunks before its own.
    u32x4 v[P];
    uint32_t my_slot[P];
    {
        uint32_t before = 0;  // slots of the segment's earlier passes
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const bool has_slot = (d[p] & kDir16Slot) != 0;
            const uint64_t ball = __builtin_amdgcn_ballot_w64(has_slot);
            my_slot[p] = before + __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(ball >> 32),
                                                           __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(ball), 0u));
            before += static_cast<uint32_t>(__builtin_popcountll(ball));
            if (has_slot) *reinterpret_cast<u32x4 *>(slots + 32u * my_slot[p]) = raw[p];
            const uint32_t nb = __builtin_amdgcn_update_dpp(0u, raw[p].x, 0x130, 0xF, 0xF, false);
            const uint32_t sh = (d[p] >> 10) & 16u;
            v[p].x = __builtin_amdgcn_alignbit(raw[p].y, raw[p].x, sh);
            v[p].y = __builtin_amdgcn_alignbit(raw[p].z, raw[p].y, sh);
            v[p].z = __builtin_amdgcn_alignbit(raw[p].w, raw[p].z, sh);
            v[p].w = __builtin_amdgcn_alignbit(nb, raw[p].w, sh);
        }
    }
    if (ln < n_q) *reinterpret_cast<u32x4 *>(slots + 32u * ln + 16u) = win_b;
    for (uint32_t q0 = 64; q0 < n_q; q0 += 64) {  // more than 64 slots in a segment: rare
        const uint32_t q = q0 + ln;
        if (q < n_q)
            *reinterpret_cast<u32x4 *>(slots + 32u * q + 16u) =
                *reinterpret_cast<const u32x4_a4 *>(yrow + (dslot8[q_lo + q].y & 0x1FFFFu));
    }
    wave_lds_fence();

    // B: selected columns -> outlier section; slots -> their 8 features.  Lanes past the
    // end repeat the last item and skip the store.
#define TPQ_HW(ptr) static_cast<uint32_t>(*reinterpret_cast<const uint16_t *>(ptr))
#define TPQ_LDS_HW(ptr) static_cast<uint32_t>(*(const __attribute__((address_space(3))) uint16_t *)(ptr))
    if (n_sel > 0) {
        uint16_t *outl = reinterpret_cast<uint16_t *>(
                             static_cast<uint8_t *>(const_cast<void *>(outlp.p[rank])) +
                             static_cast<int64_t>(t) * a.pitch_outl) + s_lo;
        for (uint32_t p0 = 0; p0 < n_sel; p0 += 64) {
            const uint32_t p = p0 + ln, pc = min(p, n_sel - 1u);
            const uint32_t e = p0 == 0 ? sel0 : dsel[s_lo + pc];
            const bool far = (e & kDirFar) != 0;
            uint32_t val = TPQ_LDS_HW(slots + (far ? 0u : e - 32u * q_lo));
            if (far) val = TPQ_HW(yrow + 2u * static_cast<uint32_t>(idx[s_lo + pc]));
            if (p < n_sel) outl[p] = static_cast<uint16_t>(val);
        }
    }
    for (uint32_t q0 = 0; q0 < n_q; q0 += 64) {
        const uint32_t q = q0 + ln, qc = min(q, n_q - 1u);
        const uint2 ent = q0 == 0 ? slot8 : dslot8[q_lo + qc];
        const uint8_t *sl = slots + 32u * qc;
        const uint32_t nib = ent.x;
        u32x4 g;
        // feature e sits at half-word (nib >> 4e) & 15 of the slot
#define TPQ_AT(e) TPQ_LDS_HW(sl + ((nib >> (4 * (e) - 1)) & 0x1Eu))
        g.x = TPQ_LDS_HW(sl + ((nib << 1) & 0x1Eu)) | (TPQ_AT(1) << 16);
        g.y = TPQ_AT(2) | (TPQ_AT(3) << 16);
        g.z = TPQ_AT(4) | (TPQ_AT(5) << 16);
        g.w = TPQ_AT(6) | (TPQ_AT(7) << 16);
#undef TPQ_AT
        if (ent.y & kDirWide8) {
            const u32x4 tab = dirr[q_lo + qc];  // the features' columns
#define TPQ_FAR(w) (TPQ_HW(yrow + 2u * ((w) & 0x7FFFu)) | (TPQ_HW(yrow + 2u * (((w) >> 16) & 0x7FFFu)) << 16))
            g.x = TPQ_FAR(tab.x);
            g.y = TPQ_FAR(tab.y);
            g.z = TPQ_FAR(tab.z);
            g.w = TPQ_FAR(tab.w);
#undef TPQ_FAR
        }
        if (q < n_q) *reinterpret_cast<u32x4 *>(slots + 32u * q) = g;
    }
#undef TPQ_HW
#undef TPQ_LDS_HW
    wave_lds_fence();
#pragma unroll
    for (int p = 0; p < P; ++p)
        if (d[p] & kDir16Slot) v[p] = *reinterpret_cast<const u32x4 *>(slots + 32u * my_slot[p]);

    // D: group min / max.  The upper feature of a word is compared as the whole
    // word: as a float the word lies between that feature and its successor in
    // magnitude, so it wins exactly where the feature would, and masking the
    // winner's low half gives the feature itself.  After the DPP reduction every
    // lane of a group holds the group's range.
    float mn[P], mx[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const float l0 = bf16_lo_to_f32(v[p].x), l1 = bf16_lo_to_f32(v[p].y);
        const float l2 = bf16_lo_to_f32(v[p].z), l3 = bf16_lo_to_f32(v[p].w);
        const float h0 = __uint_as_float(v[p].x), h1 = __uint_as_float(v[p].y);
        const float h2 = __uint_as_float(v[p].z), h3 = __uint_as_float(v[p].w);
        const float lo = fminf(fminf(fminf(l0, l1), fminf(l2, l3)),
                               fminf(fminf(h0, h1), fminf(h2, h3)));
        const float hi = fmaxf(fmaxf(fmaxf(l0, l1), fmaxf(l2, l3)),
                               fmaxf(fmaxf(h0, h1), fmaxf(h2, h3)));
        mn[p] = __uint_as_float(__float_as_uint(lo) & 0xFFFF0000u);
        mx[p] = __uint_as_float(__float_as_uint(hi) & 0xFFFF0000u);
    }
    if (last_seg) {
        // chunks beyond the row must not touch their group's range
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if ((pass0 + p) * 64u + ln >= static_cast<uint32_t>(a.chunks)) {
                mn[p] = 3.3895314e38f;   // the largest finite bf16
                mx[p] = -3.3895314e38f;
            }
        }
    }
    group_minmax_n<LPG, P>(mn, mx);

    // E: zero, bf16 scale and its reciprocal, in every lane (cheaper than a trip
    // through LDS to one lane per group).  Both divisions are exact replacements of
    // the IEEE ones: x / 15 as x * fl(1/15) with one fused correction step (equal
    // to the correctly rounded quotient for every float), 1 / scale as the hardware
    // reciprocal with one Newton step (equal to the correctly rounded reciprocal
    // for every bf16 scale whose reciprocal is a normal number, which covers every
    // finite range).  Each group's first lane parks (scale | zero << 16) in LDS, from
    // where lane g stores group g's pair.
    float inv[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        mn[p] = mn[p] + 0.0f;  // a zero minimum is stored as +0
        const float span = mx[p] - mn[p];
        const float s32 = div_by_15(span);
        const uint32_t sb = pack_bf16x2(s32, s32) & 0xFFFFu;
        const float s = bf16_bits_to_f32(sb);
        const bool constant = s < 1e-30f;
        inv[p] = constant ? 0.0f : reciprocal_of_scale(s);
        if ((ln % LPG) == 0)
            l_meta[p * (64 / LPG) + ln / LPG] = (constant ? 0u : sb) | (__float_as_uint(mn[p]) & 0xFFFF0000u);
    }
    wave_lds_fence();
    {
        uint16_t *scale = reinterpret_cast<uint16_t *>(
            static_cast<uint8_t *>(const_cast<void *>(scalep.p[rank])) +
            static_cast<int64_t>(t) * a.pitch_meta);
        uint16_t *zero = reinterpret_cast<uint16_t *>(
            static_cast<uint8_t *>(const_cast<void *>(zerop.p[rank])) +
            static_cast<int64_t>(t) * a.pitch_meta);
        const uint32_t g0 = pass0 * (64 / LPG);
        if (GPS <= 32) {
            // one store instruction for both: lanes 0..31 scales, lanes 32..63 zeros
            const uint32_t gl = ln & 31u;
            const bool is_zero = ln >= 32u;
            if (gl < static_cast<uint32_t>(GPS) && g0 + gl < static_cast<uint32_t>(a.ng)) {
                const uint32_t m = l_meta[gl];
                (is_zero ? zero : scale)[g0 + gl] = static_cast<uint16_t>(is_zero ? m >> 16 : m & 0xFFFFu);
            }
        } else {
#pragma unroll
            for (uint32_t gl0 = 0; gl0 < static_cast<uint32_t>(GPS); gl0 += 64) {
                const uint32_t gl = gl0 + ln;
                if (gl < static_cast<uint32_t>(GPS) && g0 + gl < static_cast<uint32_t>(a.ng)) {
                    const uint32_t m = l_meta[gl];
                    scale[g0 + gl] = static_cast<uint16_t>(m & 0xFFFFu);
                    zero[g0 + gl] = static_cast<uint16_t>(m >> 16);
                }
            }
        }
    }

    // F: quantise and pack.  (x - zero) * inv lies in [0, 15.06] for finite input
    // (scale is (max - min) / 15 rounded to 8 significant bits), so the rounded
    // value is a 4-bit code without a clamp.  The float -> byte conversion rounds
    // to the nearest even integer and drops the result into a byte of its
    // destination; the codes of a feature pair land swapped in neighbouring bytes,
    // so that (a << 12) | a joins each pair into one byte, and a byte permute
    // collects the four bytes.
    uint32_t *codes = reinterpret_cast<uint32_t *>(
        static_cast<uint8_t *>(const_cast<void *>(codesp.p[rank])) +
        static_cast<int64_t>(t) * a.pitch_codes);
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const uint32_t wv[4] = {v[p].x, v[p].y, v[p].z, v[p].w};
        uint32_t h[2];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            float pr[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t word = wv[half * 2 + (e >> 1)];
                const float x = (e & 1) ? bf16_hi_to_f32(word) : bf16_lo_to_f32(word);
                const float df = x - mn[p];
                pr[e] = df * inv[p];
            }
            uint32_t b = __builtin_amdgcn_cvt_pk_u8_f32(pr[1], 0u, 0u);
            b = __builtin_amdgcn_cvt_pk_u8_f32(pr[0], 1u, b);
            b = __builtin_amdgcn_cvt_pk_u8_f32(pr[3], 2u, b);
            b = __builtin_amdgcn_cvt_pk_u8_f32(pr[2], 3u, b);
            h[half] = (b << 12) | b;
        }
        uint32_t w = __builtin_amdgcn_perm(h[1], h[0], 0x07050301u);
        const uint32_t chunk = (pass0 + p) * 64u + ln;
        if (last_seg) {
            const int n_valid = a.r - 8 * static_cast<int>(chunk);
            if (n_valid < 8) w &= (1u << (4 * (n_valid & 7))) - 1u;
            if (chunk < static_cast<uint32_t>(a.chunks)) __builtin_nontemporal_store(w, codes + chunk);
        } else {
            __builtin_nontemporal_store(w, codes + chunk);
        }
    }
}

static size_t encode_row_lds(const EncodeArgs &a, int lpg)
{
    const size_t groups_padded = static_cast<size_t>(a.chunks_padded) / lpg;
    const size_t meta = (groups_padded > static_cast<size_t>(a.ng) ? groups_padded : a.ng) * 8;
    return static_cast<size_t>(a.E) * 2 + (meta + 15) / 16 * 16;
}

// Passes per segment: rows are cut into segments of at most 6 passes (3072 features).
// Short segments keep a wave's registers and LDS small, so that 16 waves fit on a CU.
static int pick_seg_passes(int passes, int *segs)
{
    const int n_seg = (passes + 5) / 6;
    const int p = (passes + n_seg - 1) / n_seg;
    *segs = (passes + p - 1) / p;
    return p;
}

template <int LPG>
static hipError_t launch_stream_lpg(EncodeArgs &a, const RankPtrs &Y, const RankPtrs &codes,
                                    const RankPtrs &scale, const RankPtrs &zero,
                                    const RankPtrs &outl, int blocks_x, hipStream_t s)
{
    const int P = a.seg_passes;
    const size_t meta_bytes = (static_cast<size_t>(64 * P / LPG) * 8 + 15) / 16 * 16;
    const size_t stage_bytes = (static_cast<size_t>(8) * (P + 1) * 37 * 4 + 15) / 16 * 16;
    const size_t per_wave = stage_bytes + 16u * a.patch_slots + meta_bytes;
    const size_t tables = 16u * a.patch_slots + ((2u * a.k + 15u) & ~static_cast<size_t>(15));
    const size_t lds = tables + 4 * per_wave;
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    const dim3 grid(static_cast<unsigned>(blocks_x), static_cast<unsigned>(a.n_ranks),
                    static_cast<unsigned>(a.segs));
    hipError_t e = hipSuccess;
#define TPQ_CASE(PP)                                                                         \
    case PP:                                                                                 \
        if (lds > 65536)                                                                     \
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_encode_stream<LPG, PP>), \
                                    hipFuncAttributeMaxDynamicSharedMemorySize,              \
                                    static_cast<int>(lds));                                  \
        if (e == hipSuccess)                                                                 \
            k_encode_stream<LPG, PP><<<grid, 256, lds, s>>>(a, Y, codes, scale, zero, outl); \
        break;
    switch (P) {
        TPQ_CASE(1) TPQ_CASE(2) TPQ_CASE(3) TPQ_CASE(4) TPQ_CASE(5) TPQ_CASE(6)
    default: return hipErrorInvalidValue;
    }
#undef TPQ_CASE
    if (e != hipSuccess) return e;
    return hipGetLastError();
}

template <int LPG, int P>
static hipError_t launch_direct_lp(const EncodeArgs &a, const RankPtrs &Y, const RankPtrs &codes,
                                   const RankPtrs &scale, const RankPtrs &zero,
                                   const RankPtrs &outl, size_t lds, dim3 grid, hipStream_t s)
{
    hipError_t e = hipSuccess;
    if (lds > 65536)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_encode_direct<LPG, P>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return e;
    k_encode_direct<LPG, P><<<grid, 256, lds, s>>>(a, Y, codes, scale, zero, outl);
    return hipGetLastError();
}

// Direct path: one wave per (rank, row, segment).
static hipError_t launch_direct(const EncodeArgs &a_in, const RankPtrs &Y_in, const RankPtrs &codes_in,
                                const RankPtrs &scale_in, const RankPtrs &zero_in,
                                const RankPtrs &outl_in, hipStream_t s)
{
    EncodeArgs a = a_in;
    const int lpg = a.G / 8;
    const int passes = a.chunks_padded / 64;
    const int P = dir_passes_of(passes);
    a.seg_passes = P;
    a.segs = (passes + P - 1) / P;
    a.segs_magic = a.segs > 1 ? static_cast<uint32_t>((1ull << 32) / a.segs + 1) : 0u;  // unused for 1
    a.dslots = dir_slots_of(a.k, a.r);
    {
        const PlanOffsets o = plan_offsets(a.k, a.r, a.G);
        a.off_idx = o.idx;
        a.off_dirr = o.dirr;
        a.off_dsel = o.dsel;
        a.off_dpos16 = o.dpos16;
        a.off_dslot8 = o.dslot8;
        a.off_dseg = o.dseg;
        a.off_drec = o.drec;
    }
    a.patch_slots = a.dslots < 64 * P ? a.dslots : 64 * P;
    const size_t lds = 4 * (32u * static_cast<size_t>(a.patch_slots) + 4u * (64 * P / lpg));

    // task numbers of a rank stay below 2^32 / segs (the kernel divides by multiplying)
    // and the grid's x extent below 2^31: hand over the rows in blocks
    const int64_t rows_per_launch = ((1ll << 26) - 1) / a.segs;
    hipError_t e = hipSuccess;
    for (int64_t row0 = 0; row0 < a_in.T && e == hipSuccess; row0 += rows_per_launch) {
        RankPtrs Y = Y_in, codes = codes_in, scale = scale_in, zero = zero_in, outl = outl_in;
        a.T = a_in.T - row0 < rows_per_launch ? a_in.T - row0 : rows_per_launch;
        for (int i = 0; i < a.n_ranks; ++i) {
            Y.p[i] = static_cast<const uint8_t *>(Y.p[i]) + row0 * a.ldY * 2;
            codes.p[i] = static_cast<const uint8_t *>(codes.p[i]) + row0 * a.pitch_codes;
            scale.p[i] = static_cast<const uint8_t *>(scale.p[i]) + row0 * a.pitch_meta;
            zero.p[i] = static_cast<const uint8_t *>(zero.p[i]) + row0 * a.pitch_meta;
            if (outl.p[i]) outl.p[i] = static_cast<const uint8_t *>(outl.p[i]) + row0 * a.pitch_outl;
        }
        a.n_tasks = a.T * a.segs;  // per rank
        const dim3 grid(static_cast<unsigned>((a.n_tasks + 3) / 4), static_cast<unsigned>(a.n_ranks));
#define TPQ_DIRECT_P(LPG, PP) \
    case PP: e = launch_direct_lp<LPG, PP>(a, Y, codes, scale, zero, outl, lds, grid, s); break;
#define TPQ_DIRECT(LPG)                                                                      \
    switch (P) {                                                                             \
        TPQ_DIRECT_P(LPG, 1) TPQ_DIRECT_P(LPG, 2) TPQ_DIRECT_P(LPG, 3) TPQ_DIRECT_P(LPG, 4)  \
        TPQ_DIRECT_P(LPG, 5)                                                                 \
    default: return hipErrorInvalidValue;                                                    \
    }
        switch (lpg) {
        case 4: TPQ_DIRECT(4) break;
        case 8: TPQ_DIRECT(8) break;
        case 16: TPQ_DIRECT(16) break;
        case 32: TPQ_DIRECT(32) break;
        default: return hipErrorInvalidValue;
        }
#undef TPQ_DIRECT
#undef TPQ_DIRECT_P
    }
    return e;
}

int launch_encode(const EncodeArgs &a_in, const RankPtrs &Y, const RankPtrs &codes,
                  const RankPtrs &scale, const RankPtrs &zero, const RankPtrs &outl,
                  hipStream_t s)
{
    EncodeArgs a = a_in;
    const int lpg = a.G / 8;
    hipError_t e = hipSuccess;
    if (lpg != 4 && lpg != 8 && lpg != 16 && lpg != 32) return TPQ_ERR_UNSUPPORTED;

    if (a.r > 0 && a.T > 0) {
        e = launch_direct(a, Y, codes, scale, zero, outl, s);
        if (e != hipErrorInvalidValue) return hip_result(e);
        e = hipSuccess;
    }

    // Streaming path: needs at least one quantised feature, an LDS patch area (k + 1
    // slots of 16 bytes per wave) of moderate size and a shift of at most 62 chunks.
    const int slots = irr_slots_of(a.k, a.r, a.G);
    if (a.r > 0 && slots <= 1000 && (a.k + 7) / 8 + 2 <= 64) {
        a.seg_passes = pick_seg_passes(a.chunks_padded / 64, &a.segs);
        a.patch_slots = slots;
        // a segment's slice: its 64*P chunks, shifted by at most k columns, plus rounding
        {
            const int whole = a.E / 8;
            const int need = 64 * a.seg_passes + (a.k + 7) / 8 + 2;
            a.stage_chunks = need < whole ? need : whole;
        }
        a.n_tasks = a.T * a.n_ranks * a.segs;
        // persistent grid: about 16 waves per CU over the whole launch, never more
        // workgroups than there are groups of 4 rows
        const int wg_per_cu = 4;
        int64_t blocks_x = (256LL * wg_per_cu + a.n_ranks * a.segs - 1) / (a.n_ranks * a.segs);
        const int64_t row_groups = (a.T + 3) / 4;
        if (blocks_x > row_groups) blocks_x = row_groups;
        if (blocks_x < 1) blocks_x = 1;
        switch (lpg) {
        case 4: e = launch_stream_lpg<4>(a, Y, codes, scale, zero, outl, (int)blocks_x, s); break;
        case 8: e = launch_stream_lpg<8>(a, Y, codes, scale, zero, outl, (int)blocks_x, s); break;
        case 16: e = launch_stream_lpg<16>(a, Y, codes, scale, zero, outl, (int)blocks_x, s); break;
        case 32: e = launch_stream_lpg<32>(a, Y, codes, scale, zero, outl, (int)blocks_x, s); break;
        default: return TPQ_ERR_UNSUPPORTED;
        }
        return hip_result(e);
    }

    // General path: the whole row staged in LDS, any number of selected features.
    const dim3 grid(static_cast<unsigned>(a.T * a.n_ranks));
    const size_t lds = encode_row_lds(a, lpg);
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
