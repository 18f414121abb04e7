// tpq_decode_reduce kernel: dequantise the N devices' messages and add them
// (paper Sec. 2, decompression D^(i) and the sum over devices; Fig. 2 caption),
// selected features scattered back to their original columns.
#include <type_traits>

#include "tpq_device.h"
#include "tpq_internal.h"

namespace tpq {

// The 8 B-bit fields of a 64-bit word as floats: field e at bits B*e .. B*e + B - 1.
template <int B>
__device__ __forceinline__ void unpack_codes(uint64_t w, float (&c)[8])
{
#pragma unroll
    for (int e = 0; e < 8; ++e)
        c[e] = static_cast<float>(static_cast<uint32_t>(w >> (B * e)) & ((1u << B) - 1u));
}

// acc <- acc (+) x for 8 features at once, in the requested arithmetic
template <int ACC>
__device__ __forceinline__ void accumulate8(float (&acc)[8], float (&x)[8], bool first)
{
    if (ACC == TPQ_ACC_BF16) {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = round_via_bf16(x[e]);
    }
    if (first) {
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

// ---------------------------------------------------------------------------
// Stores of one pass and row.  The wave parks its 512 sums in LDS in compacted order
// (8 per lane), then lane s takes the pass's s-th store entry from the plan: a block of
// 8 consecutive features that go to 8 consecutive columns -- read back from LDS at
// whatever feature offset the block starts (two aligned 16-byte reads and a funnel
// shift), written with one 128-bit store (two for fp32 output) -- or, for the few
// features of runs shorter than 8, a single feature.  Selected columns cut the stream of
// features into runs; blocks follow the runs, so no store is split feature by feature.
// st: this wave's staging area (64 x 16 bytes for bf16 output, 128 x 16 for fp32).
// e0, e1: the entries of slots lane and 64 + lane (loaded early); further entries are
// read here.  All 64 lanes must call.
// ---------------------------------------------------------------------------
template <int OUT>
__device__ __forceinline__ void store_pass(u32x4 *st, const float (&acc)[8], uint8_t *out_row,
                                           uint32_t lane, const uint32_t *entries, uint32_t nb,
                                           uint32_t nall, uint32_t e0, uint32_t e1)
{
    if (OUT == TPQ_OUT_FP32) {
        st[2u * lane] = u32x4{__float_as_uint(acc[0]), __float_as_uint(acc[1]), __float_as_uint(acc[2]),
                              __float_as_uint(acc[3])};
        st[2u * lane + 1u] = u32x4{__float_as_uint(acc[4]), __float_as_uint(acc[5]),
                                   __float_as_uint(acc[6]), __float_as_uint(acc[7])};
    } else {
        st[lane] = u32x4{pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]),
                         pack_bf16x2(acc[4], acc[5]), pack_bf16x2(acc[6], acc[7])};
    }
    wave_lds_fence();
    for (uint32_t s0 = 0; s0 < nall; s0 += 64) {
        const uint32_t slot = s0 + lane;
        uint32_t e = s0 == 0 ? e0 : e1;
        if (s0 >= 128) e = slot < nall ? entries[slot] : 0u;
        const uint32_t col = e & 0xFFFFu, at = (e >> 16) & 0x1FFu;
        if (slot < nb) {
            if (OUT == TPQ_OUT_FP32) {
                // 8 dwords from dword `at` on: three aligned reads, shift by at % 4 dwords
                const uint32_t q = at >> 2;
                const u32x4 A = st[q], B = st[min(q + 1u, 127u)], C = st[min(q + 2u, 127u)];
                // (selects between named values: an indexed array here ends up in memory)
                const bool s2 = (at & 2u) != 0, s1 = (at & 1u) != 0;
#define TPQ_SEL(c, hi, lo) ((c) ? (hi) : (lo))
                const uint32_t u0 = TPQ_SEL(s2, A.z, A.x), u1 = TPQ_SEL(s2, A.w, A.y), u2 = TPQ_SEL(s2, B.x, A.z),
                               u3 = TPQ_SEL(s2, B.y, A.w), u4 = TPQ_SEL(s2, B.z, B.x), u5 = TPQ_SEL(s2, B.w, B.y),
                               u6 = TPQ_SEL(s2, C.x, B.z), u7 = TPQ_SEL(s2, C.y, B.w), u8 = TPQ_SEL(s2, C.z, C.x);
                const uint32_t o[8] = {TPQ_SEL(s1, u1, u0), TPQ_SEL(s1, u2, u1), TPQ_SEL(s1, u3, u2),
                                       TPQ_SEL(s1, u4, u3), TPQ_SEL(s1, u5, u4), TPQ_SEL(s1, u6, u5),
                                       TPQ_SEL(s1, u7, u6), TPQ_SEL(s1, u8, u7)};
                __builtin_nontemporal_store(u32x4{o[0], o[1], o[2], o[3]},
                                            reinterpret_cast<u32x4_a4 *>(out_row + 4u * col));
                __builtin_nontemporal_store(u32x4{o[4], o[5], o[6], o[7]},
                                            reinterpret_cast<u32x4_a4 *>(out_row + 4u * col + 16u));
            } else {
                // 8 half-words from half-word `at` on: two aligned reads, shift by at % 8
                const uint32_t q = at >> 3;
                const u32x4 A = st[q], B = st[min(q + 1u, 63u)];
                const bool s2 = (at & 4u) != 0, s1 = (at & 2u) != 0;
                const uint32_t sh = (at & 1u) << 4;
                const uint32_t u0 = TPQ_SEL(s2, A.z, A.x), u1 = TPQ_SEL(s2, A.w, A.y), u2 = TPQ_SEL(s2, B.x, A.z),
                               u3 = TPQ_SEL(s2, B.y, A.w), u4 = TPQ_SEL(s2, B.z, B.x), u5 = TPQ_SEL(s2, B.w, B.y);
                const uint32_t v0 = TPQ_SEL(s1, u1, u0), v1 = TPQ_SEL(s1, u2, u1), v2 = TPQ_SEL(s1, u3, u2),
                               v3 = TPQ_SEL(s1, u4, u3), v4 = TPQ_SEL(s1, u5, u4);
#undef TPQ_SEL
                const uint32_t o[4] = {__builtin_amdgcn_alignbit(v1, v0, sh), __builtin_amdgcn_alignbit(v2, v1, sh),
                                       __builtin_amdgcn_alignbit(v3, v2, sh), __builtin_amdgcn_alignbit(v4, v3, sh)};
                __builtin_nontemporal_store(u32x4{o[0], o[1], o[2], o[3]},
                                            reinterpret_cast<u32x4_a2 *>(out_row + 2u * col));
            }
        } else if (slot < nall) {
            const uint32_t *stw = reinterpret_cast<const uint32_t *>(st);
            if (OUT == TPQ_OUT_FP32) {
                *reinterpret_cast<uint32_t *>(out_row + 4u * col) = stw[at];
            } else {
                const uint32_t w = stw[at >> 1];
                *reinterpret_cast<uint16_t *>(out_row + 2u * col) =
                    static_cast<uint16_t>((at & 1u) ? (w >> 16) : (w & 0xFFFFu));
            }
        }
    }
    // A later call's staging writes follow these reads in program order, and a wave's LDS
    // operations execute in order: nothing to wait for (a fence here would also hold the
    // wave until its global stores have completed).
    __builtin_amdgcn_wave_barrier();
}

// one more term of the accumulation (fp32 add; rounded to bf16 in the literal bf16 chain)
template <int ACC>
__device__ __forceinline__ float add_term(float acc, float x)
{
    const float s = acc + x;
    return ACC == TPQ_ACC_BF16 ? round_via_bf16(s) : s;
}

// ---------------------------------------------------------------------------
// store_pass with the block's epilogue (Sec. 2: the sum over the devices plus the bias):
// the sums are parked as fp32 whatever the output type, and every block adds the addend
// row's and the bias's 8 columns (one 2-byte-aligned 128-bit load each) as two more terms
// of the accumulation before it is rounded and stored.  addend_row / bias may be null.
// st: 128 x 16 bytes per wave.
// ---------------------------------------------------------------------------
template <int OUT, int ACC>
__device__ __forceinline__ void store_pass_fused(u32x4 *st, const float (&acc)[8], uint8_t *out_row,
                                                 uint32_t lane, const uint32_t *entries, uint32_t nb,
                                                 uint32_t nall, uint32_t e0, uint32_t e1,
                                                 const uint8_t *addend_row, const uint8_t *bias)
{
    st[2u * lane] = u32x4{__float_as_uint(acc[0]), __float_as_uint(acc[1]), __float_as_uint(acc[2]),
                          __float_as_uint(acc[3])};
    st[2u * lane + 1u] = u32x4{__float_as_uint(acc[4]), __float_as_uint(acc[5]), __float_as_uint(acc[6]),
                               __float_as_uint(acc[7])};
    wave_lds_fence();
    for (uint32_t s0 = 0; s0 < nall; s0 += 64) {
        const uint32_t slot = s0 + lane;
        uint32_t e = s0 == 0 ? e0 : e1;
        if (s0 >= 128) e = slot < nall ? entries[slot] : 0u;
        const uint32_t col = e & 0xFFFFu, at = (e >> 16) & 0x1FFu;
        if (slot < nb) {
            const uint32_t q = at >> 2;
            const u32x4 A = st[q], B = st[min(q + 1u, 127u)], C = st[min(q + 2u, 127u)];
            const bool s2 = (at & 2u) != 0, s1 = (at & 1u) != 0;
#define TPQ_SEL(c, hi, lo) ((c) ? (hi) : (lo))
            const uint32_t u0 = TPQ_SEL(s2, A.z, A.x), u1 = TPQ_SEL(s2, A.w, A.y), u2 = TPQ_SEL(s2, B.x, A.z),
                           u3 = TPQ_SEL(s2, B.y, A.w), u4 = TPQ_SEL(s2, B.z, B.x), u5 = TPQ_SEL(s2, B.w, B.y),
                           u6 = TPQ_SEL(s2, C.x, B.z), u7 = TPQ_SEL(s2, C.y, B.w), u8 = TPQ_SEL(s2, C.z, C.x);
            float f0 = __uint_as_float(TPQ_SEL(s1, u1, u0)), f1 = __uint_as_float(TPQ_SEL(s1, u2, u1)),
                  f2 = __uint_as_float(TPQ_SEL(s1, u3, u2)), f3 = __uint_as_float(TPQ_SEL(s1, u4, u3)),
                  f4 = __uint_as_float(TPQ_SEL(s1, u5, u4)), f5 = __uint_as_float(TPQ_SEL(s1, u6, u5)),
                  f6 = __uint_as_float(TPQ_SEL(s1, u7, u6)), f7 = __uint_as_float(TPQ_SEL(s1, u8, u7));
#undef TPQ_SEL
#define TPQ_ADD8(src)                                                                       \
    {                                                                                       \
        const u32x4 t8 = *reinterpret_cast<const u32x4_a2 *>((src) + 2u * col);             \
        f0 = add_term<ACC>(f0, bf16_lo_to_f32(t8.x)); f1 = add_term<ACC>(f1, bf16_hi_to_f32(t8.x)); \
        f2 = add_term<ACC>(f2, bf16_lo_to_f32(t8.y)); f3 = add_term<ACC>(f3, bf16_hi_to_f32(t8.y)); \
        f4 = add_term<ACC>(f4, bf16_lo_to_f32(t8.z)); f5 = add_term<ACC>(f5, bf16_hi_to_f32(t8.z)); \
        f6 = add_term<ACC>(f6, bf16_lo_to_f32(t8.w)); f7 = add_term<ACC>(f7, bf16_hi_to_f32(t8.w)); \
    }
            if (addend_row) TPQ_ADD8(addend_row)
            if (bias) TPQ_ADD8(bias)
#undef TPQ_ADD8
            if (OUT == TPQ_OUT_FP32) {
                __builtin_nontemporal_store(
                    u32x4{__float_as_uint(f0), __float_as_uint(f1), __float_as_uint(f2), __float_as_uint(f3)},
                    reinterpret_cast<u32x4_a4 *>(out_row + 4u * col));
                __builtin_nontemporal_store(
                    u32x4{__float_as_uint(f4), __float_as_uint(f5), __float_as_uint(f6), __float_as_uint(f7)},
                    reinterpret_cast<u32x4_a4 *>(out_row + 4u * col + 16u));
            } else {
                __builtin_nontemporal_store(u32x4{pack_bf16x2(f0, f1), pack_bf16x2(f2, f3), pack_bf16x2(f4, f5),
                                                  pack_bf16x2(f6, f7)},
                                            reinterpret_cast<u32x4_a2 *>(out_row + 2u * col));
            }
        } else if (slot < nall) {
            float f = __uint_as_float(reinterpret_cast<const uint32_t *>(st)[at]);
            if (addend_row)
                f = add_term<ACC>(f, bf16_bits_to_f32(*reinterpret_cast<const uint16_t *>(addend_row + 2u * col)));
            if (bias) f = add_term<ACC>(f, bf16_bits_to_f32(*reinterpret_cast<const uint16_t *>(bias + 2u * col)));
            if (OUT == TPQ_OUT_FP32)
                *reinterpret_cast<float *>(out_row + 4u * col) = f;
            else
                *reinterpret_cast<uint16_t *>(out_row + 2u * col) = static_cast<uint16_t>(pack_bf16x2(f, f));
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// ---------------------------------------------------------------------------
// One wavefront handles one pass (64 chunks = 512 compacted features) of one output
// row, or up to 64 of the row's selected features; waves are independent (no barrier;
// LDS only as each wave's private staging area for its stores), so a CU always holds
// waves in every phase and loads, arithmetic and stores overlap.
//
// Pass wave: every lane issues all its loads at once -- the pass's store entries, one
// 32-bit word of codes (8 features) per rank, the group's scale and zero per rank --
// then dequantises (code * scale + zero: one FMA, the product is exact) and
// accumulates in ascending rank order.  The sums leave through store_pass(): blocks
// of 8 consecutive columns, one 128-bit store each (2-byte aligned: removing the
// selected columns shifted the compacted stream; neighbouring lanes' stores are
// contiguous, so lines are written whole).
// Outlier wave: lane p adds the ranks' bf16 values of outlier p and stores the sum at
// its column.
// grid: (row, group of 4 waves) pairs, rounded up to a multiple of 8.
// ---------------------------------------------------------------------------
//
// GEN selects code widths other than 4 bits (Sec. 4, the experiment that varies the bits
// of the quantised features): a chunk's 8 codes are b bytes at byte chunk * b of the row,
// fetched with one 64-bit load at that byte (the row's pitch leaves room behind the last).
//
// FUSED adds the block's epilogue (an addend row and / or the bias, see store_pass_fused).
template <int LPG, int ACC, int OUT, bool GEN, bool FUSED>
__global__ __launch_bounds__(256) void k_decode_pass(DecodeArgs a, RankPtrs codesp, RankPtrs scalep,
                                                     RankPtrs zerop, RankPtrs outlp)
{
    // Nothing is stored unless the header says that the plan is good; the pass waves'
    // loads do not wait for that answer (the message sections do not depend on the plan,
    // and reads of the plan's tables are kept inside the plan buffer whatever it holds).
    const bool bad = plan_header_bad(a.plan, a.E, a.k, a.G);
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t passes = static_cast<uint32_t>(a.chunks_padded) >> 6;
    // Each XCD works through one contiguous range of (row, wave group) pairs, a row's
    // groups one after the other: the lines two neighbouring waves share (a row's scales
    // and zeros, the ends of their code ranges, the output lines at a pass boundary)
    // then meet in one L2, close in time.
    const uint32_t ny = (passes + ((static_cast<uint32_t>(a.k) + 63u) >> 6) + 3u) >> 2;
    const uint32_t logical = xcd_contiguous_index(blockIdx.x, gridDim.x);
    const uint32_t t = logical / ny;
    if (t >= static_cast<uint32_t>(a.T)) return;  // (the grid is rounded up to 8 blocks)
    const uint32_t task = (logical - t * ny) * 4u + wave;

    constexpr uint32_t OB = OUT == TPQ_OUT_FP32 ? 4u : 2u;  // bytes per output value
    const uint32_t N = static_cast<uint32_t>(a.n_ranks);
    const uint32_t ng = static_cast<uint32_t>(a.ng);
    const uint32_t chunks = static_cast<uint32_t>(a.chunks);
    uint8_t *const out_row = static_cast<uint8_t *>(a.out) + static_cast<int64_t>(t) * a.ldOut * OB;

    if (task >= passes) {
        // ---- selected features ------------------------------------------------------
        const uint32_t p = (task - passes) * 64u + lane;
        if (bad || p >= static_cast<uint32_t>(a.k)) return;
        const int32_t *idx = reinterpret_cast<const int32_t *>(a.plan + a.off_idx);
        const uint32_t off_outl = t * static_cast<uint32_t>(a.pitch_outl);
        const uint32_t j = static_cast<uint32_t>(idx[p]);
        float acc = 0.f;
        for (uint32_t i0 = 0; i0 < N; i0 += 8) {
            uint32_t v[8];
#pragma unroll
            for (int jj = 0; jj < 8; ++jj)
                v[jj] = reinterpret_cast<const uint16_t *>(
                    static_cast<const uint8_t *>(outlp.p[min(i0 + jj, N - 1u)]) + off_outl)[p];
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                if (i0 + jj < N) {
                    const float x = bf16_bits_to_f32(v[jj]);
                    if (i0 + jj == 0) {
                        acc = x;
                    } else {
                        acc = acc + x;
                        if (ACC == TPQ_ACC_BF16) acc = round_via_bf16(acc);
                    }
                }
            }
        }
        if constexpr (FUSED) {
            if (a.addend)
                acc = add_term<ACC>(acc, bf16_bits_to_f32(reinterpret_cast<const uint16_t *>(
                                             a.addend + static_cast<int64_t>(t) * a.ldAdd * 2)[j]));
            if (a.bias) acc = add_term<ACC>(acc, bf16_bits_to_f32(reinterpret_cast<const uint16_t *>(a.bias)[j]));
        }
        if (OUT == TPQ_OUT_FP32)
            *reinterpret_cast<float *>(out_row + 4u * j) = acc;
        else
            *reinterpret_cast<uint16_t *>(out_row + 2u * j) = static_cast<uint16_t>(pack_bf16x2(acc, acc));
        return;
    }

    // ---- one pass of quantised features ---------------------------------------------
    const uint32_t chunk = task * 64u + lane;
    const uint32_t g = min(chunk / LPG, ng - 1u);
    // the pass's store entries: where they start, blocks, blocks + narrow entries
    const uint4 sp = reinterpret_cast<const uint4 *>(a.plan + a.off_spass)[task];
    const uint32_t first = min(sp.x, static_cast<uint32_t>(a.sblk_cap));
    const uint32_t *entries = reinterpret_cast<const uint32_t *>(a.plan + a.off_sblk) + first;
    const uint32_t nall = min(sp.y + sp.z, static_cast<uint32_t>(a.sblk_cap) - first), nb = min(sp.y, nall);
    const uint32_t e0 = lane < nall ? entries[lane] : 0u;
    const uint32_t e1 = 64u + lane < nall ? entries[64u + lane] : 0u;
    // One 32-bit byte offset per section serves every rank (the host keeps
    // T * pitch below 2^31 per launch): the rank only changes the scalar base.
    const uint32_t off_codes = t * static_cast<uint32_t>(a.pitch_codes) +
                               (GEN ? static_cast<uint32_t>(a.bits) : 4u) * min(chunk, chunks - 1u);
    const uint32_t off_meta = t * static_cast<uint32_t>(a.pitch_meta) + 2u * g;
    float acc[8];

    // 8 ranks at a time: all 24 loads first, then the arithmetic.  FULL batches index
    // the pointer tables with constants (one wide scalar load each); the last, partial
    // batch guards every rank.
    // (the code width is a compile-time constant inside: one copy of the loop per width)
    auto batch = [&](uint32_t i0, auto full_tag, auto bits_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        constexpr int BITS = decltype(bits_tag)::value;
        uint32_t w[8], sb[8], zb[8];
        uint64_t wq[8];  // GEN
        const void *const *pc = codesp.p + i0;
        const void *const *ps = scalep.p + i0;
        const void *const *pz = zerop.p + i0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t i = FULL ? static_cast<uint32_t>(j) : min(static_cast<uint32_t>(j), N - 1u - i0);
            if constexpr (GEN)
                wq[j] = __builtin_nontemporal_load(reinterpret_cast<const u64_a1 *>(
                    static_cast<const uint8_t *>(pc[i]) + off_codes));
            else
                w[j] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(
                    static_cast<const uint8_t *>(pc[i]) + off_codes));
            sb[j] = *reinterpret_cast<const uint16_t *>(static_cast<const uint8_t *>(ps[i]) + off_meta);
            zb[j] = *reinterpret_cast<const uint16_t *>(static_cast<const uint8_t *>(pz[i]) + off_meta);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (FULL || i0 + j < N) {  // uniform
                const float sc = bf16_bits_to_f32(sb[j]), ze = bf16_bits_to_f32(zb[j]);
                // one code per byte, so that each converts with a single byte-to-float
                // instruction (the masks are hidden from the optimiser, which would
                // otherwise fold them into separate bit-field extracts)
                float x[8];
                if constexpr (GEN) {
                    float c[8];
                    unpack_codes<BITS>(wq[j], c);
#pragma unroll
                    for (int e = 0; e < 8; ++e) x[e] = __builtin_fmaf(c[e], sc, ze);  // product exact
                } else {
                    // one code per byte; the bytes 0 .. 15 read as FP8 (E4M3) are the codes
                    // times 2^-9 (subnormals and the first binade have the same spacing), so
                    // the scaled pair conversion turns two codes into floats at once
                    const uint32_t lo = w[j] & 0x0F0F0F0Fu, hi = (w[j] >> 4) & 0x0F0F0F0Fu;
                    const f32x2 c02 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(lo, 512.0f, false);
                    const f32x2 c46 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(lo, 512.0f, true);
                    const f32x2 c13 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(hi, 512.0f, false);
                    const f32x2 c57 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(hi, 512.0f, true);
                    x[0] = __builtin_fmaf(c02.x, sc, ze); x[1] = __builtin_fmaf(c13.x, sc, ze);
                    x[2] = __builtin_fmaf(c02.y, sc, ze); x[3] = __builtin_fmaf(c13.y, sc, ze);
                    x[4] = __builtin_fmaf(c46.x, sc, ze); x[5] = __builtin_fmaf(c57.x, sc, ze);
                    x[6] = __builtin_fmaf(c46.y, sc, ze); x[7] = __builtin_fmaf(c57.y, sc, ze);
                }
                accumulate8<ACC>(acc, x, i0 + j == 0);
            }
        }
    };
    auto run = [&](auto bits_tag) {
        uint32_t i0 = 0;
        for (; i0 + 8 <= N; i0 += 8) batch(i0, std::true_type{}, bits_tag);
        if (i0 < N) batch(i0, std::false_type{}, bits_tag);
    };
    if constexpr (GEN) {
        switch (a.bits) {
        case 2: run(std::integral_constant<int, 2>{}); break;
        case 3: run(std::integral_constant<int, 3>{}); break;
        case 5: run(std::integral_constant<int, 5>{}); break;
        case 6: run(std::integral_constant<int, 6>{}); break;
        default: run(std::integral_constant<int, 8>{}); break;
        }
    } else {
        run(std::integral_constant<int, 4>{});
    }
    if (bad) return;
    if constexpr (FUSED) {
        __shared__ u32x4 stage_f[4 * 128];
        store_pass_fused<OUT, ACC>(stage_f + wave * 128u, acc, out_row, lane, entries, nb, nall, e0, e1,
                                   a.addend ? a.addend + static_cast<int64_t>(t) * a.ldAdd * 2 : nullptr, a.bias);
    } else {
        __shared__ u32x4 stage[4 * 64 * (OUT == TPQ_OUT_FP32 ? 2 : 1)];
        store_pass<OUT>(stage + wave * (64u * (OUT == TPQ_OUT_FP32 ? 2u : 1u)), acc, out_row, lane, entries,
                        nb, nall, e0, e1);
    }
}

// ---------------------------------------------------------------------------
// Static symmetric mode (Sec. 3): no scale / zero sections; a feature's value is
// (nibble - 8) * step, the steps of (device, feature) read from a table in compacted
// order (8 per chunk and device: two 128-bit loads that the L2 serves).  Same wave
// roles, loads, accumulation order and stores as k_decode_pass, but a wave takes R
// consecutive rows: the rows share the step loads, which otherwise outnumber the code
// loads two to one.  Rows past the end are read as the last row and not stored.
// grid: (block of R rows, group of 4 waves) pairs, rounded up to a multiple of 8.
// ---------------------------------------------------------------------------
template <int ACC, int OUT, int R, bool GEN>
__global__ __launch_bounds__(256) void k_decode_static(DecodeArgs a, RankPtrs codesp, RankPtrs outlp)
{
    const bool bad = plan_header_bad(a.plan, a.E, a.k, a.G);  // checked before any store
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t passes = static_cast<uint32_t>(a.chunks_padded) >> 6;
    // (row block, wave group) pairs over the XCDs as in k_decode_pass
    const uint32_t ny = (passes + ((static_cast<uint32_t>(a.k) + 63u) >> 6) + 3u) >> 2;
    const uint32_t logical = xcd_contiguous_index(blockIdx.x, gridDim.x);
    const uint32_t rb = logical / ny;
    if (rb * static_cast<uint32_t>(R) >= static_cast<uint32_t>(a.T)) return;  // (grid rounded up to 8)
    const uint32_t task = (logical - rb * ny) * 4u + wave;

    constexpr uint32_t OB = OUT == TPQ_OUT_FP32 ? 4u : 2u;  // bytes per output value
    const uint32_t N = static_cast<uint32_t>(a.n_ranks);
    const uint32_t chunks = static_cast<uint32_t>(a.chunks);
    // the wave's rows; rows past the end are read as the last row and not stored
    const uint32_t t0 = rb * static_cast<uint32_t>(R);
    const uint32_t n_rows = min(static_cast<uint32_t>(R), static_cast<uint32_t>(a.T) - t0);
    uint32_t tr[R];
    uint8_t *out_row[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        tr[rr] = t0 + min(static_cast<uint32_t>(rr), n_rows - 1u);
        out_row[rr] = static_cast<uint8_t *>(a.out) + static_cast<int64_t>(tr[rr]) * a.ldOut * OB;
    }

    if (task >= passes) {
        // ---- selected features ------------------------------------------------------
        const uint32_t p = (task - passes) * 64u + lane;
        if (bad || p >= static_cast<uint32_t>(a.k)) return;
        const int32_t *idx = reinterpret_cast<const int32_t *>(a.plan + a.off_idx);
        const uint32_t j = static_cast<uint32_t>(idx[p]);
        float acc[R];
#pragma unroll
        for (int rr = 0; rr < R; ++rr) acc[rr] = 0.f;
        for (uint32_t i0 = 0; i0 < N; i0 += 8) {
            uint32_t v[R][8];
#pragma unroll
            for (int rr = 0; rr < R; ++rr)
#pragma unroll
                for (int jj = 0; jj < 8; ++jj)
                    v[rr][jj] = reinterpret_cast<const uint16_t *>(
                        static_cast<const uint8_t *>(outlp.p[min(i0 + jj, N - 1u)]) +
                        tr[rr] * static_cast<uint32_t>(a.pitch_outl))[p];
#pragma unroll
            for (int rr = 0; rr < R; ++rr)
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) {
                    if (i0 + jj < N) {
                        const float x = bf16_bits_to_f32(v[rr][jj]);
                        if (i0 + jj == 0) {
                            acc[rr] = x;
                        } else {
                            acc[rr] = acc[rr] + x;
                            if (ACC == TPQ_ACC_BF16) acc[rr] = round_via_bf16(acc[rr]);
                        }
                    }
                }
        }
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            if (static_cast<uint32_t>(rr) < n_rows) {
                if (OUT == TPQ_OUT_FP32)
                    *reinterpret_cast<float *>(out_row[rr] + 4u * j) = acc[rr];
                else
                    *reinterpret_cast<uint16_t *>(out_row[rr] + 2u * j) =
                        static_cast<uint16_t>(pack_bf16x2(acc[rr], acc[rr]));
            }
        }
        return;
    }

    // ---- one pass of quantised features ---------------------------------------------
    const uint32_t chunk = task * 64u + lane;
    // the pass's store entries: where they start, blocks, blocks + narrow entries
    const uint4 sp = reinterpret_cast<const uint4 *>(a.plan + a.off_spass)[task];
    const uint32_t first = min(sp.x, static_cast<uint32_t>(a.sblk_cap));
    const uint32_t *entries = reinterpret_cast<const uint32_t *>(a.plan + a.off_sblk) + first;
    const uint32_t nall = min(sp.y + sp.z, static_cast<uint32_t>(a.sblk_cap) - first), nb = min(sp.y, nall);
    const uint32_t e0 = lane < nall ? entries[lane] : 0u;
    const uint32_t e1 = 64u + lane < nall ? entries[64u + lane] : 0u;
    // One 32-bit byte offset per section and row serves every rank (the host keeps
    // T * pitch below 2^31 per launch): the rank only changes the scalar base.
    uint32_t off_codes[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr)
        off_codes[rr] = tr[rr] * static_cast<uint32_t>(a.pitch_codes) +
                        (GEN ? static_cast<uint32_t>(a.bits) : 4u) * min(chunk, chunks - 1u);
    float acc[R][8];

    // static mode, 4 ranks at a time: a code word per row and 8 steps each
    auto batch_static = [&](uint32_t i0, auto full_tag, auto bits_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        constexpr int BITS = decltype(bits_tag)::value;  // (one copy of the loop per width)
        uint32_t w[R][4];
        uint64_t wq[R][4];  // GEN
        float4 sa[4], sb[4];
        const void *const *pc = codesp.p + i0;
        const float *tab = a.step_c + 8u * chunk;  // chunk < chunks_padded: inside the row
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t i = FULL ? static_cast<uint32_t>(j) : min(static_cast<uint32_t>(j), N - 1u - i0);
#pragma unroll
            for (int rr = 0; rr < R; ++rr)
                if constexpr (GEN)
                    wq[rr][j] = __builtin_nontemporal_load(reinterpret_cast<const u64_a1 *>(
                        static_cast<const uint8_t *>(pc[i]) + off_codes[rr]));
                else
                    w[rr][j] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(
                        static_cast<const uint8_t *>(pc[i]) + off_codes[rr]));
            const float *row = tab + static_cast<int64_t>(i0 + i) * a.static_stride;
            sa[j] = *reinterpret_cast<const float4 *>(row);
            sb[j] = *reinterpret_cast<const float4 *>(row + 4);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (FULL || i0 + j < N) {  // uniform
                const float st[8] = {sa[j].x, sa[j].y, sa[j].z, sa[j].w, sb[j].x, sb[j].y, sb[j].z, sb[j].w};
                // (field - 8) * step as one fused multiply-add per value: -8 * step is exact, so
                // field * step - 8 * step is rounded once, from the same exact product; shared
                // by the wave's rows
                float m8[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) m8[e] = -8.0f * st[e];
#pragma unroll
                for (int rr = 0; rr < R; ++rr) {
                    float x[8];
                    if constexpr (GEN) {
                        float c[8];
                        unpack_codes<BITS>(wq[rr][j], c);
                        constexpr float half = static_cast<float>(1u << (BITS - 1));
#pragma unroll
                        for (int e = 0; e < 8; ++e) x[e] = (c[e] - half) * st[e];
                    } else {
                        // fields to floats two at a time (FP8 pair conversion, as in k_decode_pass)
                        const uint32_t lo = w[rr][j] & 0x0F0F0F0Fu, hi = (w[rr][j] >> 4) & 0x0F0F0F0Fu;
                        const f32x2 c02 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(lo, 512.0f, false);
                        const f32x2 c46 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(lo, 512.0f, true);
                        const f32x2 c13 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(hi, 512.0f, false);
                        const f32x2 c57 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(hi, 512.0f, true);
                        x[0] = __builtin_fmaf(c02.x, st[0], m8[0]); x[1] = __builtin_fmaf(c13.x, st[1], m8[1]);
                        x[2] = __builtin_fmaf(c02.y, st[2], m8[2]); x[3] = __builtin_fmaf(c13.y, st[3], m8[3]);
                        x[4] = __builtin_fmaf(c46.x, st[4], m8[4]); x[5] = __builtin_fmaf(c57.x, st[5], m8[5]);
                        x[6] = __builtin_fmaf(c46.y, st[6], m8[6]); x[7] = __builtin_fmaf(c57.y, st[7], m8[7]);
                    }
                    accumulate8<ACC>(acc[rr], x, i0 + j == 0);
                }
            }
        }
    };
    auto run = [&](auto bits_tag) {
        uint32_t i0 = 0;
        for (; i0 + 4 <= N; i0 += 4) batch_static(i0, std::true_type{}, bits_tag);
        if (i0 < N) batch_static(i0, std::false_type{}, bits_tag);
    };
    if constexpr (GEN) {
        switch (a.bits) {
        case 2: run(std::integral_constant<int, 2>{}); break;
        case 3: run(std::integral_constant<int, 3>{}); break;
        case 5: run(std::integral_constant<int, 5>{}); break;
        case 6: run(std::integral_constant<int, 6>{}); break;
        default: run(std::integral_constant<int, 8>{}); break;
        }
    } else {
        run(std::integral_constant<int, 4>{});
    }
    if (bad) return;
    __shared__ u32x4 stage[4 * 64 * (OUT == TPQ_OUT_FP32 ? 2 : 1)];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        if (static_cast<uint32_t>(rr) >= n_rows) break;  // uniform
        store_pass<OUT>(stage + wave * (64u * (OUT == TPQ_OUT_FP32 ? 2u : 1u)), acc[rr], out_row[rr], lane,
                        entries, nb, nall, e0, e1);
    }
}

#ifndef TPQ_STATIC_RPW
#define TPQ_STATIC_RPW 4
#endif
// Rows per wave.  Static mode: 4 once the launch fills the machine (the rows share the
// step table's loads); dynamic mode: 1 (measured: more rows per wave gain nothing there).
static int rows_per_wave(bool is_static, int64_t T, int tasks)
{
    return (is_static && T * tasks >= 2 * 8192) ? TPQ_STATIC_RPW : 1;
}

template <int LPG, int ACC, int OUT>
static void launch_rows(int rpw, dim3 grid, hipStream_t s, const DecodeArgs &a, const RankPtrs &codes,
                        const RankPtrs &scale, const RankPtrs &zero, const RankPtrs &outl)
{
    if constexpr (LPG == 0) {
        if (a.bits != 4) {
            if (rpw == 4)
                launch_kernel(k_decode_static<ACC, OUT, 4, true>, grid, dim3(256), 0, s, a, codes, outl);
            else
                launch_kernel(k_decode_static<ACC, OUT, 1, true>, grid, dim3(256), 0, s, a, codes, outl);
        } else if (rpw == 4) {
            launch_kernel(k_decode_static<ACC, OUT, 4, false>, grid, dim3(256), 0, s, a, codes, outl);
        } else {
            launch_kernel(k_decode_static<ACC, OUT, 1, false>, grid, dim3(256), 0, s, a, codes, outl);
        }
    } else {
        if (a.addend || a.bias)  // (4 bits only: the host refuses the epilogue at other widths)
            launch_kernel(k_decode_pass<LPG, ACC, OUT, false, true>, grid, dim3(256), 0, s, a, codes, scale, zero, outl);
        else if (a.bits != 4)
            launch_kernel(k_decode_pass<LPG, ACC, OUT, true, false>, grid, dim3(256), 0, s, a, codes, scale, zero, outl);
        else
            launch_kernel(k_decode_pass<LPG, ACC, OUT, false, false>, grid, dim3(256), 0, s, a, codes, scale, zero, outl);
    }
}

int launch_decode(const DecodeArgs &a_in, const RankPtrs &codes_in, const RankPtrs &scale_in,
                  const RankPtrs &zero_in, const RankPtrs &outl_in, int accum, int out_dtype,
                  hipStream_t s)
{
    // TPQ_ACC_FAST is evaluated as the fp32 chain (one final rounding), which is within its tolerance
    if (accum == TPQ_ACC_FAST) accum = TPQ_ACC_FP32;
    const int lpg = a_in.G / 8;
    const int tasks = a_in.chunks_padded / 64 + (a_in.k + 63) / 64;  // waves per row
    if (tasks == 0) return TPQ_OK;
    // The kernel addresses a rank's sections with 32-bit byte offsets: rows are handed
    // over in blocks whose sections stay below 2 GiB (one block unless T is huge).
    int64_t max_pitch = a_in.pitch_codes;
    if (a_in.pitch_meta > max_pitch) max_pitch = a_in.pitch_meta;
    if (a_in.pitch_outl > max_pitch) max_pitch = a_in.pitch_outl;
    int64_t rows_per_launch = max_pitch > 0 ? (0x7FFFFFFFLL / max_pitch) : a_in.T;
    if (rows_per_launch > 0x7FFFFFFFLL) rows_per_launch = 0x7FFFFFFFLL;
    if (rows_per_launch < 1) return TPQ_ERR_SHAPE;
    const int64_t ny = (tasks + 3) / 4;  // groups of 4 waves per row
    // one-dimensional grid of 256-thread workgroups: grid * block stays below 2^32
    const int64_t max_blocks = (1LL << 24) - 8;
    if (rows_per_launch > max_blocks / ny) rows_per_launch = max_blocks / ny;
    if (rows_per_launch < 1) return TPQ_ERR_SHAPE;
    const size_t ob = out_dtype == TPQ_OUT_FP32 ? 4 : 2;
    hipError_t e = hipSuccess;
    for (int64_t row0 = 0; row0 < a_in.T && e == hipSuccess; row0 += rows_per_launch) {
        DecodeArgs a = a_in;
        {
            const PlanOffsets o = plan_offsets(a.k, a.r, a.G);
            a.off_idx = o.idx;
            a.off_spass = o.spass;
            a.off_sblk = o.sblk;
            a.sblk_cap = sblk_cap_of(a.k, a.r);
        }
        RankPtrs codes = codes_in, scale = scale_in, zero = zero_in, outl = outl_in;
        a.T = a_in.T - row0 < rows_per_launch ? a_in.T - row0 : rows_per_launch;
        a.out = static_cast<uint8_t *>(a_in.out) + row0 * a_in.ldOut * ob;
        if (a_in.addend) a.addend = a_in.addend + row0 * a_in.ldAdd * 2;
        for (int i = 0; i < a_in.n_ranks; ++i) {
            if (codes.p[i]) codes.p[i] = static_cast<const uint8_t *>(codes.p[i]) + row0 * a_in.pitch_codes;
            if (scale.p[i]) scale.p[i] = static_cast<const uint8_t *>(scale.p[i]) + row0 * a_in.pitch_meta;
            if (zero.p[i]) zero.p[i] = static_cast<const uint8_t *>(zero.p[i]) + row0 * a_in.pitch_meta;
            if (outl.p[i]) outl.p[i] = static_cast<const uint8_t *>(outl.p[i]) + row0 * a_in.pitch_outl;
        }
        const int rpw = rows_per_wave(a.step_c != nullptr, a.T, tasks);
        // one dimension: (row block, wave group) pairs, dealt out over the XCDs by the kernel
        const dim3 grid(static_cast<unsigned>(((a.T + rpw - 1) / rpw * ny + 7) / 8 * 8));
#define TPQ_LAUNCH3(LPG, ACC, OUT) launch_rows<LPG, ACC, OUT>(rpw, grid, s, a, codes, scale, zero, outl)
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
        switch (a.step_c ? 0 : lpg) {
        case 0: TPQ_LAUNCH2(0); break;  // static symmetric mode
        case 4: TPQ_LAUNCH2(4); break;
        case 8: TPQ_LAUNCH2(8); break;
        case 16: TPQ_LAUNCH2(16); break;
        case 32: TPQ_LAUNCH2(32); break;
        default: return TPQ_ERR_UNSUPPORTED;
        }
#undef TPQ_LAUNCH2
#undef TPQ_LAUNCH3
        e = hipGetLastError();
    }
    return hip_result(e);
}

}  // namespace tpq
