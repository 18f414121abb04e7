// The row-parallel linear layer with the compression in its epilogue (paper Sec. 2: device i
// computes f^(i)(x^(i)) = x^(i) W^(i) and sends C^(i) of it; Sec. 3, "Selecting High Precision
// Features": the selection before the exchange is the method's overhead).  The partial sums
// never reach memory: a workgroup's tile of the product is rounded to bf16 in registers,
// and group statistics, codes and the bf16 features go straight to the message.
//
// What makes that possible without a gather: the selected features are static (Sec. 3), and so
// are the weights, so the weight rows are reordered once, offline, into message order -- the
// r features that are quantised, ascending, then the k that stay bf16 (k_gemm_weights).  The
// product then comes out compacted: output feature n < r is compacted feature n, its group is
// n / G, and the tail n >= r is the outlier section.
//
// The product itself is a dense contraction: bf16 MFMA 32x32x16, fp32 accumulators.  The
// operands are "k-contiguous" on both sides (X [T][K], Wp [E][K]), the weights are the MFMA's
// row operand and the tokens its column operand, so that a lane's 16 accumulators of a 32x32
// block are 16 features of ONE token: the per-token statistics stay inside a lane (and its
// partner 32 lanes on), and the nibbles of a chunk sit in at most two lanes.
#include "tpq_device.h"
#include "tpq_internal.h"

namespace tpq {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kGemmTF = 256;   // features per workgroup tile (2 waves of 128)
constexpr int kGemmTT = 128;   // tokens per workgroup tile (2 waves of 64)
constexpr int kGemmBK = 32;    // k per stage
constexpr int kGemmRow = 80;   // LDS bytes per operand row of a stage: 64 of data, 16 of padding
                               // (16 consecutive rows then start in 16 different 16-byte bank groups)
constexpr int kGemmStage = (kGemmTF + kGemmTT) * kGemmRow;

// Rows of Wt ([E][ldW], one row per output feature) -> Wp [E][K] in message order.
__global__ __launch_bounds__(256) void k_gemm_weights(const uint8_t *plan, int E, int k, int G, int r,
                                                      int off_idx, int off_src, const uint16_t *Wt,
                                                      int64_t ldW, int K, uint16_t *Wp)
{
    if (plan_header_bad(plan, E, k, G)) return;
    const int n = blockIdx.x;
    const int col = n < r ? reinterpret_cast<const uint16_t *>(plan + off_src)[n]
                          : reinterpret_cast<const int32_t *>(plan + off_idx)[n - r];
    const u32x4 *src = reinterpret_cast<const u32x4 *>(Wt + static_cast<int64_t>(col) * ldW);
    u32x4 *dst = reinterpret_cast<u32x4 *>(Wp + static_cast<int64_t>(n) * K);
    for (int p = threadIdx.x; p < K / 8; p += 256) dst[p] = src[p];
}

struct GemmArgs {
    const uint16_t *X;
    int64_t ldX, T;
    const uint16_t *Wp;
    int32_t K, E, k, G, r, ng, chunks;
    uint8_t *codes, *scale, *zero, *outl;
    int64_t pitch_codes, pitch_meta, pitch_outl;
    uint16_t *Ymsg;  // optional: the rounded product itself, [T][ldYm] in message order
    int64_t ldYm;
};

// One (token block of 32) of a wave's accumulators -> message.  y[fb][v]: feature
// F0 + 32 fb + 8 (v / 4) + 4 h + v % 4 of token t, h = lane / 32.  RAGGED: the wave's 128
// features are not all quantised ones (the row's last groups, the outlier section, the
// padding past E); otherwise nothing needs a mask.
template <int G, bool RAGGED>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &a, float (&y)[4][16], uint32_t F0, int64_t t,
                                              bool t_ok, uint32_t h, float *xch, uint32_t wm, uint32_t tslot)
{
    constexpr float kBig = 3.3895314e38f;  // the largest finite bf16
    const int r = a.r;
    // the rounded product, if asked for
    if (a.Ymsg && t_ok) {
        uint16_t *yrow = a.Ymsg + t * a.ldYm;
#pragma unroll
        for (int fb = 0; fb < 4; ++fb) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t f = F0 + 32u * fb + 8u * j + 4u * h;
                if (f < static_cast<uint32_t>(a.E)) {
                    const uint2 w = make_uint2(
                        (__float_as_uint(y[fb][4 * j]) >> 16) | (__float_as_uint(y[fb][4 * j + 1]) & 0xFFFF0000u),
                        (__float_as_uint(y[fb][4 * j + 2]) >> 16) | (__float_as_uint(y[fb][4 * j + 3]) & 0xFFFF0000u));
                    *reinterpret_cast<uint2 *>(yrow + f) = w;
                }
            }
        }
    }
    // min / max per block of 32 features, over the quantised ones
    float mn[4], mx[4];
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) {
        float lo = kBig, hi = -kBig;
        const int lim = r - static_cast<int>(F0 + 32u * fb + 4u * h);  // element offsets below this are quantised
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const bool ok = !RAGGED || (8 * (v >> 2) + (v & 3)) < lim;
            lo = fminf(lo, ok ? y[fb][v] : kBig);
            hi = fmaxf(hi, ok ? y[fb][v] : -kBig);
        }
        mn[fb] = fminf(lo, __shfl_xor(lo, 32, 64));
        mx[fb] = fmaxf(hi, __shfl_xor(hi, 32, 64));
    }
    if (G >= 64) {
        mn[0] = mn[1] = fminf(mn[0], mn[1]);
        mx[0] = mx[1] = fmaxf(mx[0], mx[1]);
        mn[2] = mn[3] = fminf(mn[2], mn[3]);
        mx[2] = mx[3] = fmaxf(mx[2], mx[3]);
    }
    if (G >= 128) {
        mn[0] = mn[1] = mn[2] = mn[3] = fminf(mn[0], mn[2]);
        mx[0] = mx[1] = mx[2] = mx[3] = fmaxf(mx[0], mx[2]);
    }
    if (G == 256) {
        // the group's other half is the neighbouring wave's (same tokens): through LDS
        float *mine = xch + ((wm * 2u + 0u) * 128u + tslot) * 2u;
        const float *other = xch + (((wm ^ 1u) * 2u + 0u) * 128u + tslot) * 2u;
        if (h == 0) {
            mine[0] = mn[0];
            mine[1] = mx[0];
        }
        __syncthreads();
        const float omn = other[0], omx = other[1];
        __syncthreads();
        mn[0] = mn[1] = mn[2] = mn[3] = fminf(mn[0], omn);
        mx[0] = mx[1] = mx[2] = mx[3] = fmaxf(mx[0], omx);
    }
    // zero, bf16 scale, reciprocal (the arithmetic of the stand-alone encoder); lane h = 0
    // stores the scales, its partner the zeros
    float inv[4];
    constexpr int NG = G >= 128 ? 1 : 128 / G;        // groups in the wave's 128 features
    constexpr int FB_PER_G = G >= 128 ? 4 : G / 32;   // blocks per group
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
        const int fb = gi * FB_PER_G;
        mn[fb] = mn[fb] + 0.0f;  // a zero minimum is stored as +0
        const float s32 = div_by_15(mx[fb] - mn[fb]);
        const uint32_t sb = pack_bf16x2(s32, s32) & 0xFFFFu;
        const float s = bf16_bits_to_f32(sb);
        const bool constant = s < 1e-30f;
        const float iv = constant ? 0.0f : reciprocal_of_scale(s);
#pragma unroll
        for (int q = 0; q < FB_PER_G; ++q) {
            inv[fb + q] = iv;
            mn[fb + q] = mn[fb];
        }
        const uint32_t g = G == 256 ? F0 / 256u : F0 / static_cast<uint32_t>(G) + gi;
        const bool owner = G == 256 ? wm == 0 : true;
        if (t_ok && owner && g < static_cast<uint32_t>(a.ng)) {
            uint16_t *dst = reinterpret_cast<uint16_t *>((h ? a.zero : a.scale) + t * a.pitch_meta) + g;
            *dst = static_cast<uint16_t>(h ? __float_as_uint(mn[fb]) >> 16 : (constant ? 0u : sb));
        }
    }
    // codes: a lane has 4 consecutive features of every chunk (its low or its high half)
    uint8_t *crow = a.codes + t * a.pitch_codes;
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) {
        uint32_t half[4];
        const int lim = r - static_cast<int>(F0 + 32u * fb + 4u * h);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t b = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool ok = !RAGGED || (8 * j + e) < lim;
                const float p = (y[fb][4 * j + e] - mn[fb]) * inv[fb];
                b = __builtin_amdgcn_cvt_pk_u8_f32(ok ? p : 0.0f, e, b);
            }
            const uint32_t tt = b | (b >> 4);             // bytes 0 and 2: two nibbles each
            half[j] = (tt & 0xFFu) | ((tt >> 8) & 0xFF00u);
        }
        const uint32_t p0 = half[0] | (half[1] << 16), p1 = half[2] | (half[3] << 16);
        // lane h = 0 assembles chunks 0 and 1 of the block, its partner chunks 2 and 3
        const uint32_t recv = __shfl_xor(h ? p0 : p1, 32, 64);
        const uint32_t lo = h ? recv : p0, hi = h ? p1 : recv;
        const uint32_t wa = (lo & 0xFFFFu) | (hi << 16), wb = (lo >> 16) | (hi & 0xFFFF0000u);
        const uint32_t ca = (F0 + 32u * fb) / 8u + 2u * h;
        if (t_ok) {
            if (!RAGGED || ca + 1u < static_cast<uint32_t>(a.chunks))
                *reinterpret_cast<uint2 *>(crow + 4u * ca) = make_uint2(wa, wb);
            else if (ca < static_cast<uint32_t>(a.chunks))
                *reinterpret_cast<uint32_t *>(crow + 4u * ca) = wa;
        }
    }
    // the features that stay bf16
    if (RAGGED && t_ok) {
        uint16_t *orow = reinterpret_cast<uint16_t *>(a.outl + t * a.pitch_outl);
#pragma unroll
        for (int fb = 0; fb < 4; ++fb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int f = static_cast<int>(F0 + 32u * fb + 4u * h) + 8 * (v >> 2) + (v & 3);
                if (f >= r && f < a.E) orow[f - r] = static_cast<uint16_t>(__float_as_uint(y[fb][v]) >> 16);
            }
        }
    }
}

template <int G>
__global__ __launch_bounds__(256, 2) void k_gemm_encode(GemmArgs a)
{
    extern __shared__ u32x4 smem_gemm[];
    uint8_t *lds = reinterpret_cast<uint8_t *>(smem_gemm);
    const uint32_t tid = threadIdx.x, ln = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t wm = wave >> 1, wn = wave & 1u;
    const uint32_t tileF = blockIdx.x * kGemmTF;
    const int64_t tileT = static_cast<int64_t>(blockIdx.y) * kGemmTT;
    const int K = a.K;

    // this thread's pieces of a stage: 4 of the weights' tile, 2 of the tokens'
    // (piece = 16 bytes = 8 k; row = tid / 4 + 64 i, piece tid % 4)
    const uint32_t prow = tid >> 2, pk = (tid & 3u) * 8u;
    const uint16_t *ga[4], *gb[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t f = min(tileF + prow + 64u * i, static_cast<uint32_t>(a.E) - 1u);
        ga[i] = a.Wp + static_cast<int64_t>(f) * K;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int64_t t = min(tileT + prow + 64 * i, a.T - 1);
        gb[i] = a.X + t * a.ldX;
    }
    const uint32_t lds_piece = prow * kGemmRow + (tid & 3u) * 16u;

    u32x4 ra[4], rb[2];
    auto load_stage = [&](int k0) {
        const int kk = k0 + static_cast<int>(pk);
        const bool ok = kk < K;           // (K is a multiple of 8: a piece is inside or outside)
        const int ks = ok ? kk : 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            ra[i] = *reinterpret_cast<const u32x4 *>(ga[i] + ks);
            if (!ok) ra[i] = u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            rb[i] = *reinterpret_cast<const u32x4 *>(gb[i] + ks);
            if (!ok) rb[i] = u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto store_stage = [&](int s) {
        uint8_t *base = lds + s * kGemmStage;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<u32x4 *>(base + lds_piece + 64u * i * kGemmRow) = ra[i];
#pragma unroll
        for (int i = 0; i < 2; ++i)
            *reinterpret_cast<u32x4 *>(base + kGemmTF * kGemmRow + lds_piece + 64u * i * kGemmRow) = rb[i];
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[fb][tb][v] = 0.0f;

    // operand fetch: lane = (row of the 32x32 block, half of the 16 k)
    const uint32_t frag = (ln & 31u) * kGemmRow + (ln >> 5) * 16u;
    const uint32_t fa = (128u * wm) * kGemmRow + frag;
    const uint32_t fbt = kGemmTF * kGemmRow + (64u * wn) * kGemmRow + frag;

    const int nkt = (K + kGemmBK - 1) / kGemmBK;
    load_stage(0);
    store_stage(0);
    __syncthreads();
    for (int kt = 0; kt < nkt; ++kt) {
        const bool more = kt + 1 < nkt;
        if (more) load_stage((kt + 1) * kGemmBK);
        const uint8_t *st = lds + (kt & 1) * kGemmStage;
#pragma unroll
        for (int ks = 0; ks < kGemmBK / 16; ++ks) {
            u32x4 av[4], bv[2];
#pragma unroll
            for (int fb = 0; fb < 4; ++fb)
                av[fb] = *reinterpret_cast<const u32x4 *>(st + fa + 32u * fb * kGemmRow + 32u * ks);
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
                bv[tb] = *reinterpret_cast<const u32x4 *>(st + fbt + 32u * tb * kGemmRow + 32u * ks);
#pragma unroll
            for (int fb = 0; fb < 4; ++fb)
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
                    acc[fb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8_t, av[fb]), __builtin_bit_cast(bf16x8_t, bv[tb]), acc[fb][tb], 0, 0, 0);
        }
        if (more) store_stage((kt + 1) & 1);
        __syncthreads();
    }

    // epilogue, one block of 32 tokens at a time
    const uint32_t F0 = tileF + 128u * wm;
    const uint32_t h = ln >> 5;
    float *xch = reinterpret_cast<float *>(lds);  // (the stages are done with: the last barrier has passed)
    const bool ragged = F0 + 128u > static_cast<uint32_t>(a.r);
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        const int64_t t = tileT + 64 * wn + 32 * tb + (ln & 31u);
        const bool t_ok = t < a.T;
        float y[4][16];
#pragma unroll
        for (int fb = 0; fb < 4; ++fb)
#pragma unroll
            for (int v = 0; v < 16; ++v) y[fb][v] = round_via_bf16(acc[fb][tb][v]);
        const uint32_t tslot = 64u * wn + 32u * tb + (ln & 31u);
        const int64_t tc = t_ok ? t : 0;
        if (G == 256) {
            // (both waves of a group pass the barriers inside: one code path for everybody)
            gemm_epilogue<G, true>(a, y, F0, tc, t_ok, h, xch, wm, tslot);
        } else if (ragged) {
            gemm_epilogue<G, true>(a, y, F0, tc, t_ok, h, xch, wm, tslot);
        } else {
            gemm_epilogue<G, false>(a, y, F0, tc, t_ok, h, xch, wm, tslot);
        }
    }
}

int launch_gemm_weights(const tpq_layout *L, const void *plan, const uint16_t *Wt, int64_t ldW, int K,
                        uint16_t *Wp, hipStream_t s)
{
    const PlanOffsets o = plan_offsets(L->k, L->r, L->G);
    k_gemm_weights<<<L->E, 256, 0, s>>>(static_cast<const uint8_t *>(plan), L->E, L->k, L->G, L->r, o.idx, o.src,
                                        Wt, ldW, K, Wp);
    return hip_result(hipGetLastError());
}

int launch_gemm_encode(const tpq_layout *L, const uint16_t *X, int64_t T, int64_t ldX, int K,
                       const uint16_t *Wp, uint8_t *codes, uint16_t *scale, uint16_t *zero,
                       uint16_t *outl, uint16_t *Ymsg, int64_t ldYm, hipStream_t s)
{
    GemmArgs a;
    a.X = X;
    a.ldX = ldX;
    a.T = T;
    a.Wp = Wp;
    a.K = K;
    a.E = L->E;
    a.k = L->k;
    a.G = L->G;
    a.r = L->r;
    a.ng = L->ng;
    a.chunks = chunks_of(L->r);
    a.codes = codes;
    a.scale = reinterpret_cast<uint8_t *>(scale);
    a.zero = reinterpret_cast<uint8_t *>(zero);
    a.outl = reinterpret_cast<uint8_t *>(outl);
    a.pitch_codes = L->pitch_codes;
    a.pitch_meta = L->pitch_meta;
    a.pitch_outl = L->pitch_outl;
    a.Ymsg = Ymsg;
    a.ldYm = ldYm;
    const int64_t tiles_t = (T + kGemmTT - 1) / kGemmTT;
    if (tiles_t > 65535) return TPQ_ERR_SHAPE;
    const dim3 grid(static_cast<unsigned>((L->E + kGemmTF - 1) / kGemmTF), static_cast<unsigned>(tiles_t));
    const size_t lds = 2 * kGemmStage;
    hipError_t e = hipSuccess;
#define TPQ_GEMM(GG)                                                                                     \
    case GG:                                                                                             \
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_encode<GG>),                      \
                                hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));      \
        if (e == hipSuccess) launch_kernel(k_gemm_encode<GG>, grid, dim3(256), lds, s, a);               \
        break;
    switch (L->G) {
        TPQ_GEMM(32)
        TPQ_GEMM(64)
        TPQ_GEMM(128)
        TPQ_GEMM(256)
    default: return TPQ_ERR_UNSUPPORTED;
    }
#undef TPQ_GEMM
    if (e != hipSuccess) return hip_result(e);
    return hip_result(hipGetLastError());
}

}  // namespace tpq
