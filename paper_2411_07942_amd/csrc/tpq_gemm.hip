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

// k per stage: a row of a stage is 128 bytes, one whole cache line per request to L2
constexpr int kGemmBK = 64;
constexpr int kGemmPPR = kGemmBK / 8;        // 16-byte pieces per operand row of a stage
constexpr int kGemmRow = kGemmBK * 2;        // LDS bytes per operand row of a stage
// piece p of row m sits at slot p ^ (m % 8): the lanes that fetch the same piece of consecutive
// rows (an MFMA operand) spread over all banks, and so do the lanes that write a row's pieces
__device__ __forceinline__ uint32_t gemm_swz(uint32_t row) { return row & 7u; }

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
// F0 + 32 fb + 8 (v / 4) + 4 h + v % 4 of token t, h = lane / 32 (a wave has 64 features:
// fb = 0, 1).  RAGGED: the wave's 64 features are not all quantised ones (the row's last
// groups, the outlier section, the padding past E); otherwise nothing needs a mask.
// A group wider than the wave's 64 features lies in G / 64 waves of the workgroup that
// work on the same tokens: their minima and maxima meet in LDS (xch).
template <int G, int WF, bool RAGGED>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &a, float (&y)[2][16], uint32_t F0, int64_t t,
                                              bool t_ok, uint32_t h, float *xch, uint32_t wm, uint32_t tslot,
                                              uint32_t n_tslots)
{
    constexpr float kBig = 3.3895314e38f;  // the largest finite bf16
    const int r = a.r;
    // the rounded product, if asked for
    if (a.Ymsg && t_ok) {
        uint16_t *yrow = a.Ymsg + t * a.ldYm;
#pragma unroll
        for (int fb = 0; fb < 2; ++fb) {
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
    float mn[2], mx[2];
#pragma unroll
    for (int fb = 0; fb < 2; ++fb) {
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
    }
    constexpr int WPG = G > 64 ? G / 64 : 1;  // waves per group
    static_assert(WPG <= WF, "a group must lie inside the workgroup's features");
    if (WPG > 1) {
        float *mine = xch + (wm * n_tslots + tslot) * 2u;
        if (h == 0) {
            mine[0] = mn[0];
            mine[1] = mx[0];
        }
        __syncthreads();
        const uint32_t w0 = wm & ~static_cast<uint32_t>(WPG - 1);
        float lo = kBig, hi = -kBig;
#pragma unroll
        for (int q = 0; q < WPG; ++q) {
            const float *o = xch + ((w0 + q) * n_tslots + tslot) * 2u;
            lo = fminf(lo, o[0]);
            hi = fmaxf(hi, o[1]);
        }
        __syncthreads();
        mn[0] = mn[1] = lo;
        mx[0] = mx[1] = hi;
    }
    // zero, bf16 scale, reciprocal (the arithmetic of the stand-alone encoder); lane h = 0
    // stores the scales, its partner the zeros
    float inv[2];
    constexpr int NG = G == 32 ? 2 : 1;  // groups in the wave's 64 features
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
        mn[gi] = mn[gi] + 0.0f;  // a zero minimum is stored as +0
        const float s32 = div_by_15(mx[gi] - mn[gi]);
        const uint32_t sb = pack_bf16x2(s32, s32) & 0xFFFFu;
        const float s = bf16_bits_to_f32(sb);
        const bool constant = s < 1e-30f;
        inv[gi] = constant ? 0.0f : reciprocal_of_scale(s);
        const uint32_t g = G == 32 ? F0 / 32u + gi : F0 / static_cast<uint32_t>(G);
        const bool owner = WPG == 1 || (wm & (WPG - 1)) == 0;
        if (t_ok && owner && g < static_cast<uint32_t>(a.ng)) {
            uint16_t *dst = reinterpret_cast<uint16_t *>((h ? a.zero : a.scale) + t * a.pitch_meta) + g;
            *dst = static_cast<uint16_t>(h ? __float_as_uint(mn[gi]) >> 16 : (constant ? 0u : sb));
        }
    }
    if (NG == 1) {
        mn[1] = mn[0];
        inv[1] = inv[0];
    }
    // codes: a lane has 4 consecutive features of every chunk (its low or its high half)
    uint8_t *crow = a.codes + t * a.pitch_codes;
#pragma unroll
    for (int fb = 0; fb < 2; ++fb) {
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
        for (int fb = 0; fb < 2; ++fb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int f = static_cast<int>(F0 + 32u * fb + 4u * h) + 8 * (v >> 2) + (v & 3);
                if (f >= r && f < a.E) orow[f - r] = static_cast<uint16_t>(__float_as_uint(y[fb][v]) >> 16);
            }
        }
    }
}

// Workgroup = WF x WT waves, each with a tile of 64 features x 64 tokens (four 32x32 blocks);
// the workgroup's tile is 64 WF features x 64 WT tokens.  One LDS stage of 64 k; the next
// stage's operands are loaded into registers while the current one is multiplied.
template <int G, int WF, int WT>
__global__ __launch_bounds__(64 * WF * WT, 768 / (64 * WF * WT)) void k_gemm_encode(GemmArgs a)
{
    constexpr int NT = 64 * WF * WT;            // threads
    constexpr int ROWS_A = 64 * WF, ROWS_B = 64 * WT;
    constexpr int NP = (ROWS_A + ROWS_B) * kGemmPPR / NT;  // 16-byte pieces per thread and stage
    static_assert((ROWS_A + ROWS_B) * kGemmPPR % NT == 0 && (ROWS_A * kGemmPPR) % NT == 0, "pieces divide evenly");
    constexpr int NPA = ROWS_A * kGemmPPR / NT;     // ... of which the weights'
    constexpr int RPP = NT / kGemmPPR;              // rows the threads cover in one pass
    extern __shared__ u32x4 smem_gemm[];
    uint8_t *lds = reinterpret_cast<uint8_t *>(smem_gemm);
    const uint32_t tid = threadIdx.x, ln = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t wm = wave / WT, wn = wave % WT;
    const uint32_t tileF = blockIdx.x * ROWS_A;
    const int64_t tileT = static_cast<int64_t>(blockIdx.y) * ROWS_B;
    const int K = a.K;

    // this thread's pieces of a stage (piece = 16 bytes = 8 k): row tid / 8 + RPP i of the
    // weights' rows followed by the tokens' rows, piece tid % 8.  A piece's address is a
    // uniform base (operand + the stage's first k) plus a 32-bit offset that never changes, so
    // that no register is written on the way to a load but the load's own destination.
    const uint32_t prow = tid / kGemmPPR, ppc = tid % kGemmPPR;
    const int pk = static_cast<int>(ppc) * 8;
    const int pkc = min(pk, K - 8);  // (K < 64: the pieces past K read a valid one, and count as zeros)
    uint32_t voff[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        if (i < NPA) {
            const uint32_t f = min(tileF + prow + RPP * i, static_cast<uint32_t>(a.E) - 1u);
            voff[i] = (f * static_cast<uint32_t>(K) + static_cast<uint32_t>(pkc)) * 2u;
        } else {
            const int64_t t = min(tileT + prow + RPP * (i - NPA), a.T - 1);
            voff[i] = static_cast<uint32_t>((t * a.ldX + pkc) * 2);
        }
    }
    const uint32_t lds_piece = prow * kGemmRow + (ppc ^ gemm_swz(prow)) * 16u;

    // The next stage is on its way in registers while one is multiplied.  Every load is
    // unconditional: stage kt reads the 64 k from kb = min(64 kt, K - 64) on (the last, partial
    // stage reads the last 64 k of the row, the stage past the end reads them again), and what
    // a piece holds counts only if its k is inside the stage: zeros otherwise, put in when the
    // piece goes to LDS -- nothing may touch a loaded register before its stage is due, or the
    // wave waits for the load there.
    const int k_last = max(K - kGemmBK, 0);
    u32x4 rg[NP];
    // (buffer loads: descriptor and the stage's k offset in scalar registers, the piece's
    // offset in a vector register that never changes -- no address arithmetic in vector
    // registers, which the register allocator would place in the loads' destinations)
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.Wp), 0, static_cast<int>(static_cast<int64_t>(a.E) * K * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.X), 0, static_cast<int>(((a.T - 1) * a.ldX + K) * 2), 0x00020000);
    auto load_stage = [&](int kt) {
        const int kb = min(kt * kGemmBK, k_last);
#pragma unroll
        for (int i = 0; i < NP; ++i)
            rg[i] = __builtin_amdgcn_raw_buffer_load_b128(i < NPA ? ra : rb, voff[i], 2 * kb, 0);
    };
    auto store_stage = [&](int kt) {
        const int kpos = min(kt * kGemmBK, k_last) + pk;
        const bool ok = kpos >= kt * kGemmBK && kpos < K;
#pragma unroll
        for (int i = 0; i < NP; ++i)
            *reinterpret_cast<u32x4 *>(lds + lds_piece + RPP * i * kGemmRow) = ok ? rg[i] : u32x4{0u, 0u, 0u, 0u};
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int fb = 0; fb < 2; ++fb)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[fb][tb][v] = 0.0f;

    // operand fetch: lane = (row of the 32x32 block, half of the 16 k)
    const uint32_t frag = (ln & 31u) * kGemmRow;
    const uint32_t fa = (64u * wm) * kGemmRow + frag;
    const uint32_t fbt = (ROWS_A + 64u * wn) * kGemmRow + frag;
    uint32_t fk[kGemmBK / 16];  // byte offset in the row of this lane's piece of k-step ks
#pragma unroll
    for (int ks = 0; ks < kGemmBK / 16; ++ks) fk[ks] = ((2u * ks + (ln >> 5)) ^ gemm_swz(ln & 31u)) * 16u;

    const int nkt = (K + kGemmBK - 1) / kGemmBK;
    auto compute_stage = [&](const uint8_t *st) {
#pragma unroll
        for (int ks = 0; ks < kGemmBK / 16; ++ks) {
            u32x4 av[2], bv[2];
#pragma unroll
            for (int fb = 0; fb < 2; ++fb)
                av[fb] = *reinterpret_cast<const u32x4 *>(st + fa + 32u * fb * kGemmRow + fk[ks]);
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
                bv[tb] = *reinterpret_cast<const u32x4 *>(st + fbt + 32u * tb * kGemmRow + fk[ks]);
#pragma unroll
            for (int fb = 0; fb < 2; ++fb)
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
                    acc[fb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8_t, av[fb]), __builtin_bit_cast(bf16x8_t, bv[tb]),
                        acc[fb][tb], 0, 0, 0);
        }
    };
    // registers -> LDS, barrier, the next stage's loads leave, multiply, barrier
    load_stage(0);
    for (int kt = 0; kt < nkt; ++kt) {
        store_stage(kt);
        __syncthreads();
        load_stage(kt + 1);
        __builtin_amdgcn_sched_barrier(0);  // (the loads leave first: nothing is moved above them)
        compute_stage(lds);
        __syncthreads();
    }

    // epilogue, one block of 32 tokens at a time
    const uint32_t F0 = tileF + 64u * wm;
    const uint32_t h = ln >> 5;
    float *xch = reinterpret_cast<float *>(lds);  // (the stages are done with: the last barrier has passed)
    const bool ragged = F0 + 64u > static_cast<uint32_t>(a.r);
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        const int64_t t = tileT + 64 * wn + 32 * tb + (ln & 31u);
        const bool t_ok = t < a.T;
        float y[2][16];
#pragma unroll
        for (int fb = 0; fb < 2; ++fb)
#pragma unroll
            for (int v = 0; v < 16; ++v) y[fb][v] = round_via_bf16(acc[fb][tb][v]);
        const uint32_t tslot = 64u * wn + 32u * tb + (ln & 31u);
        const int64_t tc = t_ok ? t : 0;
        if (G > 64) {
            // (the waves of a group pass the barriers inside together: the workgroup takes one path)
            if (tileF + ROWS_A > static_cast<uint32_t>(a.r))
                gemm_epilogue<G, WF, true>(a, y, F0, tc, t_ok, h, xch, wm, tslot, ROWS_B);
            else
                gemm_epilogue<G, WF, false>(a, y, F0, tc, t_ok, h, xch, wm, tslot, ROWS_B);
        } else if (ragged) {
            gemm_epilogue<G, WF, true>(a, y, F0, tc, t_ok, h, xch, wm, tslot, ROWS_B);
        } else {
            gemm_epilogue<G, WF, false>(a, y, F0, tc, t_ok, h, xch, wm, tslot, ROWS_B);
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
    hipError_t e = hipSuccess;
    // groups up to 128: workgroups of 2 x 2 waves (128 features x 128 tokens); groups of 256
    // need 256 features in the workgroup: 4 x 1 waves (256 features x 64 tokens)
#define TPQ_GEMM(GG, WF, WT)                                                                              \
    case GG: {                                                                                            \
        const int64_t tiles_t = (T + 64 * WT - 1) / (64 * WT);                                            \
        if (tiles_t > 65535) return TPQ_ERR_SHAPE;                                                        \
        const dim3 grid(static_cast<unsigned>((L->E + 64 * WF - 1) / (64 * WF)), static_cast<unsigned>(tiles_t)); \
        const size_t lds = 64 * (WF + WT) * kGemmRow;                                                 \
        launch_kernel(k_gemm_encode<GG, WF, WT>, grid, dim3(64 * WF * WT), lds, s, a);                    \
        break;                                                                                            \
    }
    switch (L->G) {
        TPQ_GEMM(32, 2, 2)
        TPQ_GEMM(64, 2, 2)
        TPQ_GEMM(128, 2, 2)
        TPQ_GEMM(256, 4, 1)
    default: return TPQ_ERR_UNSUPPORTED;
    }
#undef TPQ_GEMM
    if (e != hipSuccess) return hip_result(e);
    return hip_result(hipGetLastError());
}

}  // namespace tpq
