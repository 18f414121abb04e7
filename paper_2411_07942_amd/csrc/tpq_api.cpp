// Host side of the C ABI: layout arithmetic, argument validation, dispatch.
// Every check here runs before anything is enqueued.
#include <string.h>

#include "tpq_internal.h"

namespace tpq {

static thread_local int g_last_hip_error = 0;

void set_last_hip_error(hipError_t e) { g_last_hip_error = static_cast<int>(e); }

thread_local LaunchTimer g_launch_timer = {nullptr, nullptr};

int hip_result(hipError_t e)
{
    if (e == hipSuccess) return TPQ_OK;
    set_last_hip_error(e);
    return TPQ_ERR_HIP;
}

static bool group_ok(int G) { return G == 32 || G == 64 || G == 128 || G == 256; }

static bool bits_ok(int b) { return b == 2 || b == 3 || b == 4 || b == 5 || b == 6 || b == 8; }

static int64_t round16(int64_t v) { return (v + 15) / 16 * 16; }

// Bytes of a row of codes, and the least pitch: 4 bits: the last 32-bit word is stored
// whole; other widths: whole chunks of 8 codes are stored, and the decoder reads 8 bytes
// from the start of every chunk.
static int64_t code_bytes_of(int r, int bits) { return (static_cast<int64_t>(r) * bits + 7) / 8; }
static int64_t min_pitch_codes(int r, int bits)
{
    if (bits == 4) return round16(code_bytes_of(r, 4));
    return r > 0 ? round16(static_cast<int64_t>(chunks_of(r)) * bits + 8) : 0;
}

int check_layout(const tpq_layout *L)
{
    if (!L) return TPQ_ERR_NULL;
    if (!bits_ok(L->bits) || !group_ok(L->G)) return TPQ_ERR_UNSUPPORTED;
    if (L->E < 8 || L->E > TPQ_MAX_E || (L->E % 8) != 0) return TPQ_ERR_SHAPE;
    if (L->k < 0 || L->k > L->E) return TPQ_ERR_SHAPE;
    const int r = L->E - L->k;
    if (L->r != r || L->ng != (r + L->G - 1) / L->G || L->code_bytes != code_bytes_of(r, L->bits))
        return TPQ_ERR_SHAPE;
    if (L->wire_bytes_per_row != 2LL * L->k + L->code_bytes + 4LL * L->ng) return TPQ_ERR_SHAPE;
    if ((L->pitch_codes % 16) || (L->pitch_meta % 16) || (L->pitch_outl % 16)) return TPQ_ERR_ALIGN;
    if (L->pitch_codes < min_pitch_codes(r, L->bits) || L->pitch_meta < 2LL * L->ng ||
        L->pitch_outl < 2LL * L->k)
        return TPQ_ERR_SHAPE;
    return TPQ_OK;
}

}  // namespace tpq

using namespace tpq;

// The argument blocks' common part: the layout's numbers, the plan, the launch's extent.
static EncodeArgs encode_args(const tpq_layout *L, const void *plan, int n_ranks, int64_t T, int64_t ldY)
{
    EncodeArgs a;
    memset(&a, 0, sizeof a);
    a.plan = static_cast<const uint8_t *>(plan);
    a.E = L->E; a.k = L->k; a.G = L->G; a.r = L->r; a.ng = L->ng;
    a.chunks = chunks_of(L->r);
    a.chunks_padded = chunks_padded_of(L->r);
    a.n_ranks = n_ranks;
    a.T = T; a.ldY = ldY;
    a.pitch_codes = L->pitch_codes; a.pitch_meta = L->pitch_meta; a.pitch_outl = L->pitch_outl;
    return a;
}

static DecodeArgs decode_args(const tpq_layout *L, const void *plan, int n_ranks, int64_t T, void *out,
                              int64_t ldOut)
{
    DecodeArgs a;
    memset(&a, 0, sizeof a);
    a.plan = static_cast<const uint8_t *>(plan);
    a.E = L->E; a.k = L->k; a.G = L->G; a.r = L->r; a.ng = L->ng;
    a.chunks = chunks_of(L->r);
    a.chunks_padded = chunks_padded_of(L->r);
    a.n_ranks = n_ranks;
    a.T = T; a.ldOut = ldOut;
    a.pitch_codes = L->pitch_codes; a.pitch_meta = L->pitch_meta; a.pitch_outl = L->pitch_outl;
    a.out = out;
    return a;
}

extern "C" {

int tpq_layout_init(tpq_layout *L, int E, int k, int G, int bits)
{
    if (!L) return TPQ_ERR_NULL;
    if (!bits_ok(bits) || !group_ok(G)) return TPQ_ERR_UNSUPPORTED;
    if (E < 8 || E > TPQ_MAX_E || (E % 8) != 0 || k < 0 || k > E) return TPQ_ERR_SHAPE;
    memset(L, 0, sizeof *L);
    L->E = E;
    L->k = k;
    L->G = G;
    L->bits = bits;
    L->r = E - k;
    L->ng = (L->r + G - 1) / G;
    L->code_bytes = static_cast<int32_t>(code_bytes_of(L->r, bits));
    L->pitch_codes = min_pitch_codes(L->r, bits);
    L->pitch_meta = round16(2LL * L->ng);
    L->pitch_outl = round16(2LL * k);
    L->wire_bytes_per_row = 2LL * k + L->code_bytes + 4LL * L->ng;
    return TPQ_OK;
}

double tpq_payload_bits(const tpq_layout *L)
{
    if (!L || L->E <= 0) return 0.0;
    return (16.0 * L->k + static_cast<double>(L->bits) * L->r) / L->E;
}

double tpq_wire_bits(const tpq_layout *L)
{
    if (!L || L->E <= 0) return 0.0;
    return 8.0 * static_cast<double>(L->wire_bytes_per_row) / L->E;
}

const char *tpq_strerror(int code)
{
    switch (code) {
    case TPQ_OK: return "ok";
    case TPQ_ERR_NULL: return "required pointer is NULL";
    case TPQ_ERR_SHAPE: return "size out of range or inconsistent";
    case TPQ_ERR_INDEX: return "outlier indices unsorted, duplicated or out of range";
    case TPQ_ERR_UNSUPPORTED: return "unsupported bit width, group size or mode";
    case TPQ_ERR_ALIGN: return "pointer or pitch not aligned";
    case TPQ_ERR_WORKSPACE: return "workspace or plan buffer too small";
    case TPQ_ERR_HIP: return "HIP runtime error";
    default: return "unknown error";
    }
}

int tpq_last_hip_error(void) { return g_last_hip_error; }

int tpq_bench_time_next_launch(void *start_event, void *stop_event)
{
    if ((start_event == nullptr) != (stop_event == nullptr)) return TPQ_ERR_NULL;
    g_launch_timer = LaunchTimer{static_cast<hipEvent_t>(start_event), static_cast<hipEvent_t>(stop_event)};
    return TPQ_OK;
}

// ---- plan ---------------------------------------------------------------------

size_t tpq_plan_bytes(const tpq_layout *L)
{
    if (check_layout(L) != TPQ_OK) return 0;
    const size_t n = static_cast<size_t>(plan_offsets(L->k, L->r, L->G).total);
    return (n + 255) / 256 * 256;
}

int tpq_plan_build(const tpq_layout *L, const int32_t *idx_sorted, void *plan,
                   size_t plan_bytes, void *stream)
{
    int rc = check_layout(L);
    if (rc) return rc;
    if (!plan || (L->k > 0 && !idx_sorted)) return TPQ_ERR_NULL;
    if (!aligned16(plan) || (reinterpret_cast<uintptr_t>(idx_sorted) & 3u)) return TPQ_ERR_ALIGN;
    if (plan_bytes < tpq_plan_bytes(L)) return TPQ_ERR_WORKSPACE;
    return launch_plan_build(L, idx_sorted, plan, static_cast<hipStream_t>(stream));
}

int tpq_plan_check(const tpq_layout *L, const void *plan, void *stream)
{
    int rc = check_layout(L);
    if (rc) return rc;
    if (!plan) return TPQ_ERR_NULL;
    PlanHeader h;
    hipStream_t s = static_cast<hipStream_t>(stream);
    rc = hip_result(hipMemcpyAsync(&h, plan, sizeof h, hipMemcpyDeviceToHost, s));
    if (rc) return rc;
    rc = hip_result(hipStreamSynchronize(s));
    if (rc) return rc;
    if (h.magic != kPlanMagic) return TPQ_ERR_SHAPE;
    if (h.status == kPlanBadIndex) return TPQ_ERR_INDEX;
    if (h.status != kPlanOk || h.E != L->E || h.k != L->k || h.G != L->G) return TPQ_ERR_SHAPE;
    return TPQ_OK;
}

// ---- calibration --------------------------------------------------------------

size_t tpq_calibrate_workspace_bytes(int64_t S, int E)
{
    if (S < 0 || E < 8 || E > TPQ_MAX_E || (E % 8)) return 0;
    return calibrate_workspace_bytes(E);
}

int tpq_calibrate(const uint16_t *Y, int64_t S, int64_t ldY, int E, int rank, int n_ranks,
                  int64_t seq_index, float gamma, float *m, float *M, void *workspace,
                  size_t ws_bytes, void *stream)
{
    if (E < 8 || E > TPQ_MAX_E || (E % 8) != 0 || S < 0 || ldY < E || n_ranks < 1 ||
        n_ranks > TPQ_MAX_RANKS || rank < 0 || rank >= n_ranks || seq_index < 0)
        return TPQ_ERR_SHAPE;
    if (!(gamma >= 0.0f && gamma <= 1.0f)) return TPQ_ERR_SHAPE;
    if (S == 0) return TPQ_OK;
    if (!Y || !m || !M || !workspace) return TPQ_ERR_NULL;
    if ((ldY % 8) != 0 || !aligned16(Y) || !aligned16(workspace) ||
        (reinterpret_cast<uintptr_t>(m) & 3u) || (reinterpret_cast<uintptr_t>(M) & 3u))
        return TPQ_ERR_ALIGN;
    if (ws_bytes < tpq_calibrate_workspace_bytes(S, E)) return TPQ_ERR_WORKSPACE;
    return launch_colminmax_ema(Y, S, ldY, E, seq_index == 0, gamma,
                                m + static_cast<int64_t>(rank) * E,
                                M + static_cast<int64_t>(rank) * E,
                                workspace, kCalMaxParts, static_cast<hipStream_t>(stream));
}

int tpq_calibrate_fixed(const uint16_t *Y, int64_t S, int64_t ldY, int E, int rank, int n_ranks,
                        int64_t seq_index, float gamma, float *m, float *M, void *stream)
{
    if (E < 8 || E > TPQ_CALIBRATE_FIXED_MAX_E || (E % 8) != 0 || S < 0 || ldY < E || n_ranks < 1 ||
        n_ranks > TPQ_MAX_RANKS || rank < 0 || rank >= n_ranks || seq_index < 0)
        return TPQ_ERR_SHAPE;
    if (!(gamma >= 0.0f && gamma <= 1.0f)) return TPQ_ERR_SHAPE;
    if (S == 0) return TPQ_OK;
    if (!Y || !m || !M) return TPQ_ERR_NULL;
    if ((ldY % 8) != 0 || !aligned16(Y) || (reinterpret_cast<uintptr_t>(m) & 3u) ||
        (reinterpret_cast<uintptr_t>(M) & 3u))
        return TPQ_ERR_ALIGN;
    void *scratch = nullptr;
    const int rc = calibrate_fixed_scratch(&scratch);
    if (rc) return rc;
    return launch_colminmax_ema(Y, S, ldY, E, seq_index == 0, gamma,
                                m + static_cast<int64_t>(rank) * E,
                                M + static_cast<int64_t>(rank) * E, scratch, kCalFixedMaxParts,
                                static_cast<hipStream_t>(stream));
}

size_t tpq_calibrate_finalize_workspace_bytes(int E)
{
    if (E < 8 || E > TPQ_MAX_E || (E % 8)) return 0;
    return static_cast<size_t>(E) * sizeof(int32_t);
}

int tpq_calibrate_finalize(const float *m, const float *M, int n_ranks, int E, int k, float *R,
                           float *Rbar, int32_t *idx_sorted, int32_t *idx_ranked,
                           void *workspace, size_t ws_bytes, void *stream)
{
    if (E < 8 || E > TPQ_MAX_E || (E % 8) != 0 || n_ranks < 1 || n_ranks > TPQ_MAX_RANKS ||
        k < 0 || k > E)
        return TPQ_ERR_SHAPE;
    if (!m || !M || !Rbar || !workspace || (k > 0 && !idx_sorted)) return TPQ_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(m) & 3u) || (reinterpret_cast<uintptr_t>(M) & 3u) ||
        (reinterpret_cast<uintptr_t>(R) & 3u) || (reinterpret_cast<uintptr_t>(Rbar) & 3u) ||
        (reinterpret_cast<uintptr_t>(idx_sorted) & 3u) ||
        (reinterpret_cast<uintptr_t>(idx_ranked) & 3u) ||
        (reinterpret_cast<uintptr_t>(workspace) & 3u))
        return TPQ_ERR_ALIGN;
    if (ws_bytes < tpq_calibrate_finalize_workspace_bytes(E)) return TPQ_ERR_WORKSPACE;
    return launch_finalize(m, M, n_ranks, E, k, R, Rbar, idx_sorted, idx_ranked,
                           static_cast<int32_t *>(workspace), static_cast<hipStream_t>(stream));
}

// ---- encode / decode_reduce ---------------------------------------------------

static int gather_ptrs(RankPtrs &dst, const void *const *src, int n, bool required)
{
    memset(&dst, 0, sizeof dst);
    if (!required) return TPQ_OK;
    if (!src) return TPQ_ERR_NULL;
    for (int i = 0; i < n; ++i) {
        if (!src[i]) return TPQ_ERR_NULL;
        if (!aligned16(src[i])) return TPQ_ERR_ALIGN;
        dst.p[i] = src[i];
    }
    return TPQ_OK;
}

int tpq_encode(const tpq_layout *L, const void *plan, const uint16_t *const *Y, int64_t ldY,
               int n_ranks, int64_t T, uint8_t *const *codes, uint16_t *const *scale,
               uint16_t *const *zero, uint16_t *const *outl, void *stream)
{
    int rc = check_layout(L);
    if (rc) return rc;
    if (n_ranks < 1 || n_ranks > TPQ_MAX_RANKS || T < 0 || ldY < L->E) return TPQ_ERR_SHAPE;
    if (T * n_ranks > 0x7FFFFFFFLL) return TPQ_ERR_SHAPE;
    if ((ldY % 8) != 0) return TPQ_ERR_ALIGN;
    if (!plan) return TPQ_ERR_NULL;
    if (!aligned16(plan)) return TPQ_ERR_ALIGN;
    RankPtrs pY, pc, ps, pz, po;
    const bool quant = L->r > 0, keep = L->k > 0;
    if ((rc = gather_ptrs(pY, reinterpret_cast<const void *const *>(Y), n_ranks, true))) return rc;
    if ((rc = gather_ptrs(pc, reinterpret_cast<const void *const *>(codes), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(ps, reinterpret_cast<const void *const *>(scale), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(pz, reinterpret_cast<const void *const *>(zero), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(po, reinterpret_cast<const void *const *>(outl), n_ranks, keep))) return rc;
    if (T == 0) return TPQ_OK;
    EncodeArgs a = encode_args(L, plan, n_ranks, T, ldY);
    a.bits = L->bits;
    a.qmax = static_cast<float>((1 << L->bits) - 1);
    return launch_encode(a, pY, pc, ps, pz, po, static_cast<hipStream_t>(stream));
}

int tpq_gemm_weights(const tpq_layout *L, const void *plan, const uint16_t *Wt, int64_t ldW, int K,
                     uint16_t *Wp, void *stream)
{
    int rc = check_layout(L);
    if (rc) return rc;
    if (L->bits != 4) return TPQ_ERR_UNSUPPORTED;
    if (K < 8 || ldW < K) return TPQ_ERR_SHAPE;
    if ((K % 8) != 0 || (ldW % 8) != 0) return TPQ_ERR_ALIGN;
    if (!plan || !Wt || !Wp) return TPQ_ERR_NULL;
    if (!aligned16(plan) || !aligned16(Wt) || !aligned16(Wp)) return TPQ_ERR_ALIGN;
    return launch_gemm_weights(L, plan, Wt, ldW, K, Wp, static_cast<hipStream_t>(stream));
}

int tpq_gemm_encode(const tpq_layout *L, const uint16_t *X, int64_t T, int64_t ldX, int K,
                    const uint16_t *Wp, uint8_t *codes, uint16_t *scale, uint16_t *zero,
                    uint16_t *outl, uint16_t *Y_msg, int64_t ldYm, void *stream)
{
    int rc = check_layout(L);
    if (rc) return rc;
    if (L->bits != 4) return TPQ_ERR_UNSUPPORTED;
    if (T < 0 || K < 8 || ldX < K || (Y_msg && ldYm < L->E)) return TPQ_ERR_SHAPE;
    // (the kernel addresses both operands through buffer descriptors with 31-bit sizes)
    if (static_cast<int64_t>(L->E) * K * 2 >= (1ll << 31) || T * ldX * 2 >= (1ll << 31)) return TPQ_ERR_SHAPE;
    if ((K % 8) != 0 || (ldX % 8) != 0 || (Y_msg && (ldYm % 8) != 0)) return TPQ_ERR_ALIGN;
    if (!X || !Wp) return TPQ_ERR_NULL;
    if (L->r > 0 && (!codes || !scale || !zero)) return TPQ_ERR_NULL;
    if (L->k > 0 && !outl) return TPQ_ERR_NULL;
    if (!aligned16(X) || !aligned16(Wp) || !aligned16(codes) || !aligned16(scale) || !aligned16(zero) ||
        !aligned16(outl) || !aligned16(Y_msg))
        return TPQ_ERR_ALIGN;
    if (T == 0) return TPQ_OK;
    return launch_gemm_encode(L, X, T, ldX, K, Wp, codes, scale, zero, outl, Y_msg, ldYm,
                              static_cast<hipStream_t>(stream));
}

int tpq_hop(const tpq_layout *L, const void *plan, const uint16_t *const *Y, int64_t ldY,
            int n_ranks, int64_t T, const uint8_t *const *in_codes, const uint16_t *const *in_scale,
            const uint16_t *const *in_zero, const uint16_t *const *in_outl, int accum,
            uint8_t *const *codes, uint16_t *const *scale, uint16_t *const *zero,
            uint16_t *const *outl, void *stream)
{
    int rc = check_layout(L);
    if (rc) return rc;
    if (L->bits != 4) return TPQ_ERR_UNSUPPORTED;
    if (accum != TPQ_ACC_FP32 && accum != TPQ_ACC_BF16) return TPQ_ERR_UNSUPPORTED;
    if (n_ranks < 1 || n_ranks > TPQ_MAX_HOP_RANKS || T < 0 || ldY < L->E) return TPQ_ERR_SHAPE;
    if (T * n_ranks > 0x7FFFFFFFLL) return TPQ_ERR_SHAPE;
    if ((ldY % 8) != 0) return TPQ_ERR_ALIGN;
    if (!plan) return TPQ_ERR_NULL;
    if (!aligned16(plan)) return TPQ_ERR_ALIGN;
    RankPtrs pY, pc, ps, pz, po, ic, is, iz, io;
    const bool quant = L->r > 0, keep = L->k > 0;
    if ((rc = gather_ptrs(pY, reinterpret_cast<const void *const *>(Y), n_ranks, true))) return rc;
    if ((rc = gather_ptrs(pc, reinterpret_cast<const void *const *>(codes), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(ps, reinterpret_cast<const void *const *>(scale), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(pz, reinterpret_cast<const void *const *>(zero), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(po, reinterpret_cast<const void *const *>(outl), n_ranks, keep))) return rc;
    if ((rc = gather_ptrs(ic, reinterpret_cast<const void *const *>(in_codes), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(is, reinterpret_cast<const void *const *>(in_scale), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(iz, reinterpret_cast<const void *const *>(in_zero), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(io, reinterpret_cast<const void *const *>(in_outl), n_ranks, keep))) return rc;
    if (T == 0) return TPQ_OK;
    HopIn hin;
    memset(&hin, 0, sizeof hin);
    hin.accum = accum;
    for (int i = 0; i < n_ranks; ++i) {
        hin.codes[i] = ic.p[i];
        hin.scale[i] = is.p[i];
        hin.zero[i] = iz.p[i];
        hin.outl[i] = io.p[i];
    }
    EncodeArgs a = encode_args(L, plan, n_ranks, T, ldY);
    a.bits = L->bits;
    a.qmax = 15.0f;
    return launch_encode(a, pY, pc, ps, pz, po, static_cast<hipStream_t>(stream), &hin);
}

int tpq_decode_reduce(const tpq_layout *L, const void *plan, int n_ranks, int64_t T,
                      const uint8_t *const *codes, const uint16_t *const *scale,
                      const uint16_t *const *zero, const uint16_t *const *outl, int accum,
                      int out_dtype, void *out, int64_t ldOut, void *stream)
{
    int rc = check_layout(L);
    if (rc) return rc;
    if (accum != TPQ_ACC_FP32 && accum != TPQ_ACC_BF16 && accum != TPQ_ACC_FAST) return TPQ_ERR_UNSUPPORTED;
    if (out_dtype != TPQ_OUT_BF16 && out_dtype != TPQ_OUT_FP32) return TPQ_ERR_UNSUPPORTED;
    if (n_ranks < 1 || n_ranks > TPQ_MAX_RANKS || T < 0 || ldOut < L->E) return TPQ_ERR_SHAPE;
    if (T > 0x7FFFFFFFLL) return TPQ_ERR_SHAPE;
    if ((ldOut % (out_dtype == TPQ_OUT_FP32 ? 4 : 8)) != 0) return TPQ_ERR_ALIGN;
    if (!plan || !out) return TPQ_ERR_NULL;
    if (!aligned16(plan) || !aligned16(out)) return TPQ_ERR_ALIGN;
    RankPtrs pc, ps, pz, po;
    const bool quant = L->r > 0, keep = L->k > 0;
    if ((rc = gather_ptrs(pc, reinterpret_cast<const void *const *>(codes), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(ps, reinterpret_cast<const void *const *>(scale), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(pz, reinterpret_cast<const void *const *>(zero), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(po, reinterpret_cast<const void *const *>(outl), n_ranks, keep))) return rc;
    if (T == 0) return TPQ_OK;
    DecodeArgs a = decode_args(L, plan, n_ranks, T, out, ldOut);
    a.bits = L->bits;
    return launch_decode(a, pc, ps, pz, po, accum, out_dtype, static_cast<hipStream_t>(stream));
}

int tpq_decode_reduce_fused(const tpq_layout *L, const void *plan, int n_ranks, int64_t T,
                            const uint8_t *const *codes, const uint16_t *const *scale,
                            const uint16_t *const *zero, const uint16_t *const *outl,
                            const uint16_t *addend, int64_t ldAdd, const uint16_t *bias, int accum,
                            int out_dtype, void *out, int64_t ldOut, void *stream)
{
    int rc = check_layout(L);
    if (rc) return rc;
    if (L->bits != 4) return TPQ_ERR_UNSUPPORTED;  // the epilogue is built for 4-bit codes
    if (accum != TPQ_ACC_FP32 && accum != TPQ_ACC_BF16 && accum != TPQ_ACC_FAST) return TPQ_ERR_UNSUPPORTED;
    if (out_dtype != TPQ_OUT_BF16 && out_dtype != TPQ_OUT_FP32) return TPQ_ERR_UNSUPPORTED;
    if (n_ranks < 1 || n_ranks > TPQ_MAX_RANKS || T < 0 || ldOut < L->E) return TPQ_ERR_SHAPE;
    if (T > 0x7FFFFFFFLL) return TPQ_ERR_SHAPE;
    if (addend && ldAdd < L->E) return TPQ_ERR_SHAPE;
    if ((ldOut % (out_dtype == TPQ_OUT_FP32 ? 4 : 8)) != 0) return TPQ_ERR_ALIGN;
    if (!plan || !out) return TPQ_ERR_NULL;
    if (!aligned16(plan) || !aligned16(out)) return TPQ_ERR_ALIGN;
    // rows of the addend and the bias are read with 2-byte aligned loads
    RankPtrs pc, ps, pz, po;
    const bool quant = L->r > 0, keep = L->k > 0;
    if ((rc = gather_ptrs(pc, reinterpret_cast<const void *const *>(codes), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(ps, reinterpret_cast<const void *const *>(scale), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(pz, reinterpret_cast<const void *const *>(zero), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(po, reinterpret_cast<const void *const *>(outl), n_ranks, keep))) return rc;
    if (T == 0) return TPQ_OK;
    DecodeArgs a = decode_args(L, plan, n_ranks, T, out, ldOut);
    a.bits = 4;
    a.addend = reinterpret_cast<const uint8_t *>(addend);
    a.ldAdd = ldAdd;
    a.bias = reinterpret_cast<const uint8_t *>(bias);
    return launch_decode(a, pc, ps, pz, po, accum, out_dtype, static_cast<hipStream_t>(stream));
}

// ---- static symmetric mode ----------------------------------------------------

size_t tpq_static_table_floats(const tpq_layout *L)
{
    if (check_layout(L)) return 0;
    return static_cast<size_t>(8) * chunks_padded_of(L->r);
}

int tpq_static_params(const tpq_layout *L, const void *plan, const float *m, const float *M,
                      int n_ranks, float *step, float *inv, void *stream)
{
    int rc = check_layout(L);
    if (rc) return rc;
    if (n_ranks < 1 || n_ranks > TPQ_MAX_RANKS) return TPQ_ERR_SHAPE;
    if (L->r == 0) return TPQ_OK;
    if (!plan || !m || !M || !step || !inv) return TPQ_ERR_NULL;
    if (!aligned16(plan) || !aligned16(step) || !aligned16(inv)) return TPQ_ERR_ALIGN;
    return launch_static_params(L, plan, m, M, n_ranks, step, inv, static_cast<hipStream_t>(stream));
}

int tpq_encode_static(const tpq_layout *L, const void *plan, const uint16_t *const *Y,
                      int64_t ldY, int n_ranks, int64_t T, const float *inv,
                      uint8_t *const *codes, uint16_t *const *outl, void *stream)
{
    int rc = check_layout(L);
    if (rc) return rc;
    if (n_ranks < 1 || n_ranks > TPQ_MAX_RANKS || T < 0 || ldY < L->E) return TPQ_ERR_SHAPE;
    if (T * n_ranks > 0x7FFFFFFFLL) return TPQ_ERR_SHAPE;
    if ((ldY % 8) != 0) return TPQ_ERR_ALIGN;
    if (!plan) return TPQ_ERR_NULL;
    if (!aligned16(plan)) return TPQ_ERR_ALIGN;
    RankPtrs pY, pc, po, none;
    memset(&none, 0, sizeof none);
    const bool quant = L->r > 0, keep = L->k > 0;
    if (quant && !inv) return TPQ_ERR_NULL;
    if (quant && !aligned16(inv)) return TPQ_ERR_ALIGN;
    if ((rc = gather_ptrs(pY, reinterpret_cast<const void *const *>(Y), n_ranks, true))) return rc;
    if ((rc = gather_ptrs(pc, reinterpret_cast<const void *const *>(codes), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(po, reinterpret_cast<const void *const *>(outl), n_ranks, keep))) return rc;
    if (T == 0) return TPQ_OK;
    EncodeArgs a = encode_args(L, plan, n_ranks, T, ldY);
    a.inv_c = inv;
    a.static_stride = 8 * a.chunks_padded;
    a.bits = L->bits;
    a.qmax = static_cast<float>((1 << L->bits) - 1);
    return launch_encode(a, pY, pc, none, none, po, static_cast<hipStream_t>(stream));
}

int tpq_decode_reduce_static(const tpq_layout *L, const void *plan, int n_ranks, int64_t T,
                             const uint8_t *const *codes, const uint16_t *const *outl,
                             const float *step, int accum, int out_dtype, void *out,
                             int64_t ldOut, void *stream)
{
    int rc = check_layout(L);
    if (rc) return rc;
    if (accum != TPQ_ACC_FP32 && accum != TPQ_ACC_BF16 && accum != TPQ_ACC_FAST) return TPQ_ERR_UNSUPPORTED;
    if (out_dtype != TPQ_OUT_BF16 && out_dtype != TPQ_OUT_FP32) return TPQ_ERR_UNSUPPORTED;
    if (n_ranks < 1 || n_ranks > TPQ_MAX_RANKS || T < 0 || ldOut < L->E) return TPQ_ERR_SHAPE;
    if (T > 0x7FFFFFFFLL) return TPQ_ERR_SHAPE;
    if ((ldOut % (out_dtype == TPQ_OUT_FP32 ? 4 : 8)) != 0) return TPQ_ERR_ALIGN;
    if (!plan || !out) return TPQ_ERR_NULL;
    if (!aligned16(plan) || !aligned16(out)) return TPQ_ERR_ALIGN;
    RankPtrs pc, po, none;
    memset(&none, 0, sizeof none);
    const bool quant = L->r > 0, keep = L->k > 0;
    if (quant && !step) return TPQ_ERR_NULL;
    if (quant && !aligned16(step)) return TPQ_ERR_ALIGN;
    if ((rc = gather_ptrs(pc, reinterpret_cast<const void *const *>(codes), n_ranks, quant))) return rc;
    if ((rc = gather_ptrs(po, reinterpret_cast<const void *const *>(outl), n_ranks, keep))) return rc;
    if (T == 0) return TPQ_OK;
    DecodeArgs a = decode_args(L, plan, n_ranks, T, out, ldOut);
    a.step_c = quant ? step : nullptr;
    a.static_stride = 8 * a.chunks_padded;
    a.bits = L->bits;
    return launch_decode(a, pc, none, none, po, accum, out_dtype, static_cast<hipStream_t>(stream));
}

}  // extern "C"
