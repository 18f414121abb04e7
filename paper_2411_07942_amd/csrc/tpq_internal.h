// Internal declarations shared by the library's translation units (host + device).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tpq.h"

namespace tpq {

// ---- plan (device-resident tables derived from the outlier index set) --------
//
// A "chunk" is 8 consecutive compacted features: what one lane handles, and one
// 32-bit word of packed codes.  A "pass" is 64 chunks (one wavefront).
// chunks_padded rounds the chunk count up to whole passes.
//
// Layout in the caller's plan buffer (every table starts on a 16-byte boundary):
//   PlanHeader                          64 bytes
//   idx      int32 [k rounded up to 4]  the selected features, ascending
//   src_of   uint16[chunks_padded * 8]  src_of[c] = feature index of compacted
//                                       position c; positions >= r repeat the
//                                       last real one (harmless for min / max)
//   cpos     uint32[chunks_padded]      per chunk: bits 15..0 = a column from which
//                                       16 bytes can always be read; for a "regular"
//                                       chunk (its 8 features are consecutive
//                                       columns) that is the chunk's first column
//                                       and the whole word is just that.  Bit 31 set:
//                                       an outlier splits the chunk or it is the
//                                       ragged last one ("irregular"; bits 30..16 =
//                                       its slot q in irr / irr_src), or the chunk
//                                       lies beyond the row: if it shares the last
//                                       real group it has a slot too (its 8 sources
//                                       repeat the last feature, neutral for the
//                                       group's min / max), else slot = kNoSlot.
//   flags    uint16[chunks_padded]      scratch of the build (1 = irregular)
//   irr      uint16[chunks_padded]      irr[q] = chunk number of the q-th irregular
//                                       chunk, ascending
//   pass_irr uint16[passes + 1]         irregular chunks below pass p
//   irr_src  uint16[8 * slots]          the 8 feature indices of irregular chunk q
//   pass_col uint16[passes + 1]         column of the first feature of pass p
//                                       (pass_col[passes] = E)
constexpr uint32_t kPlanMagic = 0x51505433u;  // "3TPQ"
constexpr int kPlanOk = 1;
constexpr int kPlanBadIndex = 2;
constexpr uint32_t kNotRegular = 0x80000000u;
constexpr uint32_t kNoSlot = 0x7FFFu;
// beyond the row: flag + no slot; the low bits then hold column E - 8

struct PlanHeader {
    uint32_t magic;
    int32_t status;  // kPlanOk / kPlanBadIndex; anything else: never built
    int32_t E, k, G, r;
    int32_t chunks;         // ceil(r / 8)
    int32_t chunks_padded;  // chunks rounded up to a multiple of 64
    int32_t idx_offset;     // byte offsets from the start of the plan
    int32_t src_offset;
    int32_t pos_offset;
    int32_t pass_col_offset;
    int32_t irr_offset;
    int32_t pass_irr_offset;
    int32_t n_irr;
    int32_t irr_src_offset;
};
static_assert(sizeof(PlanHeader) == 64, "plan header is 64 bytes");

__host__ __device__ inline int chunks_of(int r) { return (r + 7) / 8; }
__host__ __device__ inline int chunks_padded_of(int r) { return (chunks_of(r) + 63) / 64 * 64; }
__host__ __device__ inline int idx_bytes_of(int k) { return ((k + 3) / 4 * 4) * 4; }

// an upper bound of the irregular chunks of a row that the host can compute
__host__ __device__ inline int irr_slots_of(int k, int r, int G)
{
    // chunks split by an outlier or ragged (at most k + 1, and no more than there are
    // chunks), plus the absent chunks that share the last real group (fewer than G / 8)
    const int c = chunks_of(r);
    return (k + 1 < c ? k + 1 : c) + G / 8 - 1;
}

__host__ __device__ inline int pass_tab_bytes_of(int r) { return ((chunks_padded_of(r) / 64 + 1) * 2 + 15) / 16 * 16; }

struct PlanOffsets {
    int idx, src, pos, flags, irr, pass_irr, pass_col, irr_src, total;
};
__host__ __device__ inline PlanOffsets plan_offsets(int k, int r, int G)
{
    const int cp = chunks_padded_of(r);
    PlanOffsets o;
    o.idx = sizeof(PlanHeader);
    o.src = o.idx + idx_bytes_of(k);
    o.pos = o.src + 16 * cp;
    o.flags = o.pos + 4 * cp;
    o.irr = o.flags + 2 * cp;
    o.pass_irr = o.irr + 2 * cp;
    o.pass_col = o.pass_irr + pass_tab_bytes_of(r);
    o.irr_src = o.pass_col + pass_tab_bytes_of(r);
    o.total = o.irr_src + 16 * irr_slots_of(k, r, G);
    return o;
}

// ---- kernel argument blocks -------------------------------------------------

struct RankPtrs {
    const void *p[TPQ_MAX_RANKS];
};

struct EncodeArgs {
    const uint8_t *plan;
    int32_t E, k, G, r, ng, chunks, chunks_padded;
    int32_t n_ranks;
    int64_t T, ldY;
    int64_t pitch_codes, pitch_meta, pitch_outl;
    // streaming kernels: a row is cut into `segs` segments of `seg_passes` passes;
    // stage_chunks = 16-byte units of LDS each wave has for its slice of the row
    int32_t segs, seg_passes, patch_slots, stage_chunks;
    int64_t n_tasks;  // n_ranks * T * segs
};

struct DecodeArgs {
    const uint8_t *plan;
    int32_t E, k, G, r, ng, chunks, chunks_padded;
    int32_t n_ranks;
    int64_t T, ldOut;
    int64_t pitch_codes, pitch_meta, pitch_outl;
    void *out;
};

// ---- host-side helpers --------------------------------------------------------

int check_layout(const tpq_layout *L);  // TPQ_OK or an error code
void set_last_hip_error(hipError_t e);
int hip_result(hipError_t e);  // TPQ_OK, or records e and returns TPQ_ERR_HIP

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// kernel launchers (defined next to their kernels)
int launch_plan_build(const tpq_layout *L, const int32_t *idx, void *plan, hipStream_t s);
int launch_encode(const EncodeArgs &a, const RankPtrs &Y, const RankPtrs &codes,
                  const RankPtrs &scale, const RankPtrs &zero, const RankPtrs &outl,
                  hipStream_t s);
int launch_decode(const DecodeArgs &a, const RankPtrs &codes, const RankPtrs &scale,
                  const RankPtrs &zero, const RankPtrs &outl, int accum, int out_dtype,
                  hipStream_t s);
int launch_colminmax_ema(const uint16_t *Y, int64_t S, int64_t ldY, int E, int first,
                         float gamma, float *m, float *M, float *ws, hipStream_t s);
int calibrate_parts(int64_t S, int E);
int launch_finalize(const float *m, const float *M, int N, int E, int k, float *R,
                    float *Rbar, int32_t *idx_sorted, int32_t *idx_ranked, int32_t *ws,
                    hipStream_t s);

}  // namespace tpq
