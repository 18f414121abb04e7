// Internal declarations shared by the library's translation units (host + device).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tpq.h"

namespace tpq {

// ---- plan (device-resident tables derived from the outlier index set) --------
//
// Layout in the caller's plan buffer:
//   PlanHeader                         64 bytes
//   idx     int32 [k rounded up to 4]  the selected features, ascending
//   src_of  uint16[chunks_padded * 8]  src_of[c] = feature index of compacted
//                                      position c; positions >= r repeat the
//                                      last real one (harmless for min / max)
// A "chunk" is 8 consecutive compacted features: what one lane handles, and one
// 32-bit word of packed codes.  chunks_padded rounds the chunk count up to a
// whole number of 64-lane passes.
constexpr uint32_t kPlanMagic = 0x51505431u;  // "1TPQ"
constexpr int kPlanOk = 1;
constexpr int kPlanBadIndex = 2;

struct PlanHeader {
    uint32_t magic;
    int32_t status;  // kPlanOk / kPlanBadIndex; anything else: never built
    int32_t E, k, G, r;
    int32_t chunks;         // ceil(r / 8)
    int32_t chunks_padded;  // chunks rounded up to a multiple of 64
    int32_t idx_offset;     // byte offsets from the start of the plan
    int32_t src_offset;
    int32_t pad[6];
};
static_assert(sizeof(PlanHeader) == 64, "plan header is 64 bytes");

inline int chunks_of(int r) { return (r + 7) / 8; }
inline int chunks_padded_of(int r) { return (chunks_of(r) + 63) / 64 * 64; }
inline int idx_bytes_of(int k) { return ((k + 3) / 4 * 4) * 4; }

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
