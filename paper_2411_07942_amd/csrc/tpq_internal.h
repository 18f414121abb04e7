// Internal declarations shared by the library's translation units (host + device).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
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
//   PlanHeader                          128 bytes
//   idx      int32 [k rounded up to 4]  the selected features, ascending
//   src_of   uint16[chunks_padded * 8]  src_of[c] = feature index of compacted
//                                       position c; positions >= r repeat the
//                                       last real one (harmless for min / max)
//   pass_col uint16[passes + 1]         column of the first feature of pass p
//                                       (pass_col[passes] = E)
//
// Tables of the encoder, which reads each chunk's features with one 16-byte load
// straight from the row ("window" of 8 columns starting at an even column):
//   dpos     uint32[chunks_padded]      per chunk: bits 14..0 = first 32-bit word of its
//                                       window within the row; kDirOdd: the chunk's 8
//                                       features start at the upper half of that word and
//                                       end with the lower half of the next lane's first
//                                       word; kDirSlot: the chunk takes its features from
//                                       its slot (bits 29..16 = slot number): an outlier
//                                       splits it, it is ragged, it must lend its window to
//                                       outliers next to it, or the next lane's window
//                                       does not continue its own; kDirAbsent: beyond the row
//   dflags   uint16[chunks_padded]      scratch of the build
//   dirr     uint16[8 * dslots]         per slot: where the chunk's 8 features sit in the
//                                       32 bytes the chunk loads (two windows: its own and
//                                       the 8 columns after it, pulled back where that would
//                                       leave the row), as byte offsets 0..30; a feature out
//                                       of reach makes the slot "wide": kDirWide | column
//   dsel     uint32[k rounded up to 4]  per selected feature: (slot << 5) | byte offset in
//                                       the slot that holds it, or kDirFar: in no slot
//   pass_dirr uint16[passes + 1]        slots below pass p
//   dpos16   uint16[segs * 64 * 8]      dpos in the form the encoder loads: the row is cut
//                                       into segs segments of dir_P passes (dir_passes_of());
//                                       entry [(seg * 64 + lane) * 8 + p] belongs to lane
//                                       `lane` of the segment's pass p: bits 13..0 = first
//                                       word of the window, kDir16Odd, kDir16Slot (slots are
//                                       numbered in chunk order, so a lane finds its own by
//                                       counting the flagged lanes below it)
//   dseg     uint32[2 * segs]           per segment: word 0 = first slot | slots << 16, word 1 =
//                                       first selected feature it stores | how many << 16 (the
//                                       selected columns below the next segment's first feature
//                                       that no earlier segment owns)
//   drec     uint32[segs * 64 * 8]      what lane l of a wave working on segment sg loads
//                                       first, gathered in one 32-byte record [sg * 64 + l]:
//                                       words 0..3 = its dpos16 entries, words 4, 5 = the
//                                       dslot8 entry of the segment's l-th slot, word 6 = the
//                                       dsel entry of the l-th selected feature the segment
//                                       stores (where there is none: zero, and the
//                                       segment's first slot)
//   drec2    uint32[segs * 64 * 4]      the same for the segment's (64 + l)-th slot and selected
//                                       feature: words 0, 1 = dslot8 entry, word 2 = dsel entry
//   dslot8   uint32[2 * dslots]         per slot: word 0 = eight 4-bit half-word positions
//                                       (feature e at bits 4e..4e+3) in the slot's 32 bytes,
//                                       word 1 = byte offset of its second window in the
//                                       row | kDirWide8 for a "wide" slot (see dirr) |
//                                       kDirLoadB8 unless the next lane of the pass loads
//                                       exactly that window (the usual case: the owner then
//                                       takes it from that lane's registers)
//
// Tables of the decoder's stores.  The 512 sums of a pass (in compacted order) go to
// runs of consecutive output columns; selected columns and the pass's ends cut the
// runs.  A run of 8 or more features is covered by "blocks" of 8 consecutive features
// = 8 consecutive columns (the last block of a run is aligned to the run's end and may
// repeat features of the block before it); the features of shorter runs are stored
// one by one ("narrow" entries).
//   spass    uint32[4 * passes]         per pass: first entry in sblk, blocks, narrow
//                                       entries, 0
//   sblk     uint32[sblk_cap_of()]      per pass its blocks, then its narrow entries:
//                                       bits 15..0 = first column, bits 24..16 = first
//                                       feature's position within the pass (0..511)
constexpr uint32_t kPlanMagic = 0x51505434u;  // "4TPQ"
constexpr int kPlanOk = 1;
constexpr int kPlanBadIndex = 2;
constexpr int kPlanInternal = 3;  // a table of the build overflowed (never expected)
// beyond the row: flag + no slot; the low bits then hold column E - 8
constexpr uint32_t kDirOdd = 0x8000u;
constexpr uint32_t kDirAbsent = 0x40000000u;
constexpr uint32_t kDirSlot = 0x80000000u;
constexpr uint32_t kDirWide = 0x8000u;      // in a dirr entry
constexpr uint32_t kDirFar = 0x80000000u;   // in a dsel entry
constexpr uint32_t kDir16Odd = 0x4000u;
constexpr uint32_t kDir16Slot = 0x8000u;
constexpr uint32_t kDirWide8 = 0x80000000u;  // in word 1 of a dslot8 entry
constexpr uint32_t kDirLoadB8 = 0x40000000u; // in word 1 of a dslot8 entry: the second window is
                                             // not what the next lane loads: fetch it

struct PlanHeader {
    uint32_t magic;
    int32_t status;  // kPlanOk / kPlanBadIndex; anything else: never built
    int32_t E, k, G, r;
    int32_t chunks;         // ceil(r / 8)
    int32_t chunks_padded;  // chunks rounded up to a multiple of 64
    int32_t idx_offset;     // byte offsets from the start of the plan
    int32_t src_offset;
    int32_t pass_col_offset;
    int32_t dpos_offset;
    int32_t dirr_offset;
    int32_t dsel_offset;
    int32_t pass_dirr_offset;
    int32_t n_dirr;       // slots in use
    int32_t dslots;       // slots the tables have room for
    int32_t dpos16_offset;
    int32_t dslot8_offset;
    int32_t dir_P;        // passes per segment the dpos16 table is laid out for
    int32_t dseg_offset;
    int32_t drec_offset;
    int32_t drec2_offset;
    int32_t spass_offset;
    int32_t sblk_offset;
    int32_t sblk_cap;     // entries sblk has room for
    int32_t reserved[6];
};
static_assert(sizeof(PlanHeader) == 128, "plan header is 128 bytes");

__host__ __device__ inline int chunks_of(int r) { return (r + 7) / 8; }
__host__ __device__ inline int chunks_padded_of(int r) { return (chunks_of(r) + 63) / 64 * 64; }
__host__ __device__ inline int idx_bytes_of(int k) { return ((k + 3) / 4 * 4) * 4; }

// An upper bound of the chunks that need a slot in the encoder's tables: one per selected
// feature at most (the chunk that holds or precedes it), the ragged last chunk, the
// last chunk of every pass, and the chunks next to the row's end
__host__ __device__ inline int dir_slots_of(int k, int r)
{
    const int c = chunks_of(r);
    const int bound = k + chunks_padded_of(r) / 64 + 4;
    return bound < c ? bound : c;
}

// Passes per segment of the direct encoder: at most 5, segments as even as possible.
__host__ __device__ inline int dir_passes_of(int passes)
{
    if (passes <= 0) return 1;
    const int segs = (passes + 4) / 5;
    return (passes + segs - 1) / segs;
}
__host__ __device__ inline int dir_segs_of(int passes)
{
    const int P = dir_passes_of(passes);
    return passes > 0 ? (passes + P - 1) / P : 0;
}

// Entries of sblk: a block per chunk, one more per run (at most one run per selected
// feature and pass), up to 7 narrow entries per run -- and never more than 9 per chunk.
__host__ __device__ inline int sblk_cap_of(int k, int r)
{
    const int cp = chunks_padded_of(r);
    const int bound = cp + 8 * (k + cp / 64);
    return bound < 9 * cp ? bound : 9 * cp;
}

__host__ __device__ inline int pass_tab_bytes_of(int r) { return ((chunks_padded_of(r) / 64 + 1) * 2 + 15) / 16 * 16; }

struct PlanOffsets {
    int idx, src, pass_col;
    int dpos, dflags, dirr, dsel, pass_dirr, dpos16, dslot8, dseg, drec, drec2, spass, sblk, total;
};
__host__ __device__ inline PlanOffsets plan_offsets(int k, int r, int G)
{
    const int cp = chunks_padded_of(r);
    PlanOffsets o;
    o.idx = sizeof(PlanHeader);
    o.src = o.idx + idx_bytes_of(k);
    o.pass_col = o.src + 16 * cp;
    o.dpos = o.pass_col + pass_tab_bytes_of(r);
    o.dflags = o.dpos + 4 * cp;
    o.dirr = o.dflags + (2 * cp + 15) / 16 * 16;
    o.dsel = o.dirr + 16 * dir_slots_of(k, r);
    o.pass_dirr = o.dsel + idx_bytes_of(k);
    o.dpos16 = o.pass_dirr + pass_tab_bytes_of(r);
    o.dslot8 = o.dpos16 + dir_segs_of(cp / 64) * 64 * 8 * 2;
    o.dseg = o.dslot8 + (8 * dir_slots_of(k, r) + 15) / 16 * 16;
    o.drec = o.dseg + (8 * dir_segs_of(cp / 64) + 15) / 16 * 16;
    o.drec2 = o.drec + dir_segs_of(cp / 64) * 64 * 32;
    o.spass = o.drec2 + dir_segs_of(cp / 64) * 64 * 16;
    o.sblk = o.spass + (cp / 64) * 16;
    o.total = o.sblk + (4 * sblk_cap_of(k, r) + 15) / 16 * 16;
    return o;
}

// ---- kernel argument blocks -------------------------------------------------

struct RankPtrs {
    const void *p[TPQ_MAX_RANKS];
};

// Ring step: the message each rank has received (null pointers: plain encode).
constexpr int kMaxHopRanks = TPQ_MAX_HOP_RANKS;
struct HopIn {
    const void *codes[kMaxHopRanks];
    const void *scale[kMaxHopRanks];
    const void *zero[kMaxHopRanks];
    const void *outl[kMaxHopRanks];
    int32_t accum;  // TPQ_ACC_*
};

struct EncodeArgs {
    const uint8_t *plan;
    int32_t E, k, G, r, ng, chunks, chunks_padded;
    int32_t n_ranks;
    int64_t T, ldY;
    int64_t pitch_codes, pitch_meta, pitch_outl;
    // direct kernel: a row is cut into `segs` segments of `seg_passes` passes;
    // patch_slots = 32-byte LDS slots each wave has for split chunks
    int32_t segs, seg_passes, patch_slots;
    int64_t n_tasks;  // T * segs (per rank)
    int32_t dslots;   // slots in the plan's tables of the direct kernel
    uint32_t segs_magic;  // 2^32 / segs + 1: task / segs = mulhi(task, segs_magic)
    int32_t bits;  // code width
    float qmax;    // 2^bits - 1
    // static symmetric mode: reciprocal steps, fp32 [n_ranks][static_stride] in compacted order
    const float *inv_c;
    int32_t static_stride;
    // byte offsets of the plan's tables (what the header holds, known to the host too)
    int32_t off_idx, off_dirr, off_dsel, off_dpos16, off_dslot8, off_dseg, off_drec, off_drec2;
};

struct DecodeArgs {
    const uint8_t *plan;
    int32_t E, k, G, r, ng, chunks, chunks_padded;
    int32_t n_ranks;
    int64_t T, ldOut;
    int64_t pitch_codes, pitch_meta, pitch_outl;
    void *out;
    int32_t bits;  // code width
    // epilogue (either may be null): addend bf16 [T][ldAdd], bias bf16 [E]
    const uint8_t *addend;
    int64_t ldAdd;
    const uint8_t *bias;
    // static symmetric mode: steps, fp32 [n_ranks][static_stride] in compacted order
    const float *step_c;
    int32_t static_stride;
    // byte offsets of the plan's tables (what the header holds, known to the host too)
    int32_t off_idx, off_spass, off_sblk, sblk_cap;
};

// What a kernel checks before it trusts a plan: one wide scalar load, no branches between
// the fields.
__device__ __forceinline__ bool plan_header_bad(const uint8_t *plan, int E, int k, int G)
{
    const PlanHeader *ph = reinterpret_cast<const PlanHeader *>(plan);
    return (ph->magic != kPlanMagic) | (ph->status != kPlanOk) | (ph->E != E) | (ph->k != k) | (ph->G != G);
}

// ---- host-side helpers --------------------------------------------------------

int check_layout(const tpq_layout *L);  // TPQ_OK or an error code
void set_last_hip_error(hipError_t e);
int hip_result(hipError_t e);  // TPQ_OK, or records e and returns TPQ_ERR_HIP

// One-shot timing request of the calling thread (tpq_bench_time_next_launch): the next encode /
// ring step / decode kernel is launched with these two events attached to its dispatch.
struct LaunchTimer {
    hipEvent_t start, stop;
};
extern thread_local LaunchTimer g_launch_timer;

// kernel<<<grid, block, lds, s>>>(args...), with the pending timing events if there are any
template <typename... KArgs, typename... Args>
inline void launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t s,
                          const Args &...args)
{
    if (g_launch_timer.start) {
        const LaunchTimer t = g_launch_timer;
        g_launch_timer = LaunchTimer{nullptr, nullptr};
        hipExtLaunchKernelGGL(kernel, grid, block, static_cast<uint32_t>(lds), s, t.start, t.stop, 0u, args...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, static_cast<uint32_t>(lds), s, args...);
    }
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// kernel launchers (defined next to their kernels)
int launch_plan_build(const tpq_layout *L, const int32_t *idx, void *plan, hipStream_t s);
// hop: null for a plain encode, else the received messages (ring step)
int launch_encode(const EncodeArgs &a, const RankPtrs &Y, const RankPtrs &codes,
                  const RankPtrs &scale, const RankPtrs &zero, const RankPtrs &outl,
                  hipStream_t s, const HopIn *hop = nullptr);
int launch_decode(const DecodeArgs &a, const RankPtrs &codes, const RankPtrs &scale,
                  const RankPtrs &zero, const RankPtrs &outl, int accum, int out_dtype,
                  hipStream_t s);
int launch_gemm_weights(const tpq_layout *L, const void *plan, const uint16_t *Wt, int64_t ldW, int K,
                        uint16_t *Wp, hipStream_t s);
int launch_gemm_encode(const tpq_layout *L, const uint16_t *X, int64_t T, int64_t ldX, int K,
                       const uint16_t *Wp, uint8_t *codes, uint16_t *scale, uint16_t *zero,
                       uint16_t *outl, uint16_t *Ymsg, int64_t ldYm, hipStream_t s);
// calibration workspace: up to kCalMaxParts slices of partial minima / maxima
constexpr int kCalMaxParts = 128;
size_t calibrate_workspace_bytes(int E);
int launch_colminmax_ema(const uint16_t *Y, int64_t S, int64_t ldY, int E, int first,
                         float gamma, float *m, float *M, void *ws, int max_parts, hipStream_t s);
int calibrate_parts(int64_t S, int E, int compute_units, int max_parts);
// the library's own scratch for tpq_calibrate_fixed: its device address on the current GPU
constexpr int kCalFixedMaxParts = 64;
int calibrate_fixed_scratch(void **ptr);
int launch_static_params(const tpq_layout *L, const void *plan, const float *m, const float *M,
                         int n_ranks, float *step, float *inv, hipStream_t s);
int launch_finalize(const float *m, const float *M, int N, int E, int k, float *R,
                    float *Rbar, int32_t *idx_sorted, int32_t *idx_ranked, int32_t *ws,
                    hipStream_t s);

}  // namespace tpq
