// tpq_encode kernels: the compression function C^(i) (paper Sec. 2) in the hybrid
// form of Fig. 2 -- selected features verbatim in BF16, the rest as packed 4-bit
// codes with a per-group bf16 scale and zero.
#include "tpq_device.h"
#include "tpq_internal.h"

namespace tpq {

// ---------------------------------------------------------------------------
// k = E: nothing is quantised; the message is the row itself, column by column in
// the order of the (complete) index set.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_copy_selected(EncodeArgs a, RankPtrs Yp, RankPtrs outlp, HopIn hin)
{
    const PlanHeader *ph = reinterpret_cast<const PlanHeader *>(a.plan);
    if (ph->magic != kPlanMagic || ph->status != kPlanOk || ph->E != a.E || ph->k != a.k ||
        ph->G != a.G)
        return;
    const int32_t *idx = reinterpret_cast<const int32_t *>(a.plan + ph->idx_offset);
    const uint32_t rank = blockIdx.z;
    const int64_t t = blockIdx.y;
    const uint32_t p = blockIdx.x * 256u + threadIdx.x;
    if (p >= static_cast<uint32_t>(a.k)) return;
    const uint16_t *y = static_cast<const uint16_t *>(Yp.p[rank]) + t * a.ldY;
    uint16_t *outl = reinterpret_cast<uint16_t *>(
        static_cast<uint8_t *>(const_cast<void *>(outlp.p[rank])) + t * a.pitch_outl);
    uint32_t val = y[idx[p]];
    if (rank < static_cast<uint32_t>(kMaxHopRanks) && hin.outl[rank]) {  // ring step: received + own, in bf16
        const uint16_t *in = reinterpret_cast<const uint16_t *>(
            static_cast<const uint8_t *>(hin.outl[rank]) + t * a.pitch_outl);
        val = pack_bf16x2(bf16_bits_to_f32(in[p]) + bf16_bits_to_f32(val), 0.0f) & 0xFFFFu;
    }
    outl[p] = static_cast<uint16_t>(val);
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
// Eight codes, one per byte of (lo, hi) in feature order, as B-bit fields of a 64-bit
// word: code e at bits B*e .. B*e + B - 1.
template <int B>
__device__ __forceinline__ uint64_t pack_codes(uint32_t lo, uint32_t hi)
{
    uint64_t w = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t c = ((e < 4 ? lo : hi) >> (8 * (e & 3))) & 0xFFu;
        w |= static_cast<uint64_t>(c) << (B * e);
    }
    return w;
}

#ifndef TPQ_HOP_OCC
#define TPQ_HOP_OCC 5  // waves per SIMD of the ring step (15 more live registers than the encoder; 6: 2 % slower, 7: spills)
#endif
template <int P>
struct DirectOcc {  // waves per SIMD the register budget is set for (the static mode at other code
                    // widths and 5 passes per wave needs two registers more than 8 waves leave: 7 there)
    static constexpr int value = 8;
};

//
// STATIC selects the static symmetric mode (Sec. 3, "Calibration" and "Selecting High
// Precision Features"): the reciprocal step of every (device, feature) comes from a
// table in compacted order, nothing is measured per group, and only codes and selected
// features are written.  Everything up to the features in registers is shared.
//
// GEN selects code widths other than 4 bits (Sec. 4, the experiment that varies the
// bits of the quantised features): 2^b - 1 steps over the group's range, and the 8
// codes of a chunk are b bytes of the row's little-endian bit string.
//
// HOP makes the kernel a ring step (Sec. 5, the remark on ring all-reduce): what is
// compressed is not the row of Y itself but the message the device has received,
// dequantised, plus that row -- one more term of decode_reduce's accumulation, rounded
// to bf16.  The received chunk's codes and its group's scale and zero are loaded with
// the windows; the sums replace the features in registers before the group statistics.
template <int LPG, int P, bool STATIC, bool GEN = false, bool HOP = false>
__global__ __launch_bounds__(256, HOP ? TPQ_HOP_OCC : (STATIC && GEN && P == 5) ? 7 : DirectOcc<P>::value) void k_encode_direct(
    EncodeArgs a, RankPtrs Yp, RankPtrs codesp, RankPtrs scalep, RankPtrs zerop, RankPtrs outlp, HopIn hin)
{
    const uint32_t ln = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    const uint32_t passes = static_cast<uint32_t>(a.chunks_padded) >> 6;
    const uint32_t segs = static_cast<uint32_t>(a.segs);
    const uint32_t rank = blockIdx.y;
    uint32_t t, seg;
    bool active = true;
    if constexpr (STATIC) {
        // the four waves of a workgroup take the same segment of four consecutive rows, and
        // share that segment's slice of the device's table through LDS (workgroup =
        // (group of 4 rows, segment); the last group's waves past the last row help with the
        // table and then work on the last row again without storing anything, so that all four
        // waves reach the workgroup's one barrier at the same place)
        const uint32_t rg = segs == 1 ? blockIdx.x : __umulhi(blockIdx.x, a.segs_magic);
        seg = blockIdx.x - rg * segs;
        t = rg * 4u + wave;
        active = t < static_cast<uint32_t>(a.T);
        if (!active) t = static_cast<uint32_t>(a.T) - 1u;
    } else {
        const uint32_t task = blockIdx.x * 4u + wave;
        if (task >= static_cast<uint32_t>(a.n_tasks)) return;
        // t = task / segs by multiplication (exact below 2^32 / segs, which the host keeps)
        t = segs == 1 ? task : __umulhi(task, a.segs_magic);
        seg = task - t * segs;
    }
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
    // (where segments are likely to have more than 64 slots, the second record leaves with the
    // first instead of waiting for the segment's counts)
    const bool eager2 = a.patch_slots > 64;
    u32x4 rec2 = {0u, 0u, 0u, 0u};
    if (eager2) rec2 = reinterpret_cast<const u32x4 *>(a.plan + a.off_drec2)[seg * 64u + ln];
    const PlanHeader *ph = reinterpret_cast<const PlanHeader *>(a.plan);
    if (ph->magic != kPlanMagic || ph->status != kPlanOk || ph->E != a.E || ph->k != a.k ||
        ph->G != a.G || ph->dir_P != P)
        return;  // the whole grid takes this branch together

    // slots and selected columns of this segment
    const uint32_t q_lo = sg.x & 0xFFFFu, n_q = sg.x >> 16;
    // the wave's LDS area holds the segment's first `cap` slots; the slots past them (a
    // segment far denser in selected features than the row's average) are gathered from
    // memory, feature by feature
    const uint32_t cap = static_cast<uint32_t>(a.patch_slots);
    const uint32_t n_ql = min(n_q, cap);
    const uint32_t s_lo = sg.y & 0xFFFFu, n_sel = sg.y >> 16;

    // the segment's ln-th and (64 + ln)-th slot and selected feature (zero where there is
    // none); the second record is fetched only where a segment has that many
    const uint2 slot8 = make_uint2(rec1.x, rec1.y);
    const uint32_t sel0 = rec1.z;
    if (!eager2 && (n_q > 64 || n_sel > 64))
        rec2 = reinterpret_cast<const u32x4 *>(a.plan + a.off_drec2)[seg * 64u + ln];
    uint32_t d[P];
    {
        const uint32_t w4[4] = {dp8.x, dp8.y, dp8.z, dp8.w};
#pragma unroll
        for (int p = 0; p < P; ++p) d[p] = (p & 1) ? (w4[p >> 1] >> 16) : (w4[p >> 1] & 0xFFFFu);
    }

    // static mode: this thread's share of the segment's reciprocal steps (from L2; loaded
    // first, so that they can be parked in LDS while the windows are still on their way)
    u32x4 tab_in[(P * 128 + 255) / 256];
    if constexpr (STATIC) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(
            a.inv_c + static_cast<int64_t>(rank) * a.static_stride + 512u * pass0);
        const uint32_t n4 = (pass1 - pass0) * 128u;  // 8 steps = two 16-byte units per chunk
#pragma unroll
        for (int i = 0; i < (P * 128 + 255) / 256; ++i) {
            const uint32_t j = threadIdx.x + 256u * i;
            tab_in[i] = src[min(j, n4 - 1u)];
        }
    }

    // windows: every lane its chunk's; lane q the second window of slot q
    const uint8_t *yrow = static_cast<const uint8_t *>(Yp.p[rank]) + static_cast<int64_t>(t) * a.ldY * 2;
    u32x4 raw[P];
#pragma unroll
    for (int p = 0; p < P; ++p)
        raw[p] = __builtin_nontemporal_load(
            reinterpret_cast<const u32x4_a4 *>(yrow + 4u * (d[p] & 0x3FFFu)));
    uint32_t hop_w[P], hop_s[P], hop_z[P];  // HOP: the received chunk's codes, its group's scale and zero
    if constexpr (HOP) {
        const uint8_t *ic = static_cast<const uint8_t *>(hin.codes[rank]) + static_cast<int64_t>(t) * a.pitch_codes;
        const uint8_t *is = static_cast<const uint8_t *>(hin.scale[rank]) + static_cast<int64_t>(t) * a.pitch_meta;
        const uint8_t *iz = static_cast<const uint8_t *>(hin.zero[rank]) + static_cast<int64_t>(t) * a.pitch_meta;
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const uint32_t chunk = min((pass0 + p) * 64u + ln, static_cast<uint32_t>(a.chunks) - 1u);
            const uint32_t g = min(chunk / (LPG ? LPG : 1), static_cast<uint32_t>(a.ng) - 1u);
            hop_w[p] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(ic + 4u * chunk));
            hop_s[p] = *reinterpret_cast<const uint16_t *>(is + 2u * g);
            hop_z[p] = *reinterpret_cast<const uint16_t *>(iz + 2u * g);
        }
    }
    u32x4 win_b = {0u, 0u, 0u, 0u}, win_b2 = {0u, 0u, 0u, 0u};
    // (only where the next lane of the slot's pass does not load that window anyway)
    const bool load_b = ln < n_ql && (slot8.y & kDirLoadB8) != 0;
    const bool load_b2 = 64u + ln < n_ql && (rec2.y & kDirLoadB8) != 0;
    if (load_b) win_b = *reinterpret_cast<const u32x4_a4 *>(yrow + (slot8.y & 0x1FFFFu));
    if (load_b2) win_b2 = *reinterpret_cast<const u32x4_a4 *>(yrow + (rec2.y & 0x1FFFFu));

    constexpr int GPS = STATIC ? 0 : 64 * P / (STATIC ? 1 : LPG);  // groups per segment
    extern __shared__ u32x4 smem_direct[];
    uint8_t *slots = reinterpret_cast<uint8_t *>(smem_direct) + wave * (32u * a.patch_slots + 4u * GPS);
    uint32_t *l_meta = reinterpret_cast<uint32_t *>(slots + 32u * a.patch_slots);
    // static mode: the workgroup's table slice behind the four waves' slots, the first and
    // the second half of every chunk's 8 steps in arrays of their own (16-byte stride per lane)
    u32x4 *l_tab = reinterpret_cast<u32x4 *>(reinterpret_cast<uint8_t *>(smem_direct) + 4u * 32u * a.patch_slots);
    if constexpr (STATIC) {
#pragma unroll
        for (int i = 0; i < (P * 128 + 255) / 256; ++i) {
            const uint32_t j = threadIdx.x + 256u * i;
            if (j < static_cast<uint32_t>(P) * 128u) l_tab[(j & 1u) * (64u * P) + (j >> 1)] = tab_in[i];
        }
    }

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
            // the next lane's window: its first word completes an odd chunk, and all of it is
            // the second window of most slots
            const uint32_t nb = __builtin_amdgcn_update_dpp(0u, raw[p].x, 0x130, 0xF, 0xF, false);
            const uint32_t nby = __builtin_amdgcn_update_dpp(0u, raw[p].y, 0x130, 0xF, 0xF, false);
            const uint32_t nbz = __builtin_amdgcn_update_dpp(0u, raw[p].z, 0x130, 0xF, 0xF, false);
            const uint32_t nbw = __builtin_amdgcn_update_dpp(0u, raw[p].w, 0x130, 0xF, 0xF, false);
            if (has_slot && my_slot[p] < cap) {
                *reinterpret_cast<u32x4 *>(slots + 32u * my_slot[p]) = raw[p];
                *reinterpret_cast<u32x4 *>(slots + 32u * my_slot[p] + 16u) = u32x4{nb, nby, nbz, nbw};
            }
            const uint32_t sh = (d[p] >> 10) & 16u;
            v[p].x = __builtin_amdgcn_alignbit(raw[p].y, raw[p].x, sh);
            v[p].y = __builtin_amdgcn_alignbit(raw[p].z, raw[p].y, sh);
            v[p].z = __builtin_amdgcn_alignbit(raw[p].w, raw[p].z, sh);
            v[p].w = __builtin_amdgcn_alignbit(nb, raw[p].w, sh);
        }
    }
    if (load_b) *reinterpret_cast<u32x4 *>(slots + 32u * ln + 16u) = win_b;
    if (load_b2) *reinterpret_cast<u32x4 *>(slots + 32u * (64u + ln) + 16u) = win_b2;
    for (uint32_t q0 = 128; q0 < n_ql; q0 += 64) {  // more than 128 slots in a segment: rare
        const uint32_t q = q0 + ln;
        if (q < n_ql) {
            const uint32_t y1 = dslot8[q_lo + q].y;
            if (y1 & kDirLoadB8)
                *reinterpret_cast<u32x4 *>(slots + 32u * q + 16u) =
                    *reinterpret_cast<const u32x4_a4 *>(yrow + (y1 & 0x1FFFFu));
        }
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
            const uint32_t e = p0 == 0 ? sel0 : (p0 == 64 ? rec2.z : dsel[s_lo + pc]);
            const bool far = (e & kDirFar) != 0 || (e >> 5) - q_lo >= cap;  // in no slot, or in none that LDS holds
            uint32_t val = TPQ_LDS_HW(slots + (far ? 0u : e - 32u * q_lo));
            if (far) val = TPQ_HW(yrow + 2u * static_cast<uint32_t>(idx[s_lo + pc]));
            if constexpr (HOP) {  // received + own, in bf16
                const uint32_t in = reinterpret_cast<const uint16_t *>(
                    static_cast<const uint8_t *>(hin.outl[rank]) + static_cast<int64_t>(t) * a.pitch_outl)[s_lo + pc];
                val = pack_bf16x2(bf16_bits_to_f32(in) + bf16_bits_to_f32(val), 0.0f) & 0xFFFFu;
            }
            if (p < n_sel && active) outl[p] = static_cast<uint16_t>(val);
        }
    }
    for (uint32_t q0 = 0; q0 < n_ql; q0 += 64) {
        const uint32_t q = q0 + ln, qc = min(q, n_ql - 1u);
        const uint2 ent = q0 == 0 ? slot8 : (q0 == 64 ? make_uint2(rec2.x, rec2.y) : dslot8[q_lo + qc]);
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
        if (q < n_ql) *reinterpret_cast<u32x4 *>(slots + 32u * q) = g;
    }
    wave_lds_fence();
#pragma unroll
    for (int p = 0; p < P; ++p)
        if ((d[p] & kDir16Slot) && my_slot[p] < cap) v[p] = *reinterpret_cast<const u32x4 *>(slots + 32u * my_slot[p]);
    if (n_q > cap) {
        // the lanes whose slot LDS does not hold: a slot's entry gives each feature's column,
        // or its byte offset in the two windows (the lane's own, and the one 8 columns on,
        // pulled back to end with the row)
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if ((d[p] & kDir16Slot) && my_slot[p] >= cap) {
                const u32x4 tab = dirr[q_lo + my_slot[p]];
                const uint32_t wa = 2u * (d[p] & 0x3FFFu);
                const uint32_t wb = min(wa + 8u, static_cast<uint32_t>(a.E) - 8u);
                const uint32_t t4[4] = {tab.x, tab.y, tab.z, tab.w};
                uint32_t g4[4];
#pragma unroll
                for (int w2 = 0; w2 < 4; ++w2) {
                    uint32_t hw[2];
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2) {
                        const uint32_t en = (t4[w2] >> (16 * h2)) & 0xFFFFu;
                        const uint32_t col = (en & kDirWide) ? (en & 0x7FFFu)
                                                             : (en < 16u ? wa + (en >> 1) : wb + ((en - 16u) >> 1));
                        hw[h2] = TPQ_HW(yrow + 2u * col);
                    }
                    g4[w2] = hw[0] | (hw[1] << 16);
                }
                v[p] = u32x4{g4[0], g4[1], g4[2], g4[3]};
            }
        }
    }
#undef TPQ_HW
#undef TPQ_LDS_HW

    if constexpr (HOP) {
        // features <- bf16(x_hat (+) feature): x_hat = code * scale + zero as in decode_reduce,
        // rounded to bf16 first in the bf16 chain.  The positions of a ragged last chunk
        // past the row's end repeat the chunk's first sum (the received codes there are
        // padding), so that they stay inside their group's range.
        const bool chain = hin.accum == TPQ_ACC_BF16;
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const float sc = bf16_bits_to_f32(hop_s[p]), ze = bf16_bits_to_f32(hop_z[p]);
            const uint32_t lo = hop_w[p] & 0x0F0F0F0Fu, hi = (hop_w[p] >> 4) & 0x0F0F0F0Fu;
            const f32x2 c02 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(lo, 512.0f, false);
            const f32x2 c46 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(lo, 512.0f, true);
            const f32x2 c13 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(hi, 512.0f, false);
            const f32x2 c57 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(hi, 512.0f, true);
            float x[8] = {__builtin_fmaf(c02.x, sc, ze), __builtin_fmaf(c13.x, sc, ze), __builtin_fmaf(c02.y, sc, ze),
                          __builtin_fmaf(c13.y, sc, ze), __builtin_fmaf(c46.x, sc, ze), __builtin_fmaf(c57.x, sc, ze),
                          __builtin_fmaf(c46.y, sc, ze), __builtin_fmaf(c57.y, sc, ze)};
            if (chain) {
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = round_via_bf16(x[e]);
            }
            const uint32_t wv[4] = {v[p].x, v[p].y, v[p].z, v[p].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x[2 * e] += bf16_lo_to_f32(wv[e]);
                x[2 * e + 1] += bf16_hi_to_f32(wv[e]);
            }
            if (last_seg) {
                const int n_valid = a.r - 8 * static_cast<int>((pass0 + p) * 64u + ln);
#pragma unroll
                for (int e = 1; e < 8; ++e)
                    if (e >= n_valid) x[e] = x[0];
            }
            v[p] = u32x4{pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]),
                         pack_bf16x2(x[6], x[7])};
        }
    }

    uint32_t *codes = reinterpret_cast<uint32_t *>(
        static_cast<uint8_t *>(const_cast<void *>(codesp.p[rank])) +
        static_cast<int64_t>(t) * a.pitch_codes);
    uint32_t w[P];
    uint64_t w64[P];  // GEN
    if constexpr (STATIC) {
        // code = clamp(rint(x * inv), -8, 7), sent as code + 8.  The product is rounded
        // to fp32 before the integer rounding (a fused multiply-add would round once
        // and differ at near-ties).  Adding 1.5 * 2^23 + 8 to the clamped product leaves
        // rint(.) + 8 in the sum's low byte: the sum's unit in the last place is 1, the
        // addition rounds to nearest even, and the offset is even, so ties fall as rint's.
        __syncthreads();  // the table slice is complete (the only barrier: one per workgroup)
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const u32x4 ia = l_tab[p * 64 + ln], ib = l_tab[64 * P + p * 64 + ln];
            const float iv[8] = {__uint_as_float(ia.x), __uint_as_float(ia.y), __uint_as_float(ia.z),
                                 __uint_as_float(ia.w), __uint_as_float(ib.x), __uint_as_float(ib.y),
                                 __uint_as_float(ib.z), __uint_as_float(ib.w)};
            const uint32_t wv[4] = {v[p].x, v[p].y, v[p].z, v[p].w};
            if constexpr (GEN) {
                // b-bit codes: clamp to -2^(b-1) .. 2^(b-1) - 1, then the same rounding by
                // addition with 2^(b-1) (even for every b >= 2) in place of 8: the sum's low
                // byte is the field code + 2^(b-1)
                const float half = static_cast<float>(1u << (static_cast<uint32_t>(a.bits) - 1u));
                const float magic = 12582912.0f + half;
                uint32_t n[8];
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const float x0 = bf16_lo_to_f32(wv[e2]), x1 = bf16_hi_to_f32(wv[e2]);
                    const float c0 = __builtin_amdgcn_fmed3f(x0 * iv[2 * e2], -half, half - 1.0f);
                    const float c1 = __builtin_amdgcn_fmed3f(x1 * iv[2 * e2 + 1], -half, half - 1.0f);
                    n[2 * e2] = __float_as_uint(c0 + magic) & 0xFFu;
                    n[2 * e2 + 1] = __float_as_uint(c1 + magic) & 0xFFu;
                }
                const uint32_t lo = n[0] | (n[1] << 8) | (n[2] << 16) | (n[3] << 24);
                const uint32_t hi = n[4] | (n[5] << 8) | (n[6] << 16) | (n[7] << 24);
                switch (a.bits) {
                case 2: w64[p] = pack_codes<2>(lo, hi); break;
                case 3: w64[p] = pack_codes<3>(lo, hi); break;
                case 5: w64[p] = pack_codes<5>(lo, hi); break;
                case 6: w64[p] = pack_codes<6>(lo, hi); break;
                default: w64[p] = pack_codes<8>(lo, hi); break;
                }
            } else {
                uint32_t by[4];
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const float x0 = bf16_lo_to_f32(wv[e2]), x1 = bf16_hi_to_f32(wv[e2]);
                    const float c0 = __builtin_amdgcn_fmed3f(x0 * iv[2 * e2], -8.0f, 7.0f);
                    const float c1 = __builtin_amdgcn_fmed3f(x1 * iv[2 * e2 + 1], -8.0f, 7.0f);
                    const uint32_t n0 = __float_as_uint(c0 + 12582920.0f);
                    const uint32_t n1 = __float_as_uint(c1 + 12582920.0f);
                    by[e2] = (n1 << 4) | n0;  // low byte: the pair's two nibbles
                }
                const uint32_t lo = __builtin_amdgcn_perm(by[1], by[0], 0x00000400u);
                const uint32_t hi = __builtin_amdgcn_perm(by[3], by[2], 0x00000400u);
                w[p] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
            }
        }
    } else {
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
            const float s32 = GEN ? span / a.qmax : div_by_15(span);  // (IEEE division)
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
                if constexpr (GEN) {
                    // one code per byte, in feature order (the conversion saturates at 255,
                    // which is the clamp the 8-bit width needs; narrower widths cannot overshoot)
                    uint32_t b = __builtin_amdgcn_cvt_pk_u8_f32(pr[0], 0u, 0u);
                    b = __builtin_amdgcn_cvt_pk_u8_f32(pr[1], 1u, b);
                    b = __builtin_amdgcn_cvt_pk_u8_f32(pr[2], 2u, b);
                    b = __builtin_amdgcn_cvt_pk_u8_f32(pr[3], 3u, b);
                    h[half] = b;
                } else {
                    uint32_t b = __builtin_amdgcn_cvt_pk_u8_f32(pr[1], 0u, 0u);
                    b = __builtin_amdgcn_cvt_pk_u8_f32(pr[0], 1u, b);
                    b = __builtin_amdgcn_cvt_pk_u8_f32(pr[3], 2u, b);
                    b = __builtin_amdgcn_cvt_pk_u8_f32(pr[2], 3u, b);
                    h[half] = (b << 12) | b;
                }
            }
            if constexpr (GEN) {
                switch (a.bits) {
                case 2: w64[p] = pack_codes<2>(h[0], h[1]); break;
                case 3: w64[p] = pack_codes<3>(h[0], h[1]); break;
                case 5: w64[p] = pack_codes<5>(h[0], h[1]); break;
                case 6: w64[p] = pack_codes<6>(h[0], h[1]); break;
                default: w64[p] = pack_codes<8>(h[0], h[1]); break;
                }
            } else {
                w[p] = __builtin_amdgcn_perm(h[1], h[0], 0x07050301u);
            }
        }
    }
    if constexpr (GEN) {
        // b bytes per chunk at byte chunk * b of the row (the row's pitch has room for whole
        // chunks); a ragged last chunk's unused bits are zero.  As below, the segment's codes
        // -- one contiguous piece of the row, 64 b bytes per pass -- are parked in the wave's
        // slot area and leave as 128-bit stores; the last, partial 16 bytes go out byte by byte.
        // (Measured at the Llama shape: 58 -> 50 us at 8 bits, 57 -> 53 at 6, 52 -> 49 at 3; at 2
        // and 5 bits, and in the static mode, each lane's own narrow store is as fast or faster
        // and stays.)
        uint8_t *l_codes = slots;  // (the host gives the area 64 P b bytes at least)
        const uint32_t b = static_cast<uint32_t>(a.bits);
        if (STATIC || b == 2 || b == 5) {
            uint8_t *cb = reinterpret_cast<uint8_t *>(codes);
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const uint32_t chunk = (pass0 + p) * 64u + ln;
                uint64_t wv = w64[p];
                if (!active) continue;
                if (last_seg) {
                    const int n_valid = a.r - 8 * static_cast<int>(chunk);
                    if (n_valid < 8 && n_valid > 0) wv &= (1ull << (b * static_cast<uint32_t>(n_valid))) - 1ull;
                    if (chunk >= static_cast<uint32_t>(a.chunks)) continue;
                }
                uint8_t *dst = cb + chunk * b;
                const uint32_t lo = static_cast<uint32_t>(wv), hi = static_cast<uint32_t>(wv >> 32);
                switch (b) {
                case 2: *reinterpret_cast<uint16_t *>(dst) = static_cast<uint16_t>(lo); break;
                case 3:
                    *reinterpret_cast<u16_a1 *>(dst) = static_cast<uint16_t>(lo);
                    dst[2] = static_cast<uint8_t>(lo >> 16);
                    break;
                case 5:
                    *reinterpret_cast<u32_a1 *>(dst) = lo;
                    dst[4] = static_cast<uint8_t>(hi);
                    break;
                case 6:
                    *reinterpret_cast<u32_a2 *>(dst) = lo;
                    *reinterpret_cast<uint16_t *>(dst + 4) = static_cast<uint16_t>(hi);
                    break;
                default: *reinterpret_cast<uint2 *>(dst) = make_uint2(lo, hi); break;
                }
            }
            return;
        }
        if constexpr (!STATIC) {
    #pragma unroll
            for (int p = 0; p < P; ++p) {
                uint64_t wv = w64[p];
                if (last_seg) {
                    const int n_valid = a.r - 8 * static_cast<int>((pass0 + p) * 64u + ln);
                    if (n_valid < 8 && n_valid > 0) wv &= (1ull << (b * static_cast<uint32_t>(n_valid))) - 1ull;
                }
                uint8_t *d = l_codes + (static_cast<uint32_t>(p) * 64u + ln) * b;
                const uint32_t lo = static_cast<uint32_t>(wv), hi = static_cast<uint32_t>(wv >> 32);
                switch (b) {
                case 3:
                    d[0] = static_cast<uint8_t>(lo);
                    d[1] = static_cast<uint8_t>(lo >> 8);
                    d[2] = static_cast<uint8_t>(lo >> 16);
                    break;
                case 6:
                    *reinterpret_cast<uint16_t *>(d) = static_cast<uint16_t>(lo);
                    *reinterpret_cast<uint16_t *>(d + 2) = static_cast<uint16_t>(lo >> 16);
                    *reinterpret_cast<uint16_t *>(d + 4) = static_cast<uint16_t>(hi);
                    break;
                default: *reinterpret_cast<uint2 *>(d) = make_uint2(lo, hi); break;
                }
            }
            wave_lds_fence();
            const uint32_t nc = last_seg ? static_cast<uint32_t>(a.chunks) - pass0 * 64u : 64u * P;  // chunks to store
            const uint32_t nbytes = nc * b, full = nbytes >> 4;
            uint8_t *dst = reinterpret_cast<uint8_t *>(codes) + 64u * b * pass0;
            for (uint32_t u0 = 0; u0 < full; u0 += 64) {
                const uint32_t u = u0 + ln;
                if (u < full && active)
                    __builtin_nontemporal_store(reinterpret_cast<const u32x4 *>(l_codes)[u],
                                                reinterpret_cast<u32x4 *>(dst + 16u * u));
            }
            const uint32_t c = 16u * full + ln;
            if (c < nbytes && active) dst[c] = l_codes[c];
        }
        return;
    }
    // The segment's codes are one contiguous piece of the row (256 bytes per pass).  They leave
    // as 128-bit stores: every lane parks its P words in LDS in chunk order and takes four
    // consecutive ones back -- 1 KB per store instruction instead of 256 bytes, which the
    // memory system takes markedly better in a bare streaming kernel.
    // A last segment's final one to three words go out singly, so that nothing past the
    // row's codes is written.
    {
        // (in the wave's slot area, which nothing reads any more; the host gives it 256 P bytes at least)
        uint32_t *l_codes = reinterpret_cast<uint32_t *>(slots);
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (last_seg) {
                const int n_valid = a.r - 8 * static_cast<int>((pass0 + p) * 64u + ln);
                if (n_valid < 8) w[p] &= (1u << (4 * (n_valid & 7))) - 1u;
            }
            l_codes[p * 64 + ln] = w[p];
        }
        wave_lds_fence();
        const uint32_t nc = last_seg ? static_cast<uint32_t>(a.chunks) - pass0 * 64u : 64u * P;  // chunks to store
        const uint32_t full = nc >> 2;
        uint8_t *dst = reinterpret_cast<uint8_t *>(codes) + 256u * pass0;
#pragma unroll
        for (uint32_t u0 = 0; u0 < 16u * P; u0 += 64) {
            const uint32_t u = u0 + ln;
            if (u < full && active)
                __builtin_nontemporal_store(reinterpret_cast<const u32x4 *>(l_codes)[u],
                                            reinterpret_cast<u32x4 *>(dst + 16u * u));
        }
        const uint32_t c = 4u * full + ln;
        if (c < nc && active) __builtin_nontemporal_store(l_codes[c], reinterpret_cast<uint32_t *>(dst + 4u * c));
    }
}

template <int LPG, int P, bool STATIC, bool GEN, bool HOP = false>
static hipError_t launch_direct_lp(const EncodeArgs &a, const RankPtrs &Y, const RankPtrs &codes,
                                   const RankPtrs &scale, const RankPtrs &zero,
                                   const RankPtrs &outl, size_t lds, dim3 grid, hipStream_t s,
                                   const HopIn &hin)
{
    hipError_t e = hipSuccess;
    if (lds > 65536)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_encode_direct<LPG, P, STATIC, GEN, HOP>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return e;
    launch_kernel(k_encode_direct<LPG, P, STATIC, GEN, HOP>, grid, dim3(256), lds, s, a, Y, codes, scale, zero, outl, hin);
    return hipGetLastError();
}

// Direct path: one wave per (rank, row, segment).
static hipError_t launch_direct(const EncodeArgs &a_in, const RankPtrs &Y_in, const RankPtrs &codes_in,
                                const RankPtrs &scale_in, const RankPtrs &zero_in,
                                const RankPtrs &outl_in, hipStream_t s, const HopIn *hop)
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
        a.off_drec2 = o.drec2;
    }
    // LDS slots per wave: room for a segment with 5/4 of the row's average share of the slots
    // and 8 more (a denser segment gathers the rest from memory), never more than a segment
    // or the row can have
    a.patch_slots = (5 * a.dslots / a.segs) / 4 + 8;
    if (a.patch_slots > a.dslots) a.patch_slots = a.dslots;
    if (a.patch_slots > 64 * P) a.patch_slots = 64 * P;
    if (a.patch_slots < 8 * P) a.patch_slots = 8 * P;  // (the codes pass through the same area: 256 P bytes)
    if (a.bits != 4 && a.patch_slots < 2 * P * a.bits) a.patch_slots = 2 * P * a.bits;  // (other widths: 64 P b bytes)
    const bool is_static = a.inv_c != nullptr;
    const bool is_gen = a.bits != 4;
    // per wave: slots (+ the groups' scale / zero pairs); static mode: + the workgroup's table slice
    const size_t lds = 4 * (32u * static_cast<size_t>(a.patch_slots) + (is_static ? 0u : 4u * (64 * P / lpg))) +
                       (is_static ? 64u * 32u * static_cast<size_t>(P) : 0u);

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
            if (scale.p[i]) scale.p[i] = static_cast<const uint8_t *>(scale.p[i]) + row0 * a.pitch_meta;
            if (zero.p[i]) zero.p[i] = static_cast<const uint8_t *>(zero.p[i]) + row0 * a.pitch_meta;
            if (outl.p[i]) outl.p[i] = static_cast<const uint8_t *>(outl.p[i]) + row0 * a.pitch_outl;
        }
        HopIn hin = {};
        if (hop) {
            hin.accum = hop->accum;
            for (int i = 0; i < a.n_ranks; ++i) {
                hin.codes[i] = static_cast<const uint8_t *>(hop->codes[i]) + row0 * a.pitch_codes;
                hin.scale[i] = static_cast<const uint8_t *>(hop->scale[i]) + row0 * a.pitch_meta;
                hin.zero[i] = static_cast<const uint8_t *>(hop->zero[i]) + row0 * a.pitch_meta;
                if (hop->outl[i]) hin.outl[i] = static_cast<const uint8_t *>(hop->outl[i]) + row0 * a.pitch_outl;
            }
        }
        a.n_tasks = a.T * a.segs;  // per rank
        // workgroups of 4 tasks; static mode: (group of 4 rows, segment) pairs
        const dim3 grid(static_cast<unsigned>(is_static ? (a.T + 3) / 4 * a.segs : (a.n_tasks + 3) / 4),
                        static_cast<unsigned>(a.n_ranks));
#define TPQ_DIRECT_P(LPG, PP)                                                                       \
    case PP:                                                                                        \
        if constexpr (LPG != 0) {                                                                   \
            if (hop) {                                                                              \
                e = launch_direct_lp<LPG, PP, false, false, true>(a, Y, codes, scale, zero, outl, lds, grid, s, hin); \
                break;                                                                              \
            }                                                                                       \
        }                                                                                           \
        e = is_gen ? launch_direct_lp<LPG, PP, LPG == 0, true>(a, Y, codes, scale, zero, outl, lds, grid, s, hin) \
                   : launch_direct_lp<LPG, PP, LPG == 0, false>(a, Y, codes, scale, zero, outl, lds, grid, s, hin); \
        break;
#define TPQ_DIRECT(LPG)                                                                      \
    switch (P) {                                                                             \
        TPQ_DIRECT_P(LPG, 1) TPQ_DIRECT_P(LPG, 2) TPQ_DIRECT_P(LPG, 3) TPQ_DIRECT_P(LPG, 4)  \
        TPQ_DIRECT_P(LPG, 5)                                                                 \
    default: return hipErrorInvalidValue;                                                    \
    }
        switch (is_static ? 0 : lpg) {
        case 0: TPQ_DIRECT(0) break;  // static symmetric mode: no groups
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

int launch_encode(const EncodeArgs &a, const RankPtrs &Y, const RankPtrs &codes,
                  const RankPtrs &scale, const RankPtrs &zero, const RankPtrs &outl,
                  hipStream_t s, const HopIn *hop)
{
    const int lpg = a.G / 8;
    if (lpg != 4 && lpg != 8 && lpg != 16 && lpg != 32) return TPQ_ERR_UNSUPPORTED;
    if (a.T <= 0) return TPQ_OK;
    if (a.r > 0) return hip_result(launch_direct(a, Y, codes, scale, zero, outl, s, hop));

    // every feature selected: rows are handed over in blocks that fit the grid
    for (int64_t row0 = 0; row0 < a.T; row0 += 65535) {
        EncodeArgs b = a;
        RankPtrs Yb = Y, ob = outl;
        b.T = a.T - row0 < 65535 ? a.T - row0 : 65535;
        for (int i = 0; i < a.n_ranks; ++i) {
            Yb.p[i] = static_cast<const uint8_t *>(Y.p[i]) + row0 * a.ldY * 2;
            ob.p[i] = static_cast<const uint8_t *>(outl.p[i]) + row0 * a.pitch_outl;
        }
        const dim3 grid(static_cast<unsigned>((a.k + 255) / 256), static_cast<unsigned>(b.T),
                        static_cast<unsigned>(a.n_ranks));
        HopIn hb = {};
        if (hop)
            for (int i = 0; i < a.n_ranks; ++i)
                hb.outl[i] = static_cast<const uint8_t *>(hop->outl[i]) + row0 * a.pitch_outl;
        launch_kernel(k_copy_selected, grid, dim3(256), 0, s, b, Yb, ob, hb);
    }
    return hip_result(hipGetLastError());
}

}  // namespace tpq
