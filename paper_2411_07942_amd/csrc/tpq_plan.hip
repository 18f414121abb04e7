// Builds the compaction tables for a static outlier index set (paper Sec. 3: the
// selected features are fixed across sequences and devices, so this runs once
// per block, not per call).  Everything here is offline work on a few thousand
// table entries; clarity wins over speed.
#include "tpq_device.h"
#include "tpq_internal.h"

namespace tpq {

__global__ void k_plan_init(uint8_t *plan, int E, int k, int G, int r, int chunks,
                            int chunks_padded, PlanOffsets o)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        PlanHeader *h = reinterpret_cast<PlanHeader *>(plan);
        h->magic = kPlanMagic;
        h->status = kPlanOk;
        h->E = E;
        h->k = k;
        h->G = G;
        h->r = r;
        h->chunks = chunks;
        h->chunks_padded = chunks_padded;
        h->idx_offset = o.idx;
        h->src_offset = o.src;
        h->pos_offset = o.pos;
        h->pass_col_offset = o.pass_col;
        h->irr_offset = o.irr;
        h->pass_irr_offset = o.pass_irr;
        h->n_irr = 0;
        h->irr_src_offset = o.irr_src;
    }
}

// One thread per feature j: count the selected features below j (binary search
// in idx) and, if j itself is not selected, record src_of[j - count] = j.
// Threads p < k also validate idx[p] and copy it into the plan.
__global__ void k_plan_build(uint8_t *plan, const int32_t *__restrict__ idx, int E, int k, int r,
                             PlanOffsets o)
{
    PlanHeader *h = reinterpret_cast<PlanHeader *>(plan);
    int32_t *pidx = reinterpret_cast<int32_t *>(plan + o.idx);
    uint16_t *src = reinterpret_cast<uint16_t *>(plan + o.src);
    const int j = blockIdx.x * blockDim.x + threadIdx.x;

    if (j < k) {
        const int v = idx[j];
        bool ok = v >= 0 && v < E;
        if (j > 0) ok = ok && v > idx[j - 1];
        if (!ok) h->status = kPlanBadIndex;
        pidx[j] = ok ? v : 0;
    } else if (j < (k + 3) / 4 * 4) {
        pidx[j] = 0;
    }

    if (j < E) {
        // lower bound: number of idx entries < j
        int lo = 0, hi = k;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (idx[mid] < j) lo = mid + 1; else hi = mid;
        }
        const bool selected = lo < k && idx[lo] == j;
        const int c = j - lo;
        if (!selected && c >= 0 && c < r) src[c] = static_cast<uint16_t>(j);
    }
}

// Positions r .. 8*chunks_padded-1 repeat the last real compacted feature.
__global__ void k_plan_pad(uint8_t *plan, int r, int chunks_padded, PlanOffsets o)
{
    uint16_t *src = reinterpret_cast<uint16_t *>(plan + o.src);
    const int c = r + blockIdx.x * blockDim.x + threadIdx.x;
    if (r > 0 && c < 8 * chunks_padded) src[c] = src[r - 1];
}

// flags[c] = 1 if chunk c cannot be served by one 16-byte access: an outlier sits
// between its first and last feature, or it is the ragged last chunk.
__global__ void k_plan_flags(uint8_t *plan, int r, int chunks, int chunks_padded, int lpg,
                             PlanOffsets o)
{
    const PlanHeader *h = reinterpret_cast<const PlanHeader *>(plan);
    const uint16_t *src = reinterpret_cast<const uint16_t *>(plan + o.src);
    uint16_t *flags = reinterpret_cast<uint16_t *>(plan + o.flags);
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= chunks_padded) return;
    uint16_t f = 0;
    if (h->status == kPlanOk && chunks > 0) {
        if (c < chunks) {
            const bool ragged = 8 * c + 8 > r;
            f = (ragged || src[8 * c + 7] - src[8 * c] != 7) ? 1 : 0;
        } else {
            // beyond the row but inside the last real group: gets a slot whose sources
            // all repeat the last feature
            f = (c / lpg == (chunks - 1) / lpg) ? 1 : 0;
        }
    }
    flags[c] = f;
}

// cpos / irr / irr_src / pass_irr from the flags: the slot of an irregular chunk is
// the number of irregular chunks before it.
__global__ void k_plan_slots(uint8_t *plan, int E, int chunks, int chunks_padded, int slots,
                             PlanOffsets o)
{
    PlanHeader *h = reinterpret_cast<PlanHeader *>(plan);
    const uint16_t *src = reinterpret_cast<const uint16_t *>(plan + o.src);
    const uint16_t *flags = reinterpret_cast<const uint16_t *>(plan + o.flags);
    uint32_t *cpos = reinterpret_cast<uint32_t *>(plan + o.pos);
    uint16_t *irr = reinterpret_cast<uint16_t *>(plan + o.irr);
    uint16_t *pass_irr = reinterpret_cast<uint16_t *>(plan + o.pass_irr);
    uint16_t *irr_src = reinterpret_cast<uint16_t *>(plan + o.irr_src);
    uint16_t *pass_col = reinterpret_cast<uint16_t *>(plan + o.pass_col);
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c > chunks_padded) return;
    int q = 0;
    for (int b = 0; b < c; ++b) q += flags[b];
    if (c == chunks_padded) {  // one extra thread: the totals
        h->n_irr = q;
        pass_irr[chunks_padded / 64] = static_cast<uint16_t>(q);
        pass_col[chunks_padded / 64] = static_cast<uint16_t>(E);
        return;
    }
    if ((c & 63) == 0) {
        pass_irr[c / 64] = static_cast<uint16_t>(q);
        pass_col[c / 64] = c < chunks ? src[8 * c] : static_cast<uint16_t>(E);
    }
    if (h->status != kPlanOk || (c >= chunks && !flags[c])) {
        cpos[c] = kNotRegular | (kNoSlot << 16) | static_cast<uint32_t>(E - 8);
    } else if (flags[c] && q < slots) {
        int safe = src[8 * c];
        if (safe > E - 8) safe = E - 8;  // a 16-byte read from here stays inside the row
        cpos[c] = kNotRegular | (static_cast<uint32_t>(q) << 16) | static_cast<uint32_t>(safe);
        irr[q] = static_cast<uint16_t>(c);
        for (int e = 0; e < 8; ++e) irr_src[8 * q + e] = src[8 * c + e];
    } else {
        cpos[c] = c < chunks ? src[8 * c]
                             : (kNotRegular | (kNoSlot << 16) | static_cast<uint32_t>(E - 8));
    }
}

int launch_plan_build(const tpq_layout *L, const int32_t *idx, void *plan, hipStream_t s)
{
    const int E = L->E, k = L->k, r = L->r;
    const int chunks = chunks_of(r), cp = chunks_padded_of(r);
    const PlanOffsets o = plan_offsets(k, r, L->G);
    uint8_t *p = static_cast<uint8_t *>(plan);
    k_plan_init<<<1, 64, 0, s>>>(p, E, k, L->G, r, chunks, cp, o);
    k_plan_build<<<(E + 255) / 256, 256, 0, s>>>(p, idx, E, k, r, o);
    const int tail = 8 * cp - r;
    if (r > 0 && tail > 0) k_plan_pad<<<(tail + 255) / 256, 256, 0, s>>>(p, r, cp, o);
    if (cp > 0) k_plan_flags<<<(cp + 255) / 256, 256, 0, s>>>(p, r, chunks, cp, L->G / 8, o);
    k_plan_slots<<<(cp + 1 + 255) / 256, 256, 0, s>>>(p, E, chunks, cp, irr_slots_of(k, r, L->G), o);
    return hip_result(hipGetLastError());
}

}  // namespace tpq
