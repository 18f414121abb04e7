// Builds the compaction tables for a static outlier index set (paper Sec. 3: the
// selected features are fixed across sequences and devices, so this runs once
// per block, not per call).
#include "tpq_device.h"
#include "tpq_internal.h"

namespace tpq {

__global__ void k_plan_init(uint8_t *plan, int E, int k, int G, int r, int chunks,
                            int chunks_padded, int idx_offset, int src_offset)
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
        h->idx_offset = idx_offset;
        h->src_offset = src_offset;
        for (int i = 0; i < 6; ++i) h->pad[i] = 0;
    }
}

// One thread per feature j: count the selected features below j (binary search
// in idx) and, if j itself is not selected, record src_of[j - count] = j.
// Threads p < k also validate idx[p] and copy it into the plan.
__global__ void k_plan_build(uint8_t *plan, const int32_t *__restrict__ idx, int E, int k, int r,
                             int chunks_padded, int idx_offset, int src_offset)
{
    PlanHeader *h = reinterpret_cast<PlanHeader *>(plan);
    int32_t *pidx = reinterpret_cast<int32_t *>(plan + idx_offset);
    uint16_t *src = reinterpret_cast<uint16_t *>(plan + src_offset);
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

// Positions r .. 8*chunks_padded-1 repeat the last real compacted feature.  Runs
// after k_plan_build on the same stream.
__global__ void k_plan_pad(uint8_t *plan, int r, int chunks_padded, int src_offset)
{
    uint16_t *src = reinterpret_cast<uint16_t *>(plan + src_offset);
    const int c = r + blockIdx.x * blockDim.x + threadIdx.x;
    if (r > 0 && c < 8 * chunks_padded) src[c] = src[r - 1];
}

int launch_plan_build(const tpq_layout *L, const int32_t *idx, void *plan, hipStream_t s)
{
    const int E = L->E, k = L->k, r = L->r;
    const int chunks = chunks_of(r), cp = chunks_padded_of(r);
    const int idx_offset = sizeof(PlanHeader);
    const int src_offset = idx_offset + idx_bytes_of(k);
    uint8_t *p = static_cast<uint8_t *>(plan);
    k_plan_init<<<1, 64, 0, s>>>(p, E, k, L->G, r, chunks, cp, idx_offset, src_offset);
    k_plan_build<<<(E + 255) / 256, 256, 0, s>>>(p, idx, E, k, r, cp, idx_offset, src_offset);
    const int tail = 8 * cp - r;
    if (r > 0 && tail > 0) k_plan_pad<<<(tail + 255) / 256, 256, 0, s>>>(p, r, cp, src_offset);
    return hip_result(hipGetLastError());
}

}  // namespace tpq
