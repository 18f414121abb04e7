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
        h->pass_col_offset = o.pass_col;
        h->dpos_offset = o.dpos;
        h->dirr_offset = o.dirr;
        h->dsel_offset = o.dsel;
        h->pass_dirr_offset = o.pass_dirr;
        h->n_dirr = 0;
        h->dslots = dir_slots_of(k, r);
        h->dpos16_offset = o.dpos16;
        h->dslot8_offset = o.dslot8;
        h->dir_P = dir_passes_of(chunks_padded / 64);
        h->dseg_offset = o.dseg;
        h->drec_offset = o.drec;
        h->drec2_offset = o.drec2;
        h->spass_offset = o.spass;
        h->sblk_offset = o.sblk;
        h->sblk_cap = sblk_cap_of(k, r);
        for (int i = 0; i < 6; ++i) h->reserved[i] = 0;
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

// pass_col[p] = column of the first feature of pass p; pass_col[passes] = E
__global__ void k_plan_pass_col(uint8_t *plan, int E, int chunks, int passes, PlanOffsets o)
{
    const uint16_t *src = reinterpret_cast<const uint16_t *>(plan + o.src);
    uint16_t *pass_col = reinterpret_cast<uint16_t *>(plan + o.pass_col);
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p > passes) return;
    pass_col[p] = (p < passes && 64 * p < chunks) ? src[512 * p] : static_cast<uint16_t>(E);
}

// ---- tables of the encoder that loads each chunk straight from the row -------------

// First column of chunk c's own window: the even column at or below its first feature,
// pulled back so that 8 columns from there stay inside the row.  Chunk 0 starts its
// window at column 0 when selected features precede it and all fits in 16 columns, so
// that its slot can hold them.
__device__ inline int dir_window_a(const uint16_t *src, int c, int E, int r)
{
    const int nv = r - 8 * c < 8 ? r - 8 * c : 8;
    const int c0 = src[8 * c];
    if (c == 0 && c0 > 0 && src[nv - 1] < 16 && E >= 16) return 0;
    const int wa = c0 & ~1;
    return wa < E - 8 ? wa : E - 8;
}

// byte offset of column `col` in the 32 bytes (window a, then window b) of a slot, or -1
__device__ inline int dir_slot_offset(int col, int wa, int E)
{
    int wb = wa + 8;
    if (wb > E - 8) wb = E - 8;
    if (col >= wa && col < wa + 8) return 2 * (col - wa);
    if (col >= wb && col < wb + 8) return 16 + 2 * (col - wb);
    return -1;
}

// dflags[c] = 1 if chunk c needs a slot.
__global__ void k_plan_dflags(uint8_t *plan, int E, int r, int chunks, int chunks_padded,
                              PlanOffsets o)
{
    const PlanHeader *h = reinterpret_cast<const PlanHeader *>(plan);
    const uint16_t *src = reinterpret_cast<const uint16_t *>(plan + o.src);
    uint16_t *dflags = reinterpret_cast<uint16_t *>(plan + o.dflags);
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= chunks_padded) return;
    uint16_t f = 0;
    if (h->status == kPlanOk && c < chunks) {
        const int nv = r - 8 * c < 8 ? r - 8 * c : 8;
        const int c0 = src[8 * c], clast = src[8 * c + nv - 1];
        const int next0 = 8 * c + 8 < r ? src[8 * c + 8] : -1;
        const bool contiguous = nv == 8 && clast == c0 + 7;
        // selected features inside the chunk, between it and the next one (or the row's
        // end), or before the first chunk: this chunk's slot holds them
        const bool hosts = clast - c0 != nv - 1 || (next0 >= 0 ? next0 : E) - clast - 1 > 0 ||
                           (c == 0 && c0 > 0);
        bool slot = !contiguous || hosts;
        if (!slot && (c0 & 1)) {
            // the 8th feature is the first half-word of the next lane's window
            const bool next_ok = (c & 63) != 63 && next0 == c0 + 8 &&
                                 dir_window_a(src, c + 1, E, r) == (c0 & ~1) + 8;
            slot = !next_ok;
        }
        f = slot ? 1 : 0;
    }
    dflags[c] = f;
}

__global__ void k_plan_dslots(uint8_t *plan, int E, int r, int chunks, int chunks_padded,
                              int dslots, PlanOffsets o)
{
    PlanHeader *h = reinterpret_cast<PlanHeader *>(plan);
    const uint16_t *src = reinterpret_cast<const uint16_t *>(plan + o.src);
    const uint16_t *dflags = reinterpret_cast<const uint16_t *>(plan + o.dflags);
    uint32_t *dpos = reinterpret_cast<uint32_t *>(plan + o.dpos);
    uint16_t *dirr = reinterpret_cast<uint16_t *>(plan + o.dirr);
    uint16_t *pass_dirr = reinterpret_cast<uint16_t *>(plan + o.pass_dirr);
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c > chunks_padded) return;
    int q = 0;
    for (int b = 0; b < c; ++b) q += dflags[b];
    if (c == chunks_padded) {
        h->n_dirr = q;
        pass_dirr[chunks_padded / 64] = static_cast<uint16_t>(q);
        return;
    }
    if ((c & 63) == 0) pass_dirr[c / 64] = static_cast<uint16_t>(q);
    // where this chunk's entry sits in the table laid out by segment
    uint16_t *dpos16 = reinterpret_cast<uint16_t *>(plan + o.dpos16);
    uint32_t *dslot8 = reinterpret_cast<uint32_t *>(plan + o.dslot8);
    const int dirP = dir_passes_of(chunks_padded / 64);
    const int pass = c / 64, seg = pass / dirP;
    uint16_t *e16 = dpos16 + (seg * 64 + (c & 63)) * 8 + (pass - seg * dirP);
    if (pass - seg * dirP == 0) {  // entries of passes the segment does not have
        const int left = chunks_padded / 64 - seg * dirP;
        for (int p = left < dirP ? left : dirP; p < 8; ++p) e16[p] = 0;
    }
    if (h->status != kPlanOk || c >= chunks) {
        dpos[c] = kDirAbsent;
        *e16 = 0;
        return;
    }
    const int c0 = src[8 * c];
    if (!dflags[c]) {
        dpos[c] = static_cast<uint32_t>(c0 >> 1) | ((c0 & 1) ? kDirOdd : 0u);
        *e16 = static_cast<uint16_t>((c0 >> 1) | ((c0 & 1) ? kDir16Odd : 0u));
        return;
    }
    if (q >= dslots) {  // the bound of dir_slots_of() does not hold: refuse the plan
        h->status = kPlanInternal;
        dpos[c] = kDirAbsent;
        *e16 = 0;
        return;
    }
    const int nv = r - 8 * c < 8 ? r - 8 * c : 8;
    const int wa = dir_window_a(src, c, E, r);
    dpos[c] = kDirSlot | (static_cast<uint32_t>(q) << 16) | static_cast<uint32_t>(wa >> 1);
    bool wide = false;
    for (int e = 0; e < 8; ++e) {
        const int col = src[8 * c + (e < nv ? e : nv - 1)];  // absent features repeat the last one
        if (dir_slot_offset(col, wa, E) < 0) wide = true;
    }
    uint32_t nib = 0;
    for (int e = 0; e < 8; ++e) {
        const int col = src[8 * c + (e < nv ? e : nv - 1)];
        dirr[8 * q + e] = wide ? static_cast<uint16_t>(kDirWide | col)
                               : static_cast<uint16_t>(dir_slot_offset(col, wa, E));
        if (!wide) nib |= static_cast<uint32_t>(dir_slot_offset(col, wa, E) >> 1) << (4 * e);
    }
    *e16 = static_cast<uint16_t>((wa >> 1) | kDir16Slot);
    int wb = wa + 8;
    if (wb > E - 8) wb = E - 8;
    // does the next lane of the pass load exactly the second window?
    bool next_has_b = false;
    if ((c & 63) != 63 && c + 1 < chunks) {
        const int next_w = dflags[c + 1] ? dir_window_a(src, c + 1, E, r) : (src[8 * (c + 1)] & ~1);
        next_has_b = next_w == wb;
    }
    dslot8[2 * q] = nib;
    dslot8[2 * q + 1] = static_cast<uint32_t>(2 * wb) | (wide ? kDirWide8 : 0u) | (next_has_b ? 0u : kDirLoadB8);
}

// One thread per selected feature: the slot that holds its column.
__global__ void k_plan_dsel(uint8_t *plan, int E, int k, int r, PlanOffsets o)
{
    const PlanHeader *h = reinterpret_cast<const PlanHeader *>(plan);
    const int32_t *pidx = reinterpret_cast<const int32_t *>(plan + o.idx);
    const uint16_t *src = reinterpret_cast<const uint16_t *>(plan + o.src);
    const uint32_t *dpos = reinterpret_cast<const uint32_t *>(plan + o.dpos);
    uint32_t *dsel = reinterpret_cast<uint32_t *>(plan + o.dsel);
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= (k + 3) / 4 * 4) return;
    uint32_t v = kDirFar;
    if (p < k && r > 0 && h->status == kPlanOk) {
        const int j = pidx[p];
        const int f = j - p;                       // compacted features before column j
        const int c = f >= 1 ? (f - 1) / 8 : 0;    // the chunk that holds the one before it
        const uint32_t d = dpos[c];
        if (d & kDirSlot) {
            const int off = dir_slot_offset(j, dir_window_a(src, c, E, r), E);
            if (off >= 0) v = (((d >> 16) & 0x3FFFu) << 5) | static_cast<uint32_t>(off);
        }
    }
    dsel[p] = v;
}

// One thread per segment of the direct encoder: its slots and selected features.
__global__ void k_plan_dseg(uint8_t *plan, int k, int chunks_padded, PlanOffsets o)
{
    const uint16_t *pass_dirr = reinterpret_cast<const uint16_t *>(plan + o.pass_dirr);
    const uint16_t *pass_col = reinterpret_cast<const uint16_t *>(plan + o.pass_col);
    uint32_t *dseg = reinterpret_cast<uint32_t *>(plan + o.dseg);
    const int passes = chunks_padded / 64, P = dir_passes_of(passes);
    const int sg = blockIdx.x * blockDim.x + threadIdx.x;
    if (sg >= dir_segs_of(passes)) return;
    const int p0 = sg * P, p1 = p0 + P < passes ? p0 + P : passes;
    const uint32_t q_lo = pass_dirr[p0], q_hi = pass_dirr[p1];
    const uint32_t s_lo = sg == 0 ? 0u : pass_col[p0] - 512u * p0;
    const uint32_t s_hi = p1 == passes ? static_cast<uint32_t>(k) : pass_col[p1] - 512u * p1;
    dseg[2 * sg] = q_lo | ((q_hi - q_lo) << 16);
    dseg[2 * sg + 1] = s_lo | ((s_hi - s_lo) << 16);
}

// One thread per (segment, lane): the record a lane of the direct encoder starts from.
__global__ void k_plan_drec(uint8_t *plan, int chunks_padded, PlanOffsets o)
{
    const uint32_t *dpos16 = reinterpret_cast<const uint32_t *>(plan + o.dpos16);
    const uint32_t *dslot8 = reinterpret_cast<const uint32_t *>(plan + o.dslot8);
    const uint32_t *dsel = reinterpret_cast<const uint32_t *>(plan + o.dsel);
    const uint32_t *dseg = reinterpret_cast<const uint32_t *>(plan + o.dseg);
    uint32_t *drec = reinterpret_cast<uint32_t *>(plan + o.drec);
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= dir_segs_of(chunks_padded / 64) * 64) return;
    const int sg = i / 64;
    const uint32_t l = i % 64;
    const uint32_t q_lo = dseg[2 * sg] & 0xFFFFu, n_q = dseg[2 * sg] >> 16;
    const uint32_t s_lo = dseg[2 * sg + 1] & 0xFFFFu, n_sel = dseg[2 * sg + 1] >> 16;
    uint32_t *rec = drec + 8 * i;
    for (int w = 0; w < 4; ++w) rec[w] = dpos16[4 * i + w];
    rec[4] = l < n_q ? dslot8[2 * (q_lo + l)] : 0u;
    rec[5] = l < n_q ? dslot8[2 * (q_lo + l) + 1] : 0u;
    rec[6] = l < n_sel ? dsel[s_lo + l] : (q_lo << 5);  // idle lanes read the segment's first slot
    rec[7] = 0u;
    uint32_t *rec2 = reinterpret_cast<uint32_t *>(plan + o.drec2) + 4 * i;
    const uint32_t l2 = l + 64u;
    rec2[0] = l2 < n_q ? dslot8[2 * (q_lo + l2)] : 0u;
    rec2[1] = l2 < n_q ? dslot8[2 * (q_lo + l2) + 1] : 0u;
    rec2[2] = l2 < n_sel ? dsel[s_lo + l2] : (q_lo << 5);
    rec2[3] = 0u;
}

// Store blocks of the decoder, one workgroup of 512 threads per pass, thread = feature.
// FILL = false: count the pass's blocks and narrow entries into spass; FILL = true
// (after k_plan_sblk_offsets): write the entries.
template <bool FILL>
__global__ __launch_bounds__(512) void k_plan_sblk(uint8_t *plan, int r, PlanOffsets o, int cap)
{
    __shared__ uint8_t start[512], kind[512];
    PlanHeader *h = reinterpret_cast<PlanHeader *>(plan);
    const uint16_t *src = reinterpret_cast<const uint16_t *>(plan + o.src);
    uint32_t *spass = reinterpret_cast<uint32_t *>(plan + o.spass);
    uint32_t *sblk = reinterpret_cast<uint32_t *>(plan + o.sblk);
    const int p = blockIdx.x, a0 = threadIdx.x;
    const int c = 512 * p + a0;
    const int n = min(512, r - 512 * p);  // features of this pass
    const bool real = a0 < n;
    start[a0] = real && (a0 == 0 || src[c] != src[c - 1] + 1);
    __syncthreads();
    int rs = a0, re = a0 + 1;  // the run [rs, re) that holds this feature
    if (real) {
        while (!start[rs]) --rs;
        while (re < n && !start[re]) ++re;
    }
    const int len = re - rs;
    // 1: leads a block; 2: narrow
    kind[a0] = !real ? 0 : (len < 8 ? 2 : ((a0 - rs) % 8 == 0 ? 1 : 0));
    __syncthreads();
    int before1 = 0, before2 = 0, n1 = 0, n2 = 0;
    for (int i = 0; i < 512; ++i) {
        const int kd = kind[i];
        n1 += kd == 1;
        n2 += kd == 2;
        if (i < a0) {
            before1 += kd == 1;
            before2 += kd == 2;
        }
    }
    if (!FILL) {
        if (a0 == 0) {
            spass[4 * p + 1] = n1;
            spass[4 * p + 2] = n2;
            spass[4 * p + 3] = 0;
        }
        return;
    }
    const int first = spass[4 * p];
    if (first + n1 + n2 > cap) {
        if (a0 == 0) h->status = kPlanInternal;
        return;
    }
    if (kind[a0] == 1) {
        const int a = a0 + 8 <= re ? a0 : re - 8;
        sblk[first + before1] = src[512 * p + a] | (static_cast<uint32_t>(a) << 16);
    } else if (kind[a0] == 2) {
        sblk[first + n1 + before2] = src[c] | (static_cast<uint32_t>(a0) << 16);
    }
}

__global__ void k_plan_sblk_offsets(uint8_t *plan, int passes, PlanOffsets o)
{
    uint32_t *spass = reinterpret_cast<uint32_t *>(plan + o.spass);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        uint32_t at = 0;
        for (int p = 0; p < passes; ++p) {
            spass[4 * p] = at;
            at += spass[4 * p + 1] + spass[4 * p + 2];
        }
    }
}

// Static symmetric mode (Sec. 3): per device i and compacted position c (feature j =
// src_of[c]): R = 2*max(-m, M), step = R/(2^bits - 1), inv = 1/step; a vanishing range gives 0, 0.
__global__ void k_static_params(const uint8_t *plan, const float *__restrict__ m,
                                const float *__restrict__ M, int E, int r, int stride, float qmax,
                                float *__restrict__ step, float *__restrict__ inv)
{
    const PlanHeader *h = reinterpret_cast<const PlanHeader *>(plan);
    const uint16_t *src = reinterpret_cast<const uint16_t *>(plan + h->src_offset);
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    const int i = blockIdx.y;
    if (c >= stride) return;
    float d = 0.0f, v = 0.0f;
    if (h->magic == kPlanMagic && h->status == kPlanOk && c < r) {
        const int j = src[c];
        const float lo = -m[static_cast<int64_t>(i) * E + j], hi = M[static_cast<int64_t>(i) * E + j];
        float R = 2.0f * (lo > hi ? lo : hi);
        R += 0.0f;
        const float q = R / qmax;
        if (q >= 1e-30f) {
            d = q;
            v = 1.0f / q;
        }
    }
    step[static_cast<int64_t>(i) * stride + c] = d;
    inv[static_cast<int64_t>(i) * stride + c] = v;
}

int launch_static_params(const tpq_layout *L, const void *plan, const float *m, const float *M,
                         int n_ranks, float *step, float *inv, hipStream_t s)
{
    const int stride = 8 * chunks_padded_of(L->r);
    if (stride == 0) return TPQ_OK;
    const dim3 grid((stride + 255) / 256, n_ranks);
    k_static_params<<<grid, 256, 0, s>>>(static_cast<const uint8_t *>(plan), m, M, L->E, L->r, stride,
                                        static_cast<float>((1 << L->bits) - 1), step, inv);
    return hip_result(hipGetLastError());
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
    k_plan_pass_col<<<1, 128, 0, s>>>(p, E, chunks, cp / 64, o);
    if (cp > 0) k_plan_dflags<<<(cp + 255) / 256, 256, 0, s>>>(p, E, r, chunks, cp, o);
    k_plan_dslots<<<(cp + 1 + 255) / 256, 256, 0, s>>>(p, E, r, chunks, cp, dir_slots_of(k, r), o);
    if (cp > 0) k_plan_dseg<<<1, 64, 0, s>>>(p, k, cp, o);
    if (k > 0) k_plan_dsel<<<((k + 3) / 4 * 4 + 255) / 256, 256, 0, s>>>(p, E, k, r, o);
    if (cp > 0) k_plan_drec<<<(dir_segs_of(cp / 64) * 64 + 255) / 256, 256, 0, s>>>(p, cp, o);
    if (cp > 0) {
        k_plan_sblk<false><<<cp / 64, 512, 0, s>>>(p, r, o, sblk_cap_of(k, r));
        k_plan_sblk_offsets<<<1, 64, 0, s>>>(p, cp / 64, o);
        k_plan_sblk<true><<<cp / 64, 512, 0, s>>>(p, r, o, sblk_cap_of(k, r));
    }
    return hip_result(hipGetLastError());
}

}  // namespace tpq
