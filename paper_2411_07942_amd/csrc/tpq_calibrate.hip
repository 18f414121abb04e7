// tpq_calibrate kernels: per-feature min / max of a calibration sequence, the
// moving-average update of Eq. (1), (2), and the final range aggregation and top-k
// selection (paper Sec. 3).
#include "tpq_device.h"
#include "tpq_internal.h"

namespace tpq {

constexpr int kStripLanes = 64;        // lanes across columns; 8 columns per lane
constexpr int kStripCols = 8 * kStripLanes;
constexpr int kWavesPerBlock = 8;      // waves of a block share columns, split rows
constexpr int kUnroll = 8;             // rows in flight per lane
// Workspace: kCalCounters 32-bit arrival counters (one per column strip; zero between calls),
// then the partial minima / maxima as [part][0 = min, 1 = max][E] floats.
constexpr int kCalCounters = TPQ_MAX_E / kStripCols;  // 64
constexpr size_t kCalCounterBytes = 256;
static_assert(kCalCounters * 4 <= kCalCounterBytes, "counters fit their area");

size_t calibrate_workspace_bytes(int E)
{
    return kCalCounterBytes + static_cast<size_t>(kCalMaxParts) * 2u * static_cast<size_t>(E) * sizeof(float);
}

// How many row slices ("parts") a sequence of S rows is cut into.  Each (column strip,
// part) is one workgroup of 8 waves; two such workgroups per compute unit keep the whole
// machine reading with nothing left over for a second round, which a partly filled round
// would make as long as a full one.
int calibrate_parts(int64_t S, int E, int compute_units, int max_parts)
{
    const int strips = (E + kStripCols - 1) / kStripCols;
    int64_t parts = (2 * static_cast<int64_t>(compute_units)) / strips;
    // at least one row per wave and unrolled step where S allows
    if (parts > S / (kWavesPerBlock * kUnroll)) parts = S / (kWavesPerBlock * kUnroll);
    if (parts > max_parts) parts = max_parts;
    if (parts < 1) parts = 1;
    return static_cast<int>(parts);
}

typedef unsigned int u32x4_cal __attribute__((ext_vector_type(4)));

// Column min / max over one slice of rows, and -- in the workgroup that finishes a strip
// last -- the moving-average update of Eq. (1), (2) for the strip's features.
// Lane l of every wave owns columns 8*(64*blockIdx.x + l) .. +7 and keeps 8 running minima
// and maxima in registers; the block's waves take interleaved rows, kUnroll 128-bit loads in
// flight each, and are combined through LDS.  The upper bf16 of a word is compared as the
// whole word (it orders like the value itself; the low half is masked off at the end).
// Partials go to `partial` as [part][0 = min, 1 = max][E]; then the workgroup takes a ticket
// from its strip's counter, and the one that draws the last ticket reads the strip's partials
// back (they are in memory: every workgroup fenced before its ticket), applies the update and
// leaves the counter at zero for the next call.  Minimum and maximum are exact and
// order-free, so the result does not depend on which workgroup comes last.
__global__ __launch_bounds__(kStripLanes *kWavesPerBlock) void k_colminmax_ema(
    const uint16_t *__restrict__ Y, int64_t S, int64_t ldY, int E, int rows_per_part, int parts,
    uint32_t *__restrict__ counters, float *__restrict__ partial, int first, float gamma,
    float *__restrict__ m, float *__restrict__ M)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int col8 = blockIdx.x * kStripLanes + lane;  // which group of 8 columns
    const bool live = col8 * 8 < E;
    const int64_t row0 = static_cast<int64_t>(blockIdx.y) * rows_per_part;
    int64_t row1 = row0 + rows_per_part;
    if (row1 > S) row1 = S;

    float mn[8], mx[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        mn[e] = 3.4028235e38f;   // every finite bf16 value lies inside (-FLT_MAX, FLT_MAX)
        mx[e] = -3.4028235e38f;
    }
    if (live) {
        const u32x4_cal *p = reinterpret_cast<const u32x4_cal *>(Y + col8 * 8);
        const int64_t stride = ldY / 8;  // in 16-byte units
        auto fold = [&](const u32x4_cal &v) {
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lo = bf16_lo_to_f32(w[e]);
                const float hi = __uint_as_float(w[e]);
                mn[2 * e] = fminf(mn[2 * e], lo);
                mx[2 * e] = fmaxf(mx[2 * e], lo);
                mn[2 * e + 1] = fminf(mn[2 * e + 1], hi);
                mx[2 * e + 1] = fmaxf(mx[2 * e + 1], hi);
            }
        };
        int64_t t = row0 + wave;
        for (; t + (kUnroll - 1) * kWavesPerBlock < row1; t += kUnroll * kWavesPerBlock) {
            u32x4_cal v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
                v[u] = __builtin_nontemporal_load(p + (t + u * kWavesPerBlock) * stride);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) fold(v[u]);
        }
        for (; t < row1; t += kWavesPerBlock) fold(__builtin_nontemporal_load(p + t * stride));
#pragma unroll
        for (int e = 1; e < 8; e += 2) {
            mn[e] = __uint_as_float(__float_as_uint(mn[e]) & 0xFFFF0000u);
            mx[e] = __uint_as_float(__float_as_uint(mx[e]) & 0xFFFF0000u);
        }
    }

    __shared__ float red[kWavesPerBlock][2][8][kStripLanes];
    __shared__ uint32_t ticket;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        red[wave][0][e][lane] = mn[e];
        red[wave][1][e][lane] = mx[e];
    }
    __syncthreads();
    // thread (wave, lane): each of the 8 waves finishes one of the 8 features of every
    // lane's column group
    const int j = col8 * 8 + wave;  // this thread's feature
    if (live) {
        float a = red[0][0][wave][lane], b = red[0][1][wave][lane];
#pragma unroll
        for (int w2 = 1; w2 < kWavesPerBlock; ++w2) {
            a = fminf(a, red[w2][0][wave][lane]);
            b = fmaxf(b, red[w2][1][wave][lane]);
        }
        partial[(static_cast<int64_t>(blockIdx.y) * 2 + 0) * E + j] = a;
        partial[(static_cast<int64_t>(blockIdx.y) * 2 + 1) * E + j] = b;
    }
    // the partials are in memory before the ticket is drawn ...
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) ticket = atomicAdd(&counters[blockIdx.x], 1u);
    __syncthreads();
    if (ticket != static_cast<uint32_t>(parts) - 1u) return;
    // ... and the last workgroup of the strip sees every other one's
    __threadfence();
    if (live) {
        float cmin = 3.4028235e38f, cmax = -3.4028235e38f;
        for (int p = 0; p < parts; ++p) {
            cmin = fminf(cmin, __hip_atomic_load(&partial[(2 * static_cast<int64_t>(p)) * E + j], __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT));
            cmax = fmaxf(cmax, __hip_atomic_load(&partial[(2 * static_cast<int64_t>(p) + 1) * E + j],
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        }
        cmin += 0.0f;  // a zero is taken as +0
        cmax += 0.0f;
        if (first) {
            m[j] = cmin;
            M[j] = cmax;
        } else {
            const float keep = 1.0f - gamma;
            float x = keep * m[j];
            float y = gamma * cmin;
            m[j] = x + y;
            x = keep * M[j];
            y = gamma * cmax;
            M[j] = x + y;
        }
    }
    if (threadIdx.x == 0) counters[blockIdx.x] = 0u;  // ready for the next call
}

int launch_colminmax_ema(const uint16_t *Y, int64_t S, int64_t ldY, int E, int first,
                         float gamma, float *m, float *M, void *ws, int max_parts, hipStream_t s)
{
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return hip_result(e);
    const int parts = calibrate_parts(S, E, cus, max_parts);
    const int rows_per_part = static_cast<int>((S + parts - 1) / parts);
    // the last parts may be empty when S is not a multiple; recompute the live count
    const int live_parts = static_cast<int>((S + rows_per_part - 1) / rows_per_part);
    const dim3 grid((E + kStripCols - 1) / kStripCols, live_parts);
    uint32_t *counters = static_cast<uint32_t *>(ws);
    float *partial = reinterpret_cast<float *>(static_cast<uint8_t *>(ws) + kCalCounterBytes);
    k_colminmax_ema<<<grid, kStripLanes * kWavesPerBlock, 0, s>>>(Y, S, ldY, E, rows_per_part, live_parts, counters,
                                                                   partial, first, gamma, m, M);
    return hip_result(hipGetLastError());
}

// ---- finalize -------------------------------------------------------------------

// R = 2*max(-m, M) per device, Rbar = sum over devices in ascending order.
__global__ void k_ranges(const float *__restrict__ m, const float *__restrict__ M, int N, int E,
                         float *__restrict__ R, float *__restrict__ Rbar)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= E) return;
    float acc = 0.f;
    for (int i = 0; i < N; ++i) {
        const float lo = -m[static_cast<int64_t>(i) * E + j];
        const float hi = M[static_cast<int64_t>(i) * E + j];
        float r = 2.0f * (lo > hi ? lo : hi);
        r += 0.0f;
        if (R) R[static_cast<int64_t>(i) * E + j] = r;
        acc = i == 0 ? r : acc + r;
    }
    Rbar[j] = acc;
}

// Rank of feature j in the order (Rbar descending, index ascending), by counting
// the features that come before it.  E <= 32768 and this runs once per block of
// the model, offline, so the quadratic count is affordable and needs no sort.
__global__ __launch_bounds__(256) void k_rank(const float *__restrict__ Rbar, int E, int k,
                                              int32_t *__restrict__ rank_of,
                                              int32_t *__restrict__ idx_ranked)
{
    __shared__ float tile[256];
    const int j = blockIdx.x * 256 + threadIdx.x;
    const float mine = j < E ? Rbar[j] : 0.f;
    int before = 0;
    for (int base = 0; base < E; base += 256) {
        const int o = base + threadIdx.x;
        tile[threadIdx.x] = o < E ? Rbar[o] : -1.0f;  // ranges are >= 0
        __syncthreads();
        const int n = E - base < 256 ? E - base : 256;
        for (int q = 0; q < n; ++q) {
            const float other = tile[q];
            before += (other > mine) || (other == mine && base + q < j);
        }
        __syncthreads();
    }
    if (j < E) {
        rank_of[j] = before;
        if (before < k && idx_ranked) idx_ranked[before] = j;
    }
}

// Ascending list of the selected features: position = selected features below j.
__global__ __launch_bounds__(256) void k_select_sorted(const int32_t *__restrict__ rank_of, int E,
                                                       int k, int32_t *__restrict__ idx_sorted)
{
    __shared__ int32_t tile[256];
    const int j = blockIdx.x * 256 + threadIdx.x;
    int below = 0;
    for (int base = 0; base <= static_cast<int>(blockIdx.x) * 256; base += 256) {
        const int o = base + threadIdx.x;
        tile[threadIdx.x] = (o < E && rank_of[o] < k) ? 1 : 0;
        __syncthreads();
        for (int q = 0; q < 256; ++q) below += (base + q < j) ? tile[q] : 0;
        __syncthreads();
    }
    if (j < E && rank_of[j] < k) idx_sorted[below] = j;
}

int launch_finalize(const float *m, const float *M, int N, int E, int k, float *R, float *Rbar,
                    int32_t *idx_sorted, int32_t *idx_ranked, int32_t *ws, hipStream_t s)
{
    const int blocks = (E + 255) / 256;
    k_ranges<<<blocks, 256, 0, s>>>(m, M, N, E, R, Rbar);
    k_rank<<<blocks, 256, 0, s>>>(Rbar, E, k, ws, idx_ranked);
    if (k > 0) k_select_sorted<<<blocks, 256, 0, s>>>(ws, E, k, idx_sorted);
    return hip_result(hipGetLastError());
}

}  // namespace tpq
