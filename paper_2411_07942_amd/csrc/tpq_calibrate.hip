// tpq_calibrate kernels: per-feature min / max of a calibration sequence, the
// moving-average update of Eq. (1), (2), and the final range aggregation and top-k
// selection (paper Sec. 3).
#include <atomic>
#include <mutex>

#include "tpq_device.h"
#include "tpq_internal.h"

namespace tpq {

constexpr int kStripLanes = 64;        // lanes across columns; 8 columns per lane
constexpr int kStripCols = 8 * kStripLanes;
constexpr int kWavesPerBlock = 8;      // waves of a block share columns, split rows
constexpr int kUnroll = 8;             // rows in flight per lane
// Workspace: the partial minima / maxima as [part][0 = min, 1 = max][E] floats.
size_t calibrate_workspace_bytes(int E)
{
    return static_cast<size_t>(kCalMaxParts) * 2u * static_cast<size_t>(E) * sizeof(float);
}

// How many row slices ("parts") a sequence of S rows is cut into.  Each (column strip,
// part) is one workgroup of 8 waves with 8 rows of loads in flight per wave; one such
// workgroup per compute unit reads fastest on this part (measured: two per unit 8 % slower,
// three and four slower still), and nothing is left over for a second round, which a partly
// filled round would make as long as a full one.
int calibrate_parts(int64_t S, int E, int compute_units, int max_parts)
{
    const int strips = (E + kStripCols - 1) / kStripCols;
    int64_t parts = static_cast<int64_t>(compute_units) / strips;
    // at least one row per wave and unrolled step where S allows
    if (parts > S / (kWavesPerBlock * kUnroll)) parts = S / (kWavesPerBlock * kUnroll);
    if (parts > max_parts) parts = max_parts;
    if (parts < 1) parts = 1;
    return static_cast<int>(parts);
}

typedef unsigned int u32x4_cal __attribute__((ext_vector_type(4)));

// Column min / max over one slice of rows.  Lane l of every wave owns columns
// 8*(64*blockIdx.x + l) .. +7 and keeps 8 running minima and maxima in registers;
// the block's waves take interleaved rows, kUnroll 128-bit loads in flight each,
// and are combined through LDS.  The upper bf16 of a word is compared as the whole
// word (it orders like the value itself; the low half is masked off at the end).
// Partials go to `partial` as [part][0 = min, 1 = max][E].
__global__ __launch_bounds__(kStripLanes *kWavesPerBlock) void k_colminmax(
    const uint16_t *__restrict__ Y, int64_t S, int64_t ldY, int E, int rows_per_part,
    float *__restrict__ partial)
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
}

// Combine the parts and apply Eq. (1), (2) to one device's state.  A block owns 64
// features; its 4 waves take interleaved parts and are combined through LDS.
__global__ __launch_bounds__(256) void k_ema(const float *__restrict__ partial, int parts, int E,
                                             int first, float gamma, float *__restrict__ m,
                                             float *__restrict__ M)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = blockIdx.x * 64 + lane;
    float cmin = 3.4028235e38f, cmax = -3.4028235e38f;
    if (j < E) {
        for (int p = wave; p < parts; p += 4) {
            cmin = fminf(cmin, partial[(2 * static_cast<int64_t>(p)) * E + j]);
            cmax = fmaxf(cmax, partial[(2 * static_cast<int64_t>(p) + 1) * E + j]);
        }
    }
    __shared__ float red[4][2][64];
    red[wave][0][lane] = cmin;
    red[wave][1][lane] = cmax;
    __syncthreads();
    if (wave != 0 || j >= E) return;
#pragma unroll
    for (int w2 = 1; w2 < 4; ++w2) {
        cmin = fminf(cmin, red[w2][0][lane]);
        cmax = fmaxf(cmax, red[w2][1][lane]);
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

// The number of compute units of the current device (looked up once per device: the query is
// slow compared with a launch).
static hipError_t compute_units_of_current_device(int *out)
{
    constexpr int kMaxDevices = 64;
    static std::atomic<int> known[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < kMaxDevices) {
        const int c = known[dev].load(std::memory_order_relaxed);
        if (c > 0) {
            *out = c;
            return hipSuccess;
        }
    }
    int cus = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    if (cus < 1) cus = 1;
    if (dev >= 0 && dev < kMaxDevices) known[dev].store(cus, std::memory_order_relaxed);
    *out = cus;
    return hipSuccess;
}

int launch_colminmax_ema(const uint16_t *Y, int64_t S, int64_t ldY, int E, int first,
                         float gamma, float *m, float *M, void *ws, int max_parts, hipStream_t s)
{
    int cus = 0;
    const hipError_t e0 = compute_units_of_current_device(&cus);
    if (e0 != hipSuccess) return hip_result(e0);
    const int parts = calibrate_parts(S, E, cus, max_parts);
    const int rows_per_part = static_cast<int>((S + parts - 1) / parts);
    // the last parts may be empty when S is not a multiple; recompute the live count
    const int live_parts = static_cast<int>((S + rows_per_part - 1) / rows_per_part);
    const dim3 grid((E + kStripCols - 1) / kStripCols, live_parts);
    float *partial = static_cast<float *>(ws);
    k_colminmax<<<grid, kStripLanes * kWavesPerBlock, 0, s>>>(Y, S, ldY, E, rows_per_part, partial);
    k_ema<<<(E + 63) / 64, 256, 0, s>>>(partial, live_parts, E, first, gamma, m, M);
    return hip_result(hipGetLastError());
}

// ---- scratch of tpq_calibrate_fixed ------------------------------------------------
// The partials for callers that cannot bring a workspace: part of the device image, so every
// GPU the library runs on holds its own copy.  Nothing in it has to start at zero: a call
// writes every partial that it reads.  In host code the array's name is only a handle: the
// device address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[TPQ_CALIBRATE_FIXED_SCRATCH_BYTES];
static_assert(TPQ_CALIBRATE_FIXED_SCRATCH_BYTES ==
                  static_cast<size_t>(kCalFixedMaxParts) * 2u * TPQ_CALIBRATE_FIXED_MAX_E * sizeof(float),
              "scratch holds kCalFixedMaxParts slices of partials at the largest E");

int calibrate_fixed_scratch(void **ptr)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *addr[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_result(e);
    if (dev < 0 || dev >= kMaxDevices) return TPQ_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_result(e);
        addr[dev] = p;
    }
    *ptr = addr[dev];
    return TPQ_OK;
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
