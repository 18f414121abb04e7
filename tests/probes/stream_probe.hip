// What the memory system of the GPU it runs on gives a kernel shaped like the codec's encoder,
// but with no arithmetic and no dependent phases: one wavefront per 10240-byte row (640 x 16
// bytes, ten 128-bit loads per lane, all issued at once), four waves per workgroup, rows of a
// 1 GiB buffer (four buffers in rotation, far beyond the caches).
//
//   read        the row is read and reduced to nothing
//   read +1     ... with every 128-bit load starting at an odd bf16 element (2-byte aligned)
//   read +2     ... at an even element that is not a multiple of 8 (4-byte aligned)
//   copy        the row is read and written (1 : 1)
//   4 : 1       the row is read and a quarter of it written -- the encoder's mix
//
// Prints GB/s of bytes moved (read + written).  A measurement aid: nothing in the library,
// the tests or bench.py depends on it.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>

typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef u4 u4_a2 __attribute__((aligned(2)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s (line %d)\n", hipGetErrorString(e_), __LINE__); exit(2); } } while (0)

constexpr int kRow16 = 640;  // 16-byte units per row

// MODE 0: read; 1: copy; 2: read, write a quarter.  OFF: element offset of every load.
template <int MODE, int OFF>
__global__ __launch_bounds__(256) void k_rows(const unsigned short *__restrict__ src, u4 *__restrict__ dst,
                                              u4 *__restrict__ sink, size_t rows)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t row = (size_t)blockIdx.x * 4 + wave;
    if (row >= rows) return;
    const unsigned short *s = src + row * kRow16 * 8;
    u4 v[10];
#pragma unroll
    for (int p = 0; p < 10; ++p) {
        const int c = p * 64 + lane;
        // (the last 16 bytes of a row are left out when the loads are shifted)
        v[p] = (OFF == 0 || c < kRow16 - 1) ? __builtin_nontemporal_load((const u4_a2 *)(s + c * 8 + OFF)) : u4{0, 0, 0, 0};
    }
    if (MODE == 0) {
        u4 acc = {0, 0, 0, 0};
#pragma unroll
        for (int p = 0; p < 10; ++p) acc ^= v[p];
        if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u) sink[0] = acc;  // never true: keeps the loads
    } else if (MODE == 1) {
        u4 *d = dst + row * kRow16;
#pragma unroll
        for (int p = 0; p < 10; ++p) __builtin_nontemporal_store(v[p], &d[p * 64 + lane]);
    } else {
        u4 *d = dst + row * (kRow16 / 4);  // 160 x 16 bytes per row
        __builtin_nontemporal_store(v[0] ^ v[3] ^ v[6] ^ v[9], &d[lane]);
        __builtin_nontemporal_store(v[1] ^ v[4] ^ v[7], &d[64 + lane]);
        if (lane < 32) __builtin_nontemporal_store(v[2] ^ v[5] ^ v[8], &d[128 + lane]);
    }
}

template <typename F>
static float time_ms(F f, int n = 10)
{
    hipEvent_t a, b;
    CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    for (int i = 0; i < 3; ++i) f(i);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(a));
    for (int i = 0; i < n; ++i) f(i);
    CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
    float ms;
    CK(hipEventElapsedTime(&ms, a, b));
    return ms / n;
}

int main()
{
    const size_t bytes = 1ull << 30;
    const size_t rows = bytes / (kRow16 * 16);
    const int NB = 4;
    unsigned short *src[NB]; u4 *dst[NB], *sink;
    for (int i = 0; i < NB; ++i) {
        CK(hipMalloc(&src[i], bytes)); CK(hipMalloc(&dst[i], bytes));
        CK(hipMemset(src[i], i + 1, bytes)); CK(hipMemset(dst[i], 0, bytes));
    }
    CK(hipMalloc(&sink, 64));
    const unsigned grid = (unsigned)((rows + 3) / 4);
    const double rb = (double)rows * kRow16 * 16;
    float ms;
    ms = time_ms([&](int i) { k_rows<0, 0><<<grid, 256>>>(src[i % NB], dst[i % NB], sink, rows); });
    printf("read              : %7.1f GB/s\n", rb / ms / 1e6);
    ms = time_ms([&](int i) { k_rows<0, 1><<<grid, 256>>>(src[i % NB], dst[i % NB], sink, rows); });
    printf("read +1 element   : %7.1f GB/s\n", rb / ms / 1e6);
    ms = time_ms([&](int i) { k_rows<0, 2><<<grid, 256>>>(src[i % NB], dst[i % NB], sink, rows); });
    printf("read +2 elements  : %7.1f GB/s\n", rb / ms / 1e6);
    ms = time_ms([&](int i) { k_rows<1, 0><<<grid, 256>>>(src[i % NB], dst[i % NB], sink, rows); });
    printf("copy (1 : 1)      : %7.1f GB/s (read + written)\n", 2.0 * rb / ms / 1e6);
    ms = time_ms([&](int i) { k_rows<2, 0><<<grid, 256>>>(src[i % NB], dst[i % NB], sink, rows); });
    printf("read 4 : write 1  : %7.1f GB/s (read + written)\n", 1.25 * rb / ms / 1e6);
    ms = time_ms([&](int i) { k_rows<2, 2><<<grid, 256>>>(src[i % NB], dst[i % NB], sink, rows); });
    printf("... loads +2 elem : %7.1f GB/s (read + written)\n", 1.25 * rb / ms / 1e6);
    return 0;
}
