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
//   decode-like the decoder's loads and stores (8 messages, 256 bytes of each per wave) alone
//   encode-like the encoder's (two waves per row, 32-bit and 2-byte stores) alone
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

// The decoder's access pattern without its arithmetic: wave (row, pass) reads 256 bytes of
// each of 8 code matrices (2528-byte rows), a 2-byte scale and zero per 16 lanes from 8 + 8
// small matrices (80-byte rows), and writes 1024 bytes of a 10240-byte output row.
struct Ptrs8 {
    const unsigned char *p[8];
};
__global__ __launch_bounds__(256) void k_decode_like(Ptrs8 codes, Ptrs8 scale, Ptrs8 zero, u4 *__restrict__ out,
                                                     unsigned rows)
{
    const unsigned lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned task = blockIdx.x * 4 + wave;  // 12 tasks per row: 10 passes, 2 idle
    const unsigned row = task / 12, pass = task % 12;
    if (row >= rows || pass >= 10) return;
    unsigned w[8], sb[8], zb[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const unsigned chunk = pass * 64 + lane < 630 ? pass * 64 + lane : 629;
        w[i] = __builtin_nontemporal_load((const unsigned *)(codes.p[i] + (size_t)row * 2528 + 4 * chunk));
        const unsigned g = chunk / 16;
        sb[i] = *(const unsigned short *)(scale.p[i] + (size_t)row * 80 + 2 * g);
        zb[i] = *(const unsigned short *)(zero.p[i] + (size_t)row * 80 + 2 * g);
    }
    unsigned x = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) x ^= w[i] ^ (sb[i] << 16) ^ zb[i];
    __builtin_nontemporal_store(u4{x, x + 1, x + 2, x + 3}, &out[(size_t)row * 640 + pass * 64 + lane]);
}

// The encoder's: two waves per 10240-byte row, five 128-bit loads each (4-byte aligned), one
// 32-bit store per load into a 2528-byte code row and a 2-byte store per 16 lanes into two
// 80-byte rows.
template <int VAR>
__global__ __launch_bounds__(256) void k_encode_like(const unsigned short *__restrict__ src,
                                                     unsigned char *__restrict__ codes,
                                                     unsigned char *__restrict__ scale,
                                                     unsigned char *__restrict__ zero, unsigned rows)
{
    const unsigned lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned task = blockIdx.x * 4 + wave;
    const unsigned row = task >> 1, seg = task & 1;
    if (row >= rows) return;
    const unsigned short *s = src + (size_t)row * 5120;
    u4 v[5];
#pragma unroll
    for (int p = 0; p < 5; ++p) {
        const unsigned c = (seg * 5 + p) * 64 + lane;
        v[p] = c < 630 ? __builtin_nontemporal_load((const u4_a2 *)(s + c * 8 + 2)) : u4{0, 0, 0, 0};
    }
    if (VAR == 1 || VAR == 3) {
        // the segment's 1280 bytes of codes as 16 bytes per lane: 64 lanes, then 16 more
        unsigned char *d = codes + (size_t)row * 2528 + seg * 1280;
        const u4 a = {v[0].x ^ v[1].y, v[1].x ^ v[2].y, v[2].x ^ v[3].y, v[3].x ^ v[4].y};
        if (seg == 0 || lane < 62) __builtin_nontemporal_store(a, (u4 *)(d + 16 * lane));
        if (lane < 16 && seg == 0) __builtin_nontemporal_store(v[4], (u4 *)(d + 1024 + 16 * lane));
    }
#pragma unroll
    for (int p = 0; p < 5; ++p) {
        const unsigned c = (seg * 5 + p) * 64 + lane;
        const unsigned x = v[p].x ^ v[p].y ^ v[p].z ^ v[p].w;
        if (VAR == 0 || VAR == 2)
            if (c < 630) __builtin_nontemporal_store(x, (unsigned *)(codes + (size_t)row * 2528 + 4 * c));
        if (VAR != 2 && (lane & 15) == 0 && c < 630) {
            *(unsigned short *)(scale + (size_t)row * 80 + 2 * (c / 16)) = (unsigned short)x;
            *(unsigned short *)(zero + (size_t)row * 80 + 2 * (c / 16)) = (unsigned short)(x >> 16);
        }
    }
}

// The encoder's reads alone: two waves per row, five 4-byte-aligned 128-bit loads each.
// TAB = 1: the loads' offsets come from a 32-byte record per lane and segment first (a
// 4 KB table that every row reads again, as the encoder's plan records are).
template <int TAB>
__global__ __launch_bounds__(256) void k_encode_reads(const unsigned short *__restrict__ src,
                                                      const u4 *__restrict__ table, u4 *__restrict__ sink,
                                                      unsigned rows)
{
    const unsigned lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned task = blockIdx.x * 4 + wave;
    const unsigned row = task >> 1, seg = task & 1;
    if (row >= rows) return;
    const unsigned short *s = src + (size_t)row * 5120;
    unsigned off[5];
    if (TAB) {
        const u4 a = table[(seg * 64 + lane) * 2], b = table[(seg * 64 + lane) * 2 + 1];
        off[0] = a.x; off[1] = a.y; off[2] = a.z; off[3] = a.w; off[4] = b.x;
    } else {
#pragma unroll
        for (int p = 0; p < 5; ++p) off[p] = ((seg * 5 + p) * 64 + lane) * 8 + 2;
    }
    u4 acc = {0, 0, 0, 0};
    u4 v[5];
#pragma unroll
    for (int p = 0; p < 5; ++p) v[p] = __builtin_nontemporal_load((const u4_a2 *)(s + (off[p] < 5110 ? off[p] : 5110)));
#pragma unroll
    for (int p = 0; p < 5; ++p) acc ^= v[p];
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u) sink[0] = acc;
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
    {   // the codec's two access patterns on their own (65536 rows: 1.4 GB and 0.9 GB per launch)
        const unsigned R = 65536;
        Ptrs8 c, sc, ze;
        for (int i = 0; i < 8; ++i) {
            unsigned char *a, *b, *d;
            CK(hipMalloc(&a, (size_t)R * 2528)); CK(hipMalloc(&b, (size_t)R * 80)); CK(hipMalloc(&d, (size_t)R * 80));
            CK(hipMemset(a, i + 1, (size_t)R * 2528)); CK(hipMemset(b, i + 2, (size_t)R * 80)); CK(hipMemset(d, i + 3, (size_t)R * 80));
            c.p[i] = a; sc.p[i] = b; ze.p[i] = d;
        }
        const double dec_bytes = (double)R * (8.0 * (2520 + 160) + 10240);
        ms = time_ms([&](int i) { k_decode_like<<<R * 12 / 4, 256>>>(c, sc, ze, dst[i % NB], R); });
        printf("decode-like       : %7.1f GB/s (8 x 256 B + 16 x 2 B read, 1 KB written per wave)\n", dec_bytes / ms / 1e6);
        const double enc_bytes = (double)R * (10240 + 2520 + 160);
        {
            u4 *tab;
            static u4 htab[256];
            for (unsigned sg = 0; sg < 2; ++sg)
                for (unsigned l = 0; l < 64; ++l) {
                    unsigned o[5];
                    for (unsigned p = 0; p < 5; ++p) o[p] = ((sg * 5 + p) * 64 + l) * 8 + 2;
                    htab[(sg * 64 + l) * 2] = u4{o[0], o[1], o[2], o[3]};
                    htab[(sg * 64 + l) * 2 + 1] = u4{o[4], 0, 0, 0};
                }
            CK(hipMalloc(&tab, sizeof htab));
            CK(hipMemcpy(tab, htab, sizeof htab, hipMemcpyHostToDevice));
            const size_t rows5 = bytes / 10240;
            ms = time_ms([&](int i) { k_encode_reads<0><<<(unsigned)(rows5 * 2 / 4), 256>>>(src[i % NB], tab, sink, (unsigned)rows5); });
            printf("encoder's reads   : %7.1f GB/s (two waves per row, five loads each)\n", (double)rows5 * 10240 / ms / 1e6);
            ms = time_ms([&](int i) { k_encode_reads<1><<<(unsigned)(rows5 * 2 / 4), 256>>>(src[i % NB], tab, sink, (unsigned)rows5); });
            printf("... offsets loaded: %7.1f GB/s (a 32-byte record per lane first)\n", (double)rows5 * 10240 / ms / 1e6);
        }
#define TPQ_ENC_LIKE(VAR)                                                                              \
    time_ms([&](int i) {                                                                               \
        k_encode_like<VAR><<<R * 2 / 4, 256>>>(src[i % NB], const_cast<unsigned char *>(c.p[i % 8]),   \
                                               const_cast<unsigned char *>(sc.p[i % 8]),               \
                                               const_cast<unsigned char *>(ze.p[i % 8]), R);           \
    })
        ms = TPQ_ENC_LIKE(0);
        printf("encode-like       : %7.1f GB/s (5 x 1 KB read, 5 x 256 B + 2-byte stores per wave)\n", enc_bytes / ms / 1e6);
        ms = TPQ_ENC_LIKE(1);
        printf("... 16-byte stores: %7.1f GB/s (the codes as 1 KB + 256 B per wave)\n", enc_bytes / ms / 1e6);
        ms = TPQ_ENC_LIKE(2);
        printf("... no 2-byte st. : %7.1f GB/s\n", (double)R * (10240 + 2520) / ms / 1e6);
    }
    return 0;
}
