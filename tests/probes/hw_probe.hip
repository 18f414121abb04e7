// Checks, on the GPU it runs on, the instruction behaviour that the codec kernels rely on for
// bit-exact results.  Each check restates the few instructions in question and compares them
// with plain IEEE arithmetic; the program exits with 0 only if every check passes.
//
//   1. DPP wave_shl:1 hands lane i the value of lane i + 1 (lane 63 keeps the "old" operand).
//   2. v_cvt_pk_u8_f32 rounds to the nearest even integer and writes the chosen byte only.
//   3. v_cvt_pk_bf16_f32 is round-to-nearest-even on the upper 16 bits.
//   4. x * fl(1/15), one fused correction step  ==  x / 15 (IEEE), on a dense sample.
//   5. hardware reciprocal + one Newton step == 1 / s (IEEE) for EVERY bf16 value s whose
//      reciprocal is a normal number and that the encoder can meet (1e-30 <= s <= 4.6e37).
//   6. v_perm_b32 byte order as used to collect the packed codes.
//   7. static mode: clamp to [-8, 7], add 1.5 * 2^23 + 8: the sum's low byte is rint(.) + 8.
//   8. one value rounded to bf16 by the pair conversion with a zero in the low half.
//   9. v_cvt_pk_u8_f32 saturates at 255 (the clamp of the 8-bit code width).
//  10. 2-, 4- and 8-byte global accesses at any byte address (code widths other than 4 bits).
//  11. the scaled FP8 (E4M3) pair conversion with scale 2^9 turns the bytes 0 .. 15 into the
//      floats 0 .. 15, from either half of the source word (4-bit codes to floats, two at once).
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s (line %d)\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__global__ void k_lane(unsigned *shl)
{
    const unsigned x = threadIdx.x + 100u;
    shl[threadIdx.x] = __builtin_amdgcn_update_dpp(7777u, x, 0x130, 0xF, 0xF, false);
}

__global__ void k_cvt(const float *f, unsigned *u8, unsigned *bf, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    u8[i] = __builtin_amdgcn_cvt_pk_u8_f32(f[i], 2u, 0xA1B2C3D4u);
    const f32x2 v = {f[i], -f[i]};
    bf[i] = __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}

__global__ void k_div15(const float *x, unsigned *fast, unsigned *ieee, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float y = 0x1.111112p-4f;
    const float q = x[i] * y;
    const float r = __builtin_fmaf(-15.0f, q, x[i]);
    fast[i] = __float_as_uint(__builtin_fmaf(r, y, q));
    ieee[i] = __float_as_uint(x[i] / 15.0f);
}

__global__ void k_recip(unsigned *fast, unsigned *ieee)
{
    const unsigned h = blockIdx.x * blockDim.x + threadIdx.x;  // a bf16 bit pattern
    if (h >= 0x8000u) return;
    const float s = __uint_as_float(h << 16);
    const float y = __builtin_amdgcn_rcpf(s);
    const float e = __builtin_fmaf(-s, y, 1.0f);
    fast[h] = __float_as_uint(__builtin_fmaf(e, y, y));
    ieee[h] = __float_as_uint(1.0f / s);
}

// static mode: clamp, then add 1.5 * 2^23 + 8: the low byte is rint(.) + 8
__global__ void k_magic(const float *p, unsigned *out, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float c = __builtin_amdgcn_fmed3f(p[i], -8.0f, 7.0f);
    out[i] = __float_as_uint(c + 12582920.0f) & 0xFFu;
}

// 8-bit codes: the float -> byte conversion saturates at 255
__global__ void k_sat(const float *p, unsigned *out, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    out[i] = __builtin_amdgcn_cvt_pk_u8_f32(p[i], 0u, 0u);
}

// byte-aligned 2-, 4- and 8-byte accesses (code widths other than 4 bits)
typedef unsigned short u16_a1 __attribute__((aligned(1)));
typedef unsigned int u32_a1 __attribute__((aligned(1)));
typedef unsigned long long u64_a1 __attribute__((aligned(1)));
__global__ void k_unaligned(unsigned char *buf, unsigned long long *loaded)
{
    const unsigned l = threadIdx.x;  // 64 lanes, 16 bytes apart, offsets l % 8
    unsigned char *p = buf + 16u * l + (l & 7u);
    loaded[l] = *reinterpret_cast<const u64_a1 *>(p);
    unsigned char *q = buf + 2048u + 16u * l + (l & 7u);
    *reinterpret_cast<u16_a1 *>(q) = static_cast<unsigned short>(0xB1A0u + l);
    *reinterpret_cast<u32_a1 *>(q + 2) = 0xC0DE0000u + l;
}

// one value rounded to bf16 by the pair conversion with a zero low half
__global__ void k_round1(const float *f, unsigned *out, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const f32x2 v = {0.0f, f[i]};
    out[i] = __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}

__global__ void k_perm(unsigned *out)
{
    out[0] = __builtin_amdgcn_perm(0x88776655u, 0x44332211u, 0x07050301u);
}

__global__ void k_fp8_codes(float *out)
{
    const unsigned b = threadIdx.x & 15u;  // bytes b, b + 1, b + 2, b + 3 (mod 16)
    const unsigned w = b | (((b + 1u) & 15u) << 8) | (((b + 2u) & 15u) << 16) | (((b + 3u) & 15u) << 24);
    const f32x2 lo = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(w, 512.0f, false);
    const f32x2 hi = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(w, 512.0f, true);
    out[4 * b] = lo.x; out[4 * b + 1] = lo.y; out[4 * b + 2] = hi.x; out[4 * b + 3] = hi.y;
}

static unsigned bf16_rne(float f)
{
    unsigned u; memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

int main()
{
    int fails = 0;
    {   // 1
        unsigned *d, h[64];
        CK(hipMalloc(&d, sizeof h));
        k_lane<<<1, 64>>>(d);
        CK(hipMemcpy(h, d, sizeof h, hipMemcpyDeviceToHost));
        int bad = 0;
        for (int i = 0; i < 63; ++i) bad += h[i] != 101u + i;
        bad += h[63] != 7777u;
        printf("wave_shl:1            : %s\n", bad ? "FAIL" : "ok");
        fails += bad != 0;
    }
    {   // 2, 3
        const int n = 1 << 20;
        float *hf = (float *)malloc(n * 4);
        for (int i = 0; i < n; ++i) hf[i] = 15.75f * (float)i / (float)n;
        for (int k = 0; k < 16; ++k) {
            hf[3 * k] = k + 0.5f;
            hf[3 * k + 1] = nextafterf(k + 0.5f, 100.f);
            hf[3 * k + 2] = nextafterf(k + 0.5f, -100.f);
        }
        float *df; unsigned *d8, *dbf;
        CK(hipMalloc(&df, n * 4)); CK(hipMalloc(&d8, n * 4)); CK(hipMalloc(&dbf, n * 4));
        CK(hipMemcpy(df, hf, n * 4, hipMemcpyHostToDevice));
        k_cvt<<<n / 256, 256>>>(df, d8, dbf, n);
        unsigned *h8 = (unsigned *)malloc(n * 4), *hbf = (unsigned *)malloc(n * 4);
        CK(hipMemcpy(h8, d8, n * 4, hipMemcpyDeviceToHost)); CK(hipMemcpy(hbf, dbf, n * 4, hipMemcpyDeviceToHost));
        long bad8 = 0, badbf = 0;
        for (int i = 0; i < n; ++i) {
            const unsigned want = (0xA1B2C3D4u & 0xFF00FFFFu) | ((unsigned)rintf(hf[i]) << 16);
            bad8 += h8[i] != want;
            const unsigned wantbf = bf16_rne(hf[i]) | (bf16_rne(-hf[i]) << 16);
            badbf += hbf[i] != wantbf;
        }
        printf("cvt_pk_u8_f32 (RNE)   : %s (%ld of %d differ)\n", bad8 ? "FAIL" : "ok", bad8, n);
        printf("cvt_pk_bf16_f32 (RNE) : %s (%ld of %d differ)\n", badbf ? "FAIL" : "ok", badbf, n);
        fails += (bad8 != 0) + (badbf != 0);
    }
    {   // 4
        const int n = 1 << 22;
        float *hx = (float *)malloc(n * 4);
        unsigned seed = 12345u;
        for (int i = 0; i < n; ++i) {  // random mantissas over a wide range of exponents
            seed = seed * 1664525u + 1013904223u;
            unsigned bits = ((seed >> 9) & 0x007FFFFFu) | ((30u + (seed & 127u) + ((seed >> 7) & 63u)) << 23);
            memcpy(&hx[i], &bits, 4);
        }
        float *dx; unsigned *da, *db;
        CK(hipMalloc(&dx, n * 4)); CK(hipMalloc(&da, n * 4)); CK(hipMalloc(&db, n * 4));
        CK(hipMemcpy(dx, hx, n * 4, hipMemcpyHostToDevice));
        k_div15<<<n / 256, 256>>>(dx, da, db, n);
        unsigned *ha = (unsigned *)malloc(n * 4), *hb = (unsigned *)malloc(n * 4);
        CK(hipMemcpy(ha, da, n * 4, hipMemcpyDeviceToHost)); CK(hipMemcpy(hb, db, n * 4, hipMemcpyDeviceToHost));
        long bad = 0, badhost = 0;
        for (int i = 0; i < n; ++i) {
            bad += ha[i] != hb[i];
            volatile float q = hx[i] / 15.0f; float qq = q; unsigned qb; memcpy(&qb, &qq, 4);
            badhost += qb != hb[i];
        }
        printf("x / 15 shortcut       : %s (%ld differ; device vs host division: %ld)\n", (bad || badhost) ? "FAIL" : "ok", bad, badhost);
        fails += (bad != 0) + (badhost != 0);
    }
    {   // 5
        unsigned *da, *db;
        static unsigned ha[0x8000], hb[0x8000];
        CK(hipMalloc(&da, sizeof ha)); CK(hipMalloc(&db, sizeof hb));
        k_recip<<<128, 256>>>(da, db);
        CK(hipMemcpy(ha, da, sizeof ha, hipMemcpyDeviceToHost)); CK(hipMemcpy(hb, db, sizeof hb, hipMemcpyDeviceToHost));
        long bad = 0, checked = 0;
        for (unsigned h = 1; h < 0x7F80u; ++h) {
            float s; unsigned b = h << 16; memcpy(&s, &b, 4);
            if (s < 1e-30f || s > 4.6e37f) continue;
            ++checked;
            bad += ha[h] != hb[h];
        }
        printf("1 / scale shortcut    : %s (%ld of %ld bf16 scales differ)\n", bad ? "FAIL" : "ok", bad, checked);
        fails += bad != 0;
    }
    {   // 6
        unsigned *d, h;
        CK(hipMalloc(&d, 4));
        k_perm<<<1, 1>>>(d);
        CK(hipMemcpy(&h, d, 4, hipMemcpyDeviceToHost));
        printf("v_perm_b32 selector   : %s (0x%08x)\n", h == 0x88664422u ? "ok" : "FAIL", h);
        fails += h != 0x88664422u;
    }
    {   // 7, 8, 9: static-mode rounding, saturation, single-value bf16 rounding
        const int n = 1 << 18;
        float *hf = (float *)malloc(n * 4);
        for (int i = 0; i < n; ++i) hf[i] = -10.0f + 20.0f * (float)i / (float)n;
        for (int k = -9; k < 9; ++k) {
            hf[3 * (k + 9)] = k + 0.5f;
            hf[3 * (k + 9) + 1] = nextafterf(k + 0.5f, 100.f);
            hf[3 * (k + 9) + 2] = nextafterf(k + 0.5f, -100.f);
        }
        float *df; unsigned *d;
        CK(hipMalloc(&df, n * 4)); CK(hipMalloc(&d, n * 4));
        CK(hipMemcpy(df, hf, n * 4, hipMemcpyHostToDevice));
        unsigned *h = (unsigned *)malloc(n * 4);
        k_magic<<<n / 256, 256>>>(df, d, n);
        CK(hipMemcpy(h, d, n * 4, hipMemcpyDeviceToHost));
        long bad = 0;
        for (int i = 0; i < n; ++i) {
            float q = rintf(hf[i]);
            q = q < -8.f ? -8.f : (q > 7.f ? 7.f : q);
            bad += h[i] != (unsigned)((int)q + 8);
        }
        printf("clamp + magic rounding: %s (%ld of %d differ)\n", bad ? "FAIL" : "ok", bad, n);
        fails += bad != 0;
        k_round1<<<n / 256, 256>>>(df, d, n);
        CK(hipMemcpy(h, d, n * 4, hipMemcpyDeviceToHost));
        bad = 0;
        for (int i = 0; i < n; ++i) bad += h[i] != (bf16_rne(hf[i]) << 16);
        printf("bf16 rounding, 1 value: %s (%ld of %d differ)\n", bad ? "FAIL" : "ok", bad, n);
        fails += bad != 0;
        for (int i = 0; i < n; ++i) hf[i] = 240.0f + 80.0f * (float)i / (float)n;
        CK(hipMemcpy(df, hf, n * 4, hipMemcpyHostToDevice));
        k_sat<<<n / 256, 256>>>(df, d, n);
        CK(hipMemcpy(h, d, n * 4, hipMemcpyDeviceToHost));
        bad = 0;
        for (int i = 0; i < n; ++i) {
            const float q = rintf(hf[i]);
            bad += h[i] != (unsigned)(q > 255.f ? 255.f : q);
        }
        printf("cvt_pk_u8 saturation  : %s (%ld of %d differ)\n", bad ? "FAIL" : "ok", bad, n);
        fails += bad != 0;
    }
    {   // 10: byte-aligned accesses
        unsigned char hb[4096], *db;
        for (int i = 0; i < 4096; ++i) hb[i] = (unsigned char)(i * 7 + 3);
        unsigned long long *dl, hl[64];
        CK(hipMalloc(&db, 4096)); CK(hipMalloc(&dl, 64 * 8));
        CK(hipMemcpy(db, hb, 4096, hipMemcpyHostToDevice));
        k_unaligned<<<1, 64>>>(db, dl);
        unsigned char after[4096];
        CK(hipMemcpy(after, db, 4096, hipMemcpyDeviceToHost));
        CK(hipMemcpy(hl, dl, 64 * 8, hipMemcpyDeviceToHost));
        long bad = 0;
        for (unsigned l = 0; l < 64; ++l) {
            unsigned long long want;
            memcpy(&want, hb + 16 * l + (l & 7), 8);
            bad += hl[l] != want;
            unsigned char *q = hb + 2048 + 16 * l + (l & 7);
            const unsigned short a = (unsigned short)(0xB1A0u + l);
            const unsigned b = 0xC0DE0000u + l;
            memcpy(q, &a, 2);
            memcpy(q + 2, &b, 4);
        }
        bad += memcmp(hb, after, 4096) != 0;
        printf("byte-aligned accesses : %s\n", bad ? "FAIL" : "ok");
        fails += bad != 0;
    }
    {   // 11: 4-bit codes to floats through the FP8 pair conversion
        float *d, h[64];
        CK(hipMalloc(&d, sizeof h));
        k_fp8_codes<<<1, 16>>>(d);
        CK(hipMemcpy(h, d, sizeof h, hipMemcpyDeviceToHost));
        int bad = 0;
        for (int b = 0; b < 16; ++b)
            for (int j = 0; j < 4; ++j) bad += h[4 * b + j] != (float)((b + j) & 15);
        printf("fp8 pair conversion   : %s\n", bad ? "FAIL" : "ok");
        fails += bad != 0;
    }
    printf("%s\n", fails ? "HW PROBE FAILED" : "HW PROBE OK");
    return fails ? 1 : 0;
}
