/*
 * TEST INFRASTRUCTURE ONLY.  A stand-alone driver that runs the oracle's routines (this file
 * includes tpq_oracle.c) on inputs read from a file and writes every result to another file.
 * tests/test_oracle_sanitized.py builds it with -fsanitize=address,undefined and compares the
 * results, byte for byte, with those of the ordinary build: any out-of-bounds access, signed
 * overflow or misaligned access in the oracle ends the run with a sanitizer report.
 *
 * input : int32 N, T, E, k, G; int32 idx[k]; uint16 Y[N][T][E]
 * output: per device outl, codes, scale, zero; the reduced sums (fp32 chain as fp32, bf16 chain
 *         as bf16); the same at 3 bits; calibration state after N sequences, ranges and indices;
 *         static parameters, static messages and their reduced sum; the fused epilogue; the linear
 *         layer on two of the tensors.
 */
#include "tpq_oracle.c"

#include <stdio.h>
#include <stdlib.h>

static void put(FILE *f, const void *p, size_t n)
{
    if (n && fwrite(p, 1, n, f) != n) exit(3);
}

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    FILE *in = fopen(argv[1], "rb");
    FILE *out = fopen(argv[2], "wb");
    if (!in || !out) return 2;
    int32_t h[5];
    if (fread(h, 4, 5, in) != 5) return 2;
    const int N = h[0], T = h[1], E = h[2], k = h[3], G = h[4];
    const int r = E - k, ng = (r + G - 1) / G;
    int32_t *idx = malloc(sizeof(int32_t) * (size_t)(k > 0 ? k : 1));
    uint16_t *Y = malloc(2u * (size_t)N * T * E);
    if (fread(idx, 4, (size_t)k, in) != (size_t)k) return 2;
    if (fread(Y, 2, (size_t)N * T * E, in) != (size_t)N * T * E) return 2;
    fclose(in);

    for (int bits = 4; bits >= 3; --bits) {   /* the 4-bit routines, then the generic ones at 3 bits */
        const size_t cb = ((size_t)r * (size_t)bits + 7) / 8;
        uint16_t **outl = malloc(sizeof(void *) * (size_t)N), **scale = malloc(sizeof(void *) * (size_t)N);
        uint16_t **zero = malloc(sizeof(void *) * (size_t)N);
        uint8_t **codes = malloc(sizeof(void *) * (size_t)N);
        for (int i = 0; i < N; ++i) {
            outl[i] = malloc(2u * (size_t)T * (size_t)(k > 0 ? k : 1));
            codes[i] = malloc((size_t)T * (cb > 0 ? cb : 1));
            scale[i] = malloc(2u * (size_t)T * (size_t)(ng > 0 ? ng : 1));
            zero[i] = malloc(2u * (size_t)T * (size_t)(ng > 0 ? ng : 1));
            const uint16_t *Yi = Y + (size_t)i * T * E;
            const int rc = bits == 4 ? orc_encode(Yi, T, E, E, k, G, idx, outl[i], codes[i], scale[i], zero[i], 1)
                                     : orc_encode_bits(Yi, T, E, E, k, G, bits, idx, outl[i], codes[i], scale[i], zero[i], 1);
            if (rc) return 4;
            put(out, outl[i], 2u * (size_t)T * k);
            put(out, codes[i], (size_t)T * cb);
            put(out, scale[i], 2u * (size_t)T * ng);
            put(out, zero[i], 2u * (size_t)T * ng);
        }
        float *s32 = malloc(4u * (size_t)T * E);
        uint16_t *s16 = malloc(2u * (size_t)T * E);
        int rc;
        if (bits == 4) {
            rc = orc_decode_reduce(N, T, E, k, G, idx, (const uint8_t *const *)codes, (const uint16_t *const *)scale,
                                   (const uint16_t *const *)zero, (const uint16_t *const *)outl, ORC_ACC_FP32, 1, s32, 1);
            rc |= orc_decode_reduce(N, T, E, k, G, idx, (const uint8_t *const *)codes, (const uint16_t *const *)scale,
                                    (const uint16_t *const *)zero, (const uint16_t *const *)outl, ORC_ACC_BF16, 0, s16, 1);
        } else {
            rc = orc_decode_reduce_bits(N, T, E, k, G, bits, idx, (const uint8_t *const *)codes,
                                        (const uint16_t *const *)scale, (const uint16_t *const *)zero,
                                        (const uint16_t *const *)outl, ORC_ACC_FP32, 1, s32, 1);
            rc |= orc_decode_reduce_bits(N, T, E, k, G, bits, idx, (const uint8_t *const *)codes,
                                         (const uint16_t *const *)scale, (const uint16_t *const *)zero,
                                         (const uint16_t *const *)outl, ORC_ACC_BF16, 0, s16, 1);
        }
        if (rc) return 5;
        put(out, s32, 4u * (size_t)T * E);
        put(out, s16, 2u * (size_t)T * E);
        if (bits == 4) {   /* the epilogue: device 0's rows as the addend, row 0 of device 1 as the bias */
            rc = orc_decode_reduce_fused(N, T, E, k, G, idx, (const uint8_t *const *)codes,
                                         (const uint16_t *const *)scale, (const uint16_t *const *)zero,
                                         (const uint16_t *const *)outl, Y, E, Y + (size_t)(N > 1 ? 1 : 0) * T * E,
                                         ORC_ACC_BF16, 0, s16, 1);
            if (rc) return 6;
            put(out, s16, 2u * (size_t)T * E);
        }
        for (int i = 0; i < N; ++i) { free(outl[i]); free(codes[i]); free(scale[i]); free(zero[i]); }
        free(outl); free(codes); free(scale); free(zero); free(s32); free(s16);
    }

    /* calibration: every device's tensor as one sequence of device 0 */
    float *m = calloc((size_t)N * E, 4), *M = calloc((size_t)N * E, 4);
    for (int i = 0; i < N; ++i)
        for (int s = 0; s < N; ++s)
            if (orc_calibrate_update(Y + (size_t)((i + s) % N) * T * E, T, E, E, s == 0, 0.25f, m + (size_t)i * E,
                                     M + (size_t)i * E))
                return 7;
    put(out, m, 4u * (size_t)N * E);
    put(out, M, 4u * (size_t)N * E);
    float *R = malloc(4u * (size_t)N * E), *Rbar = malloc(4u * (size_t)E);
    int32_t *is = malloc(4u * (size_t)(k > 0 ? k : 1)), *ir = malloc(4u * (size_t)(k > 0 ? k : 1));
    if (orc_calibrate_finalize(m, M, N, E, k, R, Rbar, is, ir)) return 8;
    put(out, R, 4u * (size_t)N * E);
    put(out, Rbar, 4u * (size_t)E);
    put(out, is, 4u * (size_t)k);
    put(out, ir, 4u * (size_t)k);

    /* static symmetric mode from that state */
    float *step = malloc(4u * (size_t)N * E), *inv = malloc(4u * (size_t)N * E);
    if (orc_static_params(m, M, N, E, step, inv)) return 9;
    put(out, step, 4u * (size_t)N * E);
    put(out, inv, 4u * (size_t)N * E);
    {
        const size_t cb = ((size_t)r + 1) / 2;
        uint16_t **outl = malloc(sizeof(void *) * (size_t)N);
        uint8_t **codes = malloc(sizeof(void *) * (size_t)N);
        for (int i = 0; i < N; ++i) {
            outl[i] = malloc(2u * (size_t)T * (size_t)(k > 0 ? k : 1));
            codes[i] = malloc((size_t)T * (cb > 0 ? cb : 1));
            if (orc_encode_static(Y + (size_t)i * T * E, T, E, E, k, idx, inv + (size_t)i * E, outl[i], codes[i], 1))
                return 10;
            put(out, outl[i], 2u * (size_t)T * k);
            put(out, codes[i], (size_t)T * cb);
        }
        uint16_t *s16 = malloc(2u * (size_t)T * E);
        if (orc_decode_reduce_static(N, T, E, k, idx, (const uint8_t *const *)codes, (const uint16_t *const *)outl, step,
                                     ORC_ACC_BF16, 0, s16, 1))
            return 11;
        put(out, s16, 2u * (size_t)T * E);
        for (int i = 0; i < N; ++i) { free(outl[i]); free(codes[i]); }
        free(outl); free(codes); free(s16);
    }
    /* the linear layer: device 0's tensor as the activations [T][E], device 1's first min(T, 7)
     * rows as a weight slice of that many output features (K = E) */
    if (N >= 2) {
        const int Eo = T < 7 ? T : 7;
        uint16_t *Yl = malloc(2u * (size_t)T * (size_t)Eo);
        double *mag = malloc(8u * (size_t)T * (size_t)Eo);
        if (orc_linear(Y, T, E, E, Y + (size_t)T * E, Eo, E, Yl, Eo, mag, 1)) return 12;
        put(out, Yl, 2u * (size_t)T * (size_t)Eo);
        put(out, mag, 8u * (size_t)T * (size_t)Eo);
        free(Yl); free(mag);
    }
    free(step); free(inv); free(R); free(Rbar); free(is); free(ir); free(m); free(M); free(Y); free(idx);
    fclose(out);
    return 0;
}
