/*
 * tpq_oracle.c -- plain scalar CPU oracle for the low-bit tensor-parallel
 * partial-sum codec (calibration, encode, decode-and-reduce).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the GPU
 * library can be checked against something written straight from the paper.
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it.  It shares no code, header, table or helper with the HIP path.
 *
 * What is computed (all arithmetic IEEE-754 binary32, round-to-nearest-even,
 * no fused contraction, denormals kept; bf16 = upper 16 bits of binary32,
 * converted with round-to-nearest-even):
 *
 *   calibration (paper Sec. 3 "Calibration", Eq. (1) and (2); Sec. 3
 *   "Selecting High Precision Features"):
 *     per sequence, per device i, per feature j: column min and max over the
 *     S rows; exponential moving average with constant gamma, the first
 *     sequence initialising the state; symmetric range R = 2*max(-m, M);
 *     aggregated range Rbar_j = sum over devices; the k features with the
 *     largest Rbar are the ones kept in BF16.
 *
 *   encode (paper Sec. 2 compression function C^(i); Fig. 2; Sec. 3): the k
 *     selected features of each row are copied verbatim as bf16; the other
 *     r = E-k features, taken in ascending feature order ("compacted"), are
 *     quantised to 4 bits.  The quantiser is the group-wise asymmetric one
 *     the workload definition asks for: per row, per group of G consecutive
 *     compacted features, zero = group minimum, scale = bf16((max-min)/15),
 *     code = rint((x - zero) * (1/scale)) clamped to 0..15; two codes per
 *     byte, low nibble first.
 *
 *   decode_reduce (paper Sec. 2 decompression D^(i) and the sum over
 *     devices; Fig. 2 caption): every device's message is dequantised
 *     (x = code*scale + zero, outliers as they are) and the N results are
 *     added in ascending device order, either in fp32 (rounded to bf16 once
 *     at the end, or left fp32) or literally in bf16 (every term and every
 *     partial sum rounded to bf16).
 *
 *   static symmetric mode (paper Sec. 3 "Calibration" and "Selecting High
 *   Precision Features": every feature on every device has static,
 *   independent quantisation parameters from calibration, the range is
 *   R = 2*max(-m, M), and all features that are not kept in BF16 are
 *   symmetrically quantised to Int4).  The paper gives neither the step nor
 *   the code set; the reading taken here is the common symmetric one with
 *   the full signed range: step = R/15, code = rint(x * (1/step)) clamped to
 *   -8..7, x^ = code * step, travelling as the nibble code + 8.  A feature
 *   whose calibrated range vanishes (step < 1e-30) is sent as code 0 and
 *   comes back as 0.  Nothing but codes and the BF16 features travels.
 *
 *   other bit widths (paper Sec. 4, the experiment that varies the number of
 *   bits of the quantised features, Fig. 3): the same dynamic group-wise
 *   quantiser with b in {2, 3, 4, 5, 6, 8} bits: 2^b - 1 steps over the group's
 *   range, scale = bf16((max-min)/(2^b - 1)), codes 0..2^b - 1.  The codes of a
 *   row form one little-endian bit string: code c occupies bits b*c .. b*c+b-1,
 *   bit n of the string being bit n%8 of byte n/8 (for b = 4 this is "two codes
 *   per byte, low nibble first").  orc_encode_bits / orc_decode_reduce_bits.
 *
 *   fused epilogue (paper Sec. 2: the block's output is the sum over the
 *   devices plus the bias, f(x) = [sum_i f^(i)(x^(i))] + b): orc_decode_reduce_fused
 *   adds, after the sum over the messages, an optional addend row (bf16 [T][E]:
 *   a residual, or the device's own partial sum when its message is left out)
 *   and then an optional bias (bf16 [E]), each as one more term of the same
 *   accumulation (fp32 add, or bf16-rounded add in the literal bf16 chain).
 *
 *   the producer of the partial sums (paper Sec. 2: device i holds the slice
 *   W^(i) of a row-parallel linear layer and computes f^(i)(x^(i)) = x^(i) W^(i),
 *   the tensor that is then compressed): orc_linear evaluates every output as the
 *   sum of its K products in binary64 (each product of two bf16 values is exact
 *   there, the sum of a few thousand of them is exact to about 2^-41 of the sum of
 *   their magnitudes) and rounds once to bf16, ties to even -- the definition, not
 *   any particular accumulation order.  orc_encode of that tensor is the
 *   reference for a GEMM that compresses in its epilogue.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py
 * (brute force over all 16 codes in float64, verbatim outliers, half-step
 * error bound, closed-form bit counts, Irwin-Hall variance of the summed
 * error, hand-worked EMA examples, numpy stable-sort top-k, plain-sum special
 * case k = E; for the static mode: half-step error inside the calibrated
 * range, saturation outside, all 16 codes by brute force in float64, the
 * worked example under tests/golden).  Parity unpinned: the byte layout of the message (nibble
 * order, pad nibble, section order) is not fixed by the paper; it is this
 * build's own choice and is only checked against its written description.
 *
 * Layouts here are dense (no row padding):
 *   outl  uint16 [T][k]          codes uint8 [T][ceil(r/2)]  (b bits: [T][ceil(r*b/8)])
 *   scale uint16 [T][ceil(r/G)]  zero  uint16 [T][ceil(r/G)]
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_ERR_ARG (-1)

/* ---- bf16 <-> binary32 ------------------------------------------------- */

static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* round-to-nearest-even on the 16 discarded bits; inputs are finite */
static uint16_t f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

static uint16_t f32_bits_hi(float f) /* exact when f is a bf16 value */
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(u >> 16);
}

static int set_threads(int threads)
{
#ifdef _OPENMP
    if (threads < 1) threads = 1;
    omp_set_num_threads(threads);
    return threads;
#else
    (void)threads;
    return 1;
#endif
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_num_procs();
#else
    return 1;
#endif
}

/* ---- calibration ------------------------------------------------------- */

/*
 * One sequence of one device (Eq. (1), (2)).  Y is bf16 [S][ldY] with E used
 * columns; m and M are that device's fp32 [E] state.  first != 0 means this is
 * the first sequence: the state is set to the column min / max.
 */
int orc_calibrate_update(const uint16_t *Y, int64_t S, int64_t ldY, int E,
                         int first, float gamma, float *m, float *M)
{
    if (!Y || !m || !M || S < 1 || E < 1 || ldY < E) return ORC_ERR_ARG;
    const float keep = 1.0f - gamma;
    for (int j = 0; j < E; ++j) {
        float cmin = bf16_to_f32(Y[j]);
        float cmax = cmin;
        for (int64_t t = 1; t < S; ++t) {
            float v = bf16_to_f32(Y[t * ldY + j]);
            if (v < cmin) cmin = v;
            if (v > cmax) cmax = v;
        }
        cmin += 0.0f; /* -0 becomes +0, so the result does not depend on */
        cmax += 0.0f; /* which of two equal zeros was met first          */
        if (first) {
            m[j] = cmin;
            M[j] = cmax;
        } else {
            float a = keep * m[j];
            float b = gamma * cmin;
            m[j] = a + b;
            a = keep * M[j];
            b = gamma * cmax;
            M[j] = a + b;
        }
    }
    return ORC_OK;
}

typedef struct {
    float key;
    int32_t j;
} orc_rank_item;

static int cmp_rank(const void *pa, const void *pb)
{
    const orc_rank_item *a = (const orc_rank_item *)pa;
    const orc_rank_item *b = (const orc_rank_item *)pb;
    if (a->key > b->key) return -1; /* larger aggregated range first */
    if (a->key < b->key) return 1;
    return (a->j > b->j) - (a->j < b->j); /* ties: lower feature first */
}

static int cmp_i32(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

/*
 * After the last sequence: R[i][j] = 2*max(-m, M); Rbar[j] = R[0][j] + R[1][j]
 * + ... in ascending device order; the k features with the largest Rbar
 * (ties to the lower index).  m, M: fp32 [N][E].  R (may be NULL): [N][E].
 * idx_ranked (may be NULL): the k features by descending Rbar.  idx_sorted:
 * the same set in ascending feature order.
 */
int orc_calibrate_finalize(const float *m, const float *M, int N, int E, int k,
                           float *R, float *Rbar, int32_t *idx_sorted,
                           int32_t *idx_ranked)
{
    if (!m || !M || !Rbar || N < 1 || E < 1 || k < 0 || k > E) return ORC_ERR_ARG;
    if (k > 0 && !idx_sorted) return ORC_ERR_ARG;
    for (int j = 0; j < E; ++j) {
        float acc = 0.0f;
        for (int i = 0; i < N; ++i) {
            float lo = -m[(int64_t)i * E + j];
            float hi = M[(int64_t)i * E + j];
            float r = 2.0f * (lo > hi ? lo : hi);
            r += 0.0f;
            if (R) R[(int64_t)i * E + j] = r;
            acc = (i == 0) ? r : acc + r;
        }
        Rbar[j] = acc;
    }
    orc_rank_item *items = (orc_rank_item *)malloc(sizeof(orc_rank_item) * (size_t)E);
    if (!items) return ORC_ERR_ARG;
    for (int j = 0; j < E; ++j) {
        items[j].key = Rbar[j];
        items[j].j = j;
    }
    qsort(items, (size_t)E, sizeof(orc_rank_item), cmp_rank);
    for (int p = 0; p < k; ++p) {
        if (idx_ranked) idx_ranked[p] = items[p].j;
        idx_sorted[p] = items[p].j;
    }
    free(items);
    if (k > 0) qsort(idx_sorted, (size_t)k, sizeof(int32_t), cmp_i32);
    return ORC_OK;
}

/* ---- shared argument checks -------------------------------------------- */

static int check_indices(const int32_t *idx, int k, int E)
{
    for (int p = 0; p < k; ++p) {
        if (idx[p] < 0 || idx[p] >= E) return 0;
        if (p > 0 && idx[p] <= idx[p - 1]) return 0;
    }
    return 1;
}

/* comp[c] = feature index of the c-th non-selected feature, ascending */
static int32_t *build_compaction(const int32_t *idx, int k, int E)
{
    int r = E - k;
    int32_t *comp = (int32_t *)malloc(sizeof(int32_t) * (size_t)(r > 0 ? r : 1));
    if (!comp) return NULL;
    int p = 0, c = 0;
    for (int j = 0; j < E; ++j) {
        if (p < k && idx[p] == j) {
            ++p;
        } else {
            comp[c++] = j;
        }
    }
    return comp;
}

/* ---- encode ------------------------------------------------------------ */

static void encode_row(const uint16_t *y, int k, int r, int G,
                       const int32_t *idx, const int32_t *comp,
                       uint16_t *outl, uint8_t *codes, uint16_t *scale,
                       uint16_t *zero)
{
    for (int p = 0; p < k; ++p) outl[p] = y[idx[p]]; /* verbatim 16-bit copy */

    int cb = (r + 1) / 2;
    memset(codes, 0, (size_t)cb);
    int ng = (r + G - 1) / G;
    for (int g = 0; g < ng; ++g) {
        int c0 = g * G;
        int c1 = c0 + G < r ? c0 + G : r;
        float mn = bf16_to_f32(y[comp[c0]]);
        float mx = mn;
        for (int c = c0 + 1; c < c1; ++c) {
            float v = bf16_to_f32(y[comp[c]]);
            if (v < mn) mn = v;
            if (v > mx) mx = v;
        }
        mn += 0.0f;
        float span = mx - mn;
        float s32 = span / 15.0f;
        uint16_t sb = f32_to_bf16(s32);
        float s = bf16_to_f32(sb);
        zero[g] = f32_bits_hi(mn); /* mn is one of the bf16 inputs: exact */
        if (s < 1e-30f) {
            /* constant (or vanishing-range) group: all codes 0, scale 0 */
            scale[g] = 0;
            continue;
        }
        scale[g] = sb;
        float inv = 1.0f / s;
        for (int c = c0; c < c1; ++c) {
            float v = bf16_to_f32(y[comp[c]]);
            float d = v - mn;
            float p = d * inv;
            float q = rintf(p); /* ties to even */
            if (q < 0.0f) q = 0.0f;
            if (q > 15.0f) q = 15.0f;
            unsigned code = (unsigned)q;
            if (c & 1)
                codes[c >> 1] |= (uint8_t)(code << 4);
            else
                codes[c >> 1] |= (uint8_t)code;
        }
    }
}

/*
 * One device's partial sums Y bf16 [T][ldY] -> message sections (dense).
 */
int orc_encode(const uint16_t *Y, int64_t T, int64_t ldY, int E, int k, int G,
               const int32_t *idx_sorted, uint16_t *outl, uint8_t *codes,
               uint16_t *scale, uint16_t *zero, int threads)
{
    if (!Y || T < 0 || E < 1 || k < 0 || k > E || G < 2 || (G & 1) || ldY < E)
        return ORC_ERR_ARG;
    if (k > 0 && (!idx_sorted || !outl)) return ORC_ERR_ARG;
    if (k < E && (!codes || !scale || !zero)) return ORC_ERR_ARG;
    if (!check_indices(idx_sorted, k, E)) return ORC_ERR_ARG;
    int r = E - k;
    int cb = (r + 1) / 2;
    int ng = (r + G - 1) / G;
    int32_t *comp = build_compaction(idx_sorted, k, E);
    if (!comp) return ORC_ERR_ARG;
    set_threads(threads);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        encode_row(Y + t * ldY, k, r, G, idx_sorted, comp,
                   outl ? outl + t * k : NULL, codes ? codes + t * cb : NULL,
                   scale ? scale + t * ng : NULL, zero ? zero + t * ng : NULL);
    }
    free(comp);
    return ORC_OK;
}

/* ---- the linear layer that produces the partial sums --------------------- */

/* nearest bf16 of a finite double, ties to even: through the two bf16 neighbours
 * of the value, compared in binary64 (no intermediate rounding to binary32) */
static uint16_t f64_to_bf16(double v)
{
    float f = (float)v;            /* within half a binary32 ulp: picks the neighbourhood */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    uint32_t lo_bits = u & 0xFFFF0000u;          /* towards zero */
    float lo, hi;
    memcpy(&lo, &lo_bits, sizeof lo);
    uint32_t hi_bits = lo_bits + 0x00010000u;    /* one bf16 step away from zero */
    memcpy(&hi, &hi_bits, sizeof hi);
    double dl = fabs(v - (double)lo), dh = fabs((double)hi - v);
    if (dl < dh) return (uint16_t)(lo_bits >> 16);
    if (dh < dl) return (uint16_t)(hi_bits >> 16);
    return (uint16_t)(((lo_bits >> 16) & 1u) ? (hi_bits >> 16) : (lo_bits >> 16));
}

/*
 * Y[t][e] = bf16( sum_k X[t][k] * Wt[e][k] ), X bf16 [T][ldX], Wt bf16 [E][ldW] (one
 * row per output feature: W^(i) transposed), Y bf16 [T][ldY].  mag (optional, double
 * [T][E]) receives sum_k |X[t][k] * Wt[e][k]|, the scale of any accumulation error.
 */
int orc_linear(const uint16_t *X, int64_t T, int64_t ldX, int K, const uint16_t *Wt, int E,
               int64_t ldW, uint16_t *Y, int64_t ldY, double *mag, int threads)
{
    if (!X || !Wt || !Y || T < 0 || K < 1 || E < 1 || ldX < K || ldW < K || ldY < E)
        return ORC_ERR_ARG;
    set_threads(threads);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            double acc = 0.0, am = 0.0;
            for (int kk = 0; kk < K; ++kk) {
                double prod = (double)bf16_to_f32(X[t * ldX + kk]) *
                              (double)bf16_to_f32(Wt[(int64_t)e * ldW + kk]);
                acc += prod;
                am += fabs(prod);
            }
            Y[t * ldY + e] = f64_to_bf16(acc);
            if (mag) mag[t * (int64_t)E + e] = am;
        }
    }
    return ORC_OK;
}

/* ---- decode + reduce --------------------------------------------------- */

#define ORC_ACC_FP32 0
#define ORC_ACC_BF16 1

static float round_to_bf16(float f) { return bf16_to_f32(f32_to_bf16(f)); }

/*
 * N messages -> out [T][E] in original feature order.
 * accum = ORC_ACC_FP32: acc = x_0; acc = acc + x_i (fp32), i ascending.
 * accum = ORC_ACC_BF16: every term and every partial sum is rounded to bf16.
 * out_fp32 != 0: out is float [T][E] (the accumulator as it is);
 * otherwise out is bf16 (uint16) [T][E], the accumulator rounded once.
 */
int orc_decode_reduce(int N, int64_t T, int E, int k, int G,
                      const int32_t *idx_sorted, const uint8_t *const *codes,
                      const uint16_t *const *scale, const uint16_t *const *zero,
                      const uint16_t *const *outl, int accum, int out_fp32,
                      void *out, int threads)
{
    if (N < 1 || T < 0 || E < 1 || k < 0 || k > E || G < 2 || (G & 1) || !out)
        return ORC_ERR_ARG;
    if (accum != ORC_ACC_FP32 && accum != ORC_ACC_BF16) return ORC_ERR_ARG;
    if (k > 0 && (!idx_sorted || !outl)) return ORC_ERR_ARG;
    if (k < E && (!codes || !scale || !zero)) return ORC_ERR_ARG;
    if (!check_indices(idx_sorted, k, E)) return ORC_ERR_ARG;
    int r = E - k;
    int cb = (r + 1) / 2;
    int ng = (r + G - 1) / G;
    int32_t *comp = build_compaction(idx_sorted, k, E);
    if (!comp) return ORC_ERR_ARG;
    set_threads(threads);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        float *of = out_fp32 ? (float *)out + t * E : NULL;
        uint16_t *ob = out_fp32 ? NULL : (uint16_t *)out + t * E;
        for (int col = 0; col < E; ++col) { /* col walks compacted, then outliers */
            int j;
            int is_outlier = col >= r;
            j = is_outlier ? idx_sorted[col - r] : comp[col];
            float acc = 0.0f;
            for (int i = 0; i < N; ++i) {
                float x;
                if (is_outlier) {
                    x = bf16_to_f32(outl[i][t * k + (col - r)]);
                } else {
                    int c = col;
                    uint8_t byte = codes[i][t * cb + (c >> 1)];
                    unsigned code = (c & 1) ? (byte >> 4) : (byte & 0x0Fu);
                    float s = bf16_to_f32(scale[i][t * ng + c / G]);
                    float z = bf16_to_f32(zero[i][t * ng + c / G]);
                    float prod = (float)code * s; /* exact: 4 bits x 8 bits */
                    x = prod + z;
                }
                if (accum == ORC_ACC_BF16) {
                    x = round_to_bf16(x);
                    acc = (i == 0) ? x : round_to_bf16(acc + x);
                } else {
                    acc = (i == 0) ? x : acc + x;
                }
            }
            if (of)
                of[j] = acc;
            else
                ob[j] = f32_to_bf16(acc);
        }
    }
    free(comp);
    return ORC_OK;
}

/* ---- decode + reduce with the block's epilogue --------------------------- */

/*
 * orc_decode_reduce (4-bit codes) followed, per element, by
 *   acc = acc (+) addend[t][j]   if addend != NULL  (bf16 [T][ldAdd])
 *   acc = acc (+) bias[j]        if bias   != NULL  (bf16 [E])
 * in this order, (+) being the accumulation's own addition: fp32, or fp32 rounded to
 * bf16 in the literal bf16 chain.  Sec. 2: f(x) = [sum_i f^(i)(x^(i))] + b.
 */
int orc_decode_reduce_fused(int N, int64_t T, int E, int k, int G,
                            const int32_t *idx_sorted, const uint8_t *const *codes,
                            const uint16_t *const *scale, const uint16_t *const *zero,
                            const uint16_t *const *outl, const uint16_t *addend, int64_t ldAdd,
                            const uint16_t *bias, int accum, int out_fp32, void *out,
                            int threads)
{
    if (N < 1 || T < 0 || E < 1 || k < 0 || k > E || G < 2 || (G & 1) || !out) return ORC_ERR_ARG;
    if (accum != ORC_ACC_FP32 && accum != ORC_ACC_BF16) return ORC_ERR_ARG;
    if (k > 0 && (!idx_sorted || !outl)) return ORC_ERR_ARG;
    if (k < E && (!codes || !scale || !zero)) return ORC_ERR_ARG;
    if (addend && ldAdd < E) return ORC_ERR_ARG;
    if (!check_indices(idx_sorted, k, E)) return ORC_ERR_ARG;
    int r = E - k;
    int cb = (r + 1) / 2;
    int ng = (r + G - 1) / G;
    int32_t *comp = build_compaction(idx_sorted, k, E);
    if (!comp) return ORC_ERR_ARG;
    set_threads(threads);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        float *of = out_fp32 ? (float *)out + t * E : NULL;
        uint16_t *ob = out_fp32 ? NULL : (uint16_t *)out + t * E;
        for (int col = 0; col < E; ++col) {
            int is_outlier = col >= r;
            int j = is_outlier ? idx_sorted[col - r] : comp[col];
            float acc = 0.0f;
            for (int i = 0; i < N; ++i) {
                float x;
                if (is_outlier) {
                    x = bf16_to_f32(outl[i][t * k + (col - r)]);
                } else {
                    uint8_t byte = codes[i][t * cb + (col >> 1)];
                    unsigned code = (col & 1) ? (byte >> 4) : (byte & 0x0Fu);
                    float sc = bf16_to_f32(scale[i][t * ng + col / G]);
                    float z = bf16_to_f32(zero[i][t * ng + col / G]);
                    float prod = (float)code * sc;
                    x = prod + z;
                }
                if (accum == ORC_ACC_BF16) {
                    x = round_to_bf16(x);
                    acc = (i == 0) ? x : round_to_bf16(acc + x);
                } else {
                    acc = (i == 0) ? x : acc + x;
                }
            }
            if (addend) {
                float a = bf16_to_f32(addend[t * ldAdd + j]);
                acc = acc + a;
                if (accum == ORC_ACC_BF16) acc = round_to_bf16(acc);
            }
            if (bias) {
                float b = bf16_to_f32(bias[j]);
                acc = acc + b;
                if (accum == ORC_ACC_BF16) acc = round_to_bf16(acc);
            }
            if (of)
                of[j] = acc;
            else
                ob[j] = f32_to_bf16(acc);
        }
    }
    free(comp);
    return ORC_OK;
}

/* ---- other bit widths ---------------------------------------------------- */

static int bits_ok(int b) { return b == 2 || b == 3 || b == 4 || b == 5 || b == 6 || b == 8; }

/* bit n of a row's code string is bit n%8 of byte n/8 */
static void put_code(uint8_t *row, int64_t c, int b, unsigned code)
{
    for (int i = 0; i < b; ++i) {
        int64_t n = (int64_t)b * c + i;
        if ((code >> i) & 1u) row[n >> 3] |= (uint8_t)(1u << (n & 7));
    }
}

static unsigned get_code(const uint8_t *row, int64_t c, int b)
{
    unsigned code = 0;
    for (int i = 0; i < b; ++i) {
        int64_t n = (int64_t)b * c + i;
        code |= (unsigned)((row[n >> 3] >> (n & 7)) & 1u) << i;
    }
    return code;
}

/*
 * orc_encode with b-bit codes (paper Sec. 4, Fig. 3: the number of bits of the
 * quantised features is varied).  codes: uint8 [T][ceil(r*b/8)].
 */
int orc_encode_bits(const uint16_t *Y, int64_t T, int64_t ldY, int E, int k, int G, int bits,
                    const int32_t *idx_sorted, uint16_t *outl, uint8_t *codes,
                    uint16_t *scale, uint16_t *zero, int threads)
{
    if (!Y || T < 0 || E < 1 || k < 0 || k > E || G < 2 || (G & 1) || ldY < E || !bits_ok(bits))
        return ORC_ERR_ARG;
    if (k > 0 && (!idx_sorted || !outl)) return ORC_ERR_ARG;
    if (k < E && (!codes || !scale || !zero)) return ORC_ERR_ARG;
    if (!check_indices(idx_sorted, k, E)) return ORC_ERR_ARG;
    int r = E - k;
    int64_t cb = ((int64_t)r * bits + 7) / 8;
    int ng = (r + G - 1) / G;
    float qmax = (float)((1 << bits) - 1);
    int32_t *comp = build_compaction(idx_sorted, k, E);
    if (!comp) return ORC_ERR_ARG;
    set_threads(threads);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const uint16_t *y = Y + t * ldY;
        for (int p = 0; p < k; ++p) outl[t * k + p] = y[idx_sorted[p]];
        uint8_t *row = codes ? codes + t * cb : NULL;
        if (row) memset(row, 0, (size_t)cb);
        for (int g = 0; g < ng; ++g) {
            int c0 = g * G;
            int c1 = c0 + G < r ? c0 + G : r;
            float mn = bf16_to_f32(y[comp[c0]]);
            float mx = mn;
            for (int c = c0 + 1; c < c1; ++c) {
                float v = bf16_to_f32(y[comp[c]]);
                if (v < mn) mn = v;
                if (v > mx) mx = v;
            }
            mn += 0.0f;
            float span = mx - mn;
            float s32 = span / qmax;
            uint16_t sb = f32_to_bf16(s32);
            float s = bf16_to_f32(sb);
            zero[t * ng + g] = f32_bits_hi(mn);
            if (s < 1e-30f) {
                scale[t * ng + g] = 0;
                continue;
            }
            scale[t * ng + g] = sb;
            float inv = 1.0f / s;
            for (int c = c0; c < c1; ++c) {
                float v = bf16_to_f32(y[comp[c]]);
                float d = v - mn;
                float p = d * inv;
                float q = rintf(p); /* ties to even */
                if (q < 0.0f) q = 0.0f;
                if (q > qmax) q = qmax;
                put_code(row, c, bits, (unsigned)q);
            }
        }
    }
    free(comp);
    return ORC_OK;
}

/* orc_decode_reduce with b-bit codes; everything else as there. */
int orc_decode_reduce_bits(int N, int64_t T, int E, int k, int G, int bits,
                           const int32_t *idx_sorted, const uint8_t *const *codes,
                           const uint16_t *const *scale, const uint16_t *const *zero,
                           const uint16_t *const *outl, int accum, int out_fp32,
                           void *out, int threads)
{
    if (N < 1 || T < 0 || E < 1 || k < 0 || k > E || G < 2 || (G & 1) || !out || !bits_ok(bits))
        return ORC_ERR_ARG;
    if (accum != ORC_ACC_FP32 && accum != ORC_ACC_BF16) return ORC_ERR_ARG;
    if (k > 0 && (!idx_sorted || !outl)) return ORC_ERR_ARG;
    if (k < E && (!codes || !scale || !zero)) return ORC_ERR_ARG;
    if (!check_indices(idx_sorted, k, E)) return ORC_ERR_ARG;
    int r = E - k;
    int64_t cb = ((int64_t)r * bits + 7) / 8;
    int ng = (r + G - 1) / G;
    int32_t *comp = build_compaction(idx_sorted, k, E);
    if (!comp) return ORC_ERR_ARG;
    set_threads(threads);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        float *of = out_fp32 ? (float *)out + t * E : NULL;
        uint16_t *ob = out_fp32 ? NULL : (uint16_t *)out + t * E;
        for (int col = 0; col < E; ++col) {
            int is_outlier = col >= r;
            int j = is_outlier ? idx_sorted[col - r] : comp[col];
            float acc = 0.0f;
            for (int i = 0; i < N; ++i) {
                float x;
                if (is_outlier) {
                    x = bf16_to_f32(outl[i][t * k + (col - r)]);
                } else {
                    unsigned code = get_code(codes[i] + t * cb, col, bits);
                    float s = bf16_to_f32(scale[i][t * ng + col / G]);
                    float z = bf16_to_f32(zero[i][t * ng + col / G]);
                    float prod = (float)code * s; /* exact: at most 8 bits x 8 bits */
                    x = prod + z;
                }
                if (accum == ORC_ACC_BF16) {
                    x = round_to_bf16(x);
                    acc = (i == 0) ? x : round_to_bf16(acc + x);
                } else {
                    acc = (i == 0) ? x : acc + x;
                }
            }
            if (of)
                of[j] = acc;
            else
                ob[j] = f32_to_bf16(acc);
        }
    }
    free(comp);
    return ORC_OK;
}

/* ---- static symmetric mode at other bit widths --------------------------- */

/*
 * The static symmetric quantiser with b-bit codes (Sec. 4, Fig. 3 varies the bits of the
 * paper's own quantiser): step = R / (2^b - 1), code = rint(x * (1/step)) clamped to
 * -2^(b-1) .. 2^(b-1) - 1, travelling as the field code + 2^(b-1) of the row's bit string.
 * b = 4 gives orc_static_params / orc_encode_static / orc_decode_reduce_static.
 */
int orc_static_params_bits(const float *m, const float *M, int N, int E, int bits, float *step,
                           float *inv)
{
    if (!m || !M || !step || !inv || N < 1 || E < 1 || !bits_ok(bits)) return ORC_ERR_ARG;
    float qmax = (float)((1 << bits) - 1);
    for (int64_t q = 0; q < (int64_t)N * E; ++q) {
        float lo = -m[q], hi = M[q];
        float R = 2.0f * (lo > hi ? lo : hi);
        R += 0.0f;
        float d = R / qmax;
        if (!(d >= 1e-30f)) {
            step[q] = 0.0f;
            inv[q] = 0.0f;
        } else {
            step[q] = d;
            inv[q] = 1.0f / d;
        }
    }
    return ORC_OK;
}

int orc_encode_static_bits(const uint16_t *Y, int64_t T, int64_t ldY, int E, int k, int bits,
                           const int32_t *idx_sorted, const float *inv, uint16_t *outl,
                           uint8_t *codes, int threads)
{
    if (!Y || T < 0 || E < 1 || k < 0 || k > E || ldY < E || !bits_ok(bits)) return ORC_ERR_ARG;
    if (k > 0 && (!idx_sorted || !outl)) return ORC_ERR_ARG;
    if (k < E && (!codes || !inv)) return ORC_ERR_ARG;
    if (!check_indices(idx_sorted, k, E)) return ORC_ERR_ARG;
    int r = E - k;
    int64_t cb = ((int64_t)r * bits + 7) / 8;
    float half = (float)(1 << (bits - 1));
    int32_t *comp = build_compaction(idx_sorted, k, E);
    if (!comp) return ORC_ERR_ARG;
    set_threads(threads);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const uint16_t *y = Y + t * ldY;
        for (int p = 0; p < k; ++p) outl[t * k + p] = y[idx_sorted[p]];
        uint8_t *row = codes ? codes + t * cb : NULL;
        if (row) memset(row, 0, (size_t)cb);
        for (int c = 0; c < r; ++c) {
            int j = comp[c];
            float x = bf16_to_f32(y[j]);
            float p = x * inv[j];
            float q = rintf(p); /* ties to even */
            if (q < -half) q = -half;
            if (q > half - 1.0f) q = half - 1.0f;
            put_code(row, c, bits, (unsigned)((int)q + (int)half));
        }
    }
    free(comp);
    return ORC_OK;
}

int orc_decode_reduce_static_bits(int N, int64_t T, int E, int k, int bits,
                                  const int32_t *idx_sorted, const uint8_t *const *codes,
                                  const uint16_t *const *outl, const float *step, int accum,
                                  int out_fp32, void *out, int threads)
{
    if (N < 1 || T < 0 || E < 1 || k < 0 || k > E || !out || !bits_ok(bits)) return ORC_ERR_ARG;
    if (accum != ORC_ACC_FP32 && accum != ORC_ACC_BF16) return ORC_ERR_ARG;
    if (k > 0 && (!idx_sorted || !outl)) return ORC_ERR_ARG;
    if (k < E && (!codes || !step)) return ORC_ERR_ARG;
    if (!check_indices(idx_sorted, k, E)) return ORC_ERR_ARG;
    int r = E - k;
    int64_t cb = ((int64_t)r * bits + 7) / 8;
    int half = 1 << (bits - 1);
    int32_t *comp = build_compaction(idx_sorted, k, E);
    if (!comp) return ORC_ERR_ARG;
    set_threads(threads);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        float *of = out_fp32 ? (float *)out + t * E : NULL;
        uint16_t *ob = out_fp32 ? NULL : (uint16_t *)out + t * E;
        for (int col = 0; col < E; ++col) {
            int is_outlier = col >= r;
            int j = is_outlier ? idx_sorted[col - r] : comp[col];
            float acc = 0.0f;
            for (int i = 0; i < N; ++i) {
                float x;
                if (is_outlier) {
                    x = bf16_to_f32(outl[i][t * k + (col - r)]);
                } else {
                    int field = (int)get_code(codes[i] + t * cb, col, bits);
                    float q = (float)(field - half);
                    x = q * step[(int64_t)i * E + j];
                }
                if (accum == ORC_ACC_BF16) {
                    x = round_to_bf16(x);
                    acc = (i == 0) ? x : round_to_bf16(acc + x);
                } else {
                    acc = (i == 0) ? x : acc + x;
                }
            }
            if (of)
                of[j] = acc;
            else
                ob[j] = f32_to_bf16(acc);
        }
    }
    free(comp);
    return ORC_OK;
}

/* ---- static symmetric mode --------------------------------------------- */

/*
 * Per device i and feature j (paper Sec. 3): R = 2*max(-m, M), step = R/15,
 * inv = 1/step; a vanishing range gives step = inv = 0.
 * m, M, step, inv: float [N][E].
 */
int orc_static_params(const float *m, const float *M, int N, int E, float *step, float *inv)
{
    if (!m || !M || !step || !inv || N < 1 || E < 1) return ORC_ERR_ARG;
    for (int64_t q = 0; q < (int64_t)N * E; ++q) {
        float lo = -m[q], hi = M[q];
        float R = 2.0f * (lo > hi ? lo : hi);
        R += 0.0f;
        float d = R / 15.0f;
        if (!(d >= 1e-30f)) {
            step[q] = 0.0f;
            inv[q] = 0.0f;
        } else {
            step[q] = d;
            inv[q] = 1.0f / d;
        }
    }
    return ORC_OK;
}

/*
 * One device's partial sums -> outl bf16 [T][k] and codes u8 [T][ceil(r/2)]
 * (two nibbles per byte, low nibble first, nibble = code + 8).
 * inv: this device's float [E], in feature order.
 */
int orc_encode_static(const uint16_t *Y, int64_t T, int64_t ldY, int E, int k,
                      const int32_t *idx_sorted, const float *inv, uint16_t *outl,
                      uint8_t *codes, int threads)
{
    if (!Y || T < 0 || E < 1 || k < 0 || k > E || ldY < E) return ORC_ERR_ARG;
    if (k > 0 && (!idx_sorted || !outl)) return ORC_ERR_ARG;
    if (k < E && (!codes || !inv)) return ORC_ERR_ARG;
    if (!check_indices(idx_sorted, k, E)) return ORC_ERR_ARG;
    int r = E - k;
    int cb = (r + 1) / 2;
    int32_t *comp = build_compaction(idx_sorted, k, E);
    if (!comp) return ORC_ERR_ARG;
    set_threads(threads);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const uint16_t *y = Y + t * ldY;
        for (int p = 0; p < k; ++p) outl[t * k + p] = y[idx_sorted[p]];
        uint8_t *row = codes ? codes + t * cb : NULL;
        if (row) memset(row, 0, (size_t)cb);
        for (int c = 0; c < r; ++c) {
            int j = comp[c];
            float x = bf16_to_f32(y[j]);
            float p = x * inv[j];
            float q = rintf(p); /* ties to even */
            if (q < -8.0f) q = -8.0f;
            if (q > 7.0f) q = 7.0f;
            unsigned nib = (unsigned)((int)q + 8);
            if (c & 1)
                row[c >> 1] |= (uint8_t)(nib << 4);
            else
                row[c >> 1] |= (uint8_t)nib;
        }
    }
    free(comp);
    return ORC_OK;
}

/*
 * N static-mode messages -> out [T][E] in original feature order; step is
 * float [N][E] in feature order.  Accumulation as in orc_decode_reduce.
 */
int orc_decode_reduce_static(int N, int64_t T, int E, int k, const int32_t *idx_sorted,
                             const uint8_t *const *codes, const uint16_t *const *outl,
                             const float *step, int accum, int out_fp32, void *out,
                             int threads)
{
    if (N < 1 || T < 0 || E < 1 || k < 0 || k > E || !out) return ORC_ERR_ARG;
    if (accum != ORC_ACC_FP32 && accum != ORC_ACC_BF16) return ORC_ERR_ARG;
    if (k > 0 && (!idx_sorted || !outl)) return ORC_ERR_ARG;
    if (k < E && (!codes || !step)) return ORC_ERR_ARG;
    if (!check_indices(idx_sorted, k, E)) return ORC_ERR_ARG;
    int r = E - k;
    int cb = (r + 1) / 2;
    int32_t *comp = build_compaction(idx_sorted, k, E);
    if (!comp) return ORC_ERR_ARG;
    set_threads(threads);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        float *of = out_fp32 ? (float *)out + t * E : NULL;
        uint16_t *ob = out_fp32 ? NULL : (uint16_t *)out + t * E;
        for (int col = 0; col < E; ++col) {
            int is_outlier = col >= r;
            int j = is_outlier ? idx_sorted[col - r] : comp[col];
            float acc = 0.0f;
            for (int i = 0; i < N; ++i) {
                float x;
                if (is_outlier) {
                    x = bf16_to_f32(outl[i][t * k + (col - r)]);
                } else {
                    uint8_t byte = codes[i][t * cb + (col >> 1)];
                    unsigned nib = (col & 1) ? (byte >> 4) : (byte & 0x0Fu);
                    float q = (float)((int)nib - 8);
                    x = q * step[(int64_t)i * E + j];
                }
                if (accum == ORC_ACC_BF16) {
                    x = round_to_bf16(x);
                    acc = (i == 0) ? x : round_to_bf16(acc + x);
                } else {
                    acc = (i == 0) ? x : acc + x;
                }
            }
            if (of)
                of[j] = acc;
            else
                ob[j] = f32_to_bf16(acc);
        }
    }
    free(comp);
    return ORC_OK;
}
