/*
 * tpq.h -- C ABI of the low-bit tensor-parallel partial-sum codec for MI355X.
 *
 * The library implements, on one GPU, the per-device hot path of hybrid
 * BF16 / 4-bit communication for tensor-parallel inference:
 *
 *   - offline calibration: per-device per-feature min/max moving averages
 *     (paper Sec. 3 "Calibration", Eq. (1), (2)), symmetric ranges, their sum
 *     over devices and the top-k features with the widest aggregated range
 *     (Sec. 3 "Selecting High Precision Features");
 *   - tpq_encode: the compression function C^(i) of Sec. 2 in the form of
 *     Fig. 2 -- the k selected features of every row are sent verbatim in
 *     BF16, the other r = E-k features as bit-packed 4-bit codes;
 *   - tpq_decode_reduce: the decompression D^(i) of all N devices' messages
 *     and their sum (Sec. 2; Fig. 2 caption), features back in original order;
 *   - further down: the static symmetric mode of Sec. 3, other code widths (Sec. 4), the
 *     block's epilogue inside decode_reduce, a ring step (Sec. 5), and the device's linear
 *     layer f^(i)(x^(i)) = x^(i) W^(i) of Sec. 2 with the compression in its epilogue.
 *
 * Quantiser (the workload definition's group-wise asymmetric form): the r
 * non-selected features of a row, taken in ascending feature order
 * ("compacted"), are cut into groups of G; per (row, group):
 *     zero  = group minimum                      (a bf16 value, stored exactly)
 *     scale = bf16_rne((max - min) / 15)         (0 if below 1e-30: constant group)
 *     code  = clamp(rint((x - zero) * (1/float(scale))), 0, 15)   (ties to even)
 *     x_hat = code * scale + zero
 * All arithmetic is IEEE binary32 without contraction.
 *
 * Other code widths (Sec. 4, the experiment that varies the number of bits of the
 * quantised features, Fig. 3): bits b in {2, 3, 5, 6, 8} beside 4, with 2^b - 1 in
 * place of 15 everywhere above.  The codes of a row then form one little-endian bit
 * string: code c occupies bits b*c .. b*c + b - 1, bit n of the string being bit
 * n % 8 of byte n / 8 (for b = 4 that is the nibble layout below).  For these
 * widths the kernels store whole chunks of 8 codes (b bytes; unused bits zero) and
 * read 8 bytes from the start of each chunk, so pitch_codes is at least
 * ceil(r/8)*b + 8, rounded up to 16.
 *
 * Message of one device for one block = four row-major matrices:
 *     outl  bf16  [T][k]             pitch_outl  bytes per row
 *     codes u8    [T][ceil(r/2)]     pitch_codes bytes per row
 *                 byte b = code 2b (bits 0-3) | code 2b+1 (bits 4-7); a final
 *                 odd nibble and the pad bytes up to a multiple of 4 are zero
 *     scale bf16  [T][ng]            pitch_meta  bytes per row, ng = ceil(r/G)
 *     zero  bf16  [T][ng]            pitch_meta  bytes per row
 *
 * General rules
 *   - Every function returns TPQ_OK (0) or a negative TPQ_ERR_* code; nothing
 *     throws.  Argument errors are detected on the host before anything is
 *     enqueued and leave all outputs untouched.
 *   - Pointers marked [device] are device memory; [host] are host memory.  bf16
 *     data is passed as uint16_t bit patterns.  Device pointers must be 16-byte
 *     aligned, leading dimensions / pitches as stated per argument.
 *   - The library never allocates, frees or retains device memory; all buffers
 *     belong to the caller.  There is no global state beyond two thread-local
 *     items (the last HIP error, a pending tpq_bench_time_next_launch request), the
 *     number of compute units of each device (looked up once), and the static device
 *     array of tpq_calibrate_fixed, the one call that brings its own scratch; calls
 *     are re-entrant across streams (tpq_calibrate_fixed: see there).
 *   - Work is enqueued on the given HIP stream (a hipStream_t passed as void*,
 *     NULL = the default stream) and the call returns without synchronising,
 *     except tpq_plan_check.
 *   - Inputs must be finite.  NaN / Inf give unspecified values, never a fault.
 *   - T = 0 (or S = 0) is a successful no-op.
 */
#ifndef TPQ_H
#define TPQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TPQ_OK 0
#define TPQ_ERR_NULL (-1)        /* a required pointer is NULL                         */
#define TPQ_ERR_SHAPE (-2)       /* a size is out of range or inconsistent             */
#define TPQ_ERR_INDEX (-3)       /* indices unsorted, duplicated or out of range       */
#define TPQ_ERR_UNSUPPORTED (-4) /* bits not in {2,3,4,5,6,8}, G not in {32,64,128,256}, bad mode */
#define TPQ_ERR_ALIGN (-5)       /* pointer or pitch alignment                         */
#define TPQ_ERR_WORKSPACE (-6)   /* workspace / plan buffer too small                  */
#define TPQ_ERR_HIP (-7)         /* a HIP call failed; see tpq_last_hip_error()        */

#define TPQ_ACC_FP32 0 /* x_0 + x_1 + ... in fp32, ascending device order              */
#define TPQ_ACC_BF16 1 /* every term and every partial sum rounded to bf16             */
#define TPQ_ACC_FAST 2 /* the bf16 accumulate mode at its tolerance instead of its letter: terms
                        * and partial sums stay fp32, one rounding at the end (the arithmetic
                        * of TPQ_ACC_FP32).  Within half a bf16 ulp of the exact sum; from the
                        * literal chain it differs by at most the chain's own rounding,
                        * (N + 1) * 2^-9 * sum_i |x_hat_i|, and by less than 1e-2 of that sum
                        * for all but a few elements per million                             */
#define TPQ_OUT_BF16 0
#define TPQ_OUT_FP32 1

#define TPQ_MAX_RANKS 64
#define TPQ_MAX_E 32768

/* Geometry of one block's message.  Fill with tpq_layout_init; the pitches may
 * then be raised by the caller (multiples of 16 bytes). */
typedef struct tpq_layout {
    int32_t E;          /* features per row; multiple of 8, <= TPQ_MAX_E               */
    int32_t k;          /* features kept in bf16, 0 <= k <= E                          */
    int32_t G;          /* quantisation group size: 32, 64, 128 or 256                 */
    int32_t bits;       /* code width b: 2, 3, 4, 5, 6 or 8                            */
    int32_t r;          /* E - k                                                       */
    int32_t ng;         /* ceil(r / G)                                                 */
    int32_t code_bytes; /* ceil(r * b / 8)                                             */
    int32_t reserved;
    int64_t pitch_codes; /* bytes per row of codes, multiple of 16, >= code_bytes      */
    int64_t pitch_meta;  /* bytes per row of scale and of zero, multiple of 16         */
    int64_t pitch_outl;  /* bytes per row of outl, multiple of 16                      */
    int64_t wire_bytes_per_row; /* 2k + code_bytes + 4*ng: what really travels         */
} tpq_layout;

/* [host] Derive the layout for (E, k, G, bits).  Pure host function. */
int tpq_layout_init(tpq_layout *L, int E, int k, int G, int bits);

/* Average bits per communicated value.  payload = (16k + b*r)/E is the paper's
 * accounting (abstract; Sec. 4: k = floor(E/64) gives 4.1875 < 4.2); wire adds
 * the per-group scale and zero: 8 * wire_bytes_per_row / E. */
double tpq_payload_bits(const tpq_layout *L);
double tpq_wire_bits(const tpq_layout *L);

const char *tpq_strerror(int code);
int tpq_last_hip_error(void); /* hipError_t of the most recent TPQ_ERR_HIP on this thread */

/* Measurement aid (for benchmarks: no part of the method).  The next kernel that
 * tpq_encode, tpq_hop, tpq_encode_static, tpq_decode_reduce, tpq_decode_reduce_fused or
 * tpq_decode_reduce_static (or tpq_gemm_encode) launches from the calling thread carries the two HIP events
 * (hipEvent_t passed as void*, created by the caller with timing enabled) on its own
 * dispatch: afterwards hipEventElapsedTime(start, stop) is that kernel's duration on
 * the GPU, without the idle time that separately recorded events put around a launch.
 * One launch only (a call that splits its rows over several launches times the first);
 * a request stays pending, also across calls that fail their argument checks, until a
 * kernel is launched or both NULL cancel it. */
int tpq_bench_time_next_launch(void *start_event, void *stop_event);

/* ---- plan: device tables derived from the static outlier index set -------
 * The selected features are fixed across sequences and devices (Sec. 3), so
 * the compaction map (which feature each compacted position reads) is built
 * once per block and reused by every encode / decode_reduce call.
 *   idx_sorted [device] int32[k], ascending, unique, in [0, E).
 *   plan       [device] tpq_plan_bytes(L) bytes, 16-byte aligned, caller-owned.
 * tpq_plan_build validates the indices on the device; encode / decode_reduce
 * given a plan that is invalid (or built for another E, k, G) write nothing.
 * The buffer handed to encode / decode_reduce / tpq_hop / the static calls must hold at
 * least tpq_plan_bytes(L) bytes for the L of THAT call, whatever it was built for: the
 * kernels fetch their first table entries, at offsets that follow from L alone, together
 * with the header that tells them whether the plan fits.
 * tpq_plan_check synchronises the stream and reports TPQ_ERR_INDEX /
 * TPQ_ERR_SHAPE for such a plan. */
size_t tpq_plan_bytes(const tpq_layout *L);
int tpq_plan_build(const tpq_layout *L, const int32_t *idx_sorted, void *plan,
                   size_t plan_bytes, void *stream);
int tpq_plan_check(const tpq_layout *L, const void *plan, void *stream);

/* ---- calibration (Sec. 3, Eq. (1), (2)) -----------------------------------
 * One call = one calibration sequence of one device:
 *   cmin_j = min_t Y[t][j], cmax_j = max_t Y[t][j]     (a zero is taken as +0)
 *   seq_index == 0:  m = cmin, M = cmax
 *   otherwise:       m = (1-gamma)*m + gamma*cmin  (three rounded fp32 ops), same for M
 *   Y         [device] bf16 [S][ldY], ldY in elements, multiple of 8, >= E
 *   m, M      [device] fp32 [n_ranks][E]; row `rank` is updated
 *   workspace [device] >= tpq_calibrate_workspace_bytes(S, E) bytes, 16-byte aligned, contents
 *             arbitrary; calls that share a workspace must not overlap in time */
size_t tpq_calibrate_workspace_bytes(int64_t S, int E);
int tpq_calibrate(const uint16_t *Y, int64_t S, int64_t ldY, int E, int rank,
                  int n_ranks, int64_t seq_index, float gamma, float *m, float *M,
                  void *workspace, size_t ws_bytes, void *stream);

/* tpq_calibrate for callers that cannot provide scratch memory they have allocated (code
 * under HIP graph capture, serving loops or harnesses that forbid hipMalloc): the same
 * kernels, with the partial minima / maxima of the row slices in a buffer that is part
 * of the library's device image (TPQ_CALIBRATE_FIXED_SCRATCH_BYTES per GPU, held until the
 * process ends) instead of a workspace argument.  Allocates nothing and calls no allocating
 * routine.  E <= TPQ_CALIBRATE_FIXED_MAX_E (TPQ_ERR_SHAPE beyond that); everything else as
 * tpq_calibrate, results bit-identical to it.  Every call on a GPU uses that GPU's one
 * buffer: calls that overlap in time on one GPU race (order them on one stream or by events). */
#define TPQ_CALIBRATE_FIXED_MAX_E 8192
#define TPQ_CALIBRATE_FIXED_SCRATCH_BYTES (64 * 2 * TPQ_CALIBRATE_FIXED_MAX_E * 4)
int tpq_calibrate_fixed(const uint16_t *Y, int64_t S, int64_t ldY, int E, int rank,
                        int n_ranks, int64_t seq_index, float gamma, float *m, float *M,
                        void *stream);

/* After the last sequence (Sec. 3):
 *   R[i][j] = 2*max(-m[i][j], M[i][j]);  Rbar[j] = R[0][j] + R[1][j] + ... (fp32, ascending i)
 *   the k features with the largest Rbar (ties: lower index first)
 *   R          [device] fp32 [n_ranks][E], may be NULL
 *   Rbar       [device] fp32 [E]
 *   idx_sorted [device] int32[k], ascending feature order (what tpq_plan_build takes)
 *   idx_ranked [device] int32[k], by descending Rbar; may be NULL
 *   workspace  [device] >= tpq_calibrate_finalize_workspace_bytes(E) bytes */
size_t tpq_calibrate_finalize_workspace_bytes(int E);
int tpq_calibrate_finalize(const float *m, const float *M, int n_ranks, int E, int k,
                           float *R, float *Rbar, int32_t *idx_sorted,
                           int32_t *idx_ranked, void *workspace, size_t ws_bytes,
                           void *stream);

/* ---- encode (Sec. 2 C^(i); Fig. 2) ----------------------------------------
 * Encodes n_ranks partial-sum tensors in one launch (n_ranks = 1 is a single
 * device's real call; larger values simulate several devices on one GPU).
 *   Y     [host] array of n_ranks [device] pointers, each bf16 [T][ldY]
 *   ldY   elements, multiple of 8, >= E
 *   codes, scale, zero, outl: [host] arrays of n_ranks [device] pointers to the
 *         message sections (see the layout above); outl entries are ignored when
 *         k = 0, the other three when k = E
 *   plan  [device] built by tpq_plan_build for the same layout */
int tpq_encode(const tpq_layout *L, const void *plan, const uint16_t *const *Y,
               int64_t ldY, int n_ranks, int64_t T, uint8_t *const *codes,
               uint16_t *const *scale, uint16_t *const *zero, uint16_t *const *outl,
               void *stream);

/* ---- ring step (Sec. 5: the closing remark that the method, made for all-reduce as
 * all-gather plus local reduction, could be adapted to ring all-reduce; the paper fixes
 * no detail, the reading here is the plainest one) ------------------------------
 * Device i has received a message and owns the partial sum Y[i]; what it sends on is
 *     tpq_encode( bf16( D(message) (+) Y[i] ) )
 * where D is the dequantisation of tpq_decode_reduce (selected features: the bf16 value
 * itself) and (+) the accumulation's addition with Y[i] as its second term: fp32 sum
 * rounded to bf16 once (TPQ_ACC_FP32), or D's value rounded to bf16 first
 * (TPQ_ACC_BF16, the literal bf16 chain).  The result equals tpq_decode_reduce_fused
 * over that one message with addend Y[i] and bf16 output, followed by tpq_encode, but
 * the sum never goes to memory.  One launch serves n_ranks devices side by side, each with
 * its own received message, partial sum and outgoing message, as tpq_encode does.
 *   in_codes, in_scale, in_zero, in_outl  [host] arrays of n_ranks [device] pointers:
 *         the received messages (layout L); must not overlap the outgoing ones
 *   n_ranks  1 .. TPQ_MAX_HOP_RANKS
 * Everything else as tpq_encode.  4-bit layouts only (TPQ_ERR_UNSUPPORTED otherwise). */
#define TPQ_MAX_HOP_RANKS 16
int tpq_hop(const tpq_layout *L, const void *plan, const uint16_t *const *Y, int64_t ldY,
            int n_ranks, int64_t T, const uint8_t *const *in_codes,
            const uint16_t *const *in_scale, const uint16_t *const *in_zero,
            const uint16_t *const *in_outl, int accum, uint8_t *const *codes,
            uint16_t *const *scale, uint16_t *const *zero, uint16_t *const *outl,
            void *stream);

/* ---- the linear layer with the compression in its epilogue (Sec. 2: device i computes
 * f^(i)(x^(i)) = x^(i) W^(i), the partial sum that C^(i) compresses; Sec. 3, "Selecting
 * High Precision Features", names the selection before the exchange as the overhead) ----
 *     message = tpq_encode( bf16( X * Wt^T ) )
 * for ONE device, without the partial sums going to memory: the product is accumulated
 * in fp32 on the matrix cores, rounded to bf16 once, and compressed from registers.  The
 * sums of the K products are taken in the matrix cores' own order, so the bf16 product can
 * differ from a product summed otherwise in its last bit where the exact sum lies next to
 * a rounding boundary; given that bf16 product, the message is exactly tpq_encode's.
 *
 * The weights are reordered once, offline (they and the selected features are static):
 *   tpq_gemm_weights: Wt [device] bf16 [E][ldW], one row per output feature (W^(i)
 *         transposed: the layout of a linear layer's weight), K columns used;
 *         Wp [device] bf16 [E][K]: the rows of Wt in message order -- the r features that are
 *         quantised, ascending, then the k selected ones, ascending.  plan as for tpq_encode.
 *   tpq_gemm_encode: X [device] bf16 [T][ldX] (K columns used), Wp from tpq_gemm_weights;
 *         codes, scale, zero, outl [device]: the device's message sections (layout L; outl is
 *         ignored when k = 0, the other three when k = E);
 *         Y_msg [device] bf16 [T][ldYm] or NULL: if given, also receives the rounded product
 *         in message order (feature n < r = compacted feature n, n >= r = selected feature
 *         n - r): what a device keeps when it takes its own partial sum unquantised.
 *   K, ldW, ldX, ldYm: elements, multiples of 8; ldW, ldX >= K; ldYm >= E.  No plan is needed
 *   by tpq_gemm_encode: the order is in Wp.  4-bit layouts only (TPQ_ERR_UNSUPPORTED
 *   otherwise); T <= 65535 * 64. */
int tpq_gemm_weights(const tpq_layout *L, const void *plan, const uint16_t *Wt, int64_t ldW,
                     int K, uint16_t *Wp, void *stream);
int tpq_gemm_encode(const tpq_layout *L, const uint16_t *X, int64_t T, int64_t ldX, int K,
                    const uint16_t *Wp, uint8_t *codes, uint16_t *scale, uint16_t *zero,
                    uint16_t *outl, uint16_t *Y_msg, int64_t ldYm, void *stream);

/* ---- decode + reduce (Sec. 2 D^(i) and the sum; Fig. 2 caption) ------------
 * out[t][j] = sum over the n_ranks messages of x_hat (selected features: the
 * bf16 value itself), in ascending device order, in original feature order.
 *   accum     TPQ_ACC_FP32 or TPQ_ACC_BF16
 *   out_dtype TPQ_OUT_BF16: out is bf16 [T][ldOut] (fp32 accumulator rounded once);
 *             TPQ_OUT_FP32: out is fp32 [T][ldOut] (needs accum = TPQ_ACC_FP32 or
 *             gives the bf16-valued accumulator widened)
 *   ldOut     elements; multiple of 8 (bf16) or 4 (fp32), >= E */
int tpq_decode_reduce(const tpq_layout *L, const void *plan, int n_ranks, int64_t T,
                      const uint8_t *const *codes, const uint16_t *const *scale,
                      const uint16_t *const *zero, const uint16_t *const *outl,
                      int accum, int out_dtype, void *out, int64_t ldOut,
                      void *stream);

/* tpq_decode_reduce followed by the block's epilogue (Sec. 2: the output of a
 * row-parallel block is the sum over the devices plus the bias,
 * f(x) = [sum_i f^(i)(x^(i))] + b), inside the same kernel:
 *     out[t][j] = ((sum over the n_ranks messages) (+) addend[t][j]) (+) bias[j]
 * where (+) is the accumulation's own addition (fp32; in TPQ_ACC_BF16 every result is
 * rounded to bf16), the terms entering in this order.
 *   addend  [device] bf16 [T][ldAdd] or NULL: a residual -- or the device's own partial
 *           sum, when the caller leaves that device's message out of the n_ranks
 *           messages (its own data then carries no quantisation error); ldAdd >= E;
 *           rows need 2-byte alignment only
 *   bias    [device] bf16 [E] or NULL
 * Everything else as tpq_decode_reduce.  4-bit layouts only (TPQ_ERR_UNSUPPORTED
 * otherwise).  With both NULL the result equals tpq_decode_reduce's. */
int tpq_decode_reduce_fused(const tpq_layout *L, const void *plan, int n_ranks, int64_t T,
                            const uint8_t *const *codes, const uint16_t *const *scale,
                            const uint16_t *const *zero, const uint16_t *const *outl,
                            const uint16_t *addend, int64_t ldAdd, const uint16_t *bias, int accum,
                            int out_dtype, void *out, int64_t ldOut, void *stream);

/* ---- static symmetric mode (the paper's own quantiser, Sec. 3) --------------
 * "Calibration": every feature on every device has static, independent
 * quantisation parameters; "Selecting High Precision Features": the range is
 * R = 2*max(-m, M) and every feature that is not kept in BF16 is symmetrically
 * quantised to Int4.  The paper gives neither the step nor the code set; this
 * library takes step = R/15 (fp32, IEEE), code = round-half-even of
 * x * (1/step) clamped to -8..7, x_hat = code * step.  A feature whose
 * calibrated range vanishes (step < 1e-30) is sent as code 0 and comes back as 0.
 * The message is the codes section (same layout; the nibble is code + 8) and the
 * outl section: nothing else travels, 4 + 12k/E bits per value.  For a layout of
 * another width b (Sec. 4, Fig. 3): step = R/(2^b - 1), codes -2^(b-1) .. 2^(b-1) - 1,
 * sent as the field code + 2^(b-1) of the row's bit string; b + (16-b)k/E bits.
 *
 * tpq_static_params turns the calibration state into the two tables the kernels
 * read, in the compacted feature order of `plan`:
 *   m, M         [device] fp32 [n_ranks][E] (as left by tpq_calibrate)
 *   step, inv    [device] fp32 [n_ranks][tpq_static_table_floats(L)], 16-byte
 *                aligned; entry c of a row belongs to the c-th feature that is not
 *                selected, entries past r are 0
 * tpq_encode_static / tpq_decode_reduce_static mirror tpq_encode /
 * tpq_decode_reduce; `inv` / `step` point at the row of the first of the n_ranks
 * devices handed over (rows of consecutive devices follow each other). */
size_t tpq_static_table_floats(const tpq_layout *L);
int tpq_static_params(const tpq_layout *L, const void *plan, const float *m, const float *M,
                      int n_ranks, float *step, float *inv, void *stream);
int tpq_encode_static(const tpq_layout *L, const void *plan, const uint16_t *const *Y,
                      int64_t ldY, int n_ranks, int64_t T, const float *inv,
                      uint8_t *const *codes, uint16_t *const *outl, void *stream);
int tpq_decode_reduce_static(const tpq_layout *L, const void *plan, int n_ranks, int64_t T,
                             const uint8_t *const *codes, const uint16_t *const *outl,
                             const float *step, int accum, int out_dtype, void *out,
                             int64_t ldOut, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TPQ_H */
