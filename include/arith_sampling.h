/*
 * arith_sampling.h -- C ABI of the MI355X (gfx950) arithmetic-sampling library.
 *
 * The library runs the data-parallel decode path of arithmetic sampling
 * (Vilnis et al., "Arithmetic Sampling: Parallel Diverse Decoding for Large
 * Language Models", arXiv 2210.15458): every sequence is driven by one code
 * point c in [0,1); at each step the code selects the token whose interval of
 * the vocabulary-order cumulative distribution holds it and is then rescaled
 * to that interval (Sec. 4.1, Algorithm 1).  N codes of one prompt sit on a
 * randomly shifted lattice (Sec. 4.2, Definition "Arithmetic sampling").
 * Codes never interact (Remark after Prop. 1), so all calls below are batched
 * over independent rows.
 *
 * Conventions for every entry point
 *   - Pointers marked DEVICE point to memory of the GPU that was current when
 *     the context was created; the caller owns them and keeps them alive until
 *     the stream has run past the call.  The library never copies them to the
 *     host and never frees them.
 *   - Calls are asynchronous: work is enqueued on the context's HIP stream and
 *     the function returns.  No call synchronises the device.
 *   - Argument errors are detected on the host before anything is launched and
 *     reported through the return code; as_last_error() gives a message.
 *     Nothing throws, aborts or prints.
 *   - Data errors (NaN logits, a code outside [0,1)) are not detected; the
 *     result for such a row is unspecified but memory safe: the emitted token
 *     lies in [0,V) and the new code in [0, 1 - 2^-24].
 *   - A logit of -inf is legal and means probability zero.
 *   - as_step / as_step_ex allocate nothing and touch only the context's
 *     fixed workspace.  as_decode, as_decode_ancestral, as_decode_fused and
 *     as_encode keep their logits and per-row state in a decode workspace that
 *     the context (re)allocates when a call needs more than any earlier call
 *     did: the first call at a size synchronises the stream, frees and
 *     allocates, and must not be made under stream capture; later calls of the
 *     same or a smaller size allocate nothing and can be captured.
 *   - One context must not be used from two host threads at once.
 */
#ifndef ARITH_SAMPLING_H
#define ARITH_SAMPLING_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct as_ctx as_ctx;
typedef struct as_model as_model;

typedef enum {
    AS_OK = 0,
    AS_ERR_INVALID_ARG = 1, /* null pointer, size out of range, bad parameter  */
    AS_ERR_UNSUPPORTED = 2, /* valid request this build cannot serve           */
    AS_ERR_ALLOC = 3,       /* device or host allocation failed                */
    AS_ERR_DEVICE = 4       /* HIP reported an error (launch, stream, ...)     */
} as_status;

/* storage type of logits and of model weights */
typedef enum { AS_F32 = 0, AS_BF16 = 1 } as_dtype;

/* ---------------------------------------------------------------- context */

/*
 * Create a context bound to the current HIP device.
 *   max_rows      largest number of rows (codes) a single call will carry, >= 1
 *   V             vocabulary size, 1 <= V <= AS_MAX_VOCAB
 *   logits_dtype  storage type of every logits tensor passed with this context
 *   hip_stream    a hipStream_t (as void*) all work is enqueued on; NULL = the
 *                 default stream.  The stream must outlive the context.
 * On success *out owns a small device workspace; release it with
 * as_ctx_destroy (which synchronises the stream first).
 */
as_status as_ctx_create(as_ctx **out, int64_t max_rows, int32_t V,
                        as_dtype logits_dtype, void *hip_stream);
as_status as_ctx_destroy(as_ctx *ctx);

/* Message for the last failing call made with this context (or, with NULL, for
 * the last failing call of this thread that had no context).  The string is
 * owned by the library and valid until the next failing call. */
const char *as_last_error(const as_ctx *ctx);

#define AS_MAX_VOCAB (1 << 21)

/*
 * Kernel choices, for tests and measurements (not part of the method; nothing
 * in the environment changes what the library runs, only this call does).  Every
 * knob starts at 0, the library's own choice; any setting gives the same results
 * up to the tolerances stated for the call, only the kernel that computes them
 * changes.  Takes effect for the calls that follow on this context.
 *   AS_TUNE_STEP_SHAPE  work-group shape of the sampling kernel: 1..5 other
 *                       (waves per row x KiB per wave) splits; 6 the general
 *                       kernel also for rows that fit the single-tile one;
 *                       9 the plain three-pass kernel (slow; any alignment)
 *   AS_TUNE_GEMM_SHAPE  logits kernel: 1 = the 128x256 tile kernel instead of
 *                       the persistent one
 *   AS_TUNE_THR_PATH    keep-threshold kernel: 1 = the radix select instead of
 *                       the register-resident / streamed kernels; 2 = the
 *                       register-resident kernel also where the single-tile
 *                       top-k and nucleus kernels apply
 *   AS_TUNE_GEMM_GM     persistent logits kernel with more row tiles than
 *                       workers: workers of one XCD along the rows (a divisor
 *                       of the workers per XCD; otherwise ignored)
 */
typedef enum {
    AS_TUNE_STEP_SHAPE = 0,
    AS_TUNE_GEMM_SHAPE = 1,
    AS_TUNE_THR_PATH = 2,
    AS_TUNE_GEMM_GM = 3
} as_tuning;
as_status as_ctx_set_tuning(as_ctx *ctx, as_tuning knob, int32_t value);

/*
 * Measurement aid (not part of the method): with profiling on, every launch of
 * the sampling kernel, the logits, threshold and interval kernels carries its
 * own start/stop HIP events, taken from the dispatch on the context's stream.
 * as_ctx_profile_read synchronises the stream, returns the summed kernel time
 * and the number of timed launches since the last read for
 *   kernel 0: fused sampling step   1: logits (bigram) kernel   2: threshold   3: interval (encode) step
 * and resets the counters.  At most 16384 launches per kernel are timed between
 * reads; further ones run untimed and are counted in *untimed.  Any output
 * pointer may be NULL.  Switching profiling on makes the first launches create
 * events (a host-side allocation).
 */
as_status as_ctx_profile(as_ctx *ctx, int enable);
as_status as_ctx_profile_read(as_ctx *ctx, int kernel, double *total_ms,
                              int64_t *launches, int64_t *untimed);
/* The single durations behind that sum, for medians and percentiles: copies the
 * milliseconds of the first min(capacity, timed launches) launches of `kernel`
 * since the last read, in launch order, to the HOST array ms_out, and stores the
 * number of timed launches in *count (may be NULL).  Synchronises the stream;
 * resets nothing, so call it before as_ctx_profile_read. */
as_status as_ctx_profile_samples(as_ctx *ctx, int kernel, float *ms_out,
                                 int64_t capacity, int64_t *count);

/* ------------------------------------------------------------ single step */

/*
 * One step of Algorithm 1 (Sec. 4.1) for `rows` independent codes.
 *
 * For row r: x_v = logits[r, v] / temp; optional top-k and nucleus masks (the
 * logit modifiers of Sec. 2; masked tokens get probability zero, Sec. 5 top-k
 * paragraph); softmax over the kept tokens; inclusive cumulative sums F in
 * VOCABULARY ORDER (the total order of Sec. 3.1); token = the first v with
 * F(v) > c, i.e. c lies in [F(v-1), F(v)); c' = (c - F(v-1)) / (F(v) -
 * F(v-1)).  Arithmetic is fp32 per element with fp64 carries.
 *
 *   logits      DEVICE [rows, ld] row-major, ctx dtype, ld >= V, any stride.
 *               Columns V..ld-1 are never used.  Memory is read in whole,
 *               aligned 16-byte pieces, so the bytes that share a 16-byte
 *               granule with a row's first or last logit may be loaded (and
 *               discarded); nothing outside those granules is touched.  Rows
 *               that start on 16 bytes and are a whole number of such pieces
 *               long (V * element size a multiple of 16) run a little faster.
 *   codes       DEVICE float[rows], each in [0,1)
 *   temp        > 0
 *   top_k       keep the k highest logits and everything tied with the k-th;
 *               <= 0 or >= V: off
 *   top_p       keep the smallest set of highest-probability value groups whose
 *               mass (after top-k) reaches top_p, whole groups; <= 0 or >= 1: off
 *   tokens_out  DEVICE int32[rows]
 *   codes_out   DEVICE float[rows]; may be the same pointer as codes
 *
 * Errors in the data on the device (NaN or infinite logits, a row without a
 * finite logit, codes outside [0,1)) are not detected, no call reads device
 * data back.  What such a row returns is unspecified but stays in range:
 * tokens_out in [0, V), codes_out in [0, 1 - 2^-24]; nothing outside the
 * buffers described here is read or written.
 */
as_status as_step(as_ctx *ctx, const void *logits, int64_t rows, int64_t ld,
                  const float *codes, float temp, int32_t top_k, float top_p,
                  int32_t *tokens_out, float *codes_out);

/*
 * as_step with the per-row state of a running decode (Algorithm 1's stopping
 * rule in its padded fixed-length form, Sec. 3.3) and optional records.
 *
 *   finished_in   DEVICE uint8[rows] or NULL.  A row with a non-zero flag emits
 *                 eos_id, keeps its code, and its logits are not read.
 *   eos_id        token that ends a sequence; < 0: none
 *   finished_out  DEVICE uint8[rows] or NULL; 1 if the row was finished on
 *                 entry or emitted eos_id now.  May alias finished_in.
 *   prob_out      DEVICE float[rows] or NULL: probability of the emitted token
 *   flo_out       DEVICE float[rows] or NULL: F(v-1), start of its interval
 *   row_ids       DEVICE int32[rows] or NULL: logits row read by each code
 *                 (several codes may share a row), each in [0, logits_rows)
 *                 (an index outside is not detected; the nearest row is read)
 *   logits_rows   number of rows in `logits` when row_ids is given
 */
as_status as_step_ex(as_ctx *ctx, const void *logits, int64_t rows, int64_t ld,
                     const float *codes, float temp, int32_t top_k, float top_p,
                     int32_t *tokens_out, float *codes_out,
                     const uint8_t *finished_in, int32_t eos_id,
                     uint8_t *finished_out, float *prob_out, float *flo_out,
                     const int32_t *row_ids, int64_t logits_rows);

/*
 * as_step for callers that cannot allocate device memory and so cannot hold a
 * context: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same kernels and same results as as_step; the per-row keep
 * thresholds that the truncation kernels hand to the sampling kernel live in a
 * fixed array inside the library's device image (AS_STATIC_MAX_ROWS floats,
 * 256 KiB, held by every GPU the library runs on until the process ends).  The
 * call allocates and frees nothing, on the device or through any library; the
 * first call on a device looks the array's address up (no allocation).
 *
 *   logits_dtype, V   what a context would carry
 *   rows              0 <= rows <= AS_STATIC_MAX_ROWS, else AS_ERR_INVALID_ARG
 *   hip_stream        hipStream_t (as void*) of the current device; NULL = default
 *   other arguments   as in as_step
 * All calls on one GPU share the array: two calls whose kernels may overlap on
 * that GPU (different streams, no ordering between them) race on it when
 * top_k / top_p is on.  Nothing in it has to start at zero; every row's entry is
 * written before it is read within one call.  Failures are reported through
 * as_last_error(NULL).
 */
#define AS_STATIC_MAX_ROWS 65536
as_status as_step_static(const void *logits, as_dtype logits_dtype, int64_t rows,
                         int64_t ld, int32_t V, const float *codes, float temp,
                         int32_t top_k, float top_p, int32_t *tokens_out,
                         float *codes_out, void *hip_stream);

/* ---------------------------------------------------------------- lattice */

/*
 * Codes of Sec. 4.2 on the circular lattice with spacing 1/N:
 * codes_out[b*N + i] = (i + u[b]) / N for i = 0..N-1, evaluated in fp64 and
 * rounded once to fp32 (then kept <= 1 - 2^-24).
 *   u          DEVICE float[B], each in [0,1): one shared shift per prompt
 *   codes_out  DEVICE float[B*N];  B*N <= ctx max_rows
 */
as_status as_lattice(as_ctx *ctx, const float *u, int32_t B, int32_t N,
                     float *codes_out);

/* ------------------------------------------- synthetic sequence model + decode */

/*
 * Low-rank bigram model standing in for P(X_t | X_<t) of Sec. 3.3:
 * logits[v] = (scale / sqrt(d)) * sum_k E[prev, k] * U[k, v].
 *   E       DEVICE [V, d] row-major, wdtype; borrowed, must outlive the model
 *   U       DEVICE [d, V] row-major, wdtype; read once here (the model keeps
 *           its own K-contiguous copy) and not needed afterwards
 *   d       rank, >= 1.  AS_BF16 weights with d a multiple of 64 and a 16-byte
 *           aligned E run on the MFMA kernel; anything else on a plain
 *           dot-product kernel meant for small models only
 * The call enqueues a re-layout kernel on the default stream and waits for it.
 */
as_status as_model_create_bigram(as_model **out, const void *E, const void *U,
                                 int32_t V, int32_t d, float scale,
                                 as_dtype wdtype);
as_status as_model_destroy(as_model *model);

/*
 * logits_out[r, :] = model logits given prev[r], for r < rows (AS_BF16 weights
 * use bf16 MFMA with fp32 accumulation; the result is rounded once to the ctx
 * logits dtype).
 *   prev        DEVICE int32[rows], each in [0,V) (a value outside is not
 *               detected; the nearest valid token is used instead)
 *   logits_out  DEVICE [rows, ld], ld >= V; columns V..ld-1 are left untouched
 */
as_status as_bigram_logits(as_ctx *ctx, const as_model *model,
                           const int32_t *prev, int64_t rows, void *logits_out,
                           int64_t ld);

/*
 * Whole decode (Algorithm 1 for every code of the lattice of Sec. 4.2):
 * codes from as_lattice, then T times { logits from the model given the
 * previous token; as_step_ex with EOS kept sticky }.  Exactly the sequence of
 * the exported calls above, enqueued back to back with no host round trip.
 *   prompts     DEVICE int32[B]: the token every code of prompt b starts from,
 *               each in [0,V) (as `prev` above)
 *   u           DEVICE float[B]
 *   tokens_out  DEVICE int32[B, N, T]
 *   codes_out   DEVICE float[B, N] final codes, or NULL
 * B*N <= ctx max_rows; model V must equal ctx V.
 */
as_status as_decode(as_ctx *ctx, const as_model *model, const int32_t *prompts,
                    int32_t B, int32_t N, int32_t T, const float *u, float temp,
                    int32_t top_k, float top_p, int32_t eos_id,
                    int32_t *tokens_out, float *codes_out);

/*
 * The two halves of the fused decode below, callable on their own.
 *
 * as_bigram_group_mass: what as_bigram_logits would give, reduced on chip to one pair
 * per row and per group g of 32 consecutive tokens: with y_v = logit_v * log2(e)/temp,
 *     mass_out[r, g] = ( sum over the group of 2^(y_v - ref), ref ),  ref = ceil(max y_v)
 * (two floats; groups are in vocabulary order, so their running sums are the cumulative
 * distribution of Sec. 3.1 sampled every 32 tokens).
 *   prev        DEVICE int32[rows]
 *   mass_out    DEVICE float[rows, ldp, 2], 16-byte aligned; ldp a multiple of 16,
 *               ldp >= ceil(V/32); entries past ceil(V/32) are not written
 *
 * as_step_fused: one step of Algorithm 1 (Sec. 4.1) from those group masses: finds the
 * group of each row's code, recomputes that group's 32 logits from the model (row
 * prev[r]), finishes the bucket search and rescales the code.  Arguments as in
 * as_step_ex; ldp <= 65536 (the library's largest vocabulary, 2^21).
 * Both need bf16 weights and a rank d that is a multiple of 64 and at least 128.
 */
as_status as_bigram_group_mass(as_ctx *ctx, const as_model *model, const int32_t *prev,
                               int64_t rows, float temp, float *mass_out, int64_t ldp);
as_status as_step_fused(as_ctx *ctx, const as_model *model, const float *mass, int64_t ldp,
                        const int32_t *prev, int64_t rows, const float *codes, float temp,
                        int32_t *tokens_out, float *codes_out, const uint8_t *finished_in,
                        int32_t eos_id, uint8_t *finished_out);

/*
 * as_decode without the logits round trip (the same Algorithm 1, Sec. 4.1, over the same
 * model): the logits kernel keeps its tile of logits on chip and leaves only, per row and
 * per group of 32 consecutive logits, the group's softmax mass; the sampling kernel finds
 * the group a code falls into, recomputes that group's 32 logits from the model and
 * finishes the bucket search and the rescaling.  Logits are used as accumulated in fp32
 * (they are never rounded to a storage type), so results agree with as_decode on an fp32
 * context only up to the accumulation order.
 * No logit modifiers (top_k / top_p); needs bf16 weights, a rank d that is a multiple of
 * 64 and at least 128; AS_ERR_UNSUPPORTED otherwise.  Arguments as in as_decode.
 */
as_status as_decode_fused(as_ctx *ctx, const as_model *model, const int32_t *prompts,
                          int32_t B, int32_t N, int32_t T, const float *u, float temp,
                          int32_t eos_id, int32_t *tokens_out, float *codes_out);

/*
 * Ancestral sampling with the same kernels (Sec. 3.3; Sec. 3.1, last paragraph: with a
 * fresh uniform per step the bucket search is inverse-CDF categorical sampling).  As
 * as_decode, except that the code of row r at step t is uniforms[t*B*N + r] and the
 * rescaled code is dropped.  The caller draws the uniforms (the library holds no
 * random number generator).
 *   uniforms    DEVICE float[T, B*N], each in [0,1)
 *   others      as in as_decode
 */
as_status as_decode_ancestral(as_ctx *ctx, const as_model *model, const int32_t *prompts,
                              int32_t B, int32_t N, int32_t T, const float *uniforms,
                              float temp, int32_t top_k, float top_p, int32_t eos_id,
                              int32_t *tokens_out);

/*
 * The estimator of Sec. 4.2, (1/N) sum_i s(x_i), per prompt, for additive per-token
 * scores: s(x) = sum of score[x_t] over the tokens of x up to and including its first
 * eos_id (the rest is padding, Sec. 3.3).  fp64 sums in a fixed order.
 *   tokens      DEVICE int32[B, N, T] (as written by as_decode / as_decode_ancestral);
 *               tokens outside [0,V) score 0
 *   score       DEVICE float[V]
 *   eos_id      < 0: none
 *   est_out     DEVICE double[B]
 * Asynchronous on the context's stream; allocates nothing.
 */
as_status as_estimate_mean(as_ctx *ctx, const int32_t *tokens, int32_t B, int32_t N,
                           int32_t T, const float *score, int32_t eos_id, double *est_out);

/*
 * Encode direction, one step (Sec. 4.1: the interval of a sequence is built by the
 * codebook recursion; Sec. 3.1: a token's sub-interval starts at the cumulative
 * probability of the tokens before it in vocabulary order and is as wide as its
 * conditional probability).  For every row r with the row's kept, tempered softmax
 *     lo[r]    += width[r] * F(tokens[r] - 1)
 *     width[r] *= P(tokens[r])
 * Start from lo = 0, width = 1; after the last token the codes in [lo, lo + width)
 * are the ones as_step decodes to that sequence (up to the rounding of an fp32 code).
 *   logits, rows, ld, temp, top_k, top_p, row_ids, logits_rows   as in as_step_ex
 *   tokens        DEVICE int32[rows]; a token outside [0,V) or outside the kept set
 *                 has probability zero (width becomes 0)
 *   lo, width     DEVICE double[rows], read and written
 *   finished_in   DEVICE uint8[rows] or NULL: nonzero rows are past their EOS
 *                 (Sec. 3.3: padding) and are left unchanged
 *   eos_id        < 0: none; required with finished_in
 *   finished_out  DEVICE uint8[rows] or NULL: set where the row is or becomes finished
 * Asynchronous on the context's stream; allocates nothing.
 */
as_status as_interval_step(as_ctx *ctx, const void *logits, int64_t rows, int64_t ld,
                           const int32_t *tokens, float temp, int32_t top_k, float top_p,
                           double *lo, double *width, const uint8_t *finished_in,
                           int32_t eos_id, uint8_t *finished_out, const int32_t *row_ids,
                           int64_t logits_rows);

/*
 * Encode direction, whole sequences under the bigram model (Sec. 4.1): the interval
 * [lo, lo + width) of each of the B*N token sequences, the inverse of as_decode.  Per
 * step: logits for the previous token (the prompt's start token first), optional keep
 * threshold, as_interval_step on column t of `tokens`; EOS is sticky as in as_decode.
 *   prompts     DEVICE int32[B]
 *   tokens      DEVICE int32[B, N, T], as written by as_decode
 *   lo_out, width_out   DEVICE double[B*N]
 * Uses (and may grow) the context's decode workspace.
 */
as_status as_encode(as_ctx *ctx, const as_model *model, const int32_t *prompts,
                    int32_t B, int32_t N, int32_t T, const int32_t *tokens, float temp,
                    int32_t top_k, float top_p, int32_t eos_id,
                    double *lo_out, double *width_out);

#ifdef __cplusplus
}
#endif
#endif /* ARITH_SAMPLING_H */
