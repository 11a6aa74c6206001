/*
 * Arithmetic sampling -- CPU oracle (TEST INFRASTRUCTURE, not the product path).
 *
 * Plain fp64 restatement of what the decode path computes.  Written straight
 * from the paper's definitions, deliberately slow and unblocked so it can be
 * checked against the paper by eye:
 *
 *   - Sec. 3.1 (arithmetic coding): with a total order on the items and
 *     w_i = sum_{j<i} P(x_j), the code c decodes to the item whose interval
 *     (w_i, w_{i+1}) holds c.
 *   - Sec. 4.1 + Algorithm 1 (sampling from a code point): per step form the
 *     vocabulary-order cumulative sums of the next-token conditional, emit the
 *     token whose interval (m, M) holds c_t, set c_{t+1} = (c_t - m)/(M - m),
 *     stop at EOS (here: EOS is sticky, the padded fixed-length form of
 *     Sec. 3.3).
 *   - Sec. 4.1 codebook recursion (the unnumbered equation for w_{i1 i2} and
 *     the one after it): interval of a sequence/prefix, the encode direction.
 *   - Sec. 4.2 Definition "Arithmetic sampling": N codes on a lattice with one
 *     shared uniform shift.
 *   - Sec. 2 / Sec. 5 (top-k paragraph): temperature, top-k and nucleus act on
 *     the conditional logits before the interval construction; everything
 *     outside the kept set gets probability zero.
 *
 * Readings taken where the paper is silent (ties, closed ends, order of the
 * logit modifiers) are listed beside each function.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code, header, table or helper with the HIP path.
 *
 * Parity pins: every exported function is pinned by tests/test_oracle_*.py
 * (brute-force enumeration of all sequence intervals, the paper's two-symbol
 * example, the floor/ceil lattice count invariant, zero variance for widths
 * k/N, unbiasedness over shifts, the App. B closed-form variance, NumPy
 * searchsorted/sort based restatements).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { AO_F32 = 0, AO_BF16 = 1, AO_F64 = 2 };

/* Result of one step for one row. */
typedef struct {
    int32_t token;     /* emitted token                                   */
    double  p;         /* its probability  M - m                          */
    double  f_lo;      /* m = w_i                                         */
    double  f_hi;      /* M = w_{i+1}                                     */
    double  c_next;    /* (c - m)/(M - m), kept in [0, 1 - 2^-53]         */
    double  delta;     /* distance from c to the nearest interior interval
                          end of the emitted token (ends at 0 and 1 are
                          not interior); +inf if there is none            */
    double  nuc_margin;/* nucleus only: |cumulative mass - top_p| at the
                          group that closes the nucleus and at the one
                          before it, whichever is smaller; +inf otherwise */
    int32_t n_kept;    /* tokens with non-zero probability after masking  */
    int32_t nuc_alt_lo;/* nucleus only: how many closings EARLIER than the
                          rule's are within `band` of being the rule's (the
                          running mass at that earlier group is already
                          within band of top_p); 0 otherwise                */
    int32_t nuc_alt_hi;/* ... and how many LATER ones (the running mass at
                          the rule's group, and at the ones after it,
                          exceeds top_p by less than band)                  */
    int32_t tok_prev;  /* nearest token before the emitted one that has
                          non-zero probability, -1 if none                  */
    int32_t tok_next;  /* nearest such token after it, -1 if none           */
    double  p_prev;    /* their probabilities (0 if none)                   */
    double  p_next;
} ao_step_result;

/* Which nucleus to form.  The rule (shift 0) closes the nucleus with the first
 * group of equal logits at which the running mass reaches top_p.  An
 * implementation in finite precision may legitimately close one group earlier
 * or later when that mass passes within a hair of top_p; `shift` asks for the
 * kept set that closes that many groups later (negative: earlier), so that a
 * checker can compare against every admissible alternative, and `band` is the
 * width of the hair used to count the alternatives. */
typedef struct {
    int32_t shift;
    double  band;
} ao_nucleus_opt;

/* ------------------------------------------------------------------ */
/* storage widening                                                    */
/* ------------------------------------------------------------------ */

/* bfloat16 is the upper half of an IEEE binary32. */
static double widen_bf16(uint16_t h)
{
    uint32_t bits = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static double load_elem(const void *base, int dtype, int64_t idx)
{
    switch (dtype) {
    case AO_F32:  return (double)((const float *)base)[idx];
    case AO_BF16: return widen_bf16(((const uint16_t *)base)[idx]);
    default:      return ((const double *)base)[idx];
    }
}

/* round-to-nearest-even narrowing used when the decode loop is asked to store
 * its logits the way the device does (bf16 or fp32) before sampling from them */
static double round_to_bf16(double x)
{
    float f = (float)x;           /* fp64 -> fp32, RNE */
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    if ((bits & 0x7fffffffu) > 0x7f800000u) return (double)f;   /* NaN */
    uint32_t lsb = (bits >> 16) & 1u;
    bits += 0x7fffu + lsb;
    bits &= 0xffff0000u;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* ------------------------------------------------------------------ */
/* Sec. 4.2: lattice of codes                                          */
/* ------------------------------------------------------------------ */

/* Circular lattice with spacing exactly 1/N: c_i = (i + u)/N, i = 0..N-1,
 * u in [0,1).  This is the evenly spaced shifted lattice for which the
 * zero-variance statement of Sec. 4.4 (interval widths that are multiples of
 * 1/N) holds exactly. */
void ao_lattice(int32_t N, double u, double *codes)
{
    for (int32_t i = 0; i < N; ++i)
        codes[i] = ((double)i + u) / (double)N;
}

/* The lattice as the Definition in Sec. 4.2 prints it: i/(N+1) + b mod 1,
 * i = 1..N (the two-symbol example fixes the index range: N=1 gives 0.5). */
void ao_lattice_paper(int32_t N, double b, double *codes)
{
    for (int32_t i = 1; i <= N; ++i) {
        double c = (double)i / (double)(N + 1) + b;
        codes[i - 1] = c - floor(c);
    }
}

/* ------------------------------------------------------------------ */
/* Sec. 2 / Sec. 5: logit modifiers -> unnormalised kept weights       */
/* ------------------------------------------------------------------ */

/* descending; a NaN (no logit at all: outside the method) orders after every
 * number so that the order stays total */
static int cmp_desc(const void *a, const void *b)
{
    double x = *(const double *)a, y = *(const double *)b;
    int xn = isnan(x), yn = isnan(y);
    if (xn || yn) return xn - yn;
    return (x < y) - (x > y);
}

/*
 * Fill e[v] = exp(x_v/temp - max) for kept tokens and 0 for the others.
 * Order of the modifiers: temperature, then top-k, then nucleus, then the
 * softmax over the survivors.
 *
 * top-k  (0 < k < V): threshold = k-th largest logit counted with
 *        multiplicity; every logit >= threshold is kept (ties at the threshold
 *        all stay).
 * top-p  (0 < p < 1): over the tokens that survived top-k, group equal
 *        logits, order groups by value descending, accumulate their softmax
 *        mass; the nucleus closes with the first group at which the running
 *        mass reaches top_p; that group is kept whole.
 *
 * Returns the sum of e in vocabulary order; writes n_kept and nuc_margin.
 */
static double kept_weights(const double *x, int32_t V, double temp,
                           int32_t top_k, double top_p, ao_nucleus_opt nuc,
                           double *e, double *scratch,
                           int32_t *n_kept, double *nuc_margin,
                           int32_t *nuc_alt_lo, int32_t *nuc_alt_hi)
{
    double thr = -INFINITY;           /* keep x_v >= thr */
    *nuc_margin = INFINITY;
    *nuc_alt_lo = 0;
    *nuc_alt_hi = 0;

    if (top_k > 0 && top_k < V) {
        memcpy(scratch, x, (size_t)V * sizeof(double));
        qsort(scratch, (size_t)V, sizeof(double), cmp_desc);
        thr = scratch[top_k - 1];
        if (isnan(thr)) thr = -INFINITY;   /* fewer than k numbers: keep them all */
    }

    if (top_p > 0.0 && top_p < 1.0) {
        /* softmax over the current survivors */
        double m = -INFINITY;
        for (int32_t v = 0; v < V; ++v)
            if (x[v] >= thr && x[v] / temp > m) m = x[v] / temp;
        int32_t n = 0;
        for (int32_t v = 0; v < V; ++v)
            if (x[v] >= thr) scratch[n++] = x[v];
        if (n > 0 && m > -INFINITY) {
            qsort(scratch, (size_t)n, sizeof(double), cmp_desc);
            double total = 0.0;
            for (int32_t j = 0; j < n; ++j) total += exp(scratch[j] / temp - m);

            /* groups of equal logits, descending: value gval[g] (kept in place at
             * the front of scratch), running mass gcum[g] up to and including it
             * (e is free until the weights are written below) */
            double *gval = scratch, *gcum = e;
            int32_t ng = 0, j = 0;
            double cum = 0.0;
            while (j < n) {
                double val = scratch[j];
                double grp = 0.0;
                while (j < n && scratch[j] == val) {
                    grp += exp(scratch[j] / temp - m);
                    ++j;
                }
                cum += grp / total;
                gval[ng] = val;
                gcum[ng] = cum;
                ++ng;
            }
            /* the rule: first group at which the running mass reaches top_p */
            int32_t close = ng - 1;
            for (int32_t g = 0; g < ng; ++g)
                if (gcum[g] >= top_p) { close = g; break; }
            double a = fabs(gcum[close] - top_p);
            double b = close > 0 ? fabs(gcum[close - 1] - top_p) : fabs(0.0 - top_p);
            *nuc_margin = a < b ? a : b;
            /* alternatives within the band */
            for (int32_t g = close - 1; g >= 0 && gcum[g] >= top_p - nuc.band; --g)
                ++*nuc_alt_lo;
            for (int32_t g = close; g < ng - 1 && gcum[g] < top_p + nuc.band; ++g)
                ++*nuc_alt_hi;
            int32_t use = close + nuc.shift;
            if (use < 0) use = 0;
            if (use > ng - 1) use = ng - 1;
            double new_thr = gval[use];
            if (new_thr > thr) thr = new_thr;
        }
    }

    double m = -INFINITY;
    for (int32_t v = 0; v < V; ++v)
        if (x[v] >= thr && x[v] / temp > m) m = x[v] / temp;

    double S = 0.0;
    int32_t kept = 0;
    for (int32_t v = 0; v < V; ++v) {
        if (x[v] >= thr && m > -INFINITY) {
            e[v] = exp(x[v] / temp - m);
            if (e[v] > 0.0) ++kept;
        } else {
            e[v] = 0.0;
        }
        S += e[v];
    }
    *n_kept = kept;
    return S;
}

/* ------------------------------------------------------------------ */
/* Algorithm 1, loop body                                              */
/* ------------------------------------------------------------------ */

/*
 * One step for one row.  x[V] are the logits already widened to fp64.
 *
 * Interval ends: the paper's test is strict on both sides and leaves c = w_i
 * undefined; here intervals are half open, [w_i, w_{i+1}), so the emitted
 * token is the first one whose inclusive cumulative sum exceeds c.  Tokens of
 * probability zero have empty intervals and are never emitted.  The comparison
 * is done on unnormalised sums (c*S against the running sum) so that no
 * division sits between the exponentials and the decision.
 */
static void step_row(const double *x, int32_t V, double c, double temp,
                     int32_t top_k, double top_p, ao_nucleus_opt nuc,
                     double *e, double *scratch, ao_step_result *out)
{
    int32_t n_kept, alt_lo, alt_hi;
    double nuc_margin;
    double S = kept_weights(x, V, temp, top_k, top_p, nuc, e, scratch,
                            &n_kept, &nuc_margin, &alt_lo, &alt_hi);
    out->nuc_margin = nuc_margin;
    out->n_kept = n_kept;
    out->nuc_alt_lo = alt_lo;
    out->nuc_alt_hi = alt_hi;
    out->tok_prev = -1; out->tok_next = -1;
    out->p_prev = 0.0;  out->p_next = 0.0;
    if (!(S > 0.0)) {
        /* a row without any weight (no finite logit): nothing can be emitted.
         * Defined sentinel: token -1, probability 0, the code unchanged. */
        out->token = -1;
        out->p = 0.0; out->f_lo = 0.0; out->f_hi = 0.0;
        out->c_next = c;
        out->delta = INFINITY;
        return;
    }

    double target = c * S;
    double run = 0.0, before = 0.0;
    int32_t tok = -1, first_nz = -1, last_nz = -1;
    double before_last = 0.0;
    for (int32_t v = 0; v < V; ++v) {
        if (e[v] > 0.0) {
            if (first_nz < 0) first_nz = v;
            last_nz = v;
            before_last = run;
        }
        double next = run + e[v];
        if (tok < 0 && next > target) { tok = v; before = run; }
        run = next;
    }
    if (tok < 0) {            /* only by rounding (c*S >= full sum) */
        tok = last_nz;
        before = before_last;
    }

    out->token = tok;
    out->p = e[tok] / S;
    out->f_lo = before / S;
    out->f_hi = (before + e[tok]) / S;
    double cn = (target - before) / e[tok];
    const double top = 1.0 - ldexp(1.0, -53);
    if (cn < 0.0) cn = 0.0;
    if (cn > top) cn = top;
    out->c_next = cn;

    double d = INFINITY;
    if (tok != first_nz) d = c - out->f_lo;
    if (tok != last_nz) {
        double d2 = out->f_hi - c;
        if (d2 < d) d = d2;
    }
    out->delta = fabs(d);

    /* neighbours in the cumulative order: the tokens whose intervals touch
     * the emitted one's (tokens of probability zero have empty intervals) */
    for (int32_t v = tok - 1; v >= 0; --v)
        if (e[v] > 0.0) { out->tok_prev = v; out->p_prev = e[v] / S; break; }
    for (int32_t v = tok + 1; v < V; ++v)
        if (e[v] > 0.0) { out->tok_next = v; out->p_next = e[v] / S; break; }
}

/*
 * Batched step over `rows` independent rows (rows never interact: Remark after
 * Prop. 1).  logits is [rows, ld] row-major in the stored type; row r reads
 * logits row row_ids[r] if row_ids is given.  finished rows (finished_in[r]
 * != 0) emit eos_id with probability one, keep their code and do not look at
 * their logits.  A row that emits eos_id is marked finished on output.
 * Every output pointer may be NULL.  nthreads <= 1 runs serially.
 * nuc_shift / nuc_band: see ao_nucleus_opt (0, 0 for the rule itself);
 * nuc_alt is [rows, 2] (admissible earlier, later closings), tok_nb and p_nb are
 * [rows, 2] (previous, next token with non-zero probability; -1 / 0 if none).
 * A row without any weight returns token -1, p = 0 and its code unchanged.
 * Returns 0, or -1 on an allocation failure.
 */
int ao_step_rows(const void *logits, int dtype, int64_t rows, int64_t ld,
                 int32_t V, const int64_t *row_ids, const double *codes,
                 double temp, int32_t top_k, double top_p,
                 const uint8_t *finished_in, int32_t eos_id,
                 int32_t *tokens, double *codes_next, double *p, double *f_lo,
                 double *f_hi, double *delta, double *nuc_margin,
                 int32_t *n_kept, uint8_t *finished_out, int nthreads,
                 int32_t nuc_shift, double nuc_band, int32_t *nuc_alt,
                 int32_t *tok_nb, double *p_nb)
{
    ao_nucleus_opt nuc = { nuc_shift, nuc_band };
    int failed = 0;
#ifdef _OPENMP
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel num_threads(nthreads)
#endif
    {
        double *x = (double *)malloc((size_t)V * sizeof(double));
        double *e = (double *)malloc((size_t)V * sizeof(double));
        double *s = (double *)malloc((size_t)V * sizeof(double));
        if (!x || !e || !s) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp barrier
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t r = 0; r < rows; ++r) {
            if (failed) continue;
            ao_step_result res;
            if (finished_in && finished_in[r]) {
                res.token = eos_id; res.p = 1.0; res.f_lo = 0.0; res.f_hi = 1.0;
                res.c_next = codes[r]; res.delta = INFINITY;
                res.nuc_margin = INFINITY; res.n_kept = 1;
                res.nuc_alt_lo = 0; res.nuc_alt_hi = 0;
                res.tok_prev = -1; res.tok_next = -1;
                res.p_prev = 0.0; res.p_next = 0.0;
                if (finished_out) finished_out[r] = 1;
            } else {
                int64_t src = row_ids ? row_ids[r] : r;
                for (int32_t v = 0; v < V; ++v)
                    x[v] = load_elem(logits, dtype, src * ld + v);
                step_row(x, V, codes[r], temp, top_k, top_p, nuc, e, s, &res);
                if (finished_out)
                    finished_out[r] = (eos_id >= 0 && res.token == eos_id) ? 1 : 0;
            }
            if (tokens)     tokens[r] = res.token;
            if (codes_next) codes_next[r] = res.c_next;
            if (p)          p[r] = res.p;
            if (f_lo)       f_lo[r] = res.f_lo;
            if (f_hi)       f_hi[r] = res.f_hi;
            if (delta)      delta[r] = res.delta;
            if (nuc_margin) nuc_margin[r] = res.nuc_margin;
            if (n_kept)     n_kept[r] = res.n_kept;
            if (nuc_alt) { nuc_alt[2 * r] = res.nuc_alt_lo; nuc_alt[2 * r + 1] = res.nuc_alt_hi; }
            if (tok_nb)  { tok_nb[2 * r] = res.tok_prev; tok_nb[2 * r + 1] = res.tok_next; }
            if (p_nb)    { p_nb[2 * r] = res.p_prev; p_nb[2 * r + 1] = res.p_next; }
        }
        free(x); free(e); free(s);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------ */
/* the synthetic sequence model standing in for P(X_t | X_<t)          */
/* ------------------------------------------------------------------ */

/*
 * Low-rank bigram conditional: logits[v] = (scale/sqrt(d)) * sum_k
 * E[prev,k] * U[k,v], E is [V,d], U is [d,V], both row-major in the stored
 * type, accumulated in fp64.  round_mode: 0 keep fp64, 1 round the result to
 * fp32, 2 round it to bf16 (what a device that stores its logits narrow
 * samples from).
 */
void ao_bigram_logits(const void *E, const void *U, int wdtype, int32_t V,
                      int32_t d, double scale, int32_t prev, int round_mode,
                      double *x)
{
    double f = scale / sqrt((double)d);
    for (int32_t v = 0; v < V; ++v) x[v] = 0.0;
    for (int32_t k = 0; k < d; ++k) {
        double a = load_elem(E, wdtype, (int64_t)prev * d + k);
        for (int32_t v = 0; v < V; ++v)
            x[v] += a * load_elem(U, wdtype, (int64_t)k * V + v);
    }
    for (int32_t v = 0; v < V; ++v) {
        double y = x[v] * f;
        if (round_mode == 1) y = (double)(float)y;
        else if (round_mode == 2) y = round_to_bf16(y);
        x[v] = y;
    }
}

/* ------------------------------------------------------------------ */
/* Algorithm 1 + Definition of Sec. 4.2: whole decode                  */
/* ------------------------------------------------------------------ */

/*
 * Decode B prompts x N codes for T steps.  codes0 is [B*N] (the caller builds
 * the lattice, so any lattice variant can be decoded); prompts[b] is the start
 * token every code of prompt b conditions on.  tokens is [B*N, T].  Once a
 * code has emitted eos_id (>= 0) it keeps emitting eos_id and its code value
 * stops changing.  Optional per-step records p_out / delta_out are [B*N, T];
 * codes_final is [B*N].
 */
int ao_decode(const void *E, const void *U, int wdtype, int32_t V, int32_t d,
              double scale, int round_mode, const int32_t *prompts, int32_t B,
              int32_t N, int32_t T, const double *codes0, double temp,
              int32_t top_k, double top_p, int32_t eos_id, int32_t *tokens,
              double *codes_final, double *p_out, double *delta_out,
              int nthreads)
{
    int64_t R = (int64_t)B * N;
    int failed = 0;
#ifdef _OPENMP
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel num_threads(nthreads)
#endif
    {
        double *x = (double *)malloc((size_t)V * sizeof(double));
        double *e = (double *)malloc((size_t)V * sizeof(double));
        double *s = (double *)malloc((size_t)V * sizeof(double));
        if (!x || !e || !s) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp barrier
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t r = 0; r < R; ++r) {
            if (failed) continue;
            double c = codes0[r];
            int32_t prev = prompts[r / N];
            int done = 0;
            for (int32_t t = 0; t < T; ++t) {
                if (done) {
                    tokens[r * T + t] = eos_id;
                    if (p_out) p_out[r * T + t] = 1.0;
                    if (delta_out) delta_out[r * T + t] = INFINITY;
                    continue;
                }
                ao_bigram_logits(E, U, wdtype, V, d, scale, prev, round_mode, x);
                ao_step_result res;
                const ao_nucleus_opt rule = { 0, 0.0 };
                step_row(x, V, c, temp, top_k, top_p, rule, e, s, &res);
                tokens[r * T + t] = res.token;
                if (res.token < 0) {        /* a row without weight ends here */
                    for (int32_t tt = t; tt < T; ++tt) {
                        tokens[r * T + tt] = -1;
                        if (p_out) p_out[r * T + tt] = 0.0;
                        if (delta_out) delta_out[r * T + tt] = INFINITY;
                    }
                    break;
                }
                if (p_out) p_out[r * T + t] = res.p;
                if (delta_out) delta_out[r * T + t] = res.delta;
                c = res.c_next;
                prev = res.token;
                if (eos_id >= 0 && res.token == eos_id) done = 1;
            }
            if (codes_final) codes_final[r] = c;
        }
        free(x); free(e); free(s);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------ */
/* Sec. 4.1 codebook recursion: sequence -> interval                   */
/* ------------------------------------------------------------------ */

/*
 * One step of the codebook recursion of Sec. 4.1 for a given next token:
 * within the current prefix's interval the token's sub-interval starts at
 * the cumulative probability of the tokens before it in vocabulary order
 * and has the token's conditional probability as its width (Sec. 3.1).
 * x holds the row's logits; e, s are scratch of V doubles.
 */
static void token_interval(const double *x, int32_t V, double temp,
                           int32_t top_k, double top_p, int32_t nuc_shift,
                           int32_t token,
                           double *e, double *s, double *f_lo, double *p)
{
    int32_t n_kept, alo, ahi; double nm;
    const ao_nucleus_opt rule = { nuc_shift, 0.0 };
    double S = kept_weights(x, V, temp, top_k, top_p, rule, e, s, &n_kept, &nm,
                            &alo, &ahi);
    if (!(S > 0.0) || token < 0 || token >= V) { *f_lo = 0.0; *p = 0.0; return; }
    double before = 0.0;
    for (int32_t v = 0; v < token; ++v) before += e[v];
    *f_lo = before / S;
    *p = e[token] / S;
}

/*
 * token_interval over rows of stored logits (layout and dtype as in
 * ao_step_rows): f_lo[r], p[r] for tokens[r].  Finished rows (already past
 * their EOS, Sec. 3.3) do not narrow the interval: f_lo = 0, p = 1.
 * nuc_shift as in ao_nucleus_opt (0: the rule).
 * Returns 0, -1 on allocation failure.
 */
int ao_token_interval_rows(const void *logits, int dtype, int64_t rows,
                           int64_t ld, int32_t V, const int64_t *row_ids,
                           const int32_t *tokens, double temp, int32_t top_k,
                           double top_p, const uint8_t *finished_in,
                           double *f_lo, double *p, int nthreads,
                           int32_t nuc_shift)
{
    int failed = 0;
#ifdef _OPENMP
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel num_threads(nthreads)
#endif
    {
        double *x = (double *)malloc((size_t)V * sizeof(double));
        double *e = (double *)malloc((size_t)V * sizeof(double));
        double *s = (double *)malloc((size_t)V * sizeof(double));
        if (!x || !e || !s) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp barrier
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t r = 0; r < rows; ++r) {
            if (failed) continue;
            if (finished_in && finished_in[r]) {
                f_lo[r] = 0.0; p[r] = 1.0;
                continue;
            }
            int64_t src = row_ids ? row_ids[r] : r;
            for (int32_t v = 0; v < V; ++v)
                x[v] = load_elem(logits, dtype, src * ld + v);
            token_interval(x, V, temp, top_k, top_p, nuc_shift, tokens[r], e, s,
                           &f_lo[r], &p[r]);
        }
        free(x); free(e); free(s);
    }
    return failed ? -1 : 0;
}

/*
 * Interval [w, w + P) of the prefix seq[0..L) under the same model and logit
 * modifiers: w grows by P(prefix so far) times the cumulative probability of
 * the tokens ordered before the next one; P(prefix) is multiplied by that
 * token's conditional.  A sequence is complete at its first eos_id: later
 * positions are padding and do not narrow the interval.  Returns 0, -1 on
 * allocation failure.
 */
int ao_encode(const void *E, const void *U, int wdtype, int32_t V, int32_t d,
              double scale, int round_mode, int32_t prompt, const int32_t *seq,
              int32_t L, double temp, int32_t top_k, double top_p,
              int32_t eos_id, double *w_out, double *P_out)
{
    double *x = (double *)malloc((size_t)V * sizeof(double));
    double *e = (double *)malloc((size_t)V * sizeof(double));
    double *s = (double *)malloc((size_t)V * sizeof(double));
    if (!x || !e || !s) { free(x); free(e); free(s); return -1; }
    double w = 0.0, P = 1.0;
    int32_t prev = prompt;
    for (int32_t t = 0; t < L; ++t) {
        ao_bigram_logits(E, U, wdtype, V, d, scale, prev, round_mode, x);
        double f_lo, p;
        token_interval(x, V, temp, top_k, top_p, 0, seq[t], e, s, &f_lo, &p);
        w += P * f_lo;
        P *= p;
        prev = seq[t];
        if (eos_id >= 0 && seq[t] == eos_id) break;
    }
    *w_out = w;
    *P_out = P;
    free(x); free(e); free(s);
    return 0;
}

/*
 * The estimator of Sec. 4.2, (1/N) sum_i s(x_i), per prompt, for additive
 * per-token scores: s(x) = sum of score[x_t] over the sequence's tokens up to
 * and including its first eos_id (the rest is padding, Sec. 3.3).  tokens is
 * [B, N, T]; est is [B].
 */
void ao_estimate_mean(const int32_t *tokens, int32_t B, int32_t N, int32_t T,
                      const double *score, int32_t eos_id, double *est)
{
    for (int32_t b = 0; b < B; ++b) {
        double total = 0.0;
        for (int32_t i = 0; i < N; ++i) {
            const int32_t *seq = tokens + ((int64_t)b * N + i) * T;
            double s = 0.0;
            for (int32_t t = 0; t < T; ++t) {
                s += score[seq[t]];
                if (eos_id >= 0 && seq[t] == eos_id) break;
            }
            total += s;
        }
        est[b] = total / (double)N;
    }
}

int ao_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
