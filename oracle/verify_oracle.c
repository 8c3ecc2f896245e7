/*
 * CPU oracle for draft verification in speculative decoding.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, double-precision
 * statement of what Token Verification (Alg. 1) and Block Verification
 * (Alg. 2) of "Block Verification Accelerates Speculative Decoding" compute.
 * It shares no code with the HIP library, and nothing in the product path may
 * call it.  Only the tests, the smoke check and the benchmark's CPU-baseline
 * leg load it.
 *
 * The paper fixes the *law* of (tau, Y) given the inputs.  To make the result
 * a function of the inputs we add three conventions of our own (the paper is
 * silent on them): uniforms live in [0,1) and a test "accepts" iff eta < h;
 * the categorical draw for Y is an inverse-CDF walk in vocabulary-index order
 * with a strict ">" (a token of zero weight is never returned); and
 * h_i = 1 whenever w_i >= 1 (the 0/0 of the acceptance formula when the two
 * models agree on a row).
 *
 * Notation (the paper writes p_i for what is called w_i here):
 *   p_i(.) = M_b(. | c, X^i), i = 0..gamma      target row i
 *   q_i(.) = M_s(. | c, X^i), i = 0..gamma-1    draft row i;  q_gamma == 0
 *   X_i    = i-th draft token (drawn from q_{i-1}), stored at tokens[i-1]
 *   r_i    = p_{i-1}(X_i) / q_{i-1}(X_i)        ratio in the acceptance rule (Sec. 1)
 *   w_i    = min(w_{i-1} r_i, 1), w_0 = 1       Alg. 2, recursion for its p_i
 *   S_i    = sum_x max(w_i p_i(x) - q_i(x), 0)  numerator of the block acceptance formula
 *   eta_i  = uniforms[i-1], i = 1..gamma;  u = uniforms[gamma] draws Y.
 *
 * Everything is evaluated in double, one sequence at a time, in the order the
 * algorithms state it: no blocking, no fusion.  Sums run in index order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };   /* F64: tests only (exact tiny tables) */
enum { ORACLE_LOGITS = 0, ORACLE_PROBS = 1 };               /* what the rows hold */
enum { ORACLE_BLOCK = 0, ORACLE_TOKEN = 1, ORACLE_GREEDY = 2 };

/* number of doubles per (sequence, position) in the debug block */
#define ORACLE_DBG_STRIDE 6
/* dbg[b][i][0..5] = w_i, S_i, h_i, logZ target row i, logZ draft row i (NaN at
 * i = gamma), log r_i (NaN at i = 0).                                         */

/* A logit as a double, exactly.  bf16 is the upper half of an IEEE float.     */
static double logit_at(const void *base, int dtype, size_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    if (dtype == ORACLE_F64)
        return ((const double *)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* Temperature softmax of one row: a(x) = logit(x) / T, the row's
 * log-normaliser log sum_x exp(a(x)), and prob(x) = exp(a(x) - logZ).
 * `scaled` receives a(x), `prob` the probabilities.  Returns logZ.            */
static double softmax_row(const void *base, int dtype, size_t off, int V, double T,
                          double *scaled, double *prob)
{
    double amax = -INFINITY;
    for (int x = 0; x < V; ++x) {
        scaled[x] = logit_at(base, dtype, off + (size_t)x) / T;
        if (scaled[x] > amax) amax = scaled[x];
    }
    double z = 0.0;
    for (int x = 0; x < V; ++x) z += exp(scaled[x] - amax);
    double logz = amax + log(z);
    for (int x = 0; x < V; ++x) prob[x] = exp(scaled[x] - logz);
    return logz;
}

/* A row that already holds a distribution (the p_i, q_i of Alg. 1 / Alg. 2 handed over as they are, the
 * form of the arrays in App. A): prob(x) is the stored value, used as given (not renormalised), and
 * `scaled` receives its log (-inf for a zero), so that with a log-normaliser of 0 the rest of the
 * oracle reads the row exactly like a softmax row.  Returns that 0.                              */
static double given_row(const void *base, int dtype, size_t off, int V, double *scaled, double *prob)
{
    for (int x = 0; x < V; ++x) {
        prob[x] = logit_at(base, dtype, off + (size_t)x);
        scaled[x] = log(prob[x]);
    }
    return 0.0;
}

/* Inverse-CDF draw: rho(x) >= 0 are unnormalised weights.  C_x = sum_{x'<=x} rho,
 * t = u * C_{V-1}, Y = min{x : C_x > t}.  If rounding leaves no such x, Y is the
 * last x with rho(x) > 0.  Returns -1 when every weight is zero.  `margin`
 * receives min(t - C_{Y-1}, C_Y - t) / C_{V-1}: how far, relative to the total,
 * t lies from the nearest edge of the chosen token's cell.                    */
static int inverse_cdf(const double *rho, int V, double u, double *margin)
{
    double total = 0.0;
    for (int x = 0; x < V; ++x) total += rho[x];
    *margin = 0.0;
    if (!(total > 0.0)) return -1;
    double t = u * total, c = 0.0;
    int last_positive = -1;
    for (int x = 0; x < V; ++x) {
        double below = c;
        c += rho[x];
        if (rho[x] > 0.0) last_positive = x;
        if (c > t) {
            double lo = t - below, hi = c - t;
            *margin = (lo < hi ? lo : hi) / total;
            return x;
        }
    }
    return last_positive;
}

typedef struct {
    double *a;     /* (gamma+1) x V scaled target logits */
    double *b;     /* gamma x V scaled draft logits      */
    double *p;     /* (gamma+1) x V target probabilities */
    double *q;     /* (gamma+1) x V draft probabilities; row gamma is all zero */
    double *rho;   /* V residual weights                 */
    double *w, *S, *h, *logr, *A, *Bn, *Srej;
} scratch_t;

static int scratch_alloc(scratch_t *s, int gamma, int V)
{
    size_t rows = (size_t)gamma + 1, n = rows * (size_t)V;
    s->a = malloc(n * sizeof(double));
    s->b = malloc(n * sizeof(double));
    s->p = malloc(n * sizeof(double));
    s->q = malloc(n * sizeof(double));
    s->rho = malloc((size_t)V * sizeof(double));
    s->w = malloc(rows * 7 * sizeof(double));
    if (!s->a || !s->b || !s->p || !s->q || !s->rho || !s->w) return -1;
    s->S = s->w + rows; s->h = s->S + rows; s->logr = s->h + rows;
    s->A = s->logr + rows; s->Bn = s->A + rows; s->Srej = s->Bn + rows;
    return 0;
}

static void scratch_free(scratch_t *s)
{
    free(s->a); free(s->b); free(s->p); free(s->q); free(s->rho); free(s->w);
}

/* One sequence.  Returns 1 if the degenerate all-zero-residual fallback was taken. */
static int verify_one(int algo, int form, const void *tl, const void *dl, int dtype,
                      const int32_t *X, const float *uni, int gamma, int V, double T,
                      size_t t_off, size_t d_off, scratch_t *s,
                      int32_t *tau_out, int32_t *y_out, double *dbg, double *margins)
{
    const size_t Vz = (size_t)V;

    /* The 2*gamma+1 distributions along the sample path (inputs of Alg. 1 / Alg. 2). */
    for (int i = 0; i <= gamma; ++i)
        s->A[i] = form == ORACLE_PROBS
                      ? given_row(tl, dtype, t_off + (size_t)i * Vz, V, s->a + i * Vz, s->p + i * Vz)
                      : softmax_row(tl, dtype, t_off + (size_t)i * Vz, V, T, s->a + i * Vz, s->p + i * Vz);
    for (int i = 0; i < gamma; ++i)
        s->Bn[i] = form == ORACLE_PROBS
                       ? given_row(dl, dtype, d_off + (size_t)i * Vz, V, s->b + i * Vz, s->q + i * Vz)
                       : softmax_row(dl, dtype, d_off + (size_t)i * Vz, V, T, s->b + i * Vz, s->q + i * Vz);
    /* q_gamma == 0: the padding row that makes position gamma look like the others (App. A). */
    for (int x = 0; x < V; ++x) s->q[(size_t)gamma * Vz + x] = 0.0;
    s->Bn[gamma] = NAN;

    /* r_i = p_{i-1}(X_i) / q_{i-1}(X_i), via logs so that it is finite for finite logits. */
    s->logr[0] = NAN;
    for (int i = 1; i <= gamma; ++i) {
        int xi = X[i - 1];
        double lp = s->a[(size_t)(i - 1) * Vz + xi] - s->A[i - 1];
        double lq = s->b[(size_t)(i - 1) * Vz + xi] - s->Bn[i - 1];
        s->logr[i] = lp - lq;
    }

    int tau = 0;
    double eta_margin = 1.0;   /* min |eta_i - h_i| over the tests that fixed tau */

    if (algo == ORACLE_TOKEN) {
        /* Alg. 1: h_i = min(r_i, 1); stop at the first rejection. */
        s->w[0] = 1.0; s->h[0] = 1.0;
        for (int i = 1; i <= gamma; ++i) {
            double r = exp(s->logr[i]);
            s->h[i] = r < 1.0 ? r : 1.0;
            s->w[i] = 1.0;   /* token verification has no carried weight: the residual uses p - q */
        }
        for (int i = 0; i <= gamma; ++i) {
            double acc = 0.0;
            for (int x = 0; x < V; ++x) {
                double d = s->p[(size_t)i * Vz + x] - s->q[(size_t)i * Vz + x];
                acc += d > 0.0 ? d : 0.0;
            }
            s->S[i] = acc;
        }
        for (int i = 1; i <= gamma; ++i) {
            double eta = (double)uni[i - 1];
            double gap = fabs(eta - s->h[i]);
            if (gap < eta_margin) eta_margin = gap;
            if (eta < s->h[i]) tau = i; else break;
        }
    } else if (algo == ORACLE_BLOCK) {
        /* Alg. 2: w_0 = 1, w_i = min(w_{i-1} r_i, 1). */
        s->w[0] = 1.0;
        for (int i = 1; i <= gamma; ++i) {
            double v = s->w[i - 1] * exp(s->logr[i]);
            s->w[i] = v < 1.0 ? v : 1.0;
        }
        /* S_i = sum_x max(w_i p_i(x) - q_i(x), 0); with q_gamma == 0 this is w_gamma at i = gamma. */
        for (int i = 0; i <= gamma; ++i) {
            double acc = 0.0;
            for (int x = 0; x < V; ++x) {
                double d = s->w[i] * s->p[(size_t)i * Vz + x] - s->q[(size_t)i * Vz + x];
                acc += d > 0.0 ? d : 0.0;
            }
            s->S[i] = acc;
        }
        s->S[gamma] = s->w[gamma];
        /* h_gamma = w_gamma; h_i = S_i / (S_i + 1 - w_i) for i < gamma (block acceptance formula). */
        s->h[0] = 1.0;
        for (int i = 1; i < gamma; ++i)
            s->h[i] = s->w[i] >= 1.0 ? 1.0 : s->S[i] / (s->S[i] + 1.0 - s->w[i]);
        s->h[gamma] = s->w[gamma];
        /* No break: tau is the LAST i whose test passes (longest accepted sub-block). */
        for (int i = 1; i <= gamma; ++i)
            if ((double)uni[i - 1] < s->h[i]) tau = i;
        for (int i = (tau > 1 ? tau : 1); i <= gamma; ++i) {
            double gap = fabs((double)uni[i - 1] - s->h[i]);
            if (gap < eta_margin) eta_margin = gap;
        }
    } else {
        /* Alg. 4 (greedy block verification): w~_i = w~_{i-1} r_i without the clip,
         * h_i = sum max(w~ p - q, 0) / sum max(q - w~ p, 0) for i < gamma, and the
         * last position is accepted iff eta_gamma < w~_gamma.                       */
        s->w[0] = 1.0;
        for (int i = 1; i <= gamma; ++i) s->w[i] = s->w[i - 1] * exp(s->logr[i]);
        for (int i = 0; i <= gamma; ++i) {
            double rem = 0.0, rej = 0.0;
            for (int x = 0; x < V; ++x) {
                double d = s->w[i] * s->p[(size_t)i * Vz + x] - s->q[(size_t)i * Vz + x];
                if (d > 0.0) rem += d; else rej -= d;
            }
            s->S[i] = rem; s->Srej[i] = rej;
        }
        s->h[0] = 1.0;
        for (int i = 1; i < gamma; ++i) {
            /* the ratio can exceed 1 or be x/0: every value >= 1 accepts every eta in [0,1) */
            double hv = s->Srej[i] > 0.0 ? s->S[i] / s->Srej[i] : INFINITY;
            s->h[i] = hv < 1.0 ? hv : 1.0;
        }
        s->h[gamma] = s->w[gamma] < 1.0 ? s->w[gamma] : 1.0;
        for (int i = 1; i <= gamma; ++i)
            if ((double)uni[i - 1] < s->h[i]) tau = i;
        for (int i = (tau > 1 ? tau : 1); i <= gamma; ++i) {
            double gap = fabs((double)uni[i - 1] - s->h[i]);
            if (gap < eta_margin) eta_margin = gap;
        }
    }

    /* Y: from p_gamma when everything was accepted, else from the residual at row tau
     * (token: max(p - q, 0); block / greedy: max(w_tau p - q, 0)).                  */
    int fallback = 0;
    {
        const double *pt = s->p + (size_t)tau * Vz, *qt = s->q + (size_t)tau * Vz;
        double wt = (algo == ORACLE_TOKEN) ? 1.0 : s->w[tau];
        if (tau == gamma) {
            for (int x = 0; x < V; ++x) s->rho[x] = pt[x];
        } else {
            for (int x = 0; x < V; ++x) {
                double d = wt * pt[x] - qt[x];
                s->rho[x] = d > 0.0 ? d : 0.0;
            }
        }
        double u = (double)uni[gamma], um = 0.0;
        int y = inverse_cdf(s->rho, V, u, &um);
        if (y < 0) {   /* unreachable in exact arithmetic; counted by the caller */
            fallback = 1;
            y = inverse_cdf(pt, V, u, &um);
        }
        *tau_out = tau;
        *y_out = y;
        if (margins) { margins[0] = eta_margin; margins[1] = um; }
    }

    if (dbg) {
        for (int i = 0; i <= gamma; ++i) {
            double *d = dbg + (size_t)i * ORACLE_DBG_STRIDE;
            d[0] = s->w[i]; d[1] = s->S[i]; d[2] = s->h[i];
            d[3] = s->A[i]; d[4] = s->Bn[i]; d[5] = s->logr[i];
        }
    }
    return fallback;
}

/*
 * Batched entry point (host pointers).
 *   algo            ORACLE_BLOCK, ORACLE_TOKEN or ORACLE_GREEDY
 *   target_logits   [B, gamma+1, V]   dtype, V contiguous
 *   draft_logits    [B, gamma,   V]
 *   draft_tokens    [B, gamma]        X_1..X_gamma
 *   uniforms        [B, gamma+1]      eta_1..eta_gamma, u
 *   accept_len      [B] out           tau
 *   next_token      [B] out           Y
 *   dbg             [B, gamma+1, 6] out or NULL
 *   margins         [B, 2] out or NULL  (eta margin, u margin)
 *   n_fallback      out or NULL: sequences whose residual weights were all zero
 *   nthreads        host threads over sequences (<=0: runtime default)
 * Returns 0, or -1 on a bad argument, -2 when memory runs out.
 */
static int verify_batch(int algo, int form, const void *target_logits, const void *draft_logits,
                        const int32_t *draft_tokens, const float *uniforms,
                        int B, int gamma, int V, int dtype, double temperature,
                        int32_t *accept_len, int32_t *next_token,
                        double *dbg, double *margins, int32_t *n_fallback, int nthreads)
{
    if (!target_logits || !draft_logits || !draft_tokens || !uniforms || !accept_len || !next_token)
        return -1;
    if (B < 1 || gamma < 1 || V < 1 || !(temperature > 0.0) || !isfinite(temperature)) return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F64) return -1;
    if (algo != ORACLE_BLOCK && algo != ORACLE_TOKEN && algo != ORACLE_GREEDY) return -1;
    for (size_t k = 0; k < (size_t)B * gamma; ++k)
        if (draft_tokens[k] < 0 || draft_tokens[k] >= V) return -1;

    int fail = 0, fb = 0;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
    if (nthreads > B) nthreads = B;
#pragma omp parallel num_threads(nthreads) reduction(+ : fb) reduction(| : fail)
#endif
    {
        scratch_t s;
        if (scratch_alloc(&s, gamma, V) != 0) {
            fail |= 1;
        }
#ifdef _OPENMP
#pragma omp barrier
#pragma omp for schedule(dynamic, 1)
#endif
        for (int b = 0; b < B; ++b) {
            if (fail) continue;
            fb += verify_one(algo, form, target_logits, draft_logits, dtype,
                             draft_tokens + (size_t)b * gamma, uniforms + (size_t)b * (gamma + 1),
                             gamma, V, temperature,
                             (size_t)b * (gamma + 1) * V, (size_t)b * gamma * V, &s,
                             accept_len + b, next_token + b,
                             dbg ? dbg + (size_t)b * (gamma + 1) * ORACLE_DBG_STRIDE : NULL,
                             margins ? margins + (size_t)b * 2 : NULL);
        }
        scratch_free(&s);
    }
    if (fail) return -2;
    if (n_fallback) *n_fallback = fb;
    return 0;
}

int oracle_spec_verify(int algo, const void *target_logits, const void *draft_logits,
                       const int32_t *draft_tokens, const float *uniforms,
                       int B, int gamma, int V, int dtype, double temperature,
                       int32_t *accept_len, int32_t *next_token,
                       double *dbg, double *margins, int32_t *n_fallback, int nthreads)
{
    return verify_batch(algo, ORACLE_LOGITS, target_logits, draft_logits, draft_tokens, uniforms, B, gamma, V, dtype,
                        temperature, accept_len, next_token, dbg, margins, n_fallback, nthreads);
}

/*
 * The same with the distributions themselves as inputs (the ps / qs arrays of App. A): target_probs
 * [B, gamma+1, V] holds p_i(x), draft_probs [B, gamma, V] holds q_i(x), values >= 0, q_{i-1}(X_i) > 0.
 * The rows are used as given: no temperature, no renormalisation (the draw of Y divides by the sum
 * of the weights it draws from, whatever that sum is).  dbg columns 3 and 4 are 0.
 */
int oracle_spec_verify_probs(int algo, const void *target_probs, const void *draft_probs,
                             const int32_t *draft_tokens, const float *uniforms,
                             int B, int gamma, int V, int dtype,
                             int32_t *accept_len, int32_t *next_token,
                             double *dbg, double *margins, int32_t *n_fallback, int nthreads)
{
    return verify_batch(algo, ORACLE_PROBS, target_probs, draft_probs, draft_tokens, uniforms, B, gamma, V, dtype,
                        1.0, accept_len, next_token, dbg, margins, n_fallback, nthreads);
}

/*
 * The drafting step of the outer loop of speculative decoding (Alg. 3: "sample X_1..X_gamma from
 * M_s"), for a model whose conditional distributions are handed over as rows of logits: one token
 * per row from softmax(logits / T), by the same inverse-CDF walk as the draw of Y (index order,
 * strict ">", t = u * total).
 *   logits    [rows, V]  dtype
 *   uniforms  [rows]     float32 in [0,1)
 *   tokens    [rows]     out
 *   margins   [rows]     out or NULL: distance of t to the nearest edge of the token's cell / total
 * Returns 0, or -1 on a bad argument, -2 when memory runs out.
 */
int oracle_sample_rows(const void *logits, long long rows, int V, int dtype, double temperature,
                       const float *uniforms, int32_t *tokens, double *margins)
{
    if (!logits || !uniforms || !tokens) return -1;
    if (rows < 1 || V < 1 || !(temperature > 0.0) || !isfinite(temperature)) return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return -1;
    double *scaled = (double *)malloc(sizeof(double) * (size_t)V);
    double *prob = (double *)malloc(sizeof(double) * (size_t)V);
    if (!scaled || !prob) { free(scaled); free(prob); return -2; }
    for (long long r = 0; r < rows; ++r) {
        softmax_row(logits, dtype, (size_t)r * (size_t)V, V, temperature, scaled, prob);
        double m = 0.0;
        tokens[r] = inverse_cdf(prob, V, (double)uniforms[r], &m);
        if (margins) margins[r] = m;
    }
    free(scaled);
    free(prob);
    return 0;
}

/* Threads the batched entry point would use for `requested` (<=0: default). */
int oracle_num_threads(int requested)
{
#ifdef _OPENMP
    return requested > 0 ? requested : omp_get_max_threads();
#else
    (void)requested;
    return 1;
#endif
}
