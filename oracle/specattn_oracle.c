/*
 * CPU oracle for SpecAttn's token selection and sparse attention.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file:
 * only the tests, the smoke check and the bench's cpu_baseline leg do.  It
 * shares no code, header, table or helper with the HIP library.
 *
 * Everything here is the plain definition, written for readability:
 *
 *   oracle_topp_select       Appendix A, Eq. 8 (smallest index set whose
 *                            attention mass reaches p) in the threshold form
 *                            of Algorithm 2's last step {i : a_i >= theta}:
 *                            sort the row, fp64 running sum, first prefix
 *                            that reaches p * (row sum), keep every value
 *                            that is >= the value found there.
 *   oracle_chunk_masses      the per-chunk attention mass that chunk-granular selection
 *                            (Section 4: chunks of 16 tokens) ranks instead of single
 *                            positions; the selection itself is oracle_topp_select on
 *                            the row of chunk masses.
 *   oracle_nucleus_bisection Algorithm 2 itself (value-space bisection), with
 *                            an iteration count instead of the epsilon test,
 *                            as the footnote in Section 3.4 describes.
 *   oracle_bisection_select  the same with a fixed number of halvings, as a selection
 *                            (what the paper's implementation runs, 10 halvings).
 *   oracle_masked_attention_tail  the same with the keys/values of the tokens being
 *                            verified appended causally (Algorithm 1, verification
 *                            step: gamma + 1 tokens go through the verifier at once).
 *   oracle_masked_attention  Section 3.1, Eq. 1-3: scores over ALL positions,
 *                            unselected ones masked out, softmax, times V.
 *                            The softmax is taken over the selected set (the
 *                            reading that matches attending only over the
 *                            selected K/V); with every position selected it
 *                            is Eq. 1 exactly.
 *
 * Parity pins (tests that do not depend on this file's own arithmetic):
 *   oracle_topp_select       brute force over all subsets, closed forms for
 *                            geometric and two-level rows, hand-worked tie
 *                            rows, invariants, Algorithm 2 run to convergence.
 *   oracle_chunk_masses      hand-worked rows, exact rational sums, chunk = 1 is the
 *                            identity, the masses add up to the row sum.
 *   oracle_nucleus_bisection feasibility / superset / bracket-width bounds
 *                            that follow from the algorithm's invariant.
 *   oracle_bisection_select  hand-worked rows, a separately written numpy loop, the exact
 *                            selection as a subset, equality with it after 60 halvings.
 *   oracle_masked_attention_tail  a library attention routine with an explicit
 *                            per-query boolean mask over cache + new tokens; with an
 *                            empty cache and one new token the output is that token's
 *                            value row.
 *   oracle_masked_attention  a library attention routine (with and without a
 *                            boolean mask), one-hot selections, constant keys,
 *                            the log-sum-exp merge identity, Appendix A's
 *                            error bound.
 *
 * Floating point: inputs are read exactly (fp32, or bf16 / fp16 bit patterns
 * widened) and all arithmetic is fp64.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum {
    ORACLE_ROW_INVALID = 1u,       /* NaN, negative, infinite entry, or zero row sum */
    ORACLE_ROW_NEAR_BOUNDARY = 2u  /* mass on either side of tau* within 1e-6 of p (relative to the row sum) */
};

int oracle_set_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
    return omp_get_max_threads();
#else
    (void)t;
    return 1;
#endif
}

static int cmp_desc(const void *a, const void *b)
{
    double x = *(const double *)a, y = *(const double *)b;
    return (x < y) - (x > y);
}

/*
 * Exact top-p selection of one row per (batch, kv-head).
 *
 * probs      [rows][row_stride] fp32, row r valid on [0, lens[r])
 * top_p      p in (0, 1]
 * indices    [rows][idx_stride] int32, ascending selected positions
 * counts     [rows] number selected
 * tau        [rows] the threshold value tau* (one of the row's values), 0 for invalid rows
 * flags      [rows] ORACLE_ROW_* bits
 * diag       [rows][4] fp64: row sum S, target p*S, mass of {a >= tau*}, mass of {a > tau*}
 */
int oracle_topp_select(const float *probs, int64_t row_stride, int rows, const int32_t *lens,
                       float top_p, int32_t *indices, int64_t idx_stride, int32_t *counts,
                       float *tau, uint32_t *flags, double *diag)
{
    if (!(top_p > 0.0f && top_p <= 1.0f)) return -1;
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < rows; ++r) {
        const float *a = probs + (int64_t)r * row_stride;
        const int L = lens[r];
        int32_t *out = indices + (int64_t)r * idx_stride;
        counts[r] = 0;
        tau[r] = 0.0f;
        flags[r] = 0;
        if (diag) memset(diag + 4 * (int64_t)r, 0, 4 * sizeof(double));

        int bad = (L <= 0);
        for (int i = 0; i < L && !bad; ++i)
            if (isnan(a[i]) || isinf(a[i]) || a[i] < 0.0f) bad = 1;
        if (bad) { flags[r] = ORACLE_ROW_INVALID; continue; }

        double *s = (double *)malloc(sizeof(double) * (size_t)L);   /* sorted values */
        double *c = (double *)malloc(sizeof(double) * (size_t)L);   /* running sums  */
        if (!s || !c) { free(s); free(c); status = -2; continue; }
        for (int i = 0; i < L; ++i) s[i] = (double)a[i];
        qsort(s, (size_t)L, sizeof(double), cmp_desc);
        double run = 0.0;
        for (int i = 0; i < L; ++i) { run += s[i]; c[i] = run; }
        const double S = c[L - 1];                 /* Algorithm 2: sum of the row ...            */
        if (!(S > 0.0)) { flags[r] = ORACLE_ROW_INVALID; free(s); free(c); continue; }
        const double target = (double)top_p * S;   /* ... times p is the mass to reach           */

        int kstar = 0;                             /* Eq. 8: shortest sorted prefix reaching it   */
        while (c[kstar] < target) ++kstar;
        const double t = s[kstar];                 /* tau*: the smallest value that must be kept  */

        int first = kstar, last = kstar;           /* ends of the run of values equal to tau*     */
        while (first > 0 && s[first - 1] == t) --first;
        while (last + 1 < L && s[last + 1] == t) ++last;
        const double m_incl = c[last];
        const double m_excl = first > 0 ? c[first - 1] : 0.0;

        int cnt = 0;                               /* Algorithm 2's last step: {i : a_i >= theta} */
        for (int i = 0; i < L; ++i)
            if ((double)a[i] >= t) out[cnt++] = i;
        counts[r] = cnt;
        tau[r] = (float)t;
        if (fabs(m_incl - target) <= 1e-6 * S || fabs(m_excl - target) <= 1e-6 * S)
            flags[r] |= ORACLE_ROW_NEAR_BOUNDARY;
        if (diag) {
            double *dg = diag + 4 * (int64_t)r;
            dg[0] = S; dg[1] = target; dg[2] = m_incl; dg[3] = m_excl;
        }
        free(s); free(c);
    }
    return status;
}

/*
 * Algorithm 2, inner loop, for one row: bisection on the threshold value in
 * [0, max a], `iters` halvings.  Returns both ends of the final bracket and
 * the last midpoint; the algorithm as printed selects with the last midpoint.
 * theta_low always keeps mass >= target (it starts at 0 and only moves to
 * midpoints that do), so {a >= theta_low} is the feasible choice.
 * margin (optional): the smallest |M_current - M_target| met in any iteration - how close the
 * closest of the algorithm's comparisons came to going the other way.
 */
static void bisect_row(const float *a, int L, double p, int iters,
                       double *theta_low, double *theta_high, double *theta_mid, double *total_out, double *margin)
{
    double total = 0.0, hi = 0.0, lo = 0.0, mid = 0.0, closest = INFINITY;
    for (int i = 0; i < L; ++i) { total += (double)a[i]; if ((double)a[i] > hi) hi = (double)a[i]; }
    const double target = p * total;
    for (int it = 0; it < iters; ++it) {
        mid = 0.5 * (hi + lo);
        double m = 0.0;
        for (int i = 0; i < L; ++i) if ((double)a[i] >= mid) m += (double)a[i];
        if (fabs(m - target) < closest) closest = fabs(m - target);
        if (m < target) hi = mid; else lo = mid;
    }
    *theta_low = lo; *theta_high = hi; *theta_mid = mid;
    if (total_out) *total_out = total;
    if (margin) *margin = closest;
}

int oracle_nucleus_bisection(const float *a, int L, double p, int iters,
                             double *theta_low, double *theta_high, double *theta_mid)
{
    bisect_row(a, L, p, iters, theta_low, theta_high, theta_mid, NULL, NULL);
    return 0;
}

/*
 * Algorithm 2 with a fixed number of halvings (the footnote in Section 3.4: the implementation
 * uses 10), as a selection: per row the set {j : a_j >= theta_low} in ascending j.  theta_low = 0
 * (never raised) keeps every position of the row, zeros included.
 * tau[r] is the smallest fp32 value >= theta_low, so that {a >= tau} is the same set.
 * flags: ORACLE_ROW_INVALID as for the exact selection; ORACLE_ROW_NEAR_BOUNDARY when one of the
 * comparisons M_current < M_target was decided by less than 1e-6 of the row sum.
 */
int oracle_bisection_select(const float *probs, int64_t row_stride, int rows, const int32_t *lens,
                            float top_p, int iters, int32_t *indices, int64_t idx_stride,
                            int32_t *counts, float *tau, uint32_t *flags)
{
    if (!(top_p > 0.0f && top_p <= 1.0f) || iters < 1) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < rows; ++r) {
        const float *a = probs + (int64_t)r * row_stride;
        const int L = lens[r];
        int32_t *out = indices + (int64_t)r * idx_stride;
        counts[r] = 0; tau[r] = 0.0f; flags[r] = 0;
        int bad = (L <= 0);
        for (int i = 0; i < L && !bad; ++i)
            if (isnan(a[i]) || isinf(a[i]) || a[i] < 0.0f) bad = 1;
        double lo, hi, mid, total, margin;
        if (!bad) {
            bisect_row(a, L, (double)top_p, iters, &lo, &hi, &mid, &total, &margin);
            if (!(total > 0.0)) bad = 1;
        }
        if (bad) { flags[r] = ORACLE_ROW_INVALID; continue; }
        int c = 0;
        for (int i = 0; i < L; ++i) if ((double)a[i] >= lo) out[c++] = i;
        counts[r] = c;
        float t = (float)lo;
        if ((double)t < lo) t = nextafterf(t, INFINITY);
        tau[r] = t;
        if (margin <= 1e-6 * total) flags[r] |= ORACLE_ROW_NEAR_BOUNDARY;
    }
    return 0;
}

/*
 * Chunk masses for chunk-granular selection (Section 4 evaluates with chunks of 16 tokens; the paper
 * does not say how a chunk is scored - the reading here is the chunk's attention mass, which keeps
 * the top-p guarantee: the kept chunks hold at least p of the row's mass).
 *
 * mass[r][c] = fp32( sum of probs[r][c*chunk .. min((c+1)*chunk, lens[r])) ), the sum taken in fp64 in
 * ascending position order.  A chunk that holds a NaN, negative or infinite entry gets mass NaN, which
 * makes the row invalid for the selection that follows.  Chunks past the row's end get mass 0.
 */
int oracle_chunk_masses(const float *probs, int64_t row_stride, int rows, const int32_t *lens,
                        int chunk, int n_chunks, float *mass)
{
    if (chunk <= 0) return -1;
    for (int r = 0; r < rows; ++r) {
        const float *a = probs + (int64_t)r * row_stride;
        const int L = lens[r] > 0 ? lens[r] : 0;
        for (int c = 0; c < n_chunks; ++c) {
            double sum = 0.0;
            int bad = 0;
            for (int j = c * chunk; j < (c + 1) * chunk && j < L; ++j) {
                if (isnan(a[j]) || isinf(a[j]) || a[j] < 0.0f) bad = 1;
                sum += (double)a[j];
            }
            mass[(int64_t)r * n_chunks + c] = bad ? NAN : (float)sum;
        }
    }
    return 0;
}

/* fmt: 0 = fp32, 1 = bf16 bit patterns, 2 = IEEE half (fp16) bit patterns; every value is read exactly */
static inline double load_elem(const void *base, int64_t i, int fmt)
{
    if (fmt == 1) {
        uint32_t u = (uint32_t)((const uint16_t *)base)[i] << 16;
        float f; memcpy(&f, &u, 4); return (double)f;
    }
    if (fmt == 2) {
        const uint16_t hbits = ((const uint16_t *)base)[i];
        const int sign = hbits >> 15, e = (hbits >> 10) & 31, m = hbits & 1023;
        double v;
        if (e == 0) v = ldexp((double)m, -24);                    /* zero and subnormals: m * 2^-24 */
        else if (e == 31) v = m ? NAN : INFINITY;
        else v = ldexp((double)(1024 + m), e - 25);               /* (1 + m/1024) * 2^(e-15) */
        return sign ? -v : v;
    }
    return (double)((const float *)base)[i];
}

/*
 * Masked dense attention for a list of output rows, optionally with the verifier's own new tokens.
 *
 * q      [B][H_q][T][d], k/v [B][H_kv][n][d]   (is_bf16 = 0: fp32; 1: bf16 bit patterns; 2: fp16 bit patterns)
 * mask   [B][H_kv][n] uint8, 1 = position selected for that kv head
 * lens   [B] valid context length per sequence (positions >= lens[b] never attend)
 * k_new, v_new  [B][H_kv][T][d] or NULL: keys and values of the T tokens being verified (Algorithm 1
 *        feeds the gamma draft tokens and the last accepted one through the verifier together).  They
 *        sit behind the cache, are never subject to the mask, and are seen causally: query t attends
 *        to new tokens 0..t.
 * which  [n_rows][3] = (b, h_q, t) of each requested output row
 * out    [n_rows][d] fp64, lse [n_rows] fp64 (log-sum-exp of the kept scaled scores)
 * Query head h_q reads kv head h_q / (H_q / H_kv).
 * A row with no position to attend to gives out = 0 and lse = -inf.
 */
int oracle_masked_attention_tail(const void *q, const void *k, const void *v, int is_bf16,
                                 int B, int H_q, int H_kv, int T, int d, int n,
                                 const uint8_t *mask, const int32_t *lens,
                                 const void *k_new, const void *v_new, double sm_scale,
                                 const int32_t *which, int n_rows, double *out, double *lse)
{
    if (H_q % H_kv) return -1;
    if ((k_new == NULL) != (v_new == NULL)) return -2;
    const int G = H_q / H_kv;
    (void)B;
#pragma omp parallel for schedule(dynamic, 1)
    for (int w = 0; w < n_rows; ++w) {
        const int b = which[3 * w], hq = which[3 * w + 1], t = which[3 * w + 2];
        const int hk = hq / G;
        const int L = lens[b] > 0 ? lens[b] : 0;
        const int n_tail = k_new ? t + 1 : 0;    /* causal among the new tokens */
        const int64_t qoff = (((int64_t)b * H_q + hq) * T + t) * d;
        const int64_t kvoff = ((int64_t)b * H_kv + hk) * (int64_t)n * d;
        const int64_t newoff = ((int64_t)b * H_kv + hk) * (int64_t)T * d;
        const uint8_t *m = mask + ((int64_t)b * H_kv + hk) * (int64_t)n;
        double *o = out + (int64_t)w * d;
        double *score = (double *)malloc(sizeof(double) * (size_t)(L + n_tail + 1));
        double mx = -INFINITY;
        for (int j = 0; j < L; ++j) {            /* Eq. 1: Q K^T / sqrt(d), every position */
            double acc = 0.0;
            for (int e = 0; e < d; ++e)
                acc += load_elem(q, qoff + e, is_bf16) * load_elem(k, kvoff + (int64_t)j * d + e, is_bf16);
            score[j] = m[j] ? acc * sm_scale : -INFINITY;   /* Eq. 3: unselected positions drop out */
            if (score[j] > mx) mx = score[j];
        }
        for (int p = 0; p < n_tail; ++p) {       /* the new tokens, position L + p */
            double acc = 0.0;
            for (int e = 0; e < d; ++e)
                acc += load_elem(q, qoff + e, is_bf16) * load_elem(k_new, newoff + (int64_t)p * d + e, is_bf16);
            score[L + p] = acc * sm_scale;
            if (score[L + p] > mx) mx = score[L + p];
        }
        for (int e = 0; e < d; ++e) o[e] = 0.0;
        if (mx == -INFINITY) { lse[w] = -INFINITY; free(score); continue; }
        double denom = 0.0;
        for (int j = 0; j < L + n_tail; ++j) denom += exp(score[j] - mx);
        for (int j = 0; j < L; ++j) {            /* Eq. 2: weights times V */
            if (!m[j]) continue;
            const double wj = exp(score[j] - mx) / denom;
            for (int e = 0; e < d; ++e)
                o[e] += wj * load_elem(v, kvoff + (int64_t)j * d + e, is_bf16);
        }
        for (int p = 0; p < n_tail; ++p) {
            const double wj = exp(score[L + p] - mx) / denom;
            for (int e = 0; e < d; ++e)
                o[e] += wj * load_elem(v_new, newoff + (int64_t)p * d + e, is_bf16);
        }
        lse[w] = mx + log(denom);
        free(score);
    }
    return 0;
}

/* The cache alone (no new tokens). */
int oracle_masked_attention(const void *q, const void *k, const void *v, int is_bf16,
                            int B, int H_q, int H_kv, int T, int d, int n,
                            const uint8_t *mask, const int32_t *lens, double sm_scale,
                            const int32_t *which, int n_rows, double *out, double *lse)
{
    return oracle_masked_attention_tail(q, k, v, is_bf16, B, H_q, H_kv, T, d, n, mask, lens, NULL, NULL,
                                        sm_scale, which, n_rows, out, lse);
}
