/*
 * CHECKER, NOT PRODUCT.  Test infrastructure: a serial fp64 statement of the token a
 * filtered sampling call must return.  Only the tests may call it.  It shares no code with
 * the HIP library.
 *
 * The paper samples at a set temperature (App. "Experiment settings") and names no other
 * sampler setting; min-p and top-k are the usual companions of top-p, and since the paper is
 * silent the rule is fixed here.  Filters apply in this order, each to what the previous one
 * kept:
 *
 *   1. p_i = exp((x_i - max_k x_k) / T), so the most probable token has p = 1.
 *      T == 0 is greedy: the lowest index attaining the maximum.
 *   2. min-p (min_p > 0): keep the tokens with p_i >= min_p.
 *   3. top-k (top_k > 0): order the kept tokens by (p descending, index ascending); if more
 *      than top_k are left, tau_k = p of the top_k-th, and every token with p_i >= tau_k stays
 *      (all ties with the top_k-th are kept).
 *   4. top-p over the survivors: S2 = their mass; the cut is the first position of the same
 *      order whose running mass reaches top_p * S2; tau = p at the cut; survivors with
 *      p_i >= tau stay (ties kept).  top_p >= 1 keeps every survivor.
 *   5. Z = mass of what is left, in index order; walking the vocabulary in index order the
 *      token returned is the first one left whose running mass exceeds u * Z.
 *
 * Besides the token it reports the normalised CDF interval of the returned token, the relative
 * margin of the nucleus cut, and `filter_margin`: the smallest relative distance between a
 * filter's threshold and the nearest probability that is not exactly on it (min-p: |p_i -
 * min_p| / min_p over all i; top-k: the gap between tau_k and the next smaller probability,
 * relative to tau_k).  A test uses the margins to tell a genuine mismatch from a threshold
 * that fp32 and fp64 may order differently.
 *
 * Parity pins (tests/test_oracle_sampler_filtered.py): with both filters off it is the plain
 * rule; top_k = 1 and min_p = 1 are greedy; closed forms on three and four tokens; top_k = V
 * and min_p -> 0 change nothing; the kept set is nested in k and in min_p; a brute-force
 * restatement on tiny vocabularies.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

typedef struct {
    double p;
    int32_t idx;
} fentry;

static int f_by_mass_then_index(const void *a, const void *b)
{
    const fentry *x = (const fentry *)a, *y = (const fentry *)b;
    if (x->p > y->p) return -1;
    if (x->p < y->p) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

int oracle_sample_tokens_filtered(const float *logits, int64_t rows, int64_t vocab, int64_t row_stride,
                                  const float *temperature, const float *top_p, const int32_t *top_k,
                                  const float *min_p, const float *uniforms, int32_t *token, double *cdf_lo,
                                  double *cdf_hi, double *cut_margin, double *filter_margin,
                                  int32_t *kept_count)
{
    if (vocab <= 0)
        return 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < rows; ++r) {
        const float *x = logits + r * row_stride;
        const double T = (double)temperature[r];
        double xmax = (double)x[0];
        int64_t arg = 0;
        for (int64_t i = 1; i < vocab; ++i)
            if ((double)x[i] > xmax) {
                xmax = (double)x[i];
                arg = i;
            }
        if (T == 0.0) {
            token[r] = (int32_t)arg;
            cdf_lo[r] = 0.0;
            cdf_hi[r] = 1.0;
            cut_margin[r] = INFINITY;
            filter_margin[r] = INFINITY;
            kept_count[r] = 1;
            continue;
        }
        fentry *e = (fentry *)malloc(sizeof(fentry) * (size_t)vocab);
        double fmargin = INFINITY;
        const double mp = min_p ? (double)min_p[r] : 0.0;
        int64_t n = 0;  /* survivors so far, e[0..n) */
        for (int64_t i = 0; i < vocab; ++i) {
            const double p = exp(((double)x[i] - xmax) / T);
            if (mp > 0.0) {
                const double d = fabs(p - mp) / mp;
                if (d > 0.0 && d < fmargin)
                    fmargin = d;
                if (!(p >= mp))
                    continue;
            }
            e[n].p = p;
            e[n].idx = (int32_t)i;
            ++n;
        }
        qsort(e, (size_t)n, sizeof(fentry), f_by_mass_then_index);
        const int64_t k = top_k ? (int64_t)top_k[r] : 0;
        if (k > 0 && n > k) {
            const double tau_k = e[k - 1].p;
            int64_t m = k;
            while (m < n && e[m].p >= tau_k)  /* ties with the k-th stay */
                ++m;
            if (m < n) {
                const double d = (tau_k - e[m].p) / tau_k;
                if (d < fmargin)
                    fmargin = d;
            }
            n = m;
        }
        double S2 = 0.0;
        for (int64_t i = 0; i < n; ++i)
            S2 += e[i].p;
        double tau = 0.0, margin = INFINITY;
        if ((double)top_p[r] < 1.0) {
            const double need = (double)top_p[r] * S2;
            double c = 0.0, prev = 0.0;
            int64_t cut = n - 1;
            for (int64_t i = 0; i < n; ++i) {
                prev = c;
                c += e[i].p;
                if (c >= need) {
                    cut = i;
                    break;
                }
            }
            tau = e[cut].p;
            margin = fabs(c - need) / S2;
            if (cut > 0 && fabs(prev - need) / S2 < margin)
                margin = fabs(prev - need) / S2;
            int64_t m = cut + 1;
            while (m < n && e[m].p >= tau)
                ++m;
            n = m;
        }
        /* what is left, back in vocabulary order */
        char *left = (char *)calloc((size_t)vocab, 1);
        double *pl = (double *)malloc(sizeof(double) * (size_t)vocab);
        for (int64_t i = 0; i < n; ++i) {
            left[e[i].idx] = 1;
            pl[e[i].idx] = e[i].p;
        }
        double Z = 0.0;
        for (int64_t i = 0; i < vocab; ++i)
            if (left[i])
                Z += pl[i];
        const double target = (double)uniforms[r] * Z;
        double c = 0.0, lo = 0.0;
        int64_t pick = -1, last = -1;
        for (int64_t i = 0; i < vocab; ++i) {
            if (!left[i])
                continue;
            last = i;
            lo = c;
            c += pl[i];
            if (c > target) {
                pick = i;
                break;
            }
        }
        if (pick < 0)
            pick = last;
        token[r] = (int32_t)pick;
        cdf_lo[r] = lo / Z;
        cdf_hi[r] = c / Z;
        cut_margin[r] = margin;
        filter_margin[r] = fmargin;
        kept_count[r] = (int32_t)n;
        free(left);
        free(pl);
        free(e);
    }
    return 0;
}
