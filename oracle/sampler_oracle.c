/*
 * CHECKER, NOT PRODUCT.  Test infrastructure: a serial fp64 statement of the
 * token a sampling call must return.  Only the tests, the smoke check and the
 * benchmark's CPU-baseline leg may call it.  It shares no code with the HIP
 * library.
 *
 * The paper draws completions y ~ p_theta(y | x_i, d_j) at a set temperature
 * (Alg. 1, parallel sampling; App. "Experiment settings": temperatures 0.4,
 * 0.7, 1.0) and says nothing else about the sampler, so the rule is fixed here:
 *
 *   1. p_i = exp((x_i - max_k x_k) / T), S = sum_i p_i in index order.
 *      T == 0 means greedy: the lowest index attaining the maximum.
 *   2. Nucleus: order tokens by (p descending, index ascending); the cut is the
 *      first position k whose running mass c_k >= top_p * S; tau = p at the cut.
 *      top_p >= 1 keeps everything (tau = 0).  The kept set is every token with
 *      p_i >= tau, so all ties with the threshold are kept.
 *   3. Z = sum of kept p_i in index order.  Walk the vocabulary in index order
 *      adding kept p_i; return the first kept i whose running mass c > u * Z
 *      (strict).  If rounding lets the walk finish, return the last kept index.
 *
 * Besides the token it reports the normalised CDF interval of the returned
 * token and the relative margin of the nucleus cut, so that a test can tell a
 * genuine mismatch from a uniform sitting on a boundary.
 *
 * Parity pins (tests/test_oracle_sampler.py): two- and three-token closed
 * forms, equal logits => floor(u V), T -> 0 and top_p -> 0 => argmax,
 * monotonicity in u, stratified-u frequency counts, a sort-free threshold
 * formulation, and invariance under logit shift and joint (T, logit) scaling.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

typedef struct {
    double p;
    int32_t idx;
} entry;

static int by_mass_then_index(const void *a, const void *b)
{
    const entry *x = (const entry *)a, *y = (const entry *)b;
    if (x->p > y->p) return -1;
    if (x->p < y->p) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

int oracle_sample_tokens(const float *logits, int64_t rows, int64_t vocab, int64_t row_stride,
                         const float *temperature, const float *top_p, const float *uniforms,
                         int32_t *token, double *cdf_lo, double *cdf_hi,
                         double *cut_margin, int32_t *kept_count)
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
            kept_count[r] = 1;
            continue;
        }
        double *p = (double *)malloc(sizeof(double) * (size_t)vocab);
        double S = 0.0;
        for (int64_t i = 0; i < vocab; ++i) {
            p[i] = exp(((double)x[i] - xmax) / T);
            S += p[i];
        }
        double tau = 0.0, margin = INFINITY;
        if ((double)top_p[r] < 1.0) {
            entry *e = (entry *)malloc(sizeof(entry) * (size_t)vocab);
            for (int64_t i = 0; i < vocab; ++i) {
                e[i].p = p[i];
                e[i].idx = (int32_t)i;
            }
            qsort(e, (size_t)vocab, sizeof(entry), by_mass_then_index);
            const double need = (double)top_p[r] * S;
            double c = 0.0, prev = 0.0;
            int64_t k = vocab - 1;
            for (int64_t i = 0; i < vocab; ++i) {
                prev = c;
                c += e[i].p;
                if (c >= need) {
                    k = i;
                    break;
                }
            }
            tau = e[k].p;
            margin = fabs(c - need) / S;
            if (k > 0 && fabs(prev - need) / S < margin)
                margin = fabs(prev - need) / S;
            free(e);
        }
        double Z = 0.0;
        int32_t kept = 0;
        for (int64_t i = 0; i < vocab; ++i)
            if (p[i] >= tau) {
                Z += p[i];
                ++kept;
            }
        const double target = (double)uniforms[r] * Z;
        double c = 0.0, lo = 0.0;
        int64_t pick = -1, last = -1;
        for (int64_t i = 0; i < vocab; ++i) {
            if (!(p[i] >= tau))
                continue;
            last = i;
            lo = c;
            c += p[i];
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
        kept_count[r] = kept;
        free(p);
    }
    return 0;
}
