/* Runs the fp64 checker (oracle/ *.c) under AddressSanitizer and UndefinedBehaviorSanitizer on small
 * seeded inputs that reach its corner cases: empty prefixes and suffixes, a sample with no KV at all,
 * paged KV with partly filled last pages, row subsets, one-token vocabularies, exact ties, greedy
 * rows, every filter combination.  Exit status 0 = the sanitizers saw nothing and the results are
 * finite where they must be. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_attention(int dtype, int N, int Hq, int Hkv, int D, int B, int page_size, double scale, const void *q,
                     const void *k_prefix, const void *v_prefix, const int32_t *prefix_lens,
                     const int32_t *prefix_indptr, const int32_t *prefix_page_indices, const int32_t *sample_indptr,
                     const void *k_suffix, const void *v_suffix, const int32_t *suffix_lens, int64_t max_suffix_len,
                     const int32_t *suffix_page_indptr, const int32_t *suffix_page_indices, const int64_t *rows,
                     int64_t num_rows, double *out, double *lse);
int oracle_sample_tokens(const float *logits, int64_t rows, int64_t vocab, int64_t row_stride, const float *temperature,
                         const float *top_p, const float *uniforms, int32_t *token, double *cdf_lo, double *cdf_hi,
                         double *cut_margin, int32_t *kept_count);
int oracle_sample_tokens_filtered(const float *logits, int64_t rows, int64_t vocab, int64_t row_stride,
                                  const float *temperature, const float *top_p, const int32_t *top_k,
                                  const float *min_p, const float *uniforms, int32_t *token, double *cdf_lo,
                                  double *cdf_hi, double *cut_margin, double *filter_margin, int32_t *kept_count);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static double unif(void)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(state >> 11) / 9007199254740992.0;
}
static float normalish(void) { return (float)((unif() + unif() + unif() + unif() - 2.0) * 1.7320508); }
static uint16_t bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static int attention_case(int dtype, int page, int B, int spp, int Hq, int Hkv, int D, int lp_hi, int ls_hi)
{
    const int N = B * spp, P = 16;
    const size_t elt = dtype ? 2 : 4;
    int32_t *plen = malloc(sizeof(int32_t) * B), *pind = malloc(sizeof(int32_t) * (B + 1));
    int32_t *sind = malloc(sizeof(int32_t) * (B + 1)), *slen = malloc(sizeof(int32_t) * N);
    int32_t *spind = malloc(sizeof(int32_t) * (N + 1));
    int64_t ptok = 0, ppages = 0, spages = 0;
    for (int b = 0; b < B; ++b) {
        plen[b] = b == 0 ? 0 : (int32_t)(unif() * (lp_hi + 1));   /* the first prompt is empty */
        pind[b] = (int32_t)(page ? ppages : ptok);
        ptok += plen[b];
        ppages += (plen[b] + P - 1) / P;
        sind[b] = b * spp;
    }
    pind[B] = (int32_t)(page ? ppages : ptok);
    sind[B] = N;
    for (int n = 0; n < N; ++n) {
        slen[n] = n == 0 ? 0 : (int32_t)(unif() * (ls_hi + 1));   /* sample 0 has no KV at all */
        spind[n] = (int32_t)spages;
        spages += (slen[n] + P - 1) / P;
    }
    spind[N] = (int32_t)spages;
    const int64_t pool_pages = ppages + spages;
    const int64_t kp_elems = page ? pool_pages * Hkv * P * D : (ptok > 0 ? ptok : 1) * (int64_t)Hkv * D;
    const int64_t ks_elems = page ? kp_elems : (int64_t)N * (ls_hi > 0 ? ls_hi : 1) * Hkv * D;
    void *kp = malloc(kp_elems * elt), *vp = malloc(kp_elems * elt);
    void *ks = page ? kp : malloc(ks_elems * elt), *vs = page ? vp : malloc(ks_elems * elt);
    void *q = malloc((size_t)N * Hq * D * elt);
    void *bufs[5] = {kp, vp, ks, vs, q};
    const int64_t sizes[5] = {kp_elems, kp_elems, ks_elems, ks_elems, (int64_t)N * Hq * D};
    for (int a = 0; a < 5; ++a) {
        if (page && (a == 2 || a == 3))
            continue;
        for (int64_t i = 0; i < sizes[a]; ++i) {
            if (dtype)
                ((uint16_t *)bufs[a])[i] = bf16(normalish());
            else
                ((float *)bufs[a])[i] = normalish();
        }
    }
    int32_t *ppi = NULL, *spi = NULL;
    if (page) {
        /* shuffled page ids: prefix pages then suffix pages of a random permutation */
        int32_t *perm = malloc(sizeof(int32_t) * (pool_pages > 0 ? pool_pages : 1));
        for (int64_t i = 0; i < pool_pages; ++i)
            perm[i] = (int32_t)i;
        for (int64_t i = pool_pages - 1; i > 0; --i) {
            int64_t j = (int64_t)(unif() * (i + 1));
            int32_t t = perm[i];
            perm[i] = perm[j];
            perm[j] = t;
        }
        ppi = perm;
        spi = perm + ppages;
    }
    const int64_t total = (int64_t)N * Hq;
    double *out = malloc(sizeof(double) * total * D), *lse = malloc(sizeof(double) * total);
    int rc = oracle_attention(dtype, N, Hq, Hkv, D, B, page ? P : 0, 1.0 / sqrt((double)D), q, kp, vp, plen, pind, ppi,
                              sind, ks, vs, slen, ls_hi > 0 ? ls_hi : 1, spind, spi, NULL, total, out, lse);
    int bad = rc != 0;
    for (int64_t r = 0; r < total && !bad; ++r) {
        const int n = (int)(r / Hq), b = n / spp;
        const int empty = plen[b] + slen[n] == 0;
        if (empty ? !(isinf(lse[r]) && lse[r] < 0 && out[r * D] == 0.0) : !isfinite(lse[r]))
            bad = 1;
        for (int d = 0; d < D; ++d)
            if (!isfinite(out[r * D + d]))
                bad = 1;
    }
    /* a row subset must reproduce the full result */
    int64_t rows[3] = {total - 1, 0, total / 2};
    double *o2 = malloc(sizeof(double) * 3 * D), l2[3];
    rc = oracle_attention(dtype, N, Hq, Hkv, D, B, page ? P : 0, 1.0 / sqrt((double)D), q, kp, vp, plen, pind, ppi,
                          sind, ks, vs, slen, ls_hi > 0 ? ls_hi : 1, spind, spi, rows, 3, o2, l2);
    bad |= rc != 0;
    for (int i = 0; i < 3 && !bad; ++i)
        if (memcmp(o2 + i * D, out + rows[i] * D, sizeof(double) * D) != 0)
            bad = 1;
    free(plen); free(pind); free(sind); free(slen); free(spind); free(kp); free(vp);
    if (!page) { free(ks); free(vs); }
    free(q); free(ppi); free(out); free(lse); free(o2);
    return bad;
}

static int sampler_case(int64_t rows, int64_t vocab, int64_t stride, int ties)
{
    float *x = malloc(sizeof(float) * rows * stride);
    float *T = malloc(sizeof(float) * rows), *tp = malloc(sizeof(float) * rows), *u = malloc(sizeof(float) * rows);
    float *mp = malloc(sizeof(float) * rows);
    int32_t *tk = malloc(sizeof(int32_t) * rows), *tok = malloc(sizeof(int32_t) * rows), *kept = malloc(sizeof(int32_t) * rows);
    double *lo = malloc(sizeof(double) * rows), *hi = malloc(sizeof(double) * rows), *mg = malloc(sizeof(double) * rows);
    double *fm = malloc(sizeof(double) * rows);
    const float Ts[4] = {0.0f, 0.3f, 1.0f, 1.3f}, ps[4] = {1e-6f, 0.5f, 0.95f, 1.0f}, ms[4] = {0.0f, 1e-4f, 0.3f, 1.0f};
    const int32_t ks[4] = {0, 1, 3, 1000000};
    for (int64_t i = 0; i < rows * stride; ++i)
        x[i] = ties ? (float)((int)(normalish() * 4.0f)) * 0.5f : normalish() * 3.0f;
    int bad = 0;
    for (int combo = 0; combo < 16 && !bad; ++combo) {
        for (int64_t r = 0; r < rows; ++r) {
            T[r] = Ts[(r + combo) & 3];
            tp[r] = ps[(r / 4 + combo) & 3];
            mp[r] = ms[(r + combo / 4) & 3];
            tk[r] = ks[(r / 2 + combo) & 3];
            u[r] = (float)unif() * 0.999999f;
        }
        bad |= oracle_sample_tokens(x, rows, vocab, stride, T, tp, u, tok, lo, hi, mg, kept);
        for (int64_t r = 0; r < rows; ++r)
            if (tok[r] < 0 || tok[r] >= vocab || kept[r] < 1 || !(lo[r] <= hi[r]))
                bad = 1;
        bad |= oracle_sample_tokens_filtered(x, rows, vocab, stride, T, tp, (combo & 1) ? tk : NULL,
                                             (combo & 2) ? mp : NULL, u, tok, lo, hi, mg, fm, kept);
        for (int64_t r = 0; r < rows; ++r)
            if (tok[r] < 0 || tok[r] >= vocab || kept[r] < 1 || !(lo[r] <= hi[r]) || fm[r] < 0)
                bad = 1;
    }
    free(x); free(T); free(tp); free(u); free(mp); free(tk); free(tok); free(kept); free(lo); free(hi); free(mg); free(fm);
    return bad;
}

int main(void)
{
    int bad = 0;
    bad |= attention_case(0, 0, 2, 3, 4, 2, 8, 40, 9);
    bad |= attention_case(1, 0, 3, 2, 8, 2, 16, 70, 33);
    bad |= attention_case(1, 1, 3, 4, 4, 4, 16, 50, 40);
    bad |= attention_case(0, 1, 1, 1, 2, 1, 8, 0, 0);      /* nothing anywhere */
    bad |= attention_case(1, 1, 2, 5, 6, 3, 8, 17, 0);      /* no suffixes */
    bad |= sampler_case(16, 1, 1, 0);
    bad |= sampler_case(16, 5, 8, 1);
    bad |= sampler_case(24, 333, 333, 0);
    bad |= sampler_case(8, 2048, 2051, 1);
    printf(bad ? "FAILED\n" : "ok\n");
    return bad;
}
