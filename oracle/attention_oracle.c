/*
 * CHECKER, NOT PRODUCT.  This file is test infrastructure: a plain, slow fp64
 * statement of what one decode step of shared-prefix attention must produce.
 * Only the tests, the smoke check and the benchmark's CPU-baseline leg may call
 * it.  It shares no code with the HIP library.
 *
 * What it computes.  For each sample n and query head h the single query row
 * attends over the concatenation [prefix of the sample's prompt | the sample's
 * own suffix] of KV head floor(h / G):
 *
 *      s_t = (q . k_t) * scale        w_t = exp(s_t - max_t s_t)
 *      o   = sum_t w_t v_t / sum_t w_t        lse = max_t s_t + ln sum_t w_t
 *
 * This is the plain definition the paper's attention tasks are verified
 * against (App., attn task 0: the expected output is softmax(S) applied to the
 * value rows, `bmm(softmax(E0,1), E1)`), with S = Q K^T / sqrt(D).  There is no
 * prefix/suffix split, no running maximum and no merge here on purpose: the
 * cascade in the HIP path must reproduce this result, so this file must not
 * contain it.  An empty KV list gives o = 0 and lse = -inf, the initial state
 * (-inf, 0, 0) of the paper's MaxSum recurrence (App., attn task 0, `init`).
 *
 * Parity pins (tests/test_oracle_attention.py): brute-force numpy softmax on
 * tiny odd shapes, uniform keys => mean of the value rows, a dominant key, score
 * shift invariance, constant-V-per-KV-head (head mapping), token/page
 * permutation invariance, the running (max, sum, accumulator) state of the
 * paper's attention tasks stated from its definition on growing key sets, and
 * the log-sum-exp merge identity on block-wise splits.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double widen(const void *base, int dtype, int64_t idx)
{
    if (dtype == 0)
        return (double)((const float *)base)[idx];
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* Element offset of (token t, kv head j, channel 0) of one sequence.
 * contiguous: rows are [token][kv head][D] starting at token offset `start`.
 * paged:      pool is [page][kv head][slot][D]; `pages` lists the sequence's pages. */
static int64_t row_offset(int64_t t, int j, int Hkv, int D, int page_size,
                          int64_t start, const int32_t *pages)
{
    if (page_size == 0)
        return ((start + t) * Hkv + j) * (int64_t)D;
    int64_t pg = pages[t / page_size];
    return ((pg * Hkv + j) * page_size + t % page_size) * (int64_t)D;
}

int oracle_attention(int dtype, int N, int Hq, int Hkv, int D, int B, int page_size, double scale,
                     const void *q,
                     const void *k_prefix, const void *v_prefix,
                     const int32_t *prefix_lens, const int32_t *prefix_indptr,
                     const int32_t *prefix_page_indices, const int32_t *sample_indptr,
                     const void *k_suffix, const void *v_suffix,
                     const int32_t *suffix_lens, int64_t max_suffix_len,
                     const int32_t *suffix_page_indptr, const int32_t *suffix_page_indices,
                     const int64_t *rows, int64_t num_rows,
                     double *out, double *lse)
{
    if (Hkv <= 0 || Hq % Hkv != 0 || D <= 0)
        return 1;
    const int G = Hq / Hkv;
    const int64_t total = rows ? num_rows : (int64_t)N * Hq;
    int bad = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < total; ++r) {
        const int64_t row = rows ? rows[r] : r;
        const int n = (int)(row / Hq), h = (int)(row % Hq), j = h / G;
        int b = -1;
        for (int c = 0; c < B; ++c)
            if (n >= sample_indptr[c] && n < sample_indptr[c + 1])
                b = c;
        if (b < 0) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        const int64_t Lp = prefix_lens[b], Ls = suffix_lens[n], L = Lp + Ls;
        double *o = out + r * D;
        for (int d = 0; d < D; ++d)
            o[d] = 0.0;
        if (L == 0) {
            lse[r] = -INFINITY;
            continue;
        }
        const int32_t *ppages = page_size ? prefix_page_indices + prefix_indptr[b] : NULL;
        const int32_t *spages = page_size ? suffix_page_indices + suffix_page_indptr[n] : NULL;
        const int64_t pstart = page_size ? 0 : prefix_indptr[b];
        const int64_t sstart = (int64_t)n * max_suffix_len;
        double *s = (double *)malloc(sizeof(double) * (size_t)L);
        const int64_t qoff = ((int64_t)n * Hq + h) * D;

        /* scores over the concatenated list */
        for (int64_t t = 0; t < L; ++t) {
            const int in_prefix = t < Lp;
            const void *kb = in_prefix ? k_prefix : k_suffix;
            const int64_t off = in_prefix
                ? row_offset(t, j, Hkv, D, page_size, pstart, ppages)
                : row_offset(t - Lp, j, Hkv, D, page_size, sstart, spages);
            double acc = 0.0;
            for (int d = 0; d < D; ++d)
                acc += widen(q, dtype, qoff + d) * widen(kb, dtype, off + d);
            s[t] = acc * scale;
        }
        double m = s[0];
        for (int64_t t = 1; t < L; ++t)
            if (s[t] > m)
                m = s[t];
        double l = 0.0;
        for (int64_t t = 0; t < L; ++t) {
            s[t] = exp(s[t] - m);
            l += s[t];
        }
        for (int64_t t = 0; t < L; ++t) {
            const int in_prefix = t < Lp;
            const void *vb = in_prefix ? v_prefix : v_suffix;
            const int64_t off = in_prefix
                ? row_offset(t, j, Hkv, D, page_size, pstart, ppages)
                : row_offset(t - Lp, j, Hkv, D, page_size, sstart, spages);
            for (int d = 0; d < D; ++d)
                o[d] += s[t] * widen(vb, dtype, off + d);
        }
        for (int d = 0; d < D; ++d)
            o[d] /= l;
        lse[r] = m + log(l);
        free(s);
    }
    return bad;
}
