/*
 * spdecode: one decode step of parallel sampling on MI355X (gfx950).
 *
 * The paper's self-improvement loop draws many candidate completions from one
 * long demonstration-augmented prompt (Alg. 1, "parallel sampling"; App.
 * "Experiment settings": 64 samples per temperature, at most 1024 output
 * tokens).  Inside the serving engine that step is, per generated token,
 *
 *   1. attention of every sample's single query row over the prompt's KV (shared
 *      by all samples: the "prefix") and over the sample's own generated tokens
 *      (the "suffix"), and
 *   2. temperature sampling of the next token from the logits.
 *
 * This library provides exactly those two operations.  The attention is computed
 * as a cascade: one pass treats all samples' queries of a KV head as a dense tile
 * against the shared prefix (so the prefix is read once, not once per sample), a
 * second pass streams each sample's private suffix, and the two partial softmax
 * states are combined with the log-sum-exp rescaling of the online-softmax
 * recurrence the paper prints for its attention tasks (App., attn tasks 0-2:
 * running maximum m, running sum l, unnormalised accumulator, one final
 * division).  The result equals softmax(q K^T * scale) V over the concatenated
 * KV, which is the plain definition those tasks are verified against.
 *
 * Conventions for every entry point
 *   - plain C ABI; no exceptions, no global mutable state.
 *   - every data pointer is a DEVICE pointer owned by the caller unless marked
 *     "host"; the library never allocates, frees or synchronises.  Scratch
 *     memory comes from the caller's `workspace` (size from the matching
 *     *_workspace_size call; 256-byte aligned).
 *   - work is enqueued on `stream` (a hipStream_t, may be NULL for the default
 *     stream) and the call returns without waiting.  Inputs are never written.
 *   - the return value reports host-checkable errors only (spd_status).  Values
 *     that only the device sees (lengths larger than the stated maxima, page ids
 *     out of range, NaN logits, negative temperature) are the caller's
 *     responsibility: results are then undefined.
 *   - concurrent calls are safe if their workspaces and outputs are disjoint.
 *   - range of V on the bf16 path: partial results travel between the kernels as fp16, so every
 *     value row must satisfy |v| <= 65504 (anything a softmax-weighted average of such rows can
 *     reach).  bf16 itself can hold larger magnitudes; results for them are undefined (inf or
 *     NaN).  The fp32 path has no such limit.
 */
#ifndef SPDECODE_H
#define SPDECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPD_API __attribute__((visibility("default")))

typedef enum {
    SPD_OK = 0,
    SPD_EINVAL = 1,       /* NULL pointer, non-positive size, Hq % Hkv != 0, misaligned pointer */
    SPD_EUNSUPPORTED = 2, /* dtype / head_dim / page_size outside the supported set */
    SPD_EWORKSPACE = 3,   /* workspace missing, misaligned or too small */
    SPD_ELAUNCH = 4       /* the HIP runtime refused a launch */
} spd_status;

typedef enum { SPD_F32 = 0, SPD_BF16 = 1 } spd_dtype;

/* Stages of the attention call (for tests and per-kernel timing). 0 means all. */
enum { SPD_STAGE_PREFIX = 1, SPD_STAGE_SUFFIX = 2, SPD_STAGE_MERGE = 4 };

/*
 * Problem description (host memory, read during the call only).
 *
 * N samples are grouped by prompt: prompt b owns the consecutive samples
 * sample_indptr[b] .. sample_indptr[b+1]-1.  Query head h reads KV head
 * h / (num_q_heads / num_kv_heads).
 *
 * Supported: dtype bf16 or f32, head_dim a multiple of 8 up to 256, page_size 0
 * (contiguous KV) or 16.  bf16 with head_dim 128 and at most 16 query heads per
 * KV head runs on the MFMA kernels; everything else on the plain kernels (fp32
 * arithmetic, one lane per token).
 */
typedef struct spd_attn_desc {
    int32_t dtype;                  /* spd_dtype of Q, K, V and the output */
    int32_t num_q_heads;            /* Hq */
    int32_t num_kv_heads;           /* Hkv, divides Hq */
    int32_t head_dim;               /* D */
    int32_t num_prompts;            /* B >= 1 */
    int32_t num_samples;            /* N >= 1, total over all prompts */
    int32_t max_samples_per_prompt; /* upper bound on sample_indptr[b+1]-sample_indptr[b]; 0 = N */
    int32_t page_size;              /* 0 = contiguous KV, 16 = paged */
    float sm_scale;                 /* score scale; <= 0 selects 1/sqrt(D) */
    uint32_t stages;                /* 0 = whole call; else OR of SPD_STAGE_* */
} spd_attn_desc;

/* Bytes of workspace the attention call needs for these bounds (0 on invalid desc). */
SPD_API size_t shared_prefix_decode_attn_workspace_size(const spd_attn_desc *desc,
                                                int64_t max_prefix_len,
                                                int64_t max_suffix_len);

/*
 * Attention of one decode step: out[n, h, :] = softmax(q[n, h] . K^T * scale) V
 * over [prefix of n's prompt | suffix of n], K and V of KV head h / G.
 * (Alg. 1 parallel sampling; App. attn tasks 0-2 for the softmax algebra.)
 *
 * Layouts (element type = desc->dtype, row-major, innermost dimension last):
 *   q                 [N, Hq, D]
 *   contiguous KV (page_size == 0)
 *     k_prefix/v_prefix   [sum_b Lp_b, Hkv, D]; prompt b starts at token prefix_indptr[b]
 *     k_suffix/v_suffix   [N, max_suffix_len, Hkv, D]; only the first suffix_lens[n]
 *                         tokens of slot n are read
 *   paged KV (page_size == 16)
 *     k_prefix/v_prefix and k_suffix/v_suffix are page pools [num_pages, Hkv, 16, D]
 *     (they may be the same pool).  Prompt b's pages are
 *     prefix_page_indices[prefix_indptr[b] .. prefix_indptr[b+1]); sample n's are
 *     suffix_page_indices[suffix_page_indptr[n] .. suffix_page_indptr[n+1]).  The last
 *     page of a sequence may be partly filled; slots past the length are not read.
 *   prefix_lens  int32 [B]     tokens in each prompt's prefix (0 allowed)
 *   prefix_indptr int32 [B+1]  token offsets (contiguous) or page-list offsets (paged)
 *   sample_indptr int32 [B+1]
 *   suffix_lens  int32 [N]     tokens in each sample's suffix (0 allowed)
 *   max_prefix_len / max_suffix_len  host-known upper bounds used to size the launch;
 *                         max_suffix_len is also the slot stride of contiguous suffixes
 *   out          [N, Hq, D], desc->dtype.  A sample with no KV at all gets zeros.
 *   lse_out      float [N, Hq] natural-log log-sum-exp of the scaled scores, or NULL.
 *                -inf for a sample with no KV.
 *
 * All pointers must be 16-byte aligned.  Returns spd_status.
 */
SPD_API int shared_prefix_decode_attn(const spd_attn_desc *desc,
                              const void *q,
                              const void *k_prefix, const void *v_prefix,
                              const int32_t *prefix_lens,
                              const int32_t *prefix_indptr,
                              const int32_t *prefix_page_indices,
                              const int32_t *sample_indptr,
                              const void *k_suffix, const void *v_suffix,
                              const int32_t *suffix_lens,
                              const int32_t *suffix_page_indptr,
                              const int32_t *suffix_page_indices,
                              int64_t max_prefix_len, int64_t max_suffix_len,
                              void *out, float *lse_out,
                              void *workspace, size_t workspace_bytes,
                              void *stream);

/*
 * One level of a tree of shared prefixes.  The paper's prompts nest: the base prompt is shared
 * by every task, the demonstrations by the tasks of an iteration, the task text by its samples
 * (Sec. "Adaptive self-improvement learning", Alg. 1).  At each level the N samples are cut into
 * consecutive groups; the samples of a group attend over the group's KV.
 */
typedef struct spd_prefix_level {
    const void *k, *v;              /* device; layout as k_prefix/v_prefix of the plain call */
    const int32_t *lens;            /* device int32 [num_groups]: tokens per group (0 allowed) */
    const int32_t *indptr;          /* device int32 [num_groups+1]: token or page-list offsets */
    const int32_t *page_indices;    /* device, paged KV only */
    const int32_t *sample_indptr;   /* device int32 [num_groups+1]: group g owns samples
                                       sample_indptr[g] .. sample_indptr[g+1]-1; covers 0..N */
    int32_t num_groups;             /* >= 1 */
    int32_t max_samples_per_group;  /* upper bound; 0 = N */
    int64_t max_len;                /* host-known upper bound on lens[] */
} spd_prefix_level;

#define SPD_MAX_PREFIX_LEVELS 4

/* Bytes of workspace the multi-level call needs (0 on invalid arguments).  `levels` is host
 * memory; only num_groups, max_samples_per_group and max_len are read. */
SPD_API size_t shared_prefix_decode_attn_levels_workspace_size(const spd_attn_desc *desc,
                                                       int32_t num_levels,
                                                       const spd_prefix_level *levels,
                                                       int64_t max_suffix_len);

/*
 * Attention of one decode step over a tree of shared prefixes:
 * out[n, h, :] = softmax(q[n, h] . K^T * scale) V over
 * [level 0 KV of n's group | level 1 KV of n's group | ... | suffix of n].
 * With one level this is shared_prefix_decode_attn.  desc->num_prompts and
 * desc->max_samples_per_prompt are ignored (the levels carry them); desc->stages must be 0;
 * 1 <= num_levels <= SPD_MAX_PREFIX_LEVELS; `levels` is host memory read during the call.
 * Everything else as for shared_prefix_decode_attn.  Returns spd_status.
 */
SPD_API int shared_prefix_decode_attn_levels(const spd_attn_desc *desc,
                                     const void *q,
                                     int32_t num_levels, const spd_prefix_level *levels,
                                     const void *k_suffix, const void *v_suffix,
                                     const int32_t *suffix_lens,
                                     const int32_t *suffix_page_indptr,
                                     const int32_t *suffix_page_indices,
                                     int64_t max_suffix_len,
                                     void *out, float *lse_out,
                                     void *workspace, size_t workspace_bytes,
                                     void *stream);

/* Bytes of workspace sample_tokens needs (0 on invalid sizes). */
SPD_API size_t sample_tokens_workspace_size(int64_t rows, int64_t vocab);

/*
 * Next-token sampling at a temperature (App. "Experiment settings": the paper
 * samples at temperatures 0.4, 0.7 and 1.0; it is silent on everything else, so
 * the rule is fixed here).  Per row r, with x the row's logits:
 *
 *   p_i = exp((x_i - max x) / T_r);  S = sum p_i
 *   nucleus: tau = the largest value t among the p_i with mass{p_i >= t} >= top_p_r * S
 *            (tau = 0 when top_p_r >= 1); every token with p_i >= tau is kept, ties included
 *   Z = mass of the kept tokens; walking the vocabulary in index order, the token
 *   returned is the first kept i whose running kept mass exceeds uniforms[r] * Z.
 *   T_r == 0 returns the lowest index attaining the maximum logit.
 *
 *   logits       fp32 [rows, vocab], row r at logits + r * row_stride (elements)
 *   logits_dtype must be SPD_F32
 *   temperature, top_p, uniforms   float [rows]; uniforms in [0, 1)
 *   tokens_out   int32 [rows]
 *
 * Probabilities are evaluated in fp32 and accumulated in fp64 on the device.
 * Returns spd_status.
 */
SPD_API int sample_tokens(const void *logits, int32_t logits_dtype,
                  int64_t rows, int64_t vocab, int64_t row_stride,
                  const float *temperature, const float *top_p, const float *uniforms,
                  int32_t *tokens_out,
                  void *workspace, size_t workspace_bytes,
                  void *stream);

/*
 * sample_tokens for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and result
 * as sample_tokens without the workspace; the scratch memory is an array of
 * SPD_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the process ends),
 * and the call allocates and frees nothing.
 *
 * Limit: sample_tokens_workspace_size(rows, vocab) must not exceed SPD_STATIC_SCRATCH_BYTES
 * (about 95 rows of a 128k vocabulary); larger problems return SPD_EWORKSPACE and launch nothing.
 * All calls on one GPU share that GPU's array: two calls whose kernels may overlap (different
 * streams, or the same graph launched twice at once) race on it and give undefined tokens; calls
 * that follow one another on a stream are fine, whatever their sizes (every call resets what it
 * needs to find at zero).
 */
#define SPD_STATIC_SCRATCH_BYTES (16u << 20)
SPD_API int sample_tokens_static(const void *logits, int32_t logits_dtype,
                         int64_t rows, int64_t vocab, int64_t row_stride,
                         const float *temperature, const float *top_p, const float *uniforms,
                         int32_t *tokens_out,
                         void *stream);

/*
 * sample_tokens with two more filters ahead of top-p (the paper sets only the temperature, App.
 * "Experiment settings"; min-p and top-k are the usual companions of top-p, and the rule is fixed
 * here).  Per row, each filter acts on what the previous one kept:
 *
 *   p_i = exp((x_i - max x) / T_r), so the most probable token has p = 1
 *   min-p  (min_p[r] > 0): keep p_i >= min_p[r]
 *   top-k  (top_k[r] > 0): keep the top_k[r] most probable of those, and every tie with the last
 *   top-p  over the survivors' mass S2: tau = the largest value t with
 *          mass{survivors with p_i >= t} >= top_p_r * S2; keep p_i >= tau
 *   then the walk of sample_tokens over what is left.
 *
 *   top_k   int32 [rows] or NULL (= off everywhere); 0 = off for the row
 *   min_p   float [rows] or NULL; 0 = off for the row; values in (0, 1]
 * With both NULL this is sample_tokens.  Rows with a filter run through the same kernels as
 * sample_tokens when what the filters keep lies within the few thousand most probable tokens of
 * each 16384-token stretch of the row (top-k up to about a thousand, min-p down to about 1e-3 on
 * ordinary logits); otherwise, and for rows that are not 16-byte aligned, they take a
 * one-workgroup-per-row routine that reads the row several times (exact, about ten times slower).
 * Everything else as for sample_tokens.
 */
SPD_API int sample_tokens_filtered(const void *logits, int32_t logits_dtype,
                           int64_t rows, int64_t vocab, int64_t row_stride,
                           const float *temperature, const float *top_p,
                           const int32_t *top_k, const float *min_p,
                           const float *uniforms,
                           int32_t *tokens_out,
                           void *workspace, size_t workspace_bytes,
                           void *stream);

/*
 * Between two decode steps of the sampling loop (the paper generates up to 1024
 * tokens per sample, App. "Experiment settings"): append one token's K and V to the
 * private suffix of every live sample and add one to its suffix_lens entry, all on
 * the device, so that a loop of decode steps needs no host synchronisation.
 *
 *   desc              dtype, num_kv_heads, head_dim, num_samples, page_size as for the
 *                     attention call (the other fields are ignored)
 *   k_new, v_new      [N, Hkv, D], desc->dtype: the new token of each sample
 *   k_suffix/v_suffix, suffix_page_indptr, suffix_page_indices: as for the attention
 *                     call (written here)
 *   suffix_lens       int32 [N], read and incremented
 *   max_suffix_len    capacity of a sample's slot in tokens (contiguous: the slot stride;
 *                     paged: 16 * pages in the sample's page list).  A full sample is
 *                     left unchanged.
 *   last_tokens       int32 [N] or NULL: the token each sample drew in the previous step
 *   end_token         a sample whose last token equals it is marked finished
 *   finished          int32 [N] or NULL (then no sample ever finishes); nonzero = finished.
 *                     Finished samples are left unchanged; the flags persist across calls.
 *
 * All pointers are device pointers, 16-byte aligned.  Returns spd_status.
 */
SPD_API int append_suffix_kv(const spd_attn_desc *desc,
                     const void *k_new, const void *v_new,
                     void *k_suffix, void *v_suffix,
                     int32_t *suffix_lens,
                     const int32_t *suffix_page_indptr,
                     const int32_t *suffix_page_indices,
                     int64_t max_suffix_len,
                     const int32_t *last_tokens, int32_t end_token, int32_t *finished,
                     void *stream);

/*
 * A loop of decode steps replayed from one captured step (the paper generates up to 1024 tokens
 * per sample, App. "Experiment settings"; every step is append + attention + sampling on new
 * queries, keys, values and uniforms).  The step counter lives on the device, as a pair
 * step_state = {current, next} of int64 that starts as {0, 0}:
 *
 *   decode_step_select  copies row `current` of every src (a [num_steps, row_bytes] array) to dst
 *                       (row_bytes bytes) and sets next = current + 1; rows past the last one
 *                       repeat the last one
 *   decode_step_record  copies every src (row_bytes bytes) into row next - 1 of dst (a
 *                       [num_steps, row_bytes] array; nothing is written past its end) and sets
 *                       current = next
 *
 * so a step is select, the step's calls, record.  `copies` is host memory read during the call,
 * 1 <= count <= SPD_MAX_STEP_COPIES; src, dst and step_state are device pointers; row_bytes is a
 * positive multiple of 4, src and dst are 4-byte aligned (16-byte aligned rows are moved in
 * 16-byte pieces).  Source and destination ranges must not overlap.  Both calls are kernel
 * launches only (no memset, no allocation), fit for graph capture.  Returns spd_status.
 */
typedef struct spd_row_copy {
    const void *src;
    void *dst;
    int64_t row_bytes;
} spd_row_copy;
#define SPD_MAX_STEP_COPIES 8
SPD_API int decode_step_select(int64_t *step_state, int64_t num_steps,
                       int32_t count, const spd_row_copy *copies, void *stream);
SPD_API int decode_step_record(int64_t *step_state, int64_t num_steps,
                       int32_t count, const spd_row_copy *copies, void *stream);

/*
 * Everything between two decode steps of such a loop in ONE launch (a launch between two dependent
 * kernels costs 4 to 5 us on this machine whatever it does, and select + append + record are three
 * of the seven launches of a step).  With t = current:
 *
 *   - results of the step before, if t >= 1 (and t - 1 < num_steps): every `record` src (row_bytes
 *     bytes) goes to row t - 1 of its dst ([num_steps, row_bytes]), and every sample's suffix
 *     length, as that step left it, to row t - 1 of lens_record (int32 [num_steps, N], or NULL);
 *   - inputs of this step: row t of every `select` src ([num_steps, row_bytes]) goes to its dst
 *     (rows past the last one repeat the last one);
 *   - append_suffix_kv with row t of k_steps / v_steps ([num_steps, N, Hkv, D], desc->dtype) as the
 *     new token (same rules: finished samples and full slots are left alone);
 *   - then current = next = t + 1, stored by whichever workgroup finishes last, after all have read
 *     the old value (the third word of step_state counts them and is left at 0).  No workgroup
 *     waits for another.
 *
 * step_state is int64 [3], {0, 0, 0} before the first step.  A loop is: advance, the step's calls,
 * advance, the step's calls, ...; the results of the last step are still unrecorded when the loop
 * ends, and one decode_step_record call (which writes row next - 1) records them.
 * record_count and select_count may each be 0 .. SPD_MAX_STEP_COPIES; `record` and `select` are host
 * memory read during the call; alignment rules as for decode_step_select, K/V pointers 16-byte
 * aligned; the other arguments as for append_suffix_kv.  A kernel launch only (no memset, no
 * allocation), fit for graph capture.  Calls on one step_state must not overlap.  Returns spd_status.
 */
SPD_API int decode_step_advance(int64_t *step_state, int64_t num_steps,
                        int32_t record_count, const spd_row_copy *record,
                        int32_t select_count, const spd_row_copy *select,
                        const spd_attn_desc *desc,
                        const void *k_steps, const void *v_steps,
                        void *k_suffix, void *v_suffix,
                        int32_t *suffix_lens,
                        const int32_t *suffix_page_indptr,
                        const int32_t *suffix_page_indices,
                        int64_t max_suffix_len,
                        const int32_t *last_tokens, int32_t end_token, int32_t *finished,
                        int32_t *lens_record,
                        void *stream);

/* Short description of a status code (static storage). */
SPD_API const char *spd_status_string(int status);

/*
 * Launch plan the attention call will use for these bounds (host arithmetic
 * only).  Fills, when non-NULL: tokens per prefix split, number of prefix splits,
 * tokens per suffix chunk, number of suffix chunks.  Returns spd_status.
 */
SPD_API int spd_attn_plan(const spd_attn_desc *desc, int64_t max_prefix_len, int64_t max_suffix_len,
                  int32_t *prefix_split_tokens, int32_t *num_prefix_splits,
                  int32_t *suffix_chunk_tokens, int32_t *num_suffix_chunks);

#ifdef __cplusplus
}
#endif
#endif /* SPDECODE_H */
