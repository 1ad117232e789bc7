// Launch planning of the attention calls: host arithmetic only (no HIP, no allocation), so that it
// can also be compiled and exercised on a machine without a GPU.
//
// A call is cut into prefix splits (one workgroup per (group, KV head, row tile, split)) and suffix
// chunks (one wavefront per (sample, KV head, chunk)); every (split | chunk) owns one slot of
// partial softmax state per output row, which the merge combines.
#pragma once

#include "../../include/spdecode.h"

#include <stddef.h>
#include <stdint.h>

namespace spd {
namespace plan {

struct Plan {
    int prefix_split_tokens, num_prefix_splits;
    int suffix_chunk_tokens, num_suffix_chunks;
    size_t acc_bytes, ml_bytes;
};

// Plan of a multi-level call: split size and count per level, slot offsets, suffix chunks.
struct LevelPlan {
    int split_tokens[SPD_MAX_PREFIX_LEVELS], num_splits[SPD_MAX_PREFIX_LEVELS], slot0[SPD_MAX_PREFIX_LEVELS];
    int suffix_chunk_tokens, num_suffix_chunks, num_slots;
    size_t acc_bytes, ml_bytes;
};

constexpr int kPrefixBlockRows = 128;  // query rows per prefix workgroup on the tiled path
constexpr int kMaxSplits = 64;         // the merge takes 64 prefix splits and 64 suffix chunks
constexpr long long kMaxLen = 1ll << 30;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int check_desc(const spd_attn_desc* d)
{
    if (!d)
        return SPD_EINVAL;
    if (d->num_q_heads <= 0 || d->num_kv_heads <= 0 || d->head_dim <= 0 || d->num_prompts <= 0 ||
        d->num_samples <= 0 || d->max_samples_per_prompt < 0)
        return SPD_EINVAL;
    if (d->num_q_heads % d->num_kv_heads != 0)
        return SPD_EINVAL;
    if (d->dtype != SPD_F32 && d->dtype != SPD_BF16)
        return SPD_EUNSUPPORTED;
    if (d->page_size != 0 && d->page_size != 16)
        return SPD_EUNSUPPORTED;
    if (d->head_dim > 256 || d->head_dim % 8 != 0)
        return SPD_EUNSUPPORTED;
    if (d->stages & ~(uint32_t)(SPD_STAGE_PREFIX | SPD_STAGE_SUFFIX | SPD_STAGE_MERGE))
        return SPD_EINVAL;
    return SPD_OK;
}

// Tokens per part so that at most `max_parts` parts cover `len`, in multiples of `quantum`.
inline int part_tokens(long long len, int min_tokens, int max_parts, int quantum)
{
    long long t = (len + max_parts - 1) / max_parts;
    if (t < min_tokens)
        t = min_tokens;
    t = (t + quantum - 1) / quantum * quantum;
    return (int)t;
}

// Tokens per split of a prefix level with `groups` groups of at most `spp` samples and lengths up to
// `max_prefix`, at most `max_splits` splits.
inline int plan_prefix_split(const spd_attn_desc* d, int groups, int spp, long long max_prefix, int max_splits)
{
    if (d->dtype == SPD_BF16 && d->head_dim == 128) {
        // tiled path: one workgroup per (group, KV head, row tile, split); enough splits to
        // occupy every CU once, in multiples of the 64-token tile
        const long long rows = (long long)spp * (d->num_q_heads / d->num_kv_heads);
        const long long base = (long long)groups * d->num_kv_heads * ((rows + kPrefixBlockRows - 1) / kPrefixBlockRows);
        long long want = (256 + base - 1) / base;
        if (want > max_splits) want = max_splits;
        long long t = (max_prefix + want - 1) / want;
        t = (t + 63) / 64 * 64;
        if (t < 128) t = 128;  // at least two tiles per split: a one-tile workgroup is all start-up
        return (int)t;
    }
    return part_tokens(max_prefix, 256, max_splits, 64);
}

// Tokens per suffix chunk: enough (sample, KV head, chunk) items to keep every CU busy, chunks of
// 64..320 tokens (measured on ragged suffixes of up to 2048 tokens: 320-token chunks beat 512-token
// ones by 17 %, finer balance between wavefronts), at most kMaxSplits chunks.
inline int plan_suffix_chunk(const spd_attn_desc* d, long long max_suffix)
{
    const long long pairs = (long long)d->num_samples * d->num_kv_heads;
    const long long want_chunks = (2048 + pairs - 1) / pairs;
    long long t = (max_suffix + want_chunks - 1) / want_chunks;
    t = (t + 63) / 64 * 64;
    if (t < 64) t = 64;
    if (t > 320) t = 320;
    // Chunks of 128 or 256 tokens start every wavefront of the launch at addresses that agree in
    // many low bits (the rows of a sample are 2 KB apart), which costs 5 to 20 % of the HBM rate;
    // three quarters of the size spreads them.
    if (t == 128 || t == 256) t = t / 4 * 3;
    if (max_suffix > t * kMaxSplits) t = part_tokens(max_suffix, 64, kMaxSplits, 64);
    return (int)t;
}

inline int make_plan(const spd_attn_desc* d, long long max_prefix, long long max_suffix, Plan* pl)
{
    const int rc = check_desc(d);
    if (rc != SPD_OK)
        return rc;
    if (max_prefix < 0 || max_suffix < 0 || max_prefix > kMaxLen || max_suffix > kMaxLen)
        return SPD_EINVAL;
    const int spp = d->max_samples_per_prompt > 0 ? d->max_samples_per_prompt : d->num_samples;
    pl->prefix_split_tokens = plan_prefix_split(d, d->num_prompts, spp, max_prefix, kMaxSplits);
    pl->num_prefix_splits = (int)((max_prefix + pl->prefix_split_tokens - 1) / pl->prefix_split_tokens);
    pl->suffix_chunk_tokens = plan_suffix_chunk(d, max_suffix);
    pl->num_suffix_chunks = (int)((max_suffix + pl->suffix_chunk_tokens - 1) / pl->suffix_chunk_tokens);
    const size_t rows = (size_t)d->num_samples * d->num_q_heads;
    const size_t slots = (size_t)pl->num_prefix_splits + pl->num_suffix_chunks;
    pl->acc_bytes = align_up(slots * rows * d->head_dim * sizeof(float), 256);
    pl->ml_bytes = align_up(slots * rows * 2 * sizeof(float), 256);
    return SPD_OK;
}

inline int make_level_plan(const spd_attn_desc* d, int num_levels, const spd_prefix_level* levels, long long max_suffix,
                           LevelPlan* lp)
{
    if (!d || num_levels < 1 || num_levels > SPD_MAX_PREFIX_LEVELS || !levels)
        return SPD_EINVAL;
    Plan pl;
    spd_attn_desc tmp = *d;
    tmp.num_prompts = 1;
    tmp.max_samples_per_prompt = 0;
    const int rc = make_plan(&tmp, 0, max_suffix, &pl);  // validates desc and plans the suffix chunks
    if (rc != SPD_OK)
        return rc;
    lp->suffix_chunk_tokens = pl.suffix_chunk_tokens;
    lp->num_suffix_chunks = pl.num_suffix_chunks;
    const int max_splits = kMaxSplits / num_levels;  // the merge takes kMaxSplits prefix splits in all
    int slots = 0;
    for (int l = 0; l < num_levels; ++l) {
        const spd_prefix_level& L = levels[l];
        if (L.num_groups < 1 || L.max_samples_per_group < 0 || L.max_len < 0 || L.max_len > kMaxLen)
            return SPD_EINVAL;
        const int spp = L.max_samples_per_group > 0 ? L.max_samples_per_group : d->num_samples;
        lp->split_tokens[l] = plan_prefix_split(d, L.num_groups, spp, L.max_len, max_splits);
        lp->num_splits[l] = (int)((L.max_len + lp->split_tokens[l] - 1) / lp->split_tokens[l]);
        lp->slot0[l] = slots;
        slots += lp->num_splits[l];
    }
    lp->num_slots = slots + lp->num_suffix_chunks;
    const size_t rows = (size_t)d->num_samples * d->num_q_heads;
    lp->acc_bytes = align_up((size_t)lp->num_slots * rows * d->head_dim * sizeof(float), 256);
    lp->ml_bytes = align_up((size_t)lp->num_slots * rows * 2 * sizeof(float), 256);
    return SPD_OK;
}

}  // namespace plan
}  // namespace spd
