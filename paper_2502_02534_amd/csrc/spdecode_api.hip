// C ABI of libspdecode: argument validation, launch planning, kernel launches.
#include "../../include/spdecode.h"
#include "spd_internal.h"

#include <math.h>
#include <stdlib.h>

namespace {

using spd::AttnParams;

struct Plan {
    int prefix_split_tokens, num_prefix_splits;
    int suffix_chunk_tokens, num_suffix_chunks;
    size_t acc_bytes, ml_bytes;
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int check_desc(const spd_attn_desc* d)
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
int part_tokens(long long len, int min_tokens, int max_parts, int quantum)
{
    long long t = (len + max_parts - 1) / max_parts;
    if (t < min_tokens)
        t = min_tokens;
    t = (t + quantum - 1) / quantum * quantum;
    return (int)t;
}

int make_plan(const spd_attn_desc* d, long long max_prefix, long long max_suffix, Plan* pl)
{
    const int rc = check_desc(d);
    if (rc != SPD_OK)
        return rc;
    if (max_prefix < 0 || max_suffix < 0 || max_prefix > (1ll << 30) || max_suffix > (1ll << 30))
        return SPD_EINVAL;
    if (d->dtype == SPD_BF16 && d->head_dim == 128) {
        // tiled path: one workgroup per (prompt, KV head, row tile, split); enough splits to
        // occupy every CU once, in multiples of the 64-token tile
        const int spp = d->max_samples_per_prompt > 0 ? d->max_samples_per_prompt : d->num_samples;
        const int rows = spp * (d->num_q_heads / d->num_kv_heads);
        const int block_rows = spd::prefix_mfma_block_rows(rows);
        const long long base = (long long)d->num_prompts * d->num_kv_heads * ((rows + block_rows - 1) / block_rows);
        long long want = (256 + base - 1) / base;
        if (want > 64) want = 64;
        long long t = (max_prefix + want - 1) / want;
        t = (t + 63) / 64 * 64;
        if (t < 64) t = 64;
        pl->prefix_split_tokens = (int)t;
    } else {
        pl->prefix_split_tokens = part_tokens(max_prefix, 256, 64, 64);
    }
#ifdef SPD_TUNING
    if (const char* e = getenv("SPD_TUNE_PREFIX_SPLIT")) pl->prefix_split_tokens = atoi(e);
#endif
    pl->num_prefix_splits = (int)((max_prefix + pl->prefix_split_tokens - 1) / pl->prefix_split_tokens);
    {
        // enough (sample, KV head, chunk) items to keep every CU busy, chunks of 64..320 tokens
        // (measured on ragged suffixes of up to 2048 tokens: 320-token chunks beat 512-token ones
        // by 17 %, finer balance between wavefronts; the merge can take 64 chunks)
        const long long pairs = (long long)d->num_samples * d->num_kv_heads;
        const long long want_chunks = (2048 + pairs - 1) / pairs;
        long long t = (max_suffix + want_chunks - 1) / want_chunks;
        t = (t + 63) / 64 * 64;
        if (t < 64) t = 64;
        if (t > 320) t = 320;
        // Chunks of 128 or 256 tokens start every wavefront of the launch at addresses that agree
        // in many low bits (the rows of a sample are 2 KB apart), which costs 5 to 20 % of the
        // HBM rate; three quarters of the size spreads them.
        if (t == 128 || t == 256) t = t / 4 * 3;
        if (max_suffix > t * 64) t = part_tokens(max_suffix, 64, 64, 64);
#ifdef SPD_TUNING
        if (const char* e = getenv("SPD_TUNE_SUFFIX_CHUNK")) t = atoi(e);
#endif
        pl->suffix_chunk_tokens = (int)t;
    }
    pl->num_suffix_chunks = (int)((max_suffix + pl->suffix_chunk_tokens - 1) / pl->suffix_chunk_tokens);
    const size_t rows = (size_t)d->num_samples * d->num_q_heads;
    const size_t slots = (size_t)pl->num_prefix_splits + pl->num_suffix_chunks;
    pl->acc_bytes = align_up(slots * rows * d->head_dim * sizeof(float), 256);
    pl->ml_bytes = align_up(slots * rows * sizeof(float2), 256);
    return SPD_OK;
}

inline bool misaligned(const void* p, size_t a) { return ((uintptr_t)p % a) != 0; }

}  // namespace

extern "C" {

int append_suffix_kv(const spd_attn_desc* desc, const void* k_new, const void* v_new, void* k_suffix,
                     void* v_suffix, int32_t* suffix_lens, const int32_t* suffix_page_indptr,
                     const int32_t* suffix_page_indices, int64_t max_suffix_len, const int32_t* last_tokens,
                     int32_t end_token, int32_t* finished, void* stream)
{
    if (!desc)
        return SPD_EINVAL;
    const int rc = check_desc(desc);
    if (rc != SPD_OK)
        return rc;
    if (!k_new || !v_new || !k_suffix || !v_suffix || !suffix_lens)
        return SPD_EINVAL;
    if (desc->page_size != 0 && (!suffix_page_indptr || !suffix_page_indices))
        return SPD_EINVAL;
    if (max_suffix_len < 0 || max_suffix_len > (1ll << 30))
        return SPD_EINVAL;
    const int elt = desc->dtype == SPD_BF16 ? 2 : 4;
    if ((desc->head_dim * elt) % 16 != 0)
        return SPD_EUNSUPPORTED;
    spd::KvAppendParams a;
    a.N = desc->num_samples;
    a.Hkv = desc->num_kv_heads;
    a.D = desc->head_dim;
    a.elt = elt;
    a.page_size = desc->page_size;
    a.capacity = (int)max_suffix_len;
    a.k_new = k_new;
    a.v_new = v_new;
    a.k_suffix = k_suffix;
    a.v_suffix = v_suffix;
    a.suffix_lens = suffix_lens;
    a.page_indptr = suffix_page_indptr;
    a.pages = suffix_page_indices;
    a.last_tokens = last_tokens;
    a.end_token = end_token;
    a.finished = finished;
    return spd::launch_kv_append(a, (hipStream_t)stream) == hipSuccess ? SPD_OK : SPD_ELAUNCH;
}

const char* spd_status_string(int status)
{
    switch (status) {
    case SPD_OK: return "ok";
    case SPD_EINVAL: return "invalid argument";
    case SPD_EUNSUPPORTED: return "unsupported dtype, head_dim, page_size or size";
    case SPD_EWORKSPACE: return "workspace missing, misaligned or too small";
    case SPD_ELAUNCH: return "kernel launch failed";
    default: return "unknown status";
    }
}

int spd_attn_plan(const spd_attn_desc* desc, int64_t max_prefix_len, int64_t max_suffix_len,
                  int32_t* prefix_split_tokens, int32_t* num_prefix_splits,
                  int32_t* suffix_chunk_tokens, int32_t* num_suffix_chunks)
{
    Plan pl;
    const int rc = make_plan(desc, max_prefix_len, max_suffix_len, &pl);
    if (rc != SPD_OK)
        return rc;
    if (prefix_split_tokens) *prefix_split_tokens = pl.prefix_split_tokens;
    if (num_prefix_splits) *num_prefix_splits = pl.num_prefix_splits;
    if (suffix_chunk_tokens) *suffix_chunk_tokens = pl.suffix_chunk_tokens;
    if (num_suffix_chunks) *num_suffix_chunks = pl.num_suffix_chunks;
    return SPD_OK;
}

size_t shared_prefix_decode_attn_workspace_size(const spd_attn_desc* desc, int64_t max_prefix_len,
                                                int64_t max_suffix_len)
{
    Plan pl;
    if (make_plan(desc, max_prefix_len, max_suffix_len, &pl) != SPD_OK)
        return 0;
    return pl.acc_bytes + pl.ml_bytes + 256;
}

int shared_prefix_decode_attn(const spd_attn_desc* desc, const void* q, const void* k_prefix,
                              const void* v_prefix, const int32_t* prefix_lens,
                              const int32_t* prefix_indptr, const int32_t* prefix_page_indices,
                              const int32_t* sample_indptr, const void* k_suffix,
                              const void* v_suffix, const int32_t* suffix_lens,
                              const int32_t* suffix_page_indptr, const int32_t* suffix_page_indices,
                              int64_t max_prefix_len, int64_t max_suffix_len, void* out,
                              float* lse_out, void* workspace, size_t workspace_bytes, void* stream)
{
    Plan pl;
    const int rc = make_plan(desc, max_prefix_len, max_suffix_len, &pl);
    if (rc != SPD_OK)
        return rc;
    if (!q || !prefix_lens || !prefix_indptr || !sample_indptr || !suffix_lens || !out)
        return SPD_EINVAL;
    if (max_prefix_len > 0 && (!k_prefix || !v_prefix))
        return SPD_EINVAL;
    if (max_suffix_len > 0 && (!k_suffix || !v_suffix))
        return SPD_EINVAL;
    if (desc->page_size != 0) {
        if (max_prefix_len > 0 && !prefix_page_indices)
            return SPD_EINVAL;
        if (max_suffix_len > 0 && (!suffix_page_indptr || !suffix_page_indices))
            return SPD_EINVAL;
    }
    const void* aligned16[] = {q, k_prefix, v_prefix, k_suffix, v_suffix, out};
    for (const void* ptr : aligned16)
        if (ptr && misaligned(ptr, 16))
            return SPD_EINVAL;
    const size_t need = pl.acc_bytes + pl.ml_bytes + 256;
    if (!workspace || misaligned(workspace, 256) || workspace_bytes < need)
        return SPD_EWORKSPACE;

    AttnParams p;
    p.dtype = desc->dtype;
    p.Hq = desc->num_q_heads;
    p.Hkv = desc->num_kv_heads;
    p.D = desc->head_dim;
    p.G = p.Hq / p.Hkv;
    p.B = desc->num_prompts;
    p.N = desc->num_samples;
    p.max_spp = desc->max_samples_per_prompt > 0 ? desc->max_samples_per_prompt : desc->num_samples;
    p.page_size = desc->page_size;
    const float scale = desc->sm_scale > 0.f ? desc->sm_scale : 1.0f / sqrtf((float)p.D);
    p.scale_log2 = scale * spd::kLog2e;
    p.q = q;
    p.k_prefix = k_prefix;
    p.v_prefix = v_prefix;
    p.prefix_lens = prefix_lens;
    p.prefix_indptr = prefix_indptr;
    p.prefix_pages = prefix_page_indices;
    p.sample_indptr = sample_indptr;
    p.k_suffix = k_suffix;
    p.v_suffix = v_suffix;
    p.suffix_lens = suffix_lens;
    p.suffix_page_indptr = suffix_page_indptr;
    p.suffix_pages = suffix_page_indices;
    p.max_suffix_len = max_suffix_len;
    p.prefix_split_tokens = pl.prefix_split_tokens;
    p.num_prefix_splits = pl.num_prefix_splits;
    p.suffix_chunk_tokens = pl.suffix_chunk_tokens;
    p.num_suffix_chunks = pl.num_suffix_chunks;
    p.num_slots = pl.num_prefix_splits + pl.num_suffix_chunks;
    p.prefix_slot0 = 0;
    p.suffix_slot0 = pl.num_prefix_splits;
    p.num_levels = 1;
    for (int l = 0; l < spd::kMaxLevels; ++l)
        p.mlev[l] = spd::MergeLevel{nullptr, nullptr, 0, 0, 0};
    p.mlev[0] = spd::MergeLevel{sample_indptr, prefix_lens, desc->num_prompts, pl.prefix_split_tokens, 0};
    p.part_acc = workspace;
    p.part_half = desc->dtype == SPD_BF16 ? 1 : 0;
    p.part_ml = (float2*)((char*)workspace + pl.acc_bytes);
    p.out = out;
    p.lse = lse_out;

    const uint32_t stages = desc->stages ? desc->stages
                                         : (SPD_STAGE_PREFIX | SPD_STAGE_SUFFIX | SPD_STAGE_MERGE);
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    const bool suffix_tiled = spd::suffix_mfma_supported(p);
    const bool prefix_tiled = spd::prefix_mfma_supported(p);
    e = spd::launch_attn_plain(p, (stages & SPD_STAGE_PREFIX) && !prefix_tiled,
                               (stages & SPD_STAGE_SUFFIX) && !suffix_tiled, s);
    if (e != hipSuccess)
        return SPD_ELAUNCH;
    const bool both = (stages & SPD_STAGE_PREFIX) && (stages & SPD_STAGE_SUFFIX);
    bool fused = both && spd::attn_fused_supported(p);
#ifdef SPD_TUNING
    if (getenv("SPD_TUNE_NO_FUSED")) fused = false;
#endif
    if (fused) {
        e = spd::launch_attn_fused(p, s);
        if (e != hipSuccess)
            return SPD_ELAUNCH;
    } else {
        if ((stages & SPD_STAGE_PREFIX) && prefix_tiled) {
            e = spd::launch_attn_prefix_mfma(p, s);
            if (e != hipSuccess)
                return SPD_ELAUNCH;
        }
        if ((stages & SPD_STAGE_SUFFIX) && suffix_tiled) {
            e = spd::launch_attn_suffix_mfma(p, s);
            if (e != hipSuccess)
                return SPD_ELAUNCH;
        }
    }
    if (stages & SPD_STAGE_MERGE) {
        e = spd::launch_attn_merge(p, s);
        if (e != hipSuccess)
            return SPD_ELAUNCH;
    }
    return SPD_OK;
}

size_t sample_tokens_workspace_size(int64_t rows, int64_t vocab)
{
    if (rows <= 0 || vocab <= 0)
        return 0;
    return spd::sampler_workspace_bytes(rows, vocab);
}

int sample_tokens(const void* logits, int32_t logits_dtype, int64_t rows, int64_t vocab,
                  int64_t row_stride, const float* temperature, const float* top_p,
                  const float* uniforms, int32_t* tokens_out, void* workspace,
                  size_t workspace_bytes, void* stream)
{
    if (!logits || !temperature || !top_p || !uniforms || !tokens_out)
        return SPD_EINVAL;
    if (rows <= 0 || vocab <= 0 || row_stride < vocab || rows > 0x7fffffffll)
        return SPD_EINVAL;
    if (logits_dtype != SPD_F32)
        return SPD_EUNSUPPORTED;
    if (vocab > 262144)
        return SPD_EUNSUPPORTED;
    if (misaligned(logits, 4))
        return SPD_EINVAL;
    if (!workspace || misaligned(workspace, 256) || workspace_bytes < sample_tokens_workspace_size(rows, vocab))
        return SPD_EWORKSPACE;
    spd::SamplerParams p;
    p.logits = (const float*)logits;
    p.rows = rows;
    p.vocab = vocab;
    p.stride = row_stride;
    p.temperature = temperature;
    p.top_p = top_p;
    p.uniforms = uniforms;
    p.tokens = tokens_out;
    if (spd::launch_sampler(p, workspace, (hipStream_t)stream) != hipSuccess)
        return SPD_ELAUNCH;
    return SPD_OK;
}

}  // extern "C"
