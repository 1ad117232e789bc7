// C ABI of libspdecode: argument validation, launch planning, kernel launches.
#include "../../include/spdecode.h"
#include "spd_internal.h"
#include "plan.h"

#include <math.h>
#include <stdlib.h>

#include <mutex>

// Scratch memory of sample_tokens_static: one copy per GPU, held until the process ends.  In host
// code this name only stands for the symbol; the memory is reached through the address that
// hipGetSymbolAddress returns on each device (static_scratch below).
static __device__ __align__(256) unsigned char scratch[SPD_STATIC_SCRATCH_BYTES];

namespace {

using spd::AttnParams;
using namespace spd::plan;

inline bool misaligned(const void* p, size_t a) { return ((uintptr_t)p % a) != 0; }

// Address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return SPD_ELAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr)
            return SPD_ELAUNCH;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SPD_OK;
}

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

static int step_rows(int64_t* step_state, int64_t num_steps, int32_t count, const spd_row_copy* copies,
                     bool record, void* stream)
{
    static_assert(SPD_MAX_STEP_COPIES == spd::kMaxStepCopies, "header and kernel agree on the number of copies");
    if (!step_state || misaligned(step_state, 8) || num_steps < 1 || count < 1 || count > SPD_MAX_STEP_COPIES || !copies)
        return SPD_EINVAL;
    spd::StepRowsParams a;
    a.state = (long long*)step_state;
    a.num_steps = num_steps;
    a.count = count;
    long long blocks = 0;
    for (int i = 0; i < spd::kMaxStepCopies; ++i) {
        a.first_block[i] = (int)blocks;
        a.src[i] = nullptr;
        a.dst[i] = nullptr;
        a.row_bytes[i] = 0;
        a.wide[i] = 0;
        if (i >= count)
            continue;
        const spd_row_copy& c = copies[i];
        if (!c.src || !c.dst || c.row_bytes <= 0 || c.row_bytes % 4 != 0 || misaligned(c.src, 4) || misaligned(c.dst, 4))
            return SPD_EINVAL;
        a.src[i] = c.src;
        a.dst[i] = c.dst;
        a.row_bytes[i] = c.row_bytes;
        a.wide[i] = (c.row_bytes % 16 == 0 && !misaligned(c.src, 16) && !misaligned(c.dst, 16)) ? 1 : 0;
        blocks += spd::step_rows_blocks(c.row_bytes);
        if (blocks > 0x7fffffffLL)
            return SPD_EUNSUPPORTED;
    }
    a.first_block[spd::kMaxStepCopies] = (int)blocks;
    for (int i = count; i < spd::kMaxStepCopies; ++i)
        a.first_block[i] = (int)blocks;
    return spd::launch_step_rows(a, record, (hipStream_t)stream) == hipSuccess ? SPD_OK : SPD_ELAUNCH;
}

int decode_step_select(int64_t* step_state, int64_t num_steps, int32_t count, const spd_row_copy* copies, void* stream)
{
    return step_rows(step_state, num_steps, count, copies, false, stream);
}

int decode_step_record(int64_t* step_state, int64_t num_steps, int32_t count, const spd_row_copy* copies, void* stream)
{
    return step_rows(step_state, num_steps, count, copies, true, stream);
}

int decode_step_advance(int64_t* step_state, int64_t num_steps, int32_t record_count, const spd_row_copy* record,
                        int32_t select_count, const spd_row_copy* select, const spd_attn_desc* desc,
                        const void* k_steps, const void* v_steps, void* k_suffix, void* v_suffix, int32_t* suffix_lens,
                        const int32_t* suffix_page_indptr, const int32_t* suffix_page_indices, int64_t max_suffix_len,
                        const int32_t* last_tokens, int32_t end_token, int32_t* finished, int32_t* lens_record,
                        void* stream)
{
    static_assert(2 * SPD_MAX_STEP_COPIES == spd::kMaxAdvanceCopies, "header and kernel agree on the number of copies");
    if (!step_state || misaligned(step_state, 8) || num_steps < 1 || record_count < 0 ||
        record_count > SPD_MAX_STEP_COPIES || select_count < 0 || select_count > SPD_MAX_STEP_COPIES ||
        (record_count > 0 && !record) || (select_count > 0 && !select))
        return SPD_EINVAL;
    if (!desc)
        return SPD_EINVAL;
    const int rc = check_desc(desc);
    if (rc != SPD_OK)
        return rc;
    if (!k_steps || !v_steps || !k_suffix || !v_suffix || !suffix_lens)
        return SPD_EINVAL;
    if (desc->page_size != 0 && (!suffix_page_indptr || !suffix_page_indices))
        return SPD_EINVAL;
    if (max_suffix_len < 0 || max_suffix_len > (1ll << 30))
        return SPD_EINVAL;
    const int elt = desc->dtype == SPD_BF16 ? 2 : 4;
    if ((desc->head_dim * elt) % 16 != 0)
        return SPD_EUNSUPPORTED;
    if (misaligned(k_steps, 16) || misaligned(v_steps, 16) || misaligned(k_suffix, 16) || misaligned(v_suffix, 16))
        return SPD_EINVAL;
    spd::StepAdvanceParams a;
    a.state = (long long*)step_state;
    a.num_steps = num_steps;
    a.count = record_count + select_count;
    long long blocks = 0;
    for (int i = 0; i < spd::kMaxAdvanceCopies; ++i) {
        a.first_block[i] = (int)blocks;
        a.src[i] = nullptr;
        a.dst[i] = nullptr;
        a.row_bytes[i] = 0;
        a.wide[i] = 0;
        a.record[i] = 0;
        if (i >= a.count)
            continue;
        const bool is_record = i < record_count;
        const spd_row_copy& c = is_record ? record[i] : select[i - record_count];
        if (!c.src || !c.dst || c.row_bytes <= 0 || c.row_bytes % 4 != 0 || misaligned(c.src, 4) || misaligned(c.dst, 4))
            return SPD_EINVAL;
        a.src[i] = c.src;
        a.dst[i] = c.dst;
        a.row_bytes[i] = c.row_bytes;
        a.wide[i] = (c.row_bytes % 16 == 0 && !misaligned(c.src, 16) && !misaligned(c.dst, 16)) ? 1 : 0;
        a.record[i] = is_record ? 1 : 0;
        blocks += spd::step_rows_blocks(c.row_bytes);
        if (blocks > 0x3fffffffLL)
            return SPD_EUNSUPPORTED;
    }
    a.first_block[spd::kMaxAdvanceCopies] = (int)blocks;
    a.kv.N = desc->num_samples;
    a.kv.Hkv = desc->num_kv_heads;
    a.kv.D = desc->head_dim;
    a.kv.elt = elt;
    a.kv.page_size = desc->page_size;
    a.kv.capacity = (int)max_suffix_len;
    a.kv.k_new = k_steps;
    a.kv.v_new = v_steps;
    a.kv.k_suffix = k_suffix;
    a.kv.v_suffix = v_suffix;
    a.kv.suffix_lens = suffix_lens;
    a.kv.page_indptr = suffix_page_indptr;
    a.kv.pages = suffix_page_indices;
    a.kv.last_tokens = last_tokens;
    a.kv.end_token = end_token;
    a.kv.finished = finished;
    a.lens_record = lens_record;
    if (blocks + a.kv.N > 0x7fffffffLL)
        return SPD_EUNSUPPORTED;
    return spd::launch_step_advance(a, (hipStream_t)stream) == hipSuccess ? SPD_OK : SPD_ELAUNCH;
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

}  // extern "C"

namespace {

// The attention call proper: any number of prefix levels.  `stages` as in spd_attn_desc.
int run_attention(const spd_attn_desc* desc, const void* q, int num_levels, const spd_prefix_level* levels,
                  const LevelPlan& lp, const void* k_suffix, const void* v_suffix, const int32_t* suffix_lens,
                  const int32_t* suffix_page_indptr, const int32_t* suffix_page_indices, int64_t max_suffix_len,
                  void* out, float* lse_out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!q || !suffix_lens || !out)
        return SPD_EINVAL;
    if (max_suffix_len > 0 && (!k_suffix || !v_suffix))
        return SPD_EINVAL;
    if (desc->page_size != 0 && max_suffix_len > 0 && (!suffix_page_indptr || !suffix_page_indices))
        return SPD_EINVAL;
    const void* aligned16[] = {q, k_suffix, v_suffix, out};
    for (const void* ptr : aligned16)
        if (ptr && misaligned(ptr, 16))
            return SPD_EINVAL;
    for (int l = 0; l < num_levels; ++l) {
        const spd_prefix_level& L = levels[l];
        if (!L.lens || !L.indptr || !L.sample_indptr)
            return SPD_EINVAL;
        if (L.max_len > 0 && (!L.k || !L.v || misaligned(L.k, 16) || misaligned(L.v, 16)))
            return SPD_EINVAL;
        if (desc->page_size != 0 && L.max_len > 0 && !L.page_indices)
            return SPD_EINVAL;
    }
    const size_t need = lp.acc_bytes + lp.ml_bytes + 256;
    if (!workspace || misaligned(workspace, 256) || workspace_bytes < need)
        return SPD_EWORKSPACE;

    AttnParams p;
    p.dtype = desc->dtype;
    p.Hq = desc->num_q_heads;
    p.Hkv = desc->num_kv_heads;
    p.D = desc->head_dim;
    p.G = p.Hq / p.Hkv;
    p.N = desc->num_samples;
    p.page_size = desc->page_size;
    const float scale = desc->sm_scale > 0.f ? desc->sm_scale : 1.0f / sqrtf((float)p.D);
    p.scale_log2 = scale * spd::kLog2e;
    p.q = q;
    p.k_suffix = k_suffix;
    p.v_suffix = v_suffix;
    p.suffix_lens = suffix_lens;
    p.suffix_page_indptr = suffix_page_indptr;
    p.suffix_pages = suffix_page_indices;
    p.max_suffix_len = max_suffix_len;
    p.suffix_chunk_tokens = lp.suffix_chunk_tokens;
    p.num_suffix_chunks = lp.num_suffix_chunks;
    p.num_slots = lp.num_slots;
    p.suffix_slot0 = lp.num_slots - lp.num_suffix_chunks;
    p.num_levels = num_levels;
    p.part_acc = workspace;
    p.part_half = desc->dtype == SPD_BF16 ? 1 : 0;
    p.part_ml = (float2*)((char*)workspace + lp.acc_bytes);
    p.out = out;
    p.lse = lse_out;

    const uint32_t stages = desc->stages ? desc->stages
                                         : (SPD_STAGE_PREFIX | SPD_STAGE_SUFFIX | SPD_STAGE_MERGE);
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    // Several levels, bf16 tiles everywhere: all prefix levels and the suffix pass in one launch.
    if (num_levels > 1 && stages == (SPD_STAGE_PREFIX | SPD_STAGE_SUFFIX | SPD_STAGE_MERGE)) {
        spd::FusedLevels fl;
        fl.num_levels = 0;
        long long blocks = 0;
        fl.first_block[0] = 0;
        for (int l = 0; l < num_levels; ++l) {
            if (lp.num_splits[l] <= 0)
                continue;  // an empty level has nothing to compute
            const spd_prefix_level& L = levels[l];
            spd::PrefixLevelParams& lv = fl.level[fl.num_levels];
            const int spp = L.max_samples_per_group > 0 ? L.max_samples_per_group : desc->num_samples;
            lv.k = L.k;
            lv.v = L.v;
            lv.lens = L.lens;
            lv.indptr = L.indptr;
            lv.pages = L.page_indices;
            lv.sample_indptr = L.sample_indptr;
            lv.split_tokens = lp.split_tokens[l];
            lv.num_splits = lp.num_splits[l];
            lv.slot0 = lp.slot0[l];
            lv.rowtiles = (spp * p.G + 127) / 128;
            lv.groups = L.num_groups;
            blocks += (long long)lv.num_splits * lv.rowtiles * lv.groups * p.Hkv;
            fl.first_block[++fl.num_levels] = (int)blocks;
        }
        for (int l = fl.num_levels + 1; l <= spd::kMaxLevels; ++l)
            fl.first_block[l] = (int)blocks;
        const bool one_launch = fl.num_levels >= 1 && blocks < 0x7fffffffLL && spd::attn_fused_levels_supported(p, fl);
        if (one_launch) {
            if (spd::launch_attn_fused_levels(p, fl, s) != hipSuccess)
                return SPD_ELAUNCH;
            if (spd::launch_attn_merge(p, s) != hipSuccess)
                return SPD_ELAUNCH;
            return SPD_OK;
        }
    }
    // Otherwise every level is one prefix pass over its own grouping of the samples.  The level with the most
    // tokens shares its launch with the suffix pass (where the fused kernel takes the shape), so
    // that the suffix stream overlaps with as much matrix work as possible; it is launched last.
    int with_suffix = 0;
    for (int l = 1; l < num_levels; ++l)
        if (levels[l].max_len > levels[with_suffix].max_len)
            with_suffix = l;
    for (int step = 0; step < num_levels; ++step) {
        // order: every other level first, then the one that carries the suffix pass
        const int l = step == num_levels - 1 ? with_suffix : (step < with_suffix ? step : step + 1);
        const spd_prefix_level& L = levels[l];
        p.k_prefix = L.k;
        p.v_prefix = L.v;
        p.prefix_lens = L.lens;
        p.prefix_indptr = L.indptr;
        p.prefix_pages = L.page_indices;
        p.sample_indptr = L.sample_indptr;
        p.B = L.num_groups;
        p.max_spp = L.max_samples_per_group > 0 ? L.max_samples_per_group : desc->num_samples;
        p.prefix_split_tokens = lp.split_tokens[l];
        p.num_prefix_splits = lp.num_splits[l];
        p.prefix_slot0 = lp.slot0[l];
        const bool last = l == with_suffix;
        const bool want_prefix = (stages & SPD_STAGE_PREFIX) != 0;
        const bool want_suffix = last && (stages & SPD_STAGE_SUFFIX) != 0;
        const bool suffix_tiled = spd::suffix_mfma_supported(p);
        const bool prefix_tiled = spd::prefix_mfma_supported(p);
        e = spd::launch_attn_plain(p, want_prefix && !prefix_tiled, want_suffix && !suffix_tiled, s);
        if (e != hipSuccess)
            return SPD_ELAUNCH;
        const bool fused = want_prefix && want_suffix && spd::attn_fused_supported(p);
        if (fused) {
            e = spd::launch_attn_fused(p, s);
            if (e != hipSuccess)
                return SPD_ELAUNCH;
        } else {
            if (want_prefix && prefix_tiled) {
                e = spd::launch_attn_prefix_mfma(p, s);
                if (e != hipSuccess)
                    return SPD_ELAUNCH;
            }
            if (want_suffix && suffix_tiled) {
                e = spd::launch_attn_suffix_mfma(p, s);
                if (e != hipSuccess)
                    return SPD_ELAUNCH;
            }
        }
    }
    if (stages & SPD_STAGE_MERGE) {
        e = spd::launch_attn_merge(p, s);
        if (e != hipSuccess)
            return SPD_ELAUNCH;
    }
    return SPD_OK;
}

}  // namespace

extern "C" {

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
    // one level of shared prefixes, planned exactly as spd_attn_plan reports it
    spd_prefix_level level;
    level.k = k_prefix;
    level.v = v_prefix;
    level.lens = prefix_lens;
    level.indptr = prefix_indptr;
    level.page_indices = prefix_page_indices;
    level.sample_indptr = sample_indptr;
    level.num_groups = desc->num_prompts;
    level.max_samples_per_group = desc->max_samples_per_prompt;
    level.max_len = max_prefix_len;
    LevelPlan lp;
    lp.split_tokens[0] = pl.prefix_split_tokens;
    lp.num_splits[0] = pl.num_prefix_splits;
    lp.slot0[0] = 0;
    lp.suffix_chunk_tokens = pl.suffix_chunk_tokens;
    lp.num_suffix_chunks = pl.num_suffix_chunks;
    lp.num_slots = pl.num_prefix_splits + pl.num_suffix_chunks;
    lp.acc_bytes = pl.acc_bytes;
    lp.ml_bytes = pl.ml_bytes;
    return run_attention(desc, q, 1, &level, lp, k_suffix, v_suffix, suffix_lens, suffix_page_indptr,
                         suffix_page_indices, max_suffix_len, out, lse_out, workspace, workspace_bytes, stream);
}

size_t shared_prefix_decode_attn_levels_workspace_size(const spd_attn_desc* desc, int32_t num_levels,
                                                       const spd_prefix_level* levels, int64_t max_suffix_len)
{
    LevelPlan lp;
    if (!desc || make_level_plan(desc, num_levels, levels, max_suffix_len, &lp) != SPD_OK)
        return 0;
    return lp.acc_bytes + lp.ml_bytes + 256;
}

int shared_prefix_decode_attn_levels(const spd_attn_desc* desc, const void* q, int32_t num_levels,
                                     const spd_prefix_level* levels, const void* k_suffix, const void* v_suffix,
                                     const int32_t* suffix_lens, const int32_t* suffix_page_indptr,
                                     const int32_t* suffix_page_indices, int64_t max_suffix_len, void* out,
                                     float* lse_out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!desc)
        return SPD_EINVAL;
    if (desc->stages != 0)
        return SPD_EINVAL;
    LevelPlan lp;
    const int rc = make_level_plan(desc, num_levels, levels, max_suffix_len, &lp);
    if (rc != SPD_OK)
        return rc;
    return run_attention(desc, q, num_levels, levels, lp, k_suffix, v_suffix, suffix_lens, suffix_page_indptr,
                         suffix_page_indices, max_suffix_len, out, lse_out, workspace, workspace_bytes, stream);
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
    return sample_tokens_filtered(logits, logits_dtype, rows, vocab, row_stride, temperature, top_p, nullptr,
                                  nullptr, uniforms, tokens_out, workspace, workspace_bytes, stream);
}

int sample_tokens_static(const void* logits, int32_t logits_dtype, int64_t rows, int64_t vocab,
                         int64_t row_stride, const float* temperature, const float* top_p,
                         const float* uniforms, int32_t* tokens_out, void* stream)
{
    if (rows <= 0 || vocab <= 0)
        return SPD_EINVAL;
    if (sample_tokens_workspace_size(rows, vocab) > (size_t)SPD_STATIC_SCRATCH_BYTES)
        return SPD_EWORKSPACE;  // more rows (or a larger vocabulary) than the library's own scratch holds
    void* ptr = nullptr;
    const int rc = static_scratch(&ptr);
    if (rc != SPD_OK)
        return rc;
    return sample_tokens_filtered(logits, logits_dtype, rows, vocab, row_stride, temperature, top_p, nullptr,
                                  nullptr, uniforms, tokens_out, ptr, (size_t)SPD_STATIC_SCRATCH_BYTES, stream);
}

int sample_tokens_filtered(const void* logits, int32_t logits_dtype, int64_t rows, int64_t vocab,
                           int64_t row_stride, const float* temperature, const float* top_p,
                           const int32_t* top_k, const float* min_p, const float* uniforms,
                           int32_t* tokens_out, void* workspace, size_t workspace_bytes, void* stream)
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
    p.top_k = top_k;
    p.min_p = min_p;
    if (spd::launch_sampler(p, workspace, (hipStream_t)stream) != hipSuccess)
        return SPD_ELAUNCH;
    return SPD_OK;
}

}  // extern "C"
