// Internal declarations shared by the HIP translation units of libspdecode.
// Host-side launch wrappers take a filled AttnParams / SamplerParams; they do no
// allocation and no synchronisation.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spd {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Partial softmax state of one (sample, query head) over a token range: running maximum m (in
// base-2 units of the scaled score), sum l of 2^(s - m), and the range's own normalised output
// sum 2^(s - m) v / l.  Inside a kernel the state is the deferred-division form of the paper's
// online-softmax recurrence (App., attn task 2); the division by l happens once, when the state
// is stored, which lets the bf16 path keep the stored output in fp16 (11 significant bits, three
// more than the bf16 result it is merged into) at half the traffic.  An empty range has l == 0;
// the pass that owns a slot always stores its (m, l), so the merge needs no sequence lengths.
constexpr int kMaxLevels = 4;

// One level of shared prefixes as the prefix pass sees it.
struct PrefixLevelParams {
    const void* k;
    const void* v;
    const int* lens;
    const int* indptr;
    const int* pages;
    const int* sample_indptr;
    int split_tokens;  // tokens per split
    int num_splits;
    int slot0;         // first partial-state slot of the level
    int rowtiles;      // row tiles per (group, KV head) in the launch that carries the level
    int groups;        // number of groups
};

// The levels a fused launch carries, with the range of prefix workgroups of each.
struct FusedLevels {
    int num_levels;
    int first_block[kMaxLevels + 1];  // prefix workgroups of level l: first_block[l] .. first_block[l+1]-1
    PrefixLevelParams level[kMaxLevels];
};

struct AttnParams {
    int dtype, Hq, Hkv, D, G, B, N, max_spp, page_size;
    float scale_log2;  // sm_scale * log2(e)
    const void* q;
    const void* k_prefix;
    const void* v_prefix;
    const int* prefix_lens;
    const int* prefix_indptr;
    const int* prefix_pages;
    const int* sample_indptr;
    const void* k_suffix;
    const void* v_suffix;
    const int* suffix_lens;
    const int* suffix_page_indptr;
    const int* suffix_pages;
    long long max_suffix_len;
    int prefix_split_tokens, num_prefix_splits;
    int suffix_chunk_tokens, num_suffix_chunks;
    int num_slots;    // prefix splits (of every level) + suffix chunks
    int prefix_slot0; // first slot of the prefix level the prefix fields describe
    int suffix_slot0; // first slot of the suffix chunks
    int num_levels;   // levels of shared prefixes (1 for the plain shared-prefix call)
    void* part_acc;   // [N*Hq][slots][D] normalised partial outputs, fp16 if part_half else fp32;
                      // a row's partial states are contiguous for the merge
    int part_half;
    float2* part_ml;  // [N*Hq][slots]  (m, l)
    void* out;
    float* lse;
};

// Row copies of one decode step (select: out of [steps, ...] tensors; record: into them).
constexpr int kMaxStepCopies = 8;
struct StepRowsParams {
    long long* state;      // {current step, next step}
    long long num_steps;
    int count;
    int first_block[kMaxStepCopies + 1];  // workgroups of copy i: first_block[i] .. first_block[i+1]-1
    const void* src[kMaxStepCopies];
    void* dst[kMaxStepCopies];
    long long row_bytes[kMaxStepCopies];
    int wide[kMaxStepCopies];  // 16-byte pieces (else 4-byte)
};

struct KvAppendParams {
    int N, Hkv, D, elt, page_size;
    int capacity;             // tokens a sample's slot (or page list) can hold
    const void* k_new;        // [N, Hkv, D]
    const void* v_new;
    void* k_suffix;
    void* v_suffix;
    int* suffix_lens;
    const int* page_indptr;
    const int* pages;
    const int* last_tokens;   // may be null
    int end_token;
    int* finished;            // may be null
};

// Everything between two decode steps in one launch: up to 2 * kMaxStepCopies row copies (each
// either a record of the previous step's results or a selection of this step's inputs) and the
// append, whose k_new / v_new point at [num_steps, N, Hkv, D] arrays.
constexpr int kMaxAdvanceCopies = 2 * kMaxStepCopies;
struct StepAdvanceParams {
    long long* state;      // {current step, next step, arrivals}
    long long num_steps;
    int count;
    int first_block[kMaxAdvanceCopies + 1];  // the last entry is the number of copy workgroups
    const void* src[kMaxAdvanceCopies];
    void* dst[kMaxAdvanceCopies];
    long long row_bytes[kMaxAdvanceCopies];
    int wide[kMaxAdvanceCopies];
    int record[kMaxAdvanceCopies];           // 1: into row current - 1 of dst; 0: out of row current of src
    KvAppendParams kv;
    int* lens_record;      // [num_steps, N] or null
};

struct SamplerParams {
    const float* logits;
    long long rows, vocab, stride;
    const float* temperature;
    const float* top_p;
    const float* uniforms;
    int* tokens;
    const int* top_k;    // per row, 0 = off; may be null
    const float* min_p;  // per row, 0 = off; may be null
};

// Index of the partial state of output row `row` (= n * Hq + h) in slot `slot`.
__device__ __forceinline__ long long part_index(const AttnParams& p, long long row, int slot)
{
    return row * p.num_slots + slot;
}

// Prompt that owns sample n (sample_indptr is sorted, B >= 1).
__device__ __forceinline__ int prompt_of_sample(const int* __restrict__ indptr, int B, int n)
{
    int lo = 0, hi = B - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (indptr[mid] <= n)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

// Element offset of (token t, KV head j, channel 0) inside a KV tensor.
//   contiguous: [token][Hkv][D], sequence starts at token `start`
//   paged:      [page][Hkv][page_size][D], `pages` lists the sequence's pages
__device__ __forceinline__ long long kv_row_offset(int t, int j, int Hkv, int D, int page_size,
                                                   long long start, const int* __restrict__ pages)
{
    if (page_size == 0)
        return ((start + t) * Hkv + j) * (long long)D;
    const long long pg = pages[t / page_size];
    return ((pg * Hkv + j) * page_size + (t % page_size)) * (long long)D;
}

hipError_t launch_attn_plain(const AttnParams& p, bool prefix, bool suffix, hipStream_t s);
bool prefix_mfma_supported(const AttnParams& p);
int prefix_mfma_block_rows(int rows);
hipError_t launch_attn_prefix_mfma(const AttnParams& p, hipStream_t s);
bool suffix_mfma_supported(const AttnParams& p);
hipError_t launch_attn_suffix_mfma(const AttnParams& p, hipStream_t s);
bool attn_fused_supported(const AttnParams& p);
hipError_t launch_attn_fused(const AttnParams& p, hipStream_t s);
bool attn_fused_levels_supported(const AttnParams& p, const FusedLevels& fl);
hipError_t launch_attn_fused_levels(const AttnParams& p, const FusedLevels& fl, hipStream_t s);
hipError_t launch_attn_merge(const AttnParams& p, hipStream_t s);
hipError_t launch_kv_append(const KvAppendParams& a, hipStream_t s);
long long step_rows_blocks(long long row_bytes);
hipError_t launch_step_rows(const StepRowsParams& a, bool record, hipStream_t s);
hipError_t launch_step_advance(const StepAdvanceParams& a, hipStream_t s);
size_t sampler_workspace_bytes(long long rows, long long vocab);
hipError_t launch_sampler(const SamplerParams& p, void* workspace, hipStream_t s);

}  // namespace spd
