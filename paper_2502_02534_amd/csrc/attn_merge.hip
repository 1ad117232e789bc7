// Log-sum-exp merge of partial softmax states (prefix splits and suffix chunks) into
// the normalised attention output.  With states (m_i, l_i, acc_i):
//   m = max m_i,  l = sum l_i 2^(m_i - m),  out = sum acc_i 2^(m_i - m) / l,
//   lse = (m + log2 l) ln 2.
// This is the rescaling step of the paper's online-softmax recurrence (App., attn
// task 2: `ExpMaxDiff`, `WeightedSumSingle`, `WeightedSumDouble`, `Div`) applied to
// blocks instead of single tokens.  Empty ranges are skipped, so the initial state
// (-inf, 0, 0) is the identity.
#include "spd_internal.h"

namespace spd {
namespace {

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x40);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

constexpr int kMergeThreads = 256;
constexpr int kMaxSlots = 128;   // prefix splits + suffix chunks (each at most 64)

// One workgroup merges kMergeThreads / (D/4) rows; a thread owns 4 channels of one row.
// Step 1 puts every valid partial's (m, l) in LDS, step 2 turns them into weights
// 2^(m_i - m) (0 for empty partials) and the row's m and l, step 3 combines the accumulators,
// whose loads (up to 32 independent 16-byte loads per thread) were issued before step 1.
__global__ __launch_bounds__(kMergeThreads) void attn_merge_kernel(AttnParams p, int tpr /* threads per row */)
{
    __shared__ float2 ml[kMergeThreads / 8][kMaxSlots];   // at most 32 rows per block (D = 32)
    __shared__ float wgt[kMergeThreads / 8][kMaxSlots];
    __shared__ float row_m[kMergeThreads / 8], row_l[kMergeThreads / 8];

    const int rows_per_block = kMergeThreads / tpr;
    const int r_in = threadIdx.x / tpr;
    const int c = threadIdx.x % tpr;  // channel group
    const long long total = (long long)p.N * p.Hq;
    const long long row = (long long)blockIdx.x * rows_per_block + r_in;
    const bool row_ok = row < total;

    int np = 0, ns = 0;
    if (row_ok) {
        const int n = (int)(row / p.Hq);
        const int b = prompt_of_sample(p.sample_indptr, p.B, n);
        const int Lp = p.prefix_lens[b], Ls = p.suffix_lens[n];
        np = p.prefix_split_tokens > 0 ? (Lp + p.prefix_split_tokens - 1) / p.prefix_split_tokens : 0;
        ns = p.suffix_chunk_tokens > 0 ? (Ls + p.suffix_chunk_tokens - 1) / p.suffix_chunk_tokens : 0;
    }
    const int cnt = np + ns;
    const bool ch_ok = row_ok && 4 * c < p.D;
    const float* base = p.part_acc + part_index(p, row_ok ? row : 0, 0) * p.D + 4 * c;
    auto slot_at = [&](int i) { return i < np ? i : p.num_prefix_splits + (i - np); };
    // The first batch of accumulator loads does not need the weights: it is issued together
    // with the (m, l) loads so that both round trips overlap.
    constexpr int kBatch = 32;
    float4 v[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
        v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ch_ok && u < cnt)
            v[u] = *reinterpret_cast<const float4*>(base + (long long)slot_at(u) * p.D);
    }
    for (int i = c; i < cnt; i += tpr)
        ml[r_in][i] = p.part_ml[part_index(p, row, slot_at(i))];
    __syncthreads();
    if (c == 0) {
        float m = -INFINITY;
        for (int i = 0; i < cnt; ++i)
            m = fmaxf(m, ml[r_in][i].x);
        float l = 0.f;
        for (int i = 0; i < cnt; ++i) {
            const float2 mv = ml[r_in][i];
            const float w = mv.y > 0.f ? __builtin_amdgcn_exp2f(mv.x - m) : 0.f;
            wgt[r_in][i] = w;
            l = fmaf(mv.y, w, l);
        }
        row_m[r_in] = m;
        row_l[r_in] = l;
    }
    __syncthreads();
    if (!ch_ok)
        return;
    const float l = row_l[r_in];
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i0 = 0; i0 < cnt; i0 += kBatch) {
        if (i0 > 0) {
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (i0 + u < cnt)
                    v[u] = *reinterpret_cast<const float4*>(base + (long long)slot_at(i0 + u) * p.D);
            }
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const float w = i0 + u < cnt ? wgt[r_in][i0 + u] : 0.f;
            acc.x = fmaf(v[u].x, w, acc.x);
            acc.y = fmaf(v[u].y, w, acc.y);
            acc.z = fmaf(v[u].z, w, acc.z);
            acc.w = fmaf(v[u].w, w, acc.w);
        }
    }
    const float inv = l > 0.f ? 1.f / l : 0.f;
    acc.x *= inv;
    acc.y *= inv;
    acc.z *= inv;
    acc.w *= inv;
    if (p.dtype == 0) {
        *reinterpret_cast<float4*>((float*)p.out + row * p.D + 4 * c) = acc;
    } else {
        uint2 o;
        o.x = (uint32_t)f32_to_bf16_rne(acc.x) | ((uint32_t)f32_to_bf16_rne(acc.y) << 16);
        o.y = (uint32_t)f32_to_bf16_rne(acc.z) | ((uint32_t)f32_to_bf16_rne(acc.w) << 16);
        *reinterpret_cast<uint2*>((uint16_t*)p.out + row * p.D + 4 * c) = o;
    }
    if (p.lse && c == 0)
        p.lse[row] = l > 0.f ? (row_m[r_in] + __log2f(l)) * kLn2 : -INFINITY;
}

}  // namespace

hipError_t launch_attn_merge(const AttnParams& p, hipStream_t s)
{
    // threads per row: the power of two >= max(8, D/4); lanes past D/4 idle
    int use = 8;
    while (use * 4 < p.D)
        use <<= 1;
    const int rows_per_block = kMergeThreads / use;
    const long long total = (long long)p.N * p.Hq;
    const dim3 grid((unsigned)((total + rows_per_block - 1) / rows_per_block));
    hipLaunchKernelGGL(attn_merge_kernel, grid, dim3(kMergeThreads), 0, s, p, use);
    return hipGetLastError();
}

}  // namespace spd
