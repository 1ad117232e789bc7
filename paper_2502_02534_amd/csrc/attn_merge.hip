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

// One block handles kRows rows; D threads per row (D <= 256, blockDim = kRows * Dpad).
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnParams p, int rows_per_block, int dpad)
{
    const int r_in = threadIdx.x / dpad;
    const int d = threadIdx.x % dpad;
    const long long row = (long long)blockIdx.x * rows_per_block + r_in;
    const long long total = (long long)p.N * p.Hq;
    if (r_in >= rows_per_block || row >= total)
        return;
    const int n = (int)(row / p.Hq);
    const int b = prompt_of_sample(p.sample_indptr, p.B, n);
    const int Lp = p.prefix_lens[b], Ls = p.suffix_lens[n];
    const int np = p.prefix_split_tokens > 0 ? (Lp + p.prefix_split_tokens - 1) / p.prefix_split_tokens : 0;
    const int ns = p.suffix_chunk_tokens > 0 ? (Ls + p.suffix_chunk_tokens - 1) / p.suffix_chunk_tokens : 0;

    float m = -INFINITY;
    for (int i = 0; i < np; ++i)
        m = fmaxf(m, p.part_ml[(long long)i * total + row].x);
    for (int i = 0; i < ns; ++i)
        m = fmaxf(m, p.part_ml[(long long)(p.num_prefix_splits + i) * total + row].x);

    float l = 0.f, acc = 0.f;
    const bool active = d < p.D;
    for (int i = 0; i < np + ns; ++i) {
        const long long slot = i < np ? i : p.num_prefix_splits + (i - np);
        const float2 ml = p.part_ml[slot * total + row];
        if (ml.y == 0.f)
            continue;
        const float w = __builtin_amdgcn_exp2f(ml.x - m);
        l = fmaf(ml.y, w, l);
        if (active)
            acc = fmaf(p.part_acc[(slot * total + row) * p.D + d], w, acc);
    }
    const float o = l > 0.f ? acc / l : 0.f;
    if (active) {
        if (p.dtype == 0)
            ((float*)p.out)[row * p.D + d] = o;
        else
            ((uint16_t*)p.out)[row * p.D + d] = f32_to_bf16_rne(o);
    }
    if (p.lse && d == 0)
        p.lse[row] = l > 0.f ? (m + __log2f(l)) * kLn2 : -INFINITY;
}

}  // namespace

hipError_t launch_attn_merge(const AttnParams& p, hipStream_t s)
{
    int dpad = 32;
    while (dpad < p.D)
        dpad <<= 1;
    const int rows_per_block = 256 / dpad;
    const long long total = (long long)p.N * p.Hq;
    const dim3 grid((unsigned)((total + rows_per_block - 1) / rows_per_block));
    hipLaunchKernelGGL(attn_merge_kernel, grid, dim3(256), 0, s, p, rows_per_block, dpad);
    return hipGetLastError();
}

}  // namespace spd
