// Log-sum-exp merge of partial softmax states (prefix splits and suffix chunks) into
// the normalised attention output.  With states (m_i, l_i, out_i = acc_i / l_i):
//   m = max m_i,  w_i = l_i 2^(m_i - m),  l = sum w_i,  out = sum w_i out_i / l,
//   lse = (m + log2 l) ln 2.
// This is the rescaling step of the paper's online-softmax recurrence (App., attn
// task 2: `ExpMaxDiff`, `WeightedSumSingle`, `WeightedSumDouble`, `Div`) applied to
// blocks instead of single tokens.  Empty ranges carry l = 0 and weight 0, so the initial state
// (-inf, 0, 0) is the identity.
#include "spd_internal.h"

#include <hip/hip_fp16.h>

#include <type_traits>

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
// The threads of a row share out the (m, l) pairs, find the row's m and l with shuffles and
// leave the weights l_i 2^(m_i - m) (0 for empty partials) in LDS; then every thread combines
// the partial outputs, whose loads (up to 32 independent loads per thread) were issued first.
// HALF: the partial outputs are fp16 (8 bytes per thread and partial) instead of fp32 (16).
template <bool HALF> struct PartVec;
template <> struct PartVec<false> {
    typedef float4 type;
    static __device__ __forceinline__ float4 zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    static __device__ __forceinline__ float4 widen(float4 v) { return v; }
};
template <> struct PartVec<true> {
    typedef uint2 type;
    static __device__ __forceinline__ uint2 zero() { return make_uint2(0u, 0u); }
    static __device__ __forceinline__ float4 widen(uint2 v)
    {
        const float2 a = __half22float2(*reinterpret_cast<const __half2*>(&v.x));
        const float2 b = __half22float2(*reinterpret_cast<const __half2*>(&v.y));
        return make_float4(a.x, a.y, b.x, b.y);
    }
};

// BATCH: output parts a thread loads at a time (8 when the row has at most 8 slots, else 32).
// PERLANE: (m, l) pairs a thread may have to take (kMaxSlots / tpr, rounded up).  Both only size
// register arrays: the smaller the arrays, the more workgroups a CU holds.
template <bool HALF, int BATCH, int PERLANE>
__global__ __launch_bounds__(kMergeThreads) void attn_merge_kernel(AttnParams p, int tpr /* threads per row */)
{
    typedef typename PartVec<HALF>::type vec_t;
    typedef typename std::conditional<HALF, __half, float>::type elem_t;
    __shared__ float wgt[kMergeThreads / 8][kMaxSlots];  // at most 32 rows per block (D = 32)

    const int rows_per_block = kMergeThreads / tpr;
    const int r_in = threadIdx.x / tpr;
    const int c = threadIdx.x % tpr;  // channel group
    const long long total = (long long)p.N * p.Hq;
    const long long row = (long long)blockIdx.x * rows_per_block + r_in;
    const bool row_ok = row < total;

    // Every slot of the row holds an (m, l) pair: the pass that owns a slot stores l = 0 when its
    // token range is empty (a prefix split past the group's length, a suffix chunk past the
    // sample's), and leaves the slot's output part unwritten.  The row therefore needs no lengths
    // here; a slot with l = 0 gets weight 0 and its output part, though loaded, is not used.
    const int S = row_ok ? p.num_slots : 0;
    const bool ch_ok = row_ok && 4 * c < p.D;
    const elem_t* base = (const elem_t*)p.part_acc + part_index(p, row_ok ? row : 0, 0) * p.D + 4 * c;
    // The first batch of output-part loads does not need the weights: it is issued together
    // with the (m, l) loads so that both round trips overlap.
    constexpr int kBatch = BATCH;
    vec_t v[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
        v[u] = PartVec<HALF>::zero();
        if (ch_ok && u < S)
            v[u] = *reinterpret_cast<const vec_t*>(base + (long long)u * p.D);
    }
    // Weights: the tpr threads of a row (a power of two <= 64, aligned inside a wavefront) each
    // take every tpr-th slot; maximum and sum go round the group with shuffles.
    constexpr int kPerLane = PERLANE;
    float2 mine[kPerLane];
    float m = -INFINITY;
#pragma unroll
    for (int k = 0; k < kPerLane; ++k) {
        const int i = c + k * tpr;
        mine[k] = make_float2(-INFINITY, 0.f);
        if (i < S)
            mine[k] = p.part_ml[part_index(p, row, i)];
        if (mine[k].y > 0.f)
            m = fmaxf(m, mine[k].x);
    }
    for (int o = tpr >> 1; o > 0; o >>= 1)
        m = fmaxf(m, __shfl_xor(m, o));
    float l = 0.f;
#pragma unroll
    for (int k = 0; k < kPerLane; ++k) {
        const int i = c + k * tpr;
        const float w = mine[k].y > 0.f ? mine[k].y * __builtin_amdgcn_exp2f(mine[k].x - m) : 0.f;
        if (i < S)
            wgt[r_in][i] = w;
        l += w;
    }
    for (int o = tpr >> 1; o > 0; o >>= 1)
        l += __shfl_xor(l, o);
    __syncthreads();
    if (!ch_ok)
        return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i0 = 0; i0 < S; i0 += kBatch) {
        if (i0 > 0) {
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                v[u] = PartVec<HALF>::zero();
                if (i0 + u < S)
                    v[u] = *reinterpret_cast<const vec_t*>(base + (long long)(i0 + u) * p.D);
            }
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const float w = i0 + u < S ? wgt[r_in][i0 + u] : 0.f;
            if (w != 0.f) {
                const float4 f = PartVec<HALF>::widen(v[u]);
                acc.x = fmaf(f.x, w, acc.x);
                acc.y = fmaf(f.y, w, acc.y);
                acc.z = fmaf(f.z, w, acc.z);
                acc.w = fmaf(f.w, w, acc.w);
            }
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
        p.lse[row] = l > 0.f ? (m + __log2f(l)) * kLn2 : -INFINITY;
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
    const bool few = p.num_slots <= 8, wide = use >= 32;
    const dim3 block(kMergeThreads);
#define SPD_MERGE(HALF, BATCH, PERLANE) \
    hipLaunchKernelGGL((attn_merge_kernel<HALF, BATCH, PERLANE>), grid, block, 0, s, p, use)
    if (p.part_half) {
        if (few && wide) SPD_MERGE(true, 8, kMaxSlots / 32);
        else if (wide) SPD_MERGE(true, 32, kMaxSlots / 32);
        else if (few) SPD_MERGE(true, 8, kMaxSlots / 8);
        else SPD_MERGE(true, 32, kMaxSlots / 8);
    } else {
        if (few && wide) SPD_MERGE(false, 8, kMaxSlots / 32);
        else if (wide) SPD_MERGE(false, 32, kMaxSlots / 32);
        else if (few) SPD_MERGE(false, 8, kMaxSlots / 8);
        else SPD_MERGE(false, 32, kMaxSlots / 8);
    }
#undef SPD_MERGE
    return hipGetLastError();
}

}  // namespace spd
