// Plain (non-MFMA) partial-state kernel: fp32 inputs, or any case the tiled kernels
// do not cover.  One wavefront computes the partial softmax state of one
// (sample, query head) over one token range (a prefix split or a suffix chunk),
// 64 tokens at a time: each lane scores one token, the wave reduces max and sum,
// and the weighted value rows are accumulated with lanes striding the channels.
#include "spd_internal.h"

#include <hip/hip_fp16.h>

namespace spd {
namespace {

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<uint16_t>(uint16_t v)
{
    return __uint_as_float(((uint32_t)v) << 16);
}

__device__ __forceinline__ float wave_max(float v)
{
    for (int o = 32; o > 0; o >>= 1)
        v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
    for (int o = 32; o > 0; o >>= 1)
        v += __shfl_xor(v, o);
    return v;
}

constexpr int kMaxChanPerLane = 4;  // D <= 256

template <typename T>
__global__ __launch_bounds__(64) void attn_plain_kernel(AttnParams p, int slot0, int is_prefix)
{
    const int lane = threadIdx.x;
    const int row = blockIdx.x;  // n * Hq + h
    const int part = blockIdx.y;
    const int n = row / p.Hq, h = row % p.Hq, j = h / p.G;
    const int D = p.D;

    int t0, t1;
    long long start = 0;
    const int* pages = nullptr;
    const T* kbase;
    const T* vbase;
    if (is_prefix) {
        const int b = prompt_of_sample(p.sample_indptr, p.B, n);
        const int L = p.prefix_lens[b];
        t0 = part * p.prefix_split_tokens;
        t1 = min(L, t0 + p.prefix_split_tokens);
        if (p.page_size)
            pages = p.prefix_pages + p.prefix_indptr[b];
        else
            start = p.prefix_indptr[b];
        kbase = (const T*)p.k_prefix;
        vbase = (const T*)p.v_prefix;
    } else {
        const int L = p.suffix_lens[n];
        t0 = part * p.suffix_chunk_tokens;
        t1 = min(L, t0 + p.suffix_chunk_tokens);
        if (p.page_size)
            pages = p.suffix_pages + p.suffix_page_indptr[n];
        else
            start = (long long)n * p.max_suffix_len;
        kbase = (const T*)p.k_suffix;
        vbase = (const T*)p.v_suffix;
    }
    if (t0 >= t1) {
        // empty range: l = 0 tells the merge to leave the slot out (its output part stays unwritten)
        if (lane == 0)
            p.part_ml[part_index(p, row, slot0 + part)] = make_float2(-INFINITY, 0.f);
        return;
    }

    const T* q = (const T*)p.q + (long long)row * D;
    float m = -INFINITY, l = 0.f;
    float acc[kMaxChanPerLane] = {0.f, 0.f, 0.f, 0.f};

    for (int tb = t0; tb < t1; tb += 64) {
        const int t = tb + lane;
        const bool valid = t < t1;
        float s = -INFINITY;
        long long off = 0;
        if (valid) {
            off = kv_row_offset(t, j, p.Hkv, D, p.page_size, start, pages);
            const T* k = kbase + off;
            float dot = 0.f;
            for (int d = 0; d < D; ++d)
                dot = fmaf(to_f32<T>(q[d]), to_f32<T>(k[d]), dot);
            s = dot * p.scale_log2;
        }
        const float m_new = fmaxf(m, wave_max(s));
        const float w = valid ? __builtin_amdgcn_exp2f(s - m_new) : 0.f;
        const float corr = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - m_new);
        l = l * corr + wave_sum(w);
        m = m_new;
#pragma unroll
        for (int i = 0; i < kMaxChanPerLane; ++i)
            acc[i] *= corr;
        const int cnt = min(64, t1 - tb);
        for (int u = 0; u < cnt; ++u) {
            const float wu = __shfl(w, u);
            const long long ou = __shfl(off, u);
            const T* v = vbase + ou;
#pragma unroll
            for (int i = 0; i < kMaxChanPerLane; ++i) {
                const int d = lane + 64 * i;
                if (d < D)
                    acc[i] = fmaf(wu, to_f32<T>(v[d]), acc[i]);
            }
        }
    }
    const long long prow = part_index(p, row, slot0 + part);
    const float inv_l = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
    for (int i = 0; i < kMaxChanPerLane; ++i) {
        const int d = lane + 64 * i;
        if (d < D) {
            if (p.part_half)
                ((__half*)p.part_acc)[prow * D + d] = __float2half(acc[i] * inv_l);
            else
                ((float*)p.part_acc)[prow * D + d] = acc[i] * inv_l;
        }
    }
    if (lane == 0)
        p.part_ml[prow] = make_float2(m, l);
}

}  // namespace

hipError_t launch_attn_plain(const AttnParams& p, bool prefix, bool suffix, hipStream_t s)
{
    const dim3 block(64);
    if (prefix && p.num_prefix_splits > 0) {
        const dim3 grid(p.N * p.Hq, p.num_prefix_splits);
        if (p.dtype == 0)
            hipLaunchKernelGGL(attn_plain_kernel<float>, grid, block, 0, s, p, p.prefix_slot0, 1);
        else
            hipLaunchKernelGGL(attn_plain_kernel<uint16_t>, grid, block, 0, s, p, p.prefix_slot0, 1);
    }
    if (suffix && p.num_suffix_chunks > 0) {
        const dim3 grid(p.N * p.Hq, p.num_suffix_chunks);
        if (p.dtype == 0)
            hipLaunchKernelGGL(attn_plain_kernel<float>, grid, block, 0, s, p, p.suffix_slot0, 0);
        else
            hipLaunchKernelGGL(attn_plain_kernel<uint16_t>, grid, block, 0, s, p, p.suffix_slot0, 0);
    }
    return hipGetLastError();
}

}  // namespace spd
