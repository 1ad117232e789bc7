// Suffix pass as a kernel of its own: launch wrapper around suffix_body.
#include "attn_suffix_body.h"

namespace spd {
namespace {

using namespace suffix_impl;

template <bool PAGED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void attn_suffix_mfma_kernel(AttnParams p, int slot0)
{
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    suffix_body<PAGED>(p, slot0, (long long)blockIdx.x * kWavesPerBlock + wave);
}

}  // namespace

bool suffix_mfma_supported(const AttnParams& p)
{
    return p.dtype == 1 && p.D == kD && p.G <= 16 && p.suffix_chunk_tokens % kTile == 0;
}

hipError_t launch_attn_suffix_mfma(const AttnParams& p, hipStream_t s)
{
    if (p.num_suffix_chunks <= 0)
        return hipSuccess;
    const long long total = (long long)p.N * p.Hkv * p.num_suffix_chunks;
    const dim3 grid((unsigned)((total + kWavesPerBlock - 1) / kWavesPerBlock));
    if (p.page_size)
        hipLaunchKernelGGL(attn_suffix_mfma_kernel<true>, grid, dim3(256), 0, s, p, p.suffix_slot0);
    else
        hipLaunchKernelGGL(attn_suffix_mfma_kernel<false>, grid, dim3(256), 0, s, p, p.suffix_slot0);
    return hipGetLastError();
}

}  // namespace spd
