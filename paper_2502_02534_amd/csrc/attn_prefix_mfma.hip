// Prefix (cascade) pass as a kernel of its own: launch wrappers around prefix_body.
#include "attn_prefix_body.h"

namespace spd {
namespace {

using namespace prefix_impl;

template <int WAVES, bool PAGED>
__global__ __launch_bounds__(WAVES * 64) void attn_prefix_mfma_kernel(AttnParams p)
{
    __shared__ uint4 lds[kLdsBytes / 16];
    prefix_body<WAVES, PAGED>(p, lds, blockIdx.x, blockIdx.y, blockIdx.z);
}

template <int WAVES>
hipError_t launch_waves(const AttnParams& p, hipStream_t s)
{
    constexpr int kBlockRows = 32 * WAVES;
    const int rowtiles = (p.max_spp * p.G + kBlockRows - 1) / kBlockRows;
    const dim3 grid(p.num_prefix_splits, rowtiles, p.B * p.Hkv);
    if (p.page_size)
        hipLaunchKernelGGL((attn_prefix_mfma_kernel<WAVES, true>), grid, dim3(WAVES * 64), 0, s, p);
    else
        hipLaunchKernelGGL((attn_prefix_mfma_kernel<WAVES, false>), grid, dim3(WAVES * 64), 0, s, p);
    return hipGetLastError();
}

}  // namespace

bool prefix_mfma_supported(const AttnParams& p)
{
    return p.dtype == 1 && p.D == kD && p.prefix_split_tokens % kTileN == 0 &&
           (p.page_size == 0 || p.page_size == 16) && (long long)p.B * p.Hkv <= 65535;
}

// Rows per workgroup used for a problem with `rows` query rows per (prompt, KV head):
// 32 rows per wavefront, 2 to 8 wavefronts.
int prefix_mfma_block_rows(int rows)
{
    return rows > 128 ? 256 : rows > 64 ? 128 : 64;
}

hipError_t launch_attn_prefix_mfma(const AttnParams& p, hipStream_t s)
{
    if (p.num_prefix_splits <= 0)
        return hipSuccess;
    switch (prefix_mfma_block_rows(p.max_spp * p.G)) {
    case 256: return launch_waves<8>(p, s);
    case 128: return launch_waves<4>(p, s);
    default: return launch_waves<2>(p, s);
    }
}

}  // namespace spd
