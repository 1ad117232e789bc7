// Prefix (cascade) pass as a kernel of its own: launch wrappers around prefix_body.
#include "attn_prefix_body.h"

namespace spd {
namespace {

using namespace prefix_impl;

// 128-row workgroups (4 wavefronts) take the short rings (80 KB) so that two of them share a CU;
// 256-row workgroups (8 wavefronts) keep the long rings, copies two tiles ahead.
template <int WAVES, bool PAGED>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(WAVES == 4 ? 2 : 1, 2))) void
attn_prefix_mfma_kernel(AttnParams p, int rowtiles)
{
    constexpr int KS = WAVES == 4 ? 2 : 4, VS = WAVES == 4 ? 3 : 4, AHEAD = WAVES == 4 ? 1 : 2;
    __shared__ uint4 lds[prefix_lds_bytes(KS, VS) / 16];
    const PrefixItem it = prefix_item((int)blockIdx.x, p.num_prefix_splits, rowtiles, p.B * p.Hkv);
    prefix_body<WAVES, PAGED, KS, VS, AHEAD>(p, level_of(p, rowtiles), lds, it.split, it.rowtile, it.z);
}

template <int WAVES>
hipError_t launch_waves(const AttnParams& p, hipStream_t s)
{
    constexpr int kBlockRows = 32 * WAVES;
    const int rowtiles = (p.max_spp * p.G + kBlockRows - 1) / kBlockRows;
    const long long blocks = (long long)p.num_prefix_splits * rowtiles * p.B * p.Hkv;
    if (blocks > 0x7fffffffLL)
        return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks);
    if (p.page_size)
        hipLaunchKernelGGL((attn_prefix_mfma_kernel<WAVES, true>), grid, dim3(WAVES * 64), 0, s, p, rowtiles);
    else
        hipLaunchKernelGGL((attn_prefix_mfma_kernel<WAVES, false>), grid, dim3(WAVES * 64), 0, s, p, rowtiles);
    return hipGetLastError();
}

}  // namespace

bool prefix_mfma_supported(const AttnParams& p)
{
    return p.dtype == 1 && p.D == kD && p.prefix_split_tokens % kTileN == 0 &&
           (p.page_size == 0 || p.page_size == 16) && (long long)p.B * p.Hkv <= 65535;
}

// Rows per workgroup that the split plan and the fused launch assume: 128 (four wavefronts of 32
// rows) whatever the row count.  Workgroups of 8 wavefronts and 256 rows are slower as soon as the
// pass shares a launch with the suffix pass (a 4-wavefront workgroup leaves room on its CU for a
// suffix workgroup), and smaller ones (64 rows, 128 threads) gained nothing even for a handful of
// rows, where the pass is bound by latency, not by the idle wavefronts.
int prefix_mfma_block_rows(int)
{
    return 128;
}

hipError_t launch_attn_prefix_mfma(const AttnParams& p, hipStream_t s)
{
    if (p.num_prefix_splits <= 0)
        return hipSuccess;
    // On its own (no suffix workgroups to share a CU with) a matrix-bound pass does better with
    // 256-row workgroups and the long rings, provided that still gives most CUs a workgroup;
    // the split plan does not depend on the row tile.
    const long long wide_blocks = (long long)p.num_prefix_splits * ((p.max_spp * p.G + 255) / 256) * p.B * p.Hkv;
    if (p.max_spp * p.G > 128 && wide_blocks >= 192)
        return launch_waves<8>(p, s);
    return launch_waves<4>(p, s);
}

}  // namespace spd
