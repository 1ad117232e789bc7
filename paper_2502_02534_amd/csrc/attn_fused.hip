// Prefix and suffix pass in one launch (bf16, head_dim 128).
//
// The prefix pass is bound by the matrix pipe and the vector ALU, the suffix pass by HBM, and
// neither needs the other's result before the merge.  One grid of 256-thread workgroups with
// 80 KB of LDS carries both, two workgroups per CU: the first workgroups run the prefix body
// (four wavefronts, 128 rows, K ring of 2 and V ring of 3 tiles, copies one tile ahead), the
// rest run the suffix body (four wavefront items; it uses no LDS).  Workgroups start in index order; the prefix workgroups come first (or, when there are
// more of them than CUs, evenly spread through the grid), so that a CU holds one prefix workgroup
// and, beside it, suffix workgroups: each SIMD has one wavefront that multiplies and one that
// streams, HBM is busy during the prefix pass, and there is no launch (with its ramp and tail)
// between the two passes.  Both bodies are the ones the separate kernels use.
//
// The kernel takes a table of prefix levels (a tree of shared prefixes has several; the plain call
// has one), each with its own range of prefix workgroups.
//
// Measured alternatives: 512-thread workgroups with 128 KB (one workgroup per CU, so prefix and
// suffix wavefronts never share a CU) 9 to 15 % slower; spreading the two roles evenly over the
// grid although the prefix workgroups fit one per CU another 4 to 10 % slower.
#include "attn_prefix_body.h"
#include "attn_suffix_body.h"

namespace spd {
namespace {

constexpr int kFusedWaves = 4;
constexpr int kFusedLds = prefix_impl::prefix_lds_bytes(2, 3);

template <bool PAGED>
__global__ __launch_bounds__(kFusedWaves * 64) __attribute__((amdgpu_waves_per_eu(2))) void attn_fused_kernel(
    AttnParams p, FusedLevels fl, int spread)
{
    __shared__ uint4 lds[kFusedLds / 16];
    // Which role a workgroup plays.  With at most one prefix workgroup per CU they simply come
    // first.  With more, they are spread evenly through the grid (of the first n workgroups,
    // floor(n P / T) are prefix workgroups), so that CUs keep holding one of each kind instead of
    // two prefix workgroups.
    const int prefix_blocks = fl.first_block[fl.num_levels];
    int pidx;       // index among the prefix workgroups, or -1
    long long sidx; // index among the suffix workgroups
    if (spread) {
        const long long blk = blockIdx.x, total = gridDim.x;
        const int before = (int)(blk * prefix_blocks / total);
        pidx = (int)((blk + 1) * prefix_blocks / total) > before ? before : -1;
        sidx = blk - before;
    } else {
        pidx = (int)blockIdx.x < prefix_blocks ? (int)blockIdx.x : -1;
        sidx = (long long)blockIdx.x - prefix_blocks;
    }
    if (pidx >= 0) {
        // the prefix level this workgroup belongs to
        int l = 0;
#pragma unroll
        for (int k = 1; k < kMaxLevels; ++k)
            if (k < fl.num_levels && pidx >= fl.first_block[k])
                l = k;
        const PrefixLevelParams& lv = fl.level[l];
        const prefix_impl::PrefixItem it =
            prefix_impl::prefix_item(pidx - fl.first_block[l], lv.num_splits, lv.rowtiles, lv.groups * p.Hkv);
        prefix_impl::prefix_body<kFusedWaves, PAGED, 2, 3, 1>(p, lv, lds, it.split, it.rowtile, it.z);
    } else {
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const long long item = sidx * kFusedWaves + wave;
        suffix_impl::suffix_body<PAGED>(p, p.suffix_slot0, item);
    }
}

hipError_t launch_fused(const AttnParams& p, const FusedLevels& fl, hipStream_t s)
{
    const long long prefix_blocks = fl.first_block[fl.num_levels];
    const long long items = (long long)p.N * p.Hkv * p.num_suffix_chunks;
    const long long suffix_blocks = (items + kFusedWaves - 1) / kFusedWaves;
    if (prefix_blocks + suffix_blocks > 0x7fffffffLL)
        return hipErrorInvalidValue;
    const dim3 grid((unsigned)(prefix_blocks + suffix_blocks));
    const int spread = prefix_blocks > 256 ? 1 : 0;  // more prefix workgroups than CUs
    if (p.page_size)
        hipLaunchKernelGGL(attn_fused_kernel<true>, grid, dim3(kFusedWaves * 64), 0, s, p, fl, spread);
    else
        hipLaunchKernelGGL(attn_fused_kernel<false>, grid, dim3(kFusedWaves * 64), 0, s, p, fl, spread);
    return hipGetLastError();
}

}  // namespace

// The fused launch covers the shapes for which the prefix pass uses its 128-row workgroups.
bool attn_fused_supported(const AttnParams& p)
{
    return prefix_mfma_supported(p) && suffix_mfma_supported(p) && prefix_mfma_block_rows(p.max_spp * p.G) == 128 &&
           p.num_prefix_splits > 0 && p.num_suffix_chunks > 0;
}

hipError_t launch_attn_fused(const AttnParams& p, hipStream_t s)
{
    FusedLevels fl;
    fl.num_levels = 1;
    const int rowtiles = (p.max_spp * p.G + 127) / 128;
    fl.level[0] = prefix_impl::level_of(p, rowtiles);
    fl.first_block[0] = 0;
    const long long blocks = (long long)p.num_prefix_splits * rowtiles * p.B * p.Hkv;
    if (blocks > 0x7fffffffLL)
        return hipErrorInvalidValue;
    for (int l = 1; l <= kMaxLevels; ++l)
        fl.first_block[l] = (int)blocks;
    return launch_fused(p, fl, s);
}

// Several prefix levels and the suffix pass in one launch: every level must be one the 128-row
// prefix body takes, with at least one split.
bool attn_fused_levels_supported(const AttnParams& p, const FusedLevels& fl)
{
    if (!suffix_mfma_supported(p) || p.dtype != 1 || p.D != 128 || p.num_suffix_chunks <= 0)
        return false;
    if (fl.num_levels < 1 || fl.num_levels > kMaxLevels)
        return false;
    for (int l = 0; l < fl.num_levels; ++l) {
        const PrefixLevelParams& lv = fl.level[l];
        if (lv.num_splits <= 0 || lv.split_tokens % 64 != 0 || (long long)lv.groups * p.Hkv > 65535)
            return false;
    }
    return true;
}

hipError_t launch_attn_fused_levels(const AttnParams& p, const FusedLevels& fl, hipStream_t s)
{
    return launch_fused(p, fl, s);
}

}  // namespace spd
