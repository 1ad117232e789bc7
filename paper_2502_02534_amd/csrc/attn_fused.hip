// Prefix and suffix pass in one launch (bf16, head_dim 128, more than 128 query rows per KV head).
//
// The prefix pass is bound by the matrix pipe and the vector ALU, the suffix pass by HBM, and
// neither needs the other's result before the merge.  One grid of 512-thread workgroups carries
// both: the first workgroups run the prefix body (one (prompt, KV head, row tile, split) each),
// the rest run the suffix body (eight wavefront items each).  Workgroups are handed out in
// index order, so a CU turns to suffix items as soon as its prefix workgroup is done: there is
// no launch (with its ramp and tail) between the two passes, the suffix stream starts while
// other CUs are still in their last prefix tiles, and the prefix pass's burst of partial-state
// writes overlaps with suffix reads.  Both bodies are the ones the separate kernels use.
#include "attn_prefix_body.h"
#include "attn_suffix_body.h"

namespace spd {
namespace {

constexpr int kFusedWaves = 8;
static_assert(kFusedWaves * suffix_impl::kWaveLdsBytes <= prefix_impl::kLdsBytes, "suffix tiles must fit");

template <bool PAGED>
__global__ __launch_bounds__(kFusedWaves * 64) void attn_fused_kernel(AttnParams p, int prefix_blocks,
                                                                     int rowtiles)
{
    __shared__ uint4 lds[prefix_impl::kLdsBytes / 16];
    // Prefix workgroups come first: each is one long serial chain of tiles, so they should start
    // at once; the suffix items that follow are short and fill the CUs as these finish.  (Spreading
    // the two roles evenly over the grid was measured 4 to 10 % slower.)
    const int blk = blockIdx.x;
    if (blk < prefix_blocks) {
        // split fastest, then row tile, then (prompt, KV head): the order of the 3-D prefix grid
        const int split = blk % p.num_prefix_splits;
        const int rest = blk / p.num_prefix_splits;
        prefix_impl::prefix_body<kFusedWaves, PAGED>(p, lds, split, rest % rowtiles, rest / rowtiles);
    } else {
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const long long item = (long long)(blk - prefix_blocks) * kFusedWaves + wave;
        typedef uint4 (*wave_tile_t)[suffix_impl::kRowU4];
        suffix_impl::suffix_body<PAGED>(
            p, p.num_prefix_splits, item,
            (wave_tile_t)((char*)lds + (size_t)wave * suffix_impl::kWaveLdsBytes));
    }
}

}  // namespace

// The fused launch covers the shapes for which the prefix pass would use its 256-row workgroups.
bool attn_fused_supported(const AttnParams& p)
{
    return prefix_mfma_supported(p) && suffix_mfma_supported(p) && prefix_mfma_block_rows(p.max_spp * p.G) == 256 &&
           p.num_prefix_splits > 0 && p.num_suffix_chunks > 0;
}

hipError_t launch_attn_fused(const AttnParams& p, hipStream_t s)
{
    const int rowtiles = (p.max_spp * p.G + 255) / 256;
    const long long prefix_blocks = (long long)p.num_prefix_splits * rowtiles * p.B * p.Hkv;
    const long long items = (long long)p.N * p.Hkv * p.num_suffix_chunks;
    const long long suffix_blocks = (items + kFusedWaves - 1) / kFusedWaves;
    if (prefix_blocks + suffix_blocks > 0x7fffffffLL)
        return hipErrorInvalidValue;
    const dim3 grid((unsigned)(prefix_blocks + suffix_blocks));
    if (p.page_size)
        hipLaunchKernelGGL(attn_fused_kernel<true>, grid, dim3(kFusedWaves * 64), 0, s, p, (int)prefix_blocks, rowtiles);
    else
        hipLaunchKernelGGL(attn_fused_kernel<false>, grid, dim3(kFusedWaves * 64), 0, s, p, (int)prefix_blocks, rowtiles);
    return hipGetLastError();
}

}  // namespace spd
