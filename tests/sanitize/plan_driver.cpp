// Exercises the launch planner of the attention calls (host arithmetic, paper_2502_02534_amd/csrc/plan.h)
// under AddressSanitizer and UndefinedBehaviorSanitizer over a grid of descriptions and bounds, and
// checks the invariants the kernels rely on.  Exit status 0 = nothing found.
#include "../../paper_2502_02534_amd/csrc/plan.h"

#include <cstdio>
#include <initializer_list>

using namespace spd::plan;

static int fail(const char* what, long long a, long long b)
{
    std::printf("FAILED: %s (%lld, %lld)\n", what, a, b);
    return 1;
}

int main()
{
    const long long lens[] = {0, 1, 63, 64, 65, 127, 129, 2048, 8192, 16384, 100000, 300001, 1ll << 30};
    const int samples[] = {1, 3, 16, 64, 192, 1024, 100000};
    const int prompts[] = {1, 2, 8, 26};
    int checked = 0;
    for (int dtype : {SPD_F32, SPD_BF16})
        for (int D : {64, 128, 256})
            for (int g : {1, 4, 8, 16})
                for (int hkv : {1, 8})
                    for (int B : prompts)
                        for (int N : samples)
                            for (long long lp : lens)
                                for (long long ls : lens) {
                                    if (N < B)
                                        continue;
                                    spd_attn_desc d = {dtype, g * hkv, hkv, D, B, N, (N + B - 1) / B, 0, 0.f, 0};
                                    Plan pl;
                                    if (make_plan(&d, lp, ls, &pl) != SPD_OK)
                                        return fail("make_plan refused a valid description", lp, ls);
                                    if (lp > 0 && (pl.prefix_split_tokens <= 0 || pl.prefix_split_tokens % 64))
                                        return fail("split not a positive multiple of 64", lp, pl.prefix_split_tokens);
                                    if (ls > 0 && (pl.suffix_chunk_tokens < 64 || pl.suffix_chunk_tokens % 32))
                                        return fail("chunk not a multiple of 32", ls, pl.suffix_chunk_tokens);
                                    if (pl.num_prefix_splits > kMaxSplits || pl.num_suffix_chunks > kMaxSplits)
                                        return fail("more parts than the merge takes", pl.num_prefix_splits,
                                                    pl.num_suffix_chunks);
                                    if ((long long)pl.num_prefix_splits * pl.prefix_split_tokens < lp ||
                                        (long long)pl.num_suffix_chunks * pl.suffix_chunk_tokens < ls)
                                        return fail("parts do not cover the length", lp, ls);
                                    if (pl.num_prefix_splits > 0 &&
                                        (long long)(pl.num_prefix_splits - 1) * pl.prefix_split_tokens >= lp)
                                        return fail("an empty last split", lp, pl.prefix_split_tokens);
                                    const size_t slots = (size_t)pl.num_prefix_splits + pl.num_suffix_chunks;
                                    if (pl.acc_bytes < slots * N * d.num_q_heads * D * 4 || pl.acc_bytes % 256 ||
                                        pl.ml_bytes < slots * N * d.num_q_heads * 8 || pl.ml_bytes % 256)
                                        return fail("workspace too small or misaligned", (long long)pl.acc_bytes,
                                                    (long long)pl.ml_bytes);
                                    // the same problem as a tree of one to four levels
                                    for (int levels = 1; levels <= SPD_MAX_PREFIX_LEVELS; ++levels) {
                                        spd_prefix_level lv[SPD_MAX_PREFIX_LEVELS] = {};
                                        for (int l = 0; l < levels; ++l) {
                                            lv[l].num_groups = l == 0 ? 1 : B;
                                            lv[l].max_samples_per_group = l == 0 ? 0 : (N + B - 1) / B;
                                            lv[l].max_len = l % 2 ? lp / 2 : lp;
                                        }
                                        LevelPlan lpn;
                                        if (make_level_plan(&d, levels, lv, ls, &lpn) != SPD_OK)
                                            return fail("make_level_plan refused a valid tree", levels, lp);
                                        int slots_seen = 0;
                                        for (int l = 0; l < levels; ++l) {
                                            if (lpn.slot0[l] != slots_seen)
                                                return fail("slot ranges not consecutive", l, lpn.slot0[l]);
                                            slots_seen += lpn.num_splits[l];
                                        }
                                        if (slots_seen > kMaxSplits || slots_seen + lpn.num_suffix_chunks != lpn.num_slots)
                                            return fail("slot count", slots_seen, lpn.num_slots);
                                    }
                                    ++checked;
                                }
    // refusals
    spd_attn_desc bad = {SPD_BF16, 7, 2, 128, 1, 4, 0, 0, 0.f, 0};
    Plan pl;
    if (make_plan(&bad, 10, 10, &pl) != SPD_EINVAL || make_plan(nullptr, 1, 1, &pl) != SPD_EINVAL)
        return fail("invalid description accepted", 0, 0);
    spd_attn_desc ok = {SPD_BF16, 8, 2, 128, 1, 4, 0, 0, 0.f, 0};
    if (make_plan(&ok, -1, 0, &pl) != SPD_EINVAL || make_plan(&ok, (1ll << 30) + 1, 0, &pl) != SPD_EINVAL)
        return fail("invalid bound accepted", 0, 0);
    LevelPlan lpn;
    if (make_level_plan(&ok, 0, nullptr, 0, &lpn) != SPD_EINVAL)
        return fail("empty tree accepted", 0, 0);
    std::printf("ok: %d plans\n", checked);
    return 0;
}
