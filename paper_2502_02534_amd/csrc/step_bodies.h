// Device bodies shared by the kernels that run between two decode steps of the sampling loop
// (the paper generates up to 1024 tokens per sample, App. "Experiment settings"): a block's share
// of a row copy, and the append of one sample's new K/V row.  No body returns early or uses a
// barrier, so a caller may do more work after it.
#pragma once
#include "spd_internal.h"

namespace spd {
namespace step_impl {

constexpr int kCopyThreads = 256;
constexpr int kPieces = 8;                                            // 16-byte pieces per thread
constexpr long long kBytesPerBlock = 16ll * kCopyThreads * kPieces;

// Bytes [blk * kBytesPerBlock, ...) of `nbytes` from src to dst.  All of a thread's pieces are
// requested before the first is stored (source and destination do not overlap, which the
// compiler cannot know: left to itself it waits for every load before the store that follows
// it, eight round trips instead of one).
__device__ __forceinline__ void copy_block(const char* src, char* dst, long long nbytes, long long blk, bool wide)
{
    const long long b0 = blk * kBytesPerBlock, end = min(b0 + kBytesPerBlock, nbytes);
    if (wide) {
        uint4 v[kPieces];
#pragma unroll
        for (int k = 0; k < kPieces; ++k) {
            const long long o = b0 + 16ll * (threadIdx.x + k * kCopyThreads);
            v[k] = make_uint4(0u, 0u, 0u, 0u);
            if (o < end)
                v[k] = *reinterpret_cast<const uint4*>(src + o);
        }
#pragma unroll
        for (int k = 0; k < kPieces; ++k) {
            const long long o = b0 + 16ll * (threadIdx.x + k * kCopyThreads);
            if (o < end)
                *reinterpret_cast<uint4*>(dst + o) = v[k];
        }
    } else {
        // rows that are only 4-byte aligned: the block's bytes in 4-byte pieces, kPieces at a time
        for (long long base = b0; base < end; base += 4ll * kCopyThreads * kPieces) {
            uint32_t v[kPieces];
#pragma unroll
            for (int k = 0; k < kPieces; ++k) {
                const long long o = base + 4ll * (threadIdx.x + k * kCopyThreads);
                v[k] = 0u;
                if (o < end)
                    v[k] = *reinterpret_cast<const uint32_t*>(src + o);
            }
#pragma unroll
            for (int k = 0; k < kPieces; ++k) {
                const long long o = base + 4ll * (threadIdx.x + k * kCopyThreads);
                if (o < end)
                    *reinterpret_cast<uint32_t*>(dst + o) = v[k];
            }
        }
    }
}

// Appends row n of k_new / v_new ([N, Hkv, D]) to sample n's suffix and adds one to its length,
// unless the sample is finished (its last token was the end token, now or earlier) or its slot is
// full.  `lens_out` (may be null) receives the length the sample had before this call.
// Everything that does not depend on the length is requested at once: the new token's rows (a
// thread's pieces; two rounds cover rows of up to 8 KB, longer ones loop at the end) and the
// sample's length, page range, last token and finished flag, which every thread reads for itself
// (uniform addresses), so that the body is one round trip (two with paged KV: the page number).
// Called by 256-thread workgroups, one per sample.
__device__ __forceinline__ void append_sample(const KvAppendParams& a, int n, const void* k_new, const void* v_new,
                                              int* lens_out)
{
    const int row_u4 = a.Hkv * a.D * a.elt / 16;   // 16-byte pieces of one token (all KV heads)
    const int head_u4 = a.D * a.elt / 16;
    const uint4* ks = (const uint4*)k_new + (long long)n * row_u4;
    const uint4* vs = (const uint4*)v_new + (long long)n * row_u4;
    const int i0 = threadIdx.x, i1 = threadIdx.x + 256;
    uint4 k0 = make_uint4(0u, 0u, 0u, 0u), v0 = k0, k1 = k0, v1 = k0;
    if (i0 < row_u4) {
        k0 = ks[i0];
        v0 = vs[i0];
    }
    if (i1 < row_u4) {
        k1 = ks[i1];
        v1 = vs[i1];
    }
    const int pos = a.suffix_lens[n];
    const int first_page = a.page_size != 0 ? a.page_indptr[n] : 0;
    const int num_pages = a.page_size != 0 ? a.page_indptr[n + 1] - first_page : 0;
    const int last = a.finished && a.last_tokens ? a.last_tokens[n] : 0;
    const int was_finished = a.finished ? a.finished[n] : 0;
    if (lens_out && threadIdx.x == 0)
        *lens_out = pos;
    bool live = pos < a.capacity;
    if (a.page_size != 0)  // and inside the sample's own page list
        live = live && pos / a.page_size < num_pages;
    if (a.finished) {
        const bool ends = a.last_tokens && last == a.end_token;
        if (ends && threadIdx.x == 0)
            a.finished[n] = 1;
        live = live && !ends && was_finished == 0;
    }
    if (live) {
        long long pg = 0;
        if (a.page_size != 0)
            pg = a.pages[first_page + pos / a.page_size];
        auto place = [&](int i) -> long long {
            if (a.page_size == 0)
                return ((long long)n * a.capacity + pos) * row_u4 + i;
            const int j = i / head_u4, c = i % head_u4;
            return ((pg * a.Hkv + j) * a.page_size + pos % a.page_size) * head_u4 + c;
        };
        if (i0 < row_u4) {
            ((uint4*)a.k_suffix)[place(i0)] = k0;
            ((uint4*)a.v_suffix)[place(i0)] = v0;
        }
        if (i1 < row_u4) {
            ((uint4*)a.k_suffix)[place(i1)] = k1;
            ((uint4*)a.v_suffix)[place(i1)] = v1;
        }
        for (int i = threadIdx.x + 512; i < row_u4; i += 256) {
            ((uint4*)a.k_suffix)[place(i)] = ks[i];
            ((uint4*)a.v_suffix)[place(i)] = vs[i];
        }
        if (threadIdx.x == 0)
            a.suffix_lens[n] = pos + 1;
    }
}

}  // namespace step_impl
}  // namespace spd
