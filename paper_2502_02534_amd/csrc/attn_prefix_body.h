// Prefix (cascade) pass (bf16, head_dim 128): all samples' queries of one KV head form
// a dense row tile against the shared prompt KV, so the prompt is read once per row
// tile instead of once per sample.
//
// Workgroup = (prompt b, KV head j, tile of 32*WAVES query rows, split of the prefix); WAVES is 4
// or 8.
// A query row is (sample, head in group); each wavefront owns 32 rows (one 32-wide column
// block of the transposed products).
//
// Data movement.  K and V tiles of 64 tokens go from global memory straight into LDS
// (global_load_lds_dwordx4, no registers in between), into a ring of K slots and a ring of V
// slots, one or two tiles ahead of the tile in use (K of a tile is needed one iteration before
// its V).  Both tiles are row-major [token][256 bytes] without
// padding; bank conflicts are avoided by an XOR swizzle of the 16-byte pieces of a row,
// applied on the global side of the copy (lane L of a copy instruction always lands at
// LDS offset 16 L, but it may fetch any piece).
//   K  read with ds_read_b128 as the A operand of S^T = K Q^T
//      (v_mfma_f32_32x32x16_bf16, B = query rows held in registers);
//   V  read with the transposing ds_read_b64_tr_b16 (each lane receives four tokens of one
//      channel) as the A operand of O^T += V^T P^T, B = P, which is the S^T accumulator
//      itself repacked to bf16.
// The LDS reads are issued by hand (inline assembly) a few fragments ahead of the MFMA that
// consumes them, with exact lgkmcnt waits; the compiler's own wait insertion would otherwise
// drain every outstanding copy before any LDS read.
//
// Every lane owns one query row in both products, so the online-softmax statistics and the
// accumulator rescale are lane-local.  The running state is the deferred-division form of the
// paper's online-softmax recurrence (App., attn task 2).
#pragma once

#include "spd_internal.h"

#include <hip/hip_fp16.h>

#include <utility>

namespace spd {
namespace prefix_impl {


typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kD = 128;
constexpr int kTileN = 64;               // tokens per tile
constexpr int kTileBytes = kTileN * 256;  // one K or V tile
constexpr int kRowU4 = kD * 2 / 16;
constexpr int kAhead = 4;                // LDS fragments in flight ahead of the MFMAs

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return *reinterpret_cast<bf16x8*>(&v); }
__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return *reinterpret_cast<bf16x8*>(&v); }

// Two floats to packed bf16 (round to nearest even): one v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    const bf16x2 r = __builtin_convertvector(v, bf16x2);
    return *reinterpret_cast<const uint32_t*>(&r);
}

// Swizzle of the 16-byte pieces of token row `tok` (within a tile): piece p lives in slot
// p ^ swz(tok).  Sixteen consecutive rows get sixteen different values (K operand reads: 16
// lanes, 16 rows, one piece each), and four consecutive rows land in four different 64-byte
// quarters of the 256-byte bank window (V reads: four rows, up to four neighbouring pieces each).
__device__ __forceinline__ int swz(int tok) { return ((tok & 3) << 2) | ((tok >> 2) & 3); }

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    // vmcnt(N); expcnt and lgkmcnt left alone
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// One LDS fragment: a K fragment is one ds_read_b128, a V fragment two transposing reads.
// QK: a = channel step (0..7), b = token block (0..1).  PV: a = token step (0..3), b = channel
// block (0..3).  When a region holds both products they alternate.
template <bool QK, bool PV, int K> struct Frag {
    static constexpr bool both = QK && PV;
    static constexpr int idx = both ? (K >> 1) : K;
    static constexpr bool is_pv = both ? ((K & 1) != 0) : PV;
    static constexpr int a = is_pv ? (idx >> 2) : (idx >> 1);
    static constexpr int b = is_pv ? (idx & 3) : (idx & 1);
    static constexpr int ops = is_pv ? 2 : 1;
};
template <bool QK, bool PV> constexpr int frag_count() { return (QK ? 16 : 0) + (PV ? 16 : 0); }
// LDS instructions issued after fragment K while K is the oldest outstanding one
template <bool QK, bool PV, int K> constexpr int ops_after()
{
    int n = 0;
    for (int j = K + 1; j <= K + kAhead && j < frag_count<QK, PV>(); ++j) {
        const bool both = QK && PV;
        const bool is_pv = both ? ((j & 1) != 0) : PV;
        n += is_pv ? 2 : 1;
    }
    return n;
}

template <typename F, int... I>
__device__ __forceinline__ void for_each_index(F&& f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}

// The prefix level that the prefix fields of `p` describe.
__host__ __device__ inline PrefixLevelParams level_of(const AttnParams& p, int rowtiles)
{
    PrefixLevelParams lv;
    lv.k = p.k_prefix;
    lv.v = p.v_prefix;
    lv.lens = p.prefix_lens;
    lv.indptr = p.prefix_indptr;
    lv.pages = p.prefix_pages;
    lv.sample_indptr = p.sample_indptr;
    lv.split_tokens = p.prefix_split_tokens;
    lv.num_splits = p.num_prefix_splits;
    lv.slot0 = p.prefix_slot0;
    lv.rowtiles = rowtiles;
    lv.groups = p.B;
    return lv;
}

// Which (split, row tile, z = group * Hkv + KV head) the prefix workgroup with index `local` of a
// level takes.  Workgroups go to the eight XCDs in turn (index mod 8), and every XCD has an L2 of
// its own: the row tiles of one (split, z) read the same K and V, so they are given indices that
// agree mod 8 and follow one another, which puts them on one XCD at the same time (the prompt is
// then fetched into one L2 once instead of into as many L2s as there are row tiles).  That
// takes a number of (split, z) units divisible by 8; otherwise the split runs fastest, then the
// row tile, then z.
struct PrefixItem {
    int split, rowtile, z;
};
__device__ __forceinline__ PrefixItem prefix_item(int local, int num_splits, int rowtiles, int zs)
{
    PrefixItem it;
    const int units = num_splits * zs;
    if (rowtiles > 1 && (units & 7) == 0) {
        const int slot = local >> 3;
        const int u = (local & 7) + 8 * (slot / rowtiles);
        it.rowtile = slot % rowtiles;
        it.split = u % num_splits;
        it.z = u / num_splits;
    } else {
        it.split = local % num_splits;
        const int rest = local / num_splits;
        it.rowtile = rest % rowtiles;
        it.z = rest / rowtiles;
    }
    return it;
}

// LDS of a workgroup: KS slots for K tiles followed by VS slots for V tiles.
constexpr int prefix_lds_bytes(int KS, int VS) { return (KS + VS) * kTileBytes; }

// Body of one workgroup of WAVES wavefronts for prefix level `lv`: (split, rowtile,
// z = group * Hkv + KV head).  `lds` is
// prefix_lds_bytes(KS, VS) of LDS; every wavefront of the workgroup must call it (it uses
// workgroup barriers).  Copies run AHEAD tiles ahead of the tile in use.  K of tile t is read
// in iteration t and V of tile t in iteration t + 1, and the copies of tile t + AHEAD start at
// the top of iteration t, so the rings need KS >= AHEAD + 1 and VS >= AHEAD + 2 slots.
template <int WAVES, bool PAGED, int KS = 4, int VS = 4, int AHEAD = 2>
__device__ __forceinline__ void prefix_body(const AttnParams& p, const PrefixLevelParams& lv, uint4* lds, int split,
                                            int rowtile, int z)
{
    static_assert(AHEAD == 1 || AHEAD == 2, "copy distance");
    static_assert(KS >= AHEAD + 1 && VS >= AHEAD + 2, "rings too short for the copy distance");
    constexpr int kIPW = 32 / WAVES;  // copy instructions per wave per tile

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, h = lane >> 5;

    const int b = z / p.Hkv, j = z % p.Hkv;
    const int s0 = lv.sample_indptr[b];
    const int rows_b = (lv.sample_indptr[b + 1] - s0) * p.G;
    const int row0 = rowtile * 32 * WAVES;
    const int Lp = lv.lens[b];
    const int t0 = split * lv.split_tokens;
    const int t1 = min(Lp, t0 + lv.split_tokens);
    if (row0 >= rows_b)
        return;
    if (t0 >= t1) {
        // empty split: l = 0 tells the merge to leave the slot out (its output part stays unwritten)
        const int rr = row0 + wave * 32 + col;
        if (rr < rows_b && h == 0)
            p.part_ml[part_index(p, (long long)(s0 + rr / p.G) * p.Hq + j * p.G + rr % p.G, lv.slot0 + split)] =
                make_float2(-INFINITY, 0.f);
        return;
    }

    const char* __restrict__ kg = (const char*)lv.k;
    const char* __restrict__ vg = (const char*)lv.v;
    // the page table is read with scalar loads (uniform index, constant address space)
    typedef const __attribute__((address_space(4))) int* const_int_ptr;
    const const_int_ptr pages = PAGED ? (const_int_ptr)(lv.pages + lv.indptr[b]) : nullptr;
    // byte strides of a token row and byte offset of token 0 of this KV head
    const long long tok_stride = PAGED ? 256 : (long long)p.Hkv * 256;
    const long long head_base = PAGED ? (long long)j * 16 * 256 : ((long long)lv.indptr[b] * p.Hkv + j) * 256;
    const long long page_stride = (long long)p.Hkv * 16 * 256;

    // ---- query fragments (B operand): column = this lane's row, k-slot = channels 16 s + 8 h
    bf16x8 qf[8];
    const int rr = row0 + wave * 32 + col;
    const bool row_ok = rr < rows_b;
    const long long out_row = (long long)(s0 + (row_ok ? rr : 0) / p.G) * p.Hq + j * p.G + (row_ok ? rr : 0) % p.G;
    {
        const uint4* qg = (const uint4*)p.q + out_row * kRowU4;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            uint4 v = qg[2 * s + h];
            if (!row_ok)
                v = make_uint4(0, 0, 0, 0);
            qf[s] = as_bf16x8(v);
        }
    }

    // ---- global -> LDS copies -------------------------------------------------------------------
    // A tile takes 32 copy instructions (16 for K, 16 for V), each covering 4 token rows; wave w
    // issues instructions w kIPW .. w kIPW + kIPW - 1.  Lane (r, c) of instruction q fetches piece
    // c ^ swz(row) of row 4 (q & 15) + r.  Rows past the end of the split are clamped to its last
    // token (their scores are masked later).  The four rows of an instruction lie in one page, so
    // the page number is uniform over the wavefront.
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) void*)lds;
    const int lane_row = lane >> 4;
    unsigned lane_off[kIPW];  // byte offset of this lane's piece for a full tile, relative to the group's first row
#pragma unroll
    for (int i = 0; i < kIPW; ++i) {
        const int tl = 4 * ((wave * kIPW + i) & 15) + lane_row;
        lane_off[i] = (unsigned)(lane_row * (unsigned)tok_stride + (((lane & 15) ^ swz(tl)) << 4));
    }
    // page numbers of the next tile to be copied, fetched one tile ahead of their use
    int next_page[kIPW];
    auto fetch_pages = [&](int tile) __attribute__((always_inline)) {
        if (PAGED) {
#pragma unroll
            for (int i = 0; i < kIPW; ++i) {
                const int tg = min(t0 + tile * kTileN + 4 * ((wave * kIPW + i) & 15), t1 - 1);
                next_page[i] = pages[tg >> 4];
            }
        }
    };
    fetch_pages(0);
    // Contiguous KV, whole tiles: the source of copy i is a fixed pointer (tensor, KV head, first row
    // of the group) plus a per-tile offset shared by all copies, so a copy costs one 64-bit add.
    const char* group_ptr[kIPW];
#pragma unroll
    for (int i = 0; i < kIPW; ++i) {
        const int q = wave * kIPW + i;
        group_ptr[i] = (q < 16 ? kg : vg) + head_base + (long long)(4 * (q & 15)) * tok_stride;
    }
    auto issue_tile = [&](int tile) __attribute__((always_inline)) {
        const int tb = t0 + tile * kTileN;
        const int kslot_bytes = (tile % KS) * kTileBytes, vslot_bytes = (KS + tile % VS) * kTileBytes;
        const bool full = tb + kTileN <= t1;
        if (!PAGED && full) {
            const long long tile_off = (long long)tb * tok_stride;
#pragma unroll
            for (int i = 0; i < kIPW; ++i) {
                const int q = wave * kIPW + i;
                const char* src = group_ptr[i] + tile_off + lane_off[i];
                uint4* dst = lds + ((q < 16 ? kslot_bytes : vslot_bytes) + (q & 15) * 1024) / 16;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                                 (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < kIPW; ++i) {
            const int q = wave * kIPW + i;
            const int g = 4 * (q & 15);  // first row of the group within the tile
            const int tg = min(tb + g, t1 - 1);
            long long base;              // uniform: byte offset of row tg
            if (PAGED)
                base = (long long)next_page[i] * page_stride + head_base + (tg & 15) * 256;
            else
                base = head_base + (long long)tg * tok_stride;
            unsigned off = lane_off[i];
            if (!full) {
                const int rr = min(tg + lane_row, t1 - 1) - tg;  // clamped row within the group
                off = (unsigned)(rr * (unsigned)tok_stride + (((lane & 15) ^ swz(g + lane_row)) << 4));
            }
            const char* src = (q < 16 ? kg : vg) + base + off;
            uint4* dst = lds + ((q < 16 ? kslot_bytes : vslot_bytes) + (q & 15) * 1024) / 16;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
        }
        fetch_pages(tile + 1);
    };

    // ---- per-lane LDS addresses of the MFMA operand fragments (relative to a tile) ---------------
    // K fragment (st, mb): row tl = 32 mb + col, piece (2 st + h) ^ swz(tl).  2 st has no bit 0 and
    // h is bit 0 only, so the piece is 2 st ^ (h ^ swz(tl)) and its byte offset 32 st ^ k_xor[mb].
    unsigned k_row[2], k_xor[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
        const int tl = 32 * mb + col;
        k_row[mb] = (unsigned)(tl * 256);
        k_xor[mb] = (unsigned)((h ^ swz(tl)) << 4);
    }
    // V fragment (ks, db), half `part`: source lane (r, q4) of a 16-lane group points at token
    // 16 ks + 8 part + 4 h + r, channels 32 db + 16 g16 + 4 q4 .. + 3; the transposing read then
    // hands lane i of the group the four tokens of channel 32 db + 16 g16 + i.  The token step
    // 16 ks only adds 4096 ks bytes (swz is periodic in 16) and goes into the offset field.
    unsigned v_off[4][2];
    {
        const int g16 = (lane >> 4) & 1, r = (lane & 15) >> 2, q4 = lane & 3;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int part = 0; part < 2; ++part) {
                const int tok = 8 * part + 4 * h + r;
                const int piece = 4 * db + 2 * g16 + (q4 >> 1);
                v_off[db][part] = (unsigned)(tok * 256 + ((piece ^ swz(tok)) << 4) + (q4 & 1) * 8);
            }
    }

    float m_run = -INFINITY, l_run = 0.f;
    floatx16 o[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i)
            o[db][i] = 0.f;
    floatx16 sacc[2];
    bf16x8 pf[4];  // P of the previous tile, B-operand layout

    // One MFMA region: the scores of the tile in stage `ks` (16 MFMAs) and, alternating with
    // them, O^T += V^T P^T for the previous tile in stage `vs` (16 more).  The two products are
    // independent, so their accumulator chains hide each other's latency.  Fragments are read
    // kAhead ahead of their MFMA.
    // Ring of fragment registers: kAhead + 1 reads in flight, and one more slot so that a new
    // read never targets the registers of the MFMA issued just before it.
    // A K fragment is one 128-bit read into `ring`; a V fragment is two 64-bit reads into
    // `ring_lo` / `ring_hi`, put together only after the wait that precedes its MFMA (the wait
    // names all of them as operands, so nothing that reads a fragment register can be placed
    // before the data has arrived).  What remains an assumption is that the compiler neither copies
    // nor spills a fragment register between its read and that wait; the kernels built from this
    // body use no scratch memory, and a host-side test of the build keeps it that way.
    u32x4 ring[kAhead + 2];
    u32x2 ring_lo[kAhead + 2], ring_hi[kAhead + 2];
    auto region = [&](auto qk_tag, auto pv_tag, int kstage, int vstage) __attribute__((always_inline)) {
        constexpr bool QK = decltype(qk_tag)::value, PV = decltype(pv_tag)::value;
        constexpr int NF = frag_count<QK, PV>();
        const unsigned kbase = lds_base + (unsigned)kstage * kTileBytes;
        const unsigned vbase = lds_base + (unsigned)(KS + vstage) * kTileBytes;
        if (QK) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    sacc[mb][i] = 0.f;
        }
        auto issue = [&](auto kc) __attribute__((always_inline)) {
            constexpr int K = decltype(kc)::value;
            if constexpr (K < NF) {
                using F = Frag<QK, PV, K>;
                if constexpr (!F::is_pv) {
                    const unsigned addr = kbase + k_row[F::b] + ((32u * F::a) ^ k_xor[F::b]);
                    u32x4& dst = ring[K % (kAhead + 2)];
                    asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(addr));
                } else {
                    u32x2& lo = ring_lo[K % (kAhead + 2)];
                    u32x2& hi = ring_hi[K % (kAhead + 2)];
                    const unsigned a0 = vbase + v_off[F::b][0], a1 = vbase + v_off[F::b][1];
                    asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%4\n\tds_read_b64_tr_b16 %1, %3 offset:%4"
                                 : "=&v"(lo), "=&v"(hi)
                                 : "v"(a0), "v"(a1), "n"(F::a * 4096));
                }
            }
        };
        auto consume = [&](auto kc) __attribute__((always_inline)) {
            constexpr int K = decltype(kc)::value;
            using F = Frag<QK, PV, K>;
            if constexpr (!F::is_pv) {
                u32x4& f = ring[K % (kAhead + 2)];
                asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(f) : "n"(ops_after<QK, PV, K>()));
                sacc[F::b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(f), qf[F::a], sacc[F::b], 0, 0, 0);
            } else {
                u32x2& lo = ring_lo[K % (kAhead + 2)];
                u32x2& hi = ring_hi[K % (kAhead + 2)];
                asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(lo), "+v"(hi) : "n"(ops_after<QK, PV, K>()));
                const u32x4 f = {lo[0], lo[1], hi[0], hi[1]};
                o[F::b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(f), pf[F::a], o[F::b], 0, 0, 0);
            }
        };
        for_each_index(issue, std::make_integer_sequence<int, kAhead + 1>{});
        for_each_index(
            [&](auto kc) __attribute__((always_inline)) {
                consume(kc);
                issue(std::integral_constant<int, decltype(kc)::value + kAhead + 1>{});
            },
            std::make_integer_sequence<int, NF>{});
    };

    // Online softmax of the scores in `sacc` (lane-local per row): updates (m, l), rescales O
    // (which already holds every earlier tile) and leaves P in `pf`.  Scores stay unscaled in
    // the accumulator; the scale is folded into the exponent: p = 2^(s * scale - m).
    auto softmax_tile = [&](int tb) __attribute__((always_inline)) {
        const bool full = tb + kTileN <= t1;  // only the last tile of a split can be ragged
        if (!full) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    // accumulator register i of lane-half h is token 32 mb + 8 (i/4) + 4 h + i%4
                    const int t = tb + 32 * mb + 8 * (i >> 2) + 4 * h + (i & 3);
                    if (t >= t1)
                        sacc[mb][i] = -INFINITY;
                }
        }
        float tmax = -INFINITY;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                tmax = fmaxf(tmax, sacc[mb][i]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32)) * p.scale_log2;
        // The reference maximum m only has to bound the exponents, so it is raised only when some
        // row of this wavefront exceeds it by more than kSlack (p <= 2^kSlack otherwise, exact in
        // fp32 and bf16 alike); the accumulators then need no rescale on most tiles.
        constexpr float kSlack = 8.f;
        const bool raise = __ballot(tmax > m_run + kSlack) != 0;
        float corr = 1.f;
        if (raise) {
            const float m_up = fmaxf(m_run, tmax);
            corr = __builtin_amdgcn_exp2f(m_run - m_up);
            m_run = m_up;
        }
        const float m_new = m_run;
        float psum = 0.f;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                float pv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    pv[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[mb][8 * u + e], p.scale_log2, -m_new));
                    psum += pv[e];
                }
                uint4 pu;
                pu.x = pack_bf16_rne(pv[0], pv[1]);
                pu.y = pack_bf16_rne(pv[2], pv[3]);
                pu.z = pack_bf16_rne(pv[4], pv[5]);
                pu.w = pack_bf16_rne(pv[6], pv[7]);
                pf[2 * mb + u] = as_bf16x8(pu);
            }
        l_run = l_run * corr + psum;
        if (raise) {
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    o[db][i] *= corr;
        }
    };

    // ---- pipeline over tiles ----------------------------------------------------------------------
    // Iteration `it` starts the copies of tile it+AHEAD, runs one MFMA region (scores of tile `it`
    // together with P V of tile it-1), waits until its own copies of tile it+1 have landed, meets
    // the other wavefronts at a barrier, then runs the softmax of tile `it`.
    const int ntiles = (t1 - t0 + kTileN - 1) / kTileN;
    const std::true_type yes{};
    const std::false_type no{};
    issue_tile(0);
    if (AHEAD == 2 && ntiles > 1)
        issue_tile(1);
    if (AHEAD == 2 && ntiles > 1)
        wait_vmcnt<kIPW>();
    else
        wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    // One barrier per tile, after the MFMA region (own copies of the next tile have landed by
    // then).  A copy into a ring slot is issued only after a barrier that every wavefront reaches
    // after its last read of that slot, and a tile is read only after a barrier that every
    // wavefront reaches after its copies of that tile landed.
    auto end_of_region = [&](int it) __attribute__((always_inline)) {
        if (it + 1 < ntiles) {
            if (AHEAD == 2 && it + 2 < ntiles)
                wait_vmcnt<kIPW>();
            else
                wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
        }
    };
    // first tile: scores only (kept out of the loop so that the loop body is one straight path)
    if (ntiles > AHEAD)
        issue_tile(AHEAD);
    region(yes, no, 0, 0);
    end_of_region(0);
    softmax_tile(t0);
    for (int it = 1; it < ntiles; ++it) {
        if (it + AHEAD < ntiles)
            issue_tile(it + AHEAD);
        region(yes, yes, it % KS, (it - 1) % VS);
        end_of_region(it);
        softmax_tile(t0 + it * kTileN);
    }
    region(no, yes, 0, (ntiles - 1) % VS);

    // ---- write the partial state ------------------------------------------------------------------
    const float l = l_run + __shfl_xor(l_run, 32);
    if (!row_ok)
        return;
    const long long prow = part_index(p, out_row, lv.slot0 + split);
    if (h == 0)
        p.part_ml[prow] = make_float2(m_run, l);
    // the split's own normalised output, fp16 (l > 0: a split holds at least one token)
    const float inv_l = 1.f / l;
    __half* dst = (__half*)p.part_acc + prow * kD;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            // registers 4 q4 .. 4 q4 + 3 are channels 32 db + 8 q4 + 4 h .. + 3
            const __half2 lo = __floats2half2_rn(o[db][4 * q4] * inv_l, o[db][4 * q4 + 1] * inv_l);
            const __half2 hi = __floats2half2_rn(o[db][4 * q4 + 2] * inv_l, o[db][4 * q4 + 3] * inv_l);
            uint2 v;
            v.x = *reinterpret_cast<const uint32_t*>(&lo);
            v.y = *reinterpret_cast<const uint32_t*>(&hi);
            *reinterpret_cast<uint2*>(dst + 32 * db + 8 * q4 + 4 * h) = v;
        }
}

}  // namespace prefix_impl
}  // namespace spd
