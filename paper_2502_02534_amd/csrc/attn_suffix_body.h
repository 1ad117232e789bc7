// Suffix pass (bf16, head_dim 128): streams each sample's private KV once.
//
// Work item = (sample n, KV head j, chunk of the suffix); one wavefront per item, four
// independent items per workgroup (no workgroup barriers).  The G query heads that
// share KV head j ride along as columns of one 16-wide MFMA tile, so the stream is
// read once for all of them.  Per 32-token tile:
//
//   S^T = K Q^T   v_mfma_f32_16x16x32_bf16, A = K rows (tokens) loaded from global memory
//                 straight into the operand layout (lane (c, r) takes 16 bytes of token
//                 16 blk + c at byte 64 s + 16 r for step s: four lanes cover one 64-byte
//                 stretch of a row), B = the G query rows (held in registers)
//   online softmax in the base-2 domain on the accumulator registers; the accumulator
//                 layout of S^T is exactly the A-operand layout of P, so P never moves
//   O += P V      B = V transposed inside each lane with byte permutes (a lane loads the
//                 same 16-byte column slice of 8 token rows and turns it into 8
//                 token-contiguous fragments)
//
// Global loads are 16 bytes per lane; for V 16 adjacent lanes cover one 256-byte row.  A whole
// tile is loaded from uniform bases plus per-lane offsets that are fixed for the chunk, so its
// sixteen loads cost no vector arithmetic; only a chunk's last, ragged tile clamps its rows.
// The next tile's loads are issued before the current tile is computed, and with paged KV the
// page numbers of the tile after that are fetched at the same time, so that no KV load waits
// for a page-table load.  The body uses no LDS.
// The running state is the deferred-division form of the paper's online-softmax
// recurrence (App., attn task 2): (m, l, unnormalised accumulator).
#pragma once

#include "spd_internal.h"

#include <hip/hip_fp16.h>

namespace spd {
namespace suffix_impl {


typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

constexpr int kD = 128;
constexpr int kTile = 32;        // tokens per tile
constexpr int kWavesPerBlock = 4;

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v)
{
    return *reinterpret_cast<bf16x8*>(&v);
}

// Token (relative to the tile) that load slot s (0..7) of lane-row r (0..3) covers.
// Slots 0..3 are tokens 4r..4r+3, slots 4..7 tokens 16+4r..16+4r+3: the same token
// set, in the same order, that the accumulator of S^T hands lane-row r.
__device__ __forceinline__ int tile_token(int r, int s) { return (s < 4 ? 0 : 12) + 4 * r + s; }

__device__ __forceinline__ uint32_t dword(const uint4& v, int k)
{
    return k == 0 ? v.x : k == 1 ? v.y : k == 2 ? v.z : v.w;
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Two floats to packed bf16 (round to nearest even): one v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    const bf16x2 r = __builtin_convertvector(v, bf16x2);
    return *reinterpret_cast<const uint32_t*>(&r);
}

// Body of one wavefront: work item `item`.  No LDS, no workgroup barriers.
template <bool PAGED>
__device__ __forceinline__ void suffix_body(const AttnParams& p, int slot0, long long item)
{

    const int lane = threadIdx.x & 63;
    const int r = lane >> 4, c = lane & 15;
    const int nc = p.num_suffix_chunks;
    const long long total = (long long)p.N * p.Hkv * nc;
    if (item >= total)
        return;
    // KV head fastest: the waves of a workgroup (and neighbouring workgroups) read the heads of
    // the same tokens at the same time, i.e. one contiguous stretch of the [token][head][D] cache
    const int j = (int)(item % p.Hkv);
    const int chunk = (int)((item / p.Hkv) % nc);
    const int n = (int)(item / ((long long)nc * p.Hkv));
    const int Ls = p.suffix_lens[n];
    const int t0 = chunk * p.suffix_chunk_tokens;
    const int t1 = min(Ls, t0 + p.suffix_chunk_tokens);
    const int G = p.G;
    if (t0 >= t1) {
        // empty chunk: l = 0 tells the merge to leave the slot out (its output part stays unwritten)
        if (r == 0 && c < G)
            p.part_ml[part_index(p, (long long)n * p.Hq + (long long)j * G + c, slot0 + chunk)] = make_float2(-INFINITY, 0.f);
        return;
    }

    const uint4* __restrict__ kg = (const uint4*)p.k_suffix;
    const uint4* __restrict__ vg = (const uint4*)p.v_suffix;
    const int* __restrict__ pages = PAGED ? p.suffix_pages + p.suffix_page_indptr[n] : nullptr;
    const int last_page = PAGED ? (Ls - 1) / 16 : 0;
    constexpr int kRow = kD * 2 / 16;  // uint4 per KV row

    // Page numbers of the two 16-token pages a tile covers (a tile starts on an even page).
    struct TilePages {
        long long a, b;
    };
    auto tile_pages = [&](int tb) -> TilePages {
        TilePages tp = {0, 0};
        if (PAGED) {
            tp.a = pages[min(tb >> 4, last_page)];
            tp.b = pages[min((tb >> 4) + 1, last_page)];
        }
        return tp;
    };
    // Query fragments: B operand, column n = query head j*G + c (zero beyond G),
    // k-slot (step s, lane-row r) = channels 32 s + 8 r .. + 7.
    bf16x8 qf[4];
    {
        const uint4* qg = (const uint4*)p.q + ((long long)n * p.Hq + (long long)j * G + (c < G ? c : 0)) * kRow;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            uint4 v = qg[4 * s + r];
            if (c >= G)
                v = make_uint4(0, 0, 0, 0);
            qf[s] = as_bf16x8(v);
        }
    }

    // K: register 4 blk + s of lane (c, r) = token 16 blk + c, channels 32 s + 8 r .. + 7 (the A operand of
    // step s for token block blk).  V: register s of lane (r, c) = token tile_token(r, s), 16-byte piece c.
    // Tokens past the end of the chunk are clamped to its last one (their scores are masked).
    // A whole tile is loaded from uniform bases (the tile's first row of this KV head; with paged KV
    // the first row of each of its two pages) plus 32-bit lane offsets fixed for the whole chunk,
    // so that a load costs no address arithmetic in the vector ALU; only the last, ragged tile of a
    // chunk takes the general path with its clamps.
    const unsigned row_bytes = PAGED ? 256u : (unsigned)p.Hkv * 256u;   // from one token row of the head to the next
    const unsigned koff = (unsigned)c * row_bytes + 16u * (unsigned)r;  // token c of a 16-token block, piece r (+ 64 s)
    const unsigned voff = (unsigned)(4 * r) * row_bytes + 16u * (unsigned)c;  // token 4 r (+ s rows), piece c
    uint4 kreg[8], vreg[8];
    auto load_tile = [&](int tb, const TilePages& tp, uint4 (&kk)[8], uint4 (&vv)[8]) __attribute__((always_inline)) {
        // row (of this KV head) of the tile's tokens 0 .. 15 and 16 .. 31, in units of 256 bytes
        const long long first = PAGED ? (tp.a * p.Hkv + j) * 16 : ((long long)n * p.max_suffix_len + tb) * p.Hkv + j;
        const long long second = PAGED ? (tp.b * p.Hkv + j) * 16 : first + 16ll * p.Hkv;
        const int last = t1 - 1 - tb;  // the tile's last valid token (uniform, >= 0)
        if (last >= kTile - 1) {
            const char* ka = (const char*)kg + first * 256;
            const char* kb = (const char*)kg + second * 256;
            const char* va = (const char*)vg + first * 256;
            const char* vb = (const char*)vg + second * 256;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                kk[s] = *reinterpret_cast<const uint4*>(ka + koff + 64 * s);
                kk[4 + s] = *reinterpret_cast<const uint4*>(kb + koff + 64 * s);
                // V register s holds token 4 r + s, register 4 + s token 16 + 4 r + s
                vv[s] = *reinterpret_cast<const uint4*>(va + (size_t)s * row_bytes + voff);
                vv[4 + s] = *reinterpret_cast<const uint4*>(vb + (size_t)s * row_bytes + voff);
            }
            return;
        }
        // the ragged last tile of a chunk: tokens past the end are clamped to the last one (their
        // scores are masked, and what is multiplied by their zero weights must be finite)
        const bool two = last >= 16;  // the second half holds valid tokens
        const long long sec = two ? second : first;
        const int last0 = two ? 15 : last, last1 = two ? last - 16 : last;  // clamps inside each half
        const char* ka = (const char*)kg + first * 256;
        const char* kb = (const char*)kg + sec * 256;
        const char* va = (const char*)vg + first * 256;
        const char* vb = (const char*)vg + sec * 256;
        const unsigned k0 = (unsigned)min(c, last0) * row_bytes + 16u * (unsigned)r;
        const unsigned k1 = (unsigned)(two ? min(c, last1) : last1) * row_bytes + 16u * (unsigned)r;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            kk[s] = *reinterpret_cast<const uint4*>(ka + k0 + 64 * s);
            kk[4 + s] = *reinterpret_cast<const uint4*>(kb + k1 + 64 * s);
            vv[s] = *reinterpret_cast<const uint4*>(va + (unsigned)min(4 * r + s, last0) * row_bytes + 16u * (unsigned)c);
            vv[4 + s] = *reinterpret_cast<const uint4*>(vb + (unsigned)(two ? min(4 * r + s, last1) : last1) * row_bytes +
                                                        16u * (unsigned)c);
        }
    };

    float m_run = -INFINITY;  // running maximum of query head c (replicated over lane-rows)
    float l_run = 0.f;        // this lane's share of the running sum
    floatx4 o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
        o[i] = floatx4{0.f, 0.f, 0.f, 0.f};

    // One tile: the next tile's loads go out first (into `knext` / `vnext`), then the scores, the
    // online softmax and P V of the tile held in `kcur` / `vcur`.  (Two register sets in swapped
    // roles, with the loop unrolled by two, would save the copy at the end of a round, but need
    // more registers than two wavefronts per SIMD leave.)
    TilePages pages_next = tile_pages(min(t0 + kTile, t1 - 1) & ~(kTile - 1));
    auto tile_step = [&](int tb, uint4 (&kcur)[8], uint4 (&vcur)[8], uint4 (&knext)[8], uint4 (&vnext)[8]) __attribute__((always_inline)) {
        if (tb + kTile < t1) {
            load_tile(tb + kTile, pages_next, knext, vnext);
            pages_next = tile_pages(min(tb + 2 * kTile, t1 - 1) & ~(kTile - 1));
        }

        // ---- S^T = K Q^T for the two 16-token blocks ---------------------------------------
        floatx4 sacc[2];
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            sacc[blk] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                sacc[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kcur[4 * blk + s]), qf[s], sacc[blk], 0, 0, 0);
            }
        }
        // lane (c, r) register (blk, i) = score of token tb + 16 blk + 4 r + i for head c;
        // scores stay unscaled, the scale is folded into the exponent: p = 2^(s * scale - m)
        float sv[8];
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                sv[4 * blk + i] = sacc[blk][i];
        if (tb + kTile > t1) {  // only the last tile of a chunk can be ragged
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (tb + 16 * blk + 4 * r + i >= t1)
                        sv[4 * blk + i] = -INFINITY;
        }
        float tmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            tmax = fmaxf(tmax, sv[i]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m_run, tmax * p.scale_log2);  // finite: the tile holds a valid token
        const float corr = __builtin_amdgcn_exp2f(m_run - m_new);  // 0 on the first tile
        float psum = 0.f;
        float pv[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            pv[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[i], p.scale_log2, -m_new));
            psum += pv[i];
        }
        l_run = l_run * corr + psum;
        uint4 pu;
        pu.x = pack_bf16_rne(pv[0], pv[1]);
        pu.y = pack_bf16_rne(pv[2], pv[3]);
        pu.z = pack_bf16_rne(pv[4], pv[5]);
        pu.w = pack_bf16_rne(pv[6], pv[7]);
        const bf16x8 pf = as_bf16x8(pu);

        // ---- rescale the accumulator when some head's maximum moved ---------------------------
        if (__ballot(m_new != m_run)) {
            // accumulator register i of lane-row r belongs to query head 4 r + i
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float f = __shfl(corr, (4 * r + i) & 15);
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    o[k][i] *= f;
            }
        }
        m_run = m_new;

        // ---- O += P V: transpose V in registers, one MFMA per channel residue ------------------
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
            uint4 f;
            f.x = __builtin_amdgcn_perm(dword(vcur[1], i >> 1), dword(vcur[0], i >> 1), sel);
            f.y = __builtin_amdgcn_perm(dword(vcur[3], i >> 1), dword(vcur[2], i >> 1), sel);
            f.z = __builtin_amdgcn_perm(dword(vcur[5], i >> 1), dword(vcur[4], i >> 1), sel);
            f.w = __builtin_amdgcn_perm(dword(vcur[7], i >> 1), dword(vcur[6], i >> 1), sel);
            // column c of this MFMA is channel 8 c + i
            o[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf, as_bf16x8(f), o[i], 0, 0, 0);
        }
    };

    load_tile(t0, tile_pages(t0), kreg, vreg);
    for (int tb = t0; tb < t1; tb += kTile) {
        uint4 knext[8], vnext[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            knext[s] = make_uint4(0, 0, 0, 0);
            vnext[s] = make_uint4(0, 0, 0, 0);
        }
        tile_step(tb, kreg, vreg, knext, vnext);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            kreg[s] = knext[s];
            vreg[s] = vnext[s];
        }
    }

    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);

    // ---- write the partial state ----------------------------------------------------------------
    const long long row0 = (long long)n * p.Hq + (long long)j * G;  // first of the G output rows
    if (r == 0 && c < G)
        p.part_ml[part_index(p, row0 + c, slot0 + chunk)] = make_float2(m_run, l_run);
    // the chunk's own normalised output, fp16: accumulator register i of lane-row r belongs to
    // query head 4 r + i, whose l sits in the lanes with c == 4 r + i
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int g = 4 * r + i;
        const float lg = __shfl(l_run, g & 15);
        if (g < G) {
            const float inv_l = 1.f / lg;  // > 0: the chunk holds at least one token
            __half* dst = (__half*)p.part_acc + part_index(p, row0 + g, slot0 + chunk) * kD + 8 * c;
            uint4 v;
            __half2 h2;
            h2 = __floats2half2_rn(o[0][i] * inv_l, o[1][i] * inv_l);
            v.x = *reinterpret_cast<const uint32_t*>(&h2);
            h2 = __floats2half2_rn(o[2][i] * inv_l, o[3][i] * inv_l);
            v.y = *reinterpret_cast<const uint32_t*>(&h2);
            h2 = __floats2half2_rn(o[4][i] * inv_l, o[5][i] * inv_l);
            v.z = *reinterpret_cast<const uint32_t*>(&h2);
            h2 = __floats2half2_rn(o[6][i] * inv_l, o[7][i] * inv_l);
            v.w = *reinterpret_cast<const uint32_t*>(&h2);
            *reinterpret_cast<uint4*>(dst) = v;
        }
    }
}

}  // namespace suffix_impl
}  // namespace spd
