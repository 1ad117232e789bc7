// Prefix (cascade) pass (bf16, head_dim 128): all samples' queries of one KV head form
// a dense row tile against the shared prompt KV, so the prompt is read once per row
// tile instead of once per sample.
//
// Workgroup = (prompt b, KV head j, tile of 32*WAVES query rows, split of the prefix).
// A query row is (sample, head in group); each wavefront owns 32 rows (one 32-wide
// column block of the transposed product), two wavefronts share a SIMD so that one's
// softmax overlaps the other's MFMAs.  K and V tiles of 64 tokens are loaded
// cooperatively, 16 bytes per lane with 16 adjacent lanes per 256-byte row, and
// triple-buffered in LDS:
//   K  row-major [token][channel] (padded rows), read as the A operand of
//      S^T = K Q^T          (v_mfma_f32_32x32x16_bf16, B = query rows, in registers)
//   V  transposed on the way in: a lane loads the same 8-channel slice of 8 token rows,
//      transposes the 8x8 block with byte permutes and stores 8 token-contiguous
//      fragments, read as the A operand of
//      O^T += V^T P^T       (B = P, which is the S^T accumulator itself, repacked to bf16)
// Every lane owns one query row in both products, so the online-softmax statistics and
// the accumulator rescale are lane-local.  The running state is the deferred-division
// form of the paper's online-softmax recurrence (App., attn task 2).
#include "spd_internal.h"

#include <type_traits>

namespace spd {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int kD = 128;
constexpr int kTileN = 64;    // tokens per tile
constexpr int kKRowU4 = 17;   // K tile row: 16 x 16 B + 16 B pad
constexpr int kVRowU4 = 9;    // V^T tile row (one channel): 8 fragments x 16 B + 16 B pad
constexpr int kRowU4 = kD * 2 / 16;

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return *reinterpret_cast<bf16x8*>(&v); }

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

// Token (relative to the tile) of element e (0..7) of V fragment f (0..7).  Fragment
// f = 2 ks + h feeds k-step ks, lane-half h, and must list the tokens in the order the
// S^T accumulator hands them to that lane-half: 16 ks + {4h..4h+3, 8+4h..8+4h+3}.
__device__ __forceinline__ int frag_token(int f, int e)
{
    return 16 * (f >> 1) + 4 * (f & 1) + (e < 4 ? e : e + 4);
}

template <int WAVES, int NB, bool PAGED>
__global__ __launch_bounds__(WAVES * 64) void attn_prefix_mfma_kernel(AttnParams p)
{
    constexpr int kThreads = WAVES * 64;
    constexpr int kRowsPerWave = 32 * NB;
    constexpr int kTasks = (256 + kThreads - 1) / kThreads;  // load tasks per thread per tile
    // With 512 threads a tile needs only half of them: threads 0..255 carry the even tiles and
    // threads 256..511 the odd ones, so every load has two iterations to arrive (twice the
    // bytes in flight for the same registers).
    constexpr bool kDeep = (kThreads == 512);
    __shared__ uint4 ksm[3][kTileN][kKRowU4];
    __shared__ uint4 vsm[3][kD][kVRowU4];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, h = lane >> 5;

    const int split = blockIdx.x, rowtile = blockIdx.y;
    const int b = blockIdx.z / p.Hkv, j = blockIdx.z % p.Hkv;
    const int s0 = p.sample_indptr[b];
    const int rows_b = (p.sample_indptr[b + 1] - s0) * p.G;
    const int row0 = rowtile * kRowsPerWave * WAVES;
    const int Lp = p.prefix_lens[b];
    const int t0 = split * p.prefix_split_tokens;
    const int t1 = min(Lp, t0 + p.prefix_split_tokens);
    if (row0 >= rows_b || t0 >= t1)
        return;

    const uint4* __restrict__ kg = (const uint4*)p.k_prefix;
    const uint4* __restrict__ vg = (const uint4*)p.v_prefix;
    const int* __restrict__ pages = PAGED ? p.prefix_pages + p.prefix_indptr[b] : nullptr;
    const long long start = PAGED ? 0 : p.prefix_indptr[b];

    auto row_index = [&](int t, int piece) -> long long {
        if (PAGED) {
            const long long pg = pages[t >> 4];
            return ((pg * p.Hkv + j) * 16 + (t & 15)) * kRowU4 + piece;
        }
        return ((start + t) * p.Hkv + j) * kRowU4 + piece;
    };

    // ---- query fragments (B operand): column = this lane's row, k-slot = channels 16 s + 8 h
    bf16x8 qf[NB][8];
    long long out_row[NB];
    bool row_ok[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int rr = row0 + wave * kRowsPerWave + nb * 32 + col;
        row_ok[nb] = rr < rows_b;
        const int sample = s0 + (row_ok[nb] ? rr : 0) / p.G;
        const int head = j * p.G + (row_ok[nb] ? rr : 0) % p.G;
        out_row[nb] = (long long)sample * p.Hq + head;
        const uint4* qg = (const uint4*)p.q + out_row[nb] * kRowU4;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            uint4 v = qg[2 * s + h];
            if (!row_ok[nb])
                v = make_uint4(0, 0, 0, 0);
            qf[nb][s] = as_bf16x8(v);
        }
    }

    // ---- cooperative tile loads ---------------------------------------------------------------
    // task 0..127: K rows 8 (task/16) .. + 7, piece task % 16
    // task 128..255: V fragment (task-128)/16, piece (task-128) % 16
    // The 8 loads of a task are issued two tiles ahead of their use and parked in registers.
    uint4 stage[kTasks][8];
#pragma unroll
    for (int k = 0; k < kTasks; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e)
            stage[k][e] = make_uint4(0, 0, 0, 0);
    auto issue_loads = [&](int tb) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < kTasks; ++k) {
            const int task = kDeep ? (tid & 255) : tid + k * kThreads;
            if (task < 256) {
                const int piece = task & 15;
                const int grp = (task >> 4) & 7;
                const bool is_v = task >= 128;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int tl = is_v ? frag_token(grp, e) : 8 * grp + e;
                    const int t = min(tb + tl, t1 - 1);
                    const long long idx = row_index(t, piece);
                    stage[k][e] = is_v ? vg[idx] : kg[idx];
                }
            }
        }
    };
    auto store_tile = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < kTasks; ++k) {
            const int task = kDeep ? (tid & 255) : tid + k * kThreads;
            const int piece = task & 15;
            const int grp = (task >> 4) & 7;
            if (task < 128) {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    ksm[buf][8 * grp + e][piece] = stage[k][e];
            } else if (task < 256) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
                    uint4 f;
                    f.x = __builtin_amdgcn_perm(dword(stage[k][1], i >> 1), dword(stage[k][0], i >> 1), sel);
                    f.y = __builtin_amdgcn_perm(dword(stage[k][3], i >> 1), dword(stage[k][2], i >> 1), sel);
                    f.z = __builtin_amdgcn_perm(dword(stage[k][5], i >> 1), dword(stage[k][4], i >> 1), sel);
                    f.w = __builtin_amdgcn_perm(dword(stage[k][7], i >> 1), dword(stage[k][6], i >> 1), sel);
                    // channel 8 piece + i; fragment slot swizzled by the channel group
                    vsm[buf][8 * piece + i][grp ^ (piece & 7)] = f;
                }
            }
        }
    };
    float m_run[NB], l_run[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        m_run[nb] = -INFINITY;
        l_run[nb] = 0.f;
    }
    floatx16 o[4][NB];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                o[db][nb][i] = 0.f;
    floatx16 sacc[2][NB];
    bf16x8 pf[NB][4];  // P of the previous tile, B-operand layout

    // One MFMA region: the scores of tile `kbuf` (S^T = K Q^T, 16 MFMAs per column block) and,
    // interleaved with them, O^T += V^T P^T for the previous tile `vbuf` (16 more).  The two
    // products are independent, so their accumulator chains hide each other's latency; the
    // scheduler is asked for a fragment pipeline (a few LDS reads up front, then one read per
    // MFMA) so that no MFMA waits for the read issued right before it.
    auto mfma_region = [&](auto do_qk, auto do_pv, int kbuf, int vbuf) __attribute__((always_inline)) {
        constexpr bool QK = decltype(do_qk)::value, PV = decltype(do_pv)::value;
        if (QK) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        sacc[mb][nb][i] = 0.f;
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            if (QK) {
                const int st = k >> 1, mb = k & 1;
                const bf16x8 kf = as_bf16x8(ksm[kbuf][32 * mb + col][2 * st + h]);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    sacc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[nb][st], sacc[mb][nb], 0, 0, 0);
            }
            if (PV) {
                const int ks = k >> 2, db = k & 3;
                const int ch = 32 * db + col;
                const bf16x8 vf = as_bf16x8(vsm[vbuf][ch][(2 * ks + h) ^ ((ch >> 3) & 7)]);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    o[db][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[nb][ks], o[db][nb], 0, 0, 0);
            }
        }
        constexpr int kFrags = (QK ? 16 : 0) + (PV ? 16 : 0);
        constexpr int kAhead = 6;
        __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);
#pragma unroll
        for (int k = 0; k < kFrags - kAhead; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x008, NB, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, kAhead * NB, 0);
    };

    // Online softmax of the scores in `sacc` (lane-local per row): updates (m, l), rescales O
    // (which already holds every earlier tile) and leaves P in `pf`.  Scores stay unscaled in
    // the accumulator; the scale is folded into the exponent: p = 2^(s * scale - m).
    auto softmax_tile = [&](int tb) __attribute__((always_inline)) {
        const bool full = tb + kTileN <= t1;  // only the last tile of a split can be ragged
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            if (!full) {
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        // accumulator register i of lane-half h is token 32 mb + 8 (i/4) + 4 h + i%4
                        const int t = tb + 32 * mb + 8 * (i >> 2) + 4 * h + (i & 3);
                        if (t >= t1)
                            sacc[mb][nb][i] = -INFINITY;
                    }
            }
            float tmax = -INFINITY;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    tmax = fmaxf(tmax, sacc[mb][nb][i]);
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            const float m_new = fmaxf(m_run[nb], tmax * p.scale_log2);
            const float corr = __builtin_amdgcn_exp2f(m_run[nb] - m_new);
            m_run[nb] = m_new;
            float psum = 0.f;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    float pv[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        pv[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[mb][nb][8 * u + e], p.scale_log2, -m_new));
                        psum += pv[e];
                    }
                    uint4 pu;
                    pu.x = pack_bf16_rne(pv[0], pv[1]);
                    pu.y = pack_bf16_rne(pv[2], pv[3]);
                    pu.z = pack_bf16_rne(pv[4], pv[5]);
                    pu.w = pack_bf16_rne(pv[6], pv[7]);
                    pf[nb][2 * mb + u] = as_bf16x8(pu);
                }
            l_run[nb] = l_run[nb] * corr + psum;
            if (__ballot(corr != 1.f)) {
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        o[db][nb][i] *= corr;
            }
        }
    };

    // Pipeline over tiles (three LDS buffers).  Iteration `it` issues the global loads of tile
    // it+1, runs one MFMA region (scores of tile `it` together with P V of tile it-1), then the
    // softmax of tile `it` on the vector ALU (which the other wavefront of the SIMD overlaps
    // with its own MFMA region), and parks tile it+1 in LDS.  One barrier per tile.
    const int ntiles = (t1 - t0 + kTileN - 1) / kTileN;
    const std::true_type yes{};
    const std::false_type no{};
    const int half = kDeep ? (tid >> 8) : 0;  // which tiles this thread carries (deep mode)
    auto mine = [&](int tile) { return !kDeep || (tile & 1) == half; };
    if (mine(0))
        issue_loads(t0);
    if (kDeep && mine(1) && ntiles > 1)
        issue_loads(t0 + kTileN);
    if (mine(0))
        store_tile(0);
    if (!kDeep && ntiles > 1)
        issue_loads(t0 + kTileN);
    if (kDeep && mine(2) && ntiles > 2)
        issue_loads(t0 + 2 * kTileN);
    __syncthreads();
    mfma_region(yes, no, 0, 0);
    softmax_tile(t0);
    if (ntiles > 1) {
        if (mine(1))
            store_tile(1);
        __syncthreads();
    }
    for (int it = 1; it < ntiles; ++it) {
        const int tb = t0 + it * kTileN;
        if (kDeep) {
            if (mine(it + 2) && it + 2 < ntiles)
                issue_loads(tb + 2 * kTileN);
        } else if (it + 1 < ntiles) {
            issue_loads(tb + kTileN);
        }
        mfma_region(yes, yes, it % 3, (it - 1) % 3);
        softmax_tile(tb);
        if (it + 1 < ntiles) {
            if (mine(it + 1))
                store_tile((it + 1) % 3);
            __syncthreads();
        }
    }
    mfma_region(no, yes, 0, (ntiles - 1) % 3);

    // ---- write the partial state ------------------------------------------------------------------
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const float l = l_run[nb] + __shfl_xor(l_run[nb], 32);
        if (!row_ok[nb])
            continue;
        const long long prow = part_index(p, out_row[nb], split);
        if (h == 0)
            p.part_ml[prow] = make_float2(m_run[nb], l);
        float* dst = p.part_acc + prow * kD;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                // registers 4 q4 .. 4 q4 + 3 are channels 32 db + 8 q4 + 4 h .. + 3
                float4 v = make_float4(o[db][nb][4 * q4], o[db][nb][4 * q4 + 1], o[db][nb][4 * q4 + 2],
                                       o[db][nb][4 * q4 + 3]);
                *reinterpret_cast<float4*>(dst + 32 * db + 8 * q4 + 4 * h) = v;
            }
    }
}

template <int WAVES>
hipError_t launch_waves(const AttnParams& p, hipStream_t s)
{
    constexpr int kBlockRows = 32 * WAVES;
    const int rowtiles = (p.max_spp * p.G + kBlockRows - 1) / kBlockRows;
    const dim3 grid(p.num_prefix_splits, rowtiles, p.B * p.Hkv);
    if (p.page_size)
        hipLaunchKernelGGL((attn_prefix_mfma_kernel<WAVES, 1, true>), grid, dim3(WAVES * 64), 0, s, p);
    else
        hipLaunchKernelGGL((attn_prefix_mfma_kernel<WAVES, 1, false>), grid, dim3(WAVES * 64), 0, s, p);
    return hipGetLastError();
}

}  // namespace

bool prefix_mfma_supported(const AttnParams& p)
{
    return p.dtype == 1 && p.D == kD && p.prefix_split_tokens % kTileN == 0 &&
           (long long)p.B * p.Hkv <= 65535;
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
