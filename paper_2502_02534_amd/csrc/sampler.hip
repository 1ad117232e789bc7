// Temperature / nucleus / inverse-CDF token sampler.
//
// Two paths.  The sliced path (below: two stream-ordered kernels, four for launches with many
// workgroups) reads a row from HBM once, takes a second look that caches serve when the logits
// fit, and finds the exact nucleus threshold without sorting.  The whole-row routine (one
// workgroup per row, every pass from memory) covers what the sliced path does not take: unaligned
// rows, vocabularies beyond 16 slices, the rare row whose candidate set overflows, and rows with
// a min-p or top-k filter.
//
// Probabilities are evaluated by one shared routine, p_i = 2^((x_i - max) c) with
// c = log2(e)/T carried as hi + lo floats, so every pass sees the same bits; every sum that
// decides something is carried in fp64; comparisons that define the kept set are on bit
// patterns, so all ties with the threshold are kept by construction.
#include "spd_internal.h"

#include <cstdlib>

namespace spd {
namespace {

constexpr int kBlock = 512;
constexpr int kWaves = kBlock / 64;
constexpr int kBins = 2048;
constexpr int kSeg = 256;           // elements per wave per tile (64 lanes x 4)
constexpr int kTile = kWaves * kSeg;  // elements per block iteration (64 lanes x 4 per wave)
constexpr int kMaxSegments = 1024;    // vocab <= 262144

struct RowScale {
    float max_x, c_hi, c_lo;
};

__device__ __forceinline__ float prob(float x, const RowScale& r)
{
    const float d = x - r.max_x;
    const float y = __builtin_fmaf(d, r.c_hi, d * r.c_lo);
    return __builtin_amdgcn_exp2f(y);
}

__device__ __forceinline__ double wave_sum_f64(double v)
{
    for (int o = 32; o > 0; o >>= 1)
        v += __shfl_xor(v, o);
    return v;
}

// Block-wide sum in fp64 with a fixed reduction tree (deterministic).
__device__ double block_sum_f64(double v, double* scratch /* kWaves */)
{
    v = wave_sum_f64(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0)
        scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < kWaves; ++w)
        t += scratch[w];
    return t;
}

// Chooses the refinement bin: the highest non-empty bin b whose cumulative mass
// c(b) = above + sum_{b' >= b} hist[b'] reaches `need`.  If rounding leaves even the
// total short of `need`, the lowest non-empty bin is taken (everything is kept).
// Results are left in *bin_out and *above_out (mass strictly above the chosen bin).
// Thread t owns the kBinsPerThread consecutive bins just below kBins - t * kBinsPerThread.
constexpr int kBinsPerThread = kBins / kBlock;

__device__ void pick_bin(const double* hist, double above, double need, int* bin_out,
                         int* low_out, double* above_out, double* scratch /* kWaves */)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int top = kBins - 1 - kBinsPerThread * tid;
    __syncthreads();  // callers may have just used `scratch` and the output slots
    double h[kBinsPerThread];
    double own = 0.0;
#pragma unroll
    for (int k = 0; k < kBinsPerThread; ++k) {
        h[k] = hist[top - k];
        own += h[k];
    }
    double incl = own;
    for (int o = 1; o < 64; o <<= 1) {
        const double up = __shfl_up(incl, o);
        if (lane >= o)
            incl += up;
    }
    if (tid == 0) {
        *bin_out = -1;
        *low_out = kBins;
    }
    if (lane == 63)
        scratch[wave] = incl;
    __syncthreads();
    double before = above + (incl - own);
    for (int w = 0; w < wave; ++w)
        before += scratch[w];
    int best = -1, low = kBins;
#pragma unroll
    for (int k = 0; k < kBinsPerThread; ++k) {
        if (h[k] > 0.0) {
            low = top - k;
            if (best < 0 && before + h[k] >= need)
                best = top - k;
        }
        if (best < 0)
            before += h[k];
    }
    // `before` now holds the mass strictly above `best` (when this thread found one)
    if (best >= 0)
        atomicMax(bin_out, best);
    if (low < kBins)
        atomicMin(low_out, low);
    __syncthreads();
    const int chosen = *bin_out >= 0 ? *bin_out : (*low_out < kBins ? *low_out : 0);
    const bool fallback = *bin_out < 0;
    __syncthreads();
    if (!fallback) {
        if (best == chosen)
            *above_out = before;
    } else if (chosen <= top && chosen > top - kBinsPerThread) {
        // everything above the lowest non-empty bin
        double b2 = above + (incl - own);
        for (int w = 0; w < wave; ++w)
            b2 += scratch[w];
        for (int k = 0; k < top - chosen; ++k)
            b2 += h[k];
        *above_out = b2;
    }
    if (tid == 0)
        *bin_out = chosen;
    __syncthreads();
}

// Shared-memory arrays of the row routines (one instance per workgroup).
struct RowLds {
    double hist[kBins];
    double scratch[kBlock];  // block sums and scans use the first kWaves entries
    double seg_mass[kMaxSegments];
    float red_f[kWaves];
    int red_i[kWaves];
    int sh_low;
    int sh_bin;
    double sh_above;
    int sh_token;
};

// Whole-row routine for one workgroup of kBlock threads: every pass reads the row from
// global memory.  Used when the sliced kernel cannot take a row (unaligned rows, very
// large vocabularies, candidate overflow).
__device__ void sample_row_from_memory(const SamplerParams& sp, long long r, RowLds& L)
{
    double* hist = L.hist;
    double* scratch = L.scratch;
    double* seg_mass = L.seg_mass;
    float* red_f = L.red_f;
    int* red_i = L.red_i;
    int& sh_low = L.sh_low;
    int& sh_bin = L.sh_bin;
    double& sh_above = L.sh_above;
    int& sh_token = L.sh_token;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* __restrict__ x = sp.logits + r * sp.stride;
    const int V = (int)sp.vocab;
    const float T = sp.temperature[r];

    // ---- pass 1: maximum and its lowest index -------------------------------------------
    float mx = -INFINITY;
    int mi = 0x7fffffff;
    for (int i = tid; i < V; i += kBlock) {
        const float v = x[i];
        if (v > mx) {
            mx = v;
            mi = i;
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(mx, o);
        const int oi = __shfl_xor(mi, o);
        if (ov > mx || (ov == mx && oi < mi)) {
            mx = ov;
            mi = oi;
        }
    }
    if (lane == 0) {
        red_f[wave] = mx;
        red_i[wave] = mi;
    }
    __syncthreads();
    mx = red_f[0];
    mi = red_i[0];
    for (int w = 1; w < kWaves; ++w) {
        if (red_f[w] > mx || (red_f[w] == mx && red_i[w] < mi)) {
            mx = red_f[w];
            mi = red_i[w];
        }
    }
    if (T == 0.f) {
        if (tid == 0)
            sp.tokens[r] = mi;
        return;
    }

    RowScale rs;
    rs.max_x = mx;
    {
        const double c = 1.4426950408889634 / (double)T;
        rs.c_hi = (float)c;
        rs.c_lo = (float)(c - (double)rs.c_hi);
    }

    // ---- filters ahead of the nucleus: a lower bound `lb_bits` on the bit pattern of p ----------
    // (p > 0, so patterns order like values.)  min-p: p >= min_p, and the maximum has p = 1.
    // top-k: the k-th largest pattern among what min-p left, found by radix select on counts;
    // every tie with it is kept.
    const float top_p = sp.top_p[r];
    const bool cut = top_p < 1.f;
    const float min_p = sp.min_p ? sp.min_p[r] : 0.f;
    const int top_k = sp.top_k ? sp.top_k[r] : 0;
    uint32_t lb_bits = min_p > 0.f ? __float_as_uint(min_p) : 0u;

    // Radix select over the patterns >= lb (bits 30..20, 19..9, 8..0): the highest pattern whose
    // upper set reaches `need`, counting tokens (`by_count`) or summing their probabilities.
    auto select = [&](bool by_count, double need, uint32_t lb) -> uint32_t {
        uint32_t prefix = 0u;
        double above = 0.0;
        for (int level = 0; level < 3; ++level) {
            const int shift = level == 0 ? 20 : level == 1 ? 9 : 0;
            const int bits = level == 2 ? 9 : 11;
            for (int b = tid; b < kBins; b += kBlock)
                hist[b] = 0.0;
            __syncthreads();
            for (int i = tid; i < V; i += kBlock) {
                const float pv = prob(x[i], rs);
                const uint32_t u = __float_as_uint(pv) & 0x7fffffffu;
                if (u >= lb && (level == 0 || (u >> (shift + bits)) == prefix))
                    atomicAdd(&hist[(u >> shift) & ((1u << bits) - 1u)], by_count ? 1.0 : (double)pv);
            }
            __syncthreads();
            pick_bin(hist, above, need, &sh_bin, &sh_low, &sh_above, scratch);
            prefix = (prefix << bits) | (uint32_t)sh_bin;
            above = sh_above;
            __syncthreads();
        }
        return prefix;
    };
    if (top_k > 0)
        lb_bits = max(lb_bits, select(true, (double)top_k, lb_bits));

    // ---- pass 2: mass of what the filters left; nucleus threshold among it --------------------------
    double part = 0.0;
    {
        float acc = 0.f;
        int cnt = 0;
        for (int i = tid; i < V; i += kBlock) {
            const float pv = prob(x[i], rs);
            if ((__float_as_uint(pv) & 0x7fffffffu) < lb_bits)
                continue;
            acc += pv;
            if (++cnt == 32) {  // bound the fp32 run length before widening
                part += (double)acc;
                acc = 0.f;
                cnt = 0;
            }
        }
        part += (double)acc;
    }
    const double S = block_sum_f64(part, scratch);

    uint32_t tau_bits = lb_bits;  // keep everything the filters left
    double Z = S;
    if (cut)
        tau_bits = max(lb_bits, select(false, (double)top_p * S, lb_bits));

    // ---- pass 3: kept mass per 256-element segment, in vocabulary order -----------------
    const int num_tiles = (V + kTile - 1) / kTile;
    double z_part = 0.0;
    for (int tile = 0; tile < num_tiles; ++tile) {
        const int base = tile * kTile + wave * kSeg + lane * 4;
        float s4 = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int i = base + k;
            if (i < V) {
                const float pv = prob(x[i], rs);
                if (__float_as_uint(pv) >= tau_bits)
                    s4 += pv;
            }
        }
        const double ws = wave_sum_f64((double)s4);
        if (lane == 0)
            seg_mass[tile * kWaves + wave] = ws;  // vocab <= kMaxSegments * kSeg checked on the host
        z_part += (lane == 0) ? ws : 0.0;
    }
    Z = block_sum_f64(z_part, scratch);
    const double target = (double)sp.uniforms[r] * Z;

    // ---- scan the segments (one wave), then walk inside the hit segment ------------------
    if (wave == 0) {
        const int nseg = num_tiles * kWaves;
        const int per = (nseg + 63) / 64;  // consecutive segments per lane
        double mine = 0.0;
        for (int k = 0; k < per; ++k) {
            const int sidx = lane * per + k;
            if (sidx < nseg)
                mine += seg_mass[sidx];
        }
        double incl = mine;
        for (int o = 1; o < 64; o <<= 1) {
            const double up = __shfl_up(incl, o);
            if (lane >= o)
                incl += up;
        }
        const double before_lane = incl - mine;
        // first lane whose inclusive mass exceeds the target
        const unsigned long long hit = __ballot(incl > target);
        int seg = -1;
        double before = 0.0;
        if (hit) {
            const int hl = __ffsll((long long)hit) - 1;
            double run = __shfl(before_lane, hl);
            // walk that lane's few segments (every lane does it redundantly)
            for (int k = 0; k < per; ++k) {
                const int sidx = hl * per + k;
                if (sidx >= nseg)
                    break;
                const double sm = seg_mass[sidx];
                if (run + sm > target) {
                    seg = sidx;
                    before = run;
                    break;
                }
                run += sm;
            }
        }
        int token = -1;
        if (seg >= 0) {
            const int base = seg * kSeg + lane * 4;
            float pv[4];
            bool keep[4];
            float s4 = 0.f;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int i = base + k;
                pv[k] = 0.f;
                keep[k] = false;
                if (i < V) {
                    const float q = prob(x[i], rs);
                    if (__float_as_uint(q) >= tau_bits) {
                        pv[k] = q;
                        keep[k] = true;
                        s4 += q;
                    }
                }
            }
            double incl2 = (double)s4;
            for (int o = 1; o < 64; o <<= 1) {
                const double up = __shfl_up(incl2, o);
                if (lane >= o)
                    incl2 += up;
            }
            double run = before + incl2 - (double)s4;
            int cand = 0x7fffffff;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (keep[k]) {
                    run += (double)pv[k];
                    if (run > target && cand == 0x7fffffff)
                        cand = base + k;
                }
            }
            for (int o = 32; o > 0; o >>= 1)
                cand = min(cand, __shfl_xor(cand, o));
            if (cand != 0x7fffffff)
                token = cand;
        }
        if (lane == 0)
            sh_token = token;
    }
    __syncthreads();
    if (sh_token >= 0) {
        if (tid == 0)
            sp.tokens[r] = sh_token;
        return;
    }
    // Rounding let the walk finish without crossing: return the last kept index.
    int last = -1;
    for (int i = tid; i < V; i += kBlock)
        if (__float_as_uint(prob(x[i], rs)) >= tau_bits)
            last = max(last, i);
    for (int o = 32; o > 0; o >>= 1)
        last = max(last, __shfl_xor(last, o));
    __syncthreads();
    if (lane == 0)
        red_i[wave] = last;
    __syncthreads();
    if (tid == 0) {
        int best = -1;
        for (int w = 0; w < kWaves; ++w)
            best = max(best, red_i[w]);
        sp.tokens[r] = best;
    }
}

// =============================================================================================
// Sliced path: a row is cut into `slices` contiguous pieces of at most kSliceMax elements and
// handled by two kernels in stream order (no workgroup ever waits for another):
//
//   hist    (rows x slices)  one HBM pass: slice maximum (and its lowest index) and a histogram
//           of scaled mass over bins of width 1/16 in log2 p.  The bin of a logit is
//           floor(x c 16), an integer function of x alone; a histogram built against the slice
//           maximum differs from one built against the row maximum by an integer shift.
//           Mass is accumulated in u32 fixed point relative to the bin's own reference
//           (q = 2^(frac/16) 2^15 in [32768, 34219]), which needs no maximum at all.
//   select  (rows x slices)  second look at the slice (served by cache when the logits fit).
//           Every workgroup first combines the row's slice histograms and picks the bin that
//           holds the nucleus cut, plus a neighbour when the estimate cannot decide (the same
//           arithmetic in every workgroup of a row, so they agree).  Then, with
//           p_i = 2^((x_i - row max) c) exactly as defined: slice mass in fp64, mass of the
//           certainly-kept elements per 256-element segment in vocabulary order, and the
//           elements of the cut bins as candidates (logit, index).  The workgroup of a row that
//           finishes last finds the exact threshold among the candidates by radix select on the
//           logit's bit pattern with fp64 masses, adds the kept candidates to their segments,
//           scans the segments and walks inside the segment that contains u * Z.
//
// What the workgroups of a row hand to the last one goes through memory with agent-scope
// accesses (written through, read past the local L2), ordered by an arrival counter.
// =============================================================================================
constexpr int kIter = kBlock * 4;         // elements one float4 per thread covers
constexpr int kSliceMax = 8 * kIter;      // elements per workgroup: 8 float4 per thread
constexpr int kMaxSlices = 16;
constexpr int kSegPerSlice = kSliceMax / kSeg;  // 64
constexpr int kCandCap = 4096;
constexpr int kPubBins = 1024;   // histogram bins a slice publishes (64 octaves below its maximum)
static_assert(kMaxSlices * kSegPerSlice <= kMaxSegments, "segment table too small");

struct SliceStat {
    float max_x;
    int argmax;
    double mass;    // sum of p over the slice (select kernel)
    double above;   // mass of certainly-kept elements (select kernel)
};

// Counters of a row, zeroed by the hist kernel for the select kernel that follows it.
struct RowCtl {
    unsigned arrived;     // workgroups of the row that have published their results
    unsigned cand_total;  // candidates appended so far
    int lo, hi;           // cut bins, when the per-row cut kernel ran
};

__host__ __device__ inline size_t sliced_row_bytes(int slices)
{
    return 256 + (size_t)slices * 64 + (size_t)slices * kPubBins * 4 + (size_t)slices * kSegPerSlice * 8 +
           (size_t)kCandCap * 8;
}

struct RowWs {
    RowCtl* ctl;
    SliceStat* stat;      // [slices], 64 B apart
    unsigned* hist;       // [slices][kPubBins]
    double* seg;          // [slices][kSegPerSlice]
    unsigned long long* cand;  // [kCandCap] logit bits | index << 32
};

__device__ __forceinline__ RowWs row_ws(char* base, long long row, int slices)
{
    char* p = base + row * sliced_row_bytes(slices);
    RowWs w;
    w.ctl = (RowCtl*)p;
    p += 256;
    w.stat = (SliceStat*)p;
    p += (size_t)slices * 64;
    w.hist = (unsigned*)p;
    p += (size_t)slices * kPubBins * 4;
    w.seg = (double*)p;
    p += (size_t)slices * kSegPerSlice * 8;
    w.cand = (unsigned long long*)p;
    return w;
}

__device__ __forceinline__ SliceStat* stat_at(const RowWs& w, int s)
{
    return (SliceStat*)((char*)w.stat + (size_t)s * 64);
}

// Agent-scope accesses for data that one workgroup writes and another reads inside one kernel:
// written through and read past the local L2, ordered by the row's arrival counter (the writer
// waits for its stores to be acknowledged before it counts).  A release / acquire pair on the
// counter instead was measured 13 us slower per call: an agent-scope release writes the L2 back.
// When the reader is a later kernel (`across_kernels`), ordinary stores do.
template <typename T> __device__ __forceinline__ void publish(T* p, T v, bool across_kernels)
{
    if (across_kernels)
        *p = v;
    else
        __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ __forceinline__ T observe(const T* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Monotone map of a float onto unsigned integers (larger float -> larger key).
__device__ __forceinline__ uint32_t order_key(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Bin coordinate of a logit: one multiply and a floor, the same in every kernel.
__device__ __forceinline__ float bin_coord(float x, float c16) { return floorf(x * c16); }

// Bin of a logit counted down from the bin of a maximum, clamped to [0, kBins-1].
__device__ __forceinline__ int bin_below(float kf_max, float kf)
{
    return (int)fminf(fmaxf(kf_max - kf, 0.f), (float)(kBins - 1));
}

struct RowConst {
    float c_hi, c_lo, c16;
    double cd;
};

__device__ __forceinline__ RowConst row_const(float T)
{
    RowConst k;
    k.cd = 1.4426950408889634 / (double)T;
    k.c_hi = (float)k.cd;
    k.c_lo = (float)(k.cd - (double)k.c_hi);
    k.c16 = k.c_hi * 16.f;
    return k;
}

// Loads the slice [e0, e1) of a row into 32 registers per thread (whole float4s only; lanes
// past the end hold -inf).  The last one to three logits of a row whose length is not a
// multiple of 4 (the "tail") are not loaded here: thread 0 handles them straight from memory.
struct SliceRange {
    int e0, e1, v4end, ntail;
};

__device__ __forceinline__ SliceRange slice_range(int slice, int slice_elems, int V)
{
    SliceRange g;
    g.e0 = slice * slice_elems;
    g.e1 = min(V, g.e0 + slice_elems);
    g.v4end = g.e1 & ~3;
    g.ntail = (g.e1 == V && g.e0 < V) ? (V & 3) : 0;
    return g;
}

// Every load is unconditional (lanes past the end re-read the slice's last float4), so that the
// hardware's in-order load counter stays exact for the compiler and later loads need not wait
// for these.  SPD_MASK_SLICE, applied where the values are first needed, replaces what lies
// past the end by -inf.  Every slice holds at least one whole float4 (the host sends rows
// shorter than that to the whole-row kernel, and slices are never shorter than about 2000).
#define SPD_LOAD_SLICE(xv, x, g, tid)                                                   \
    _Pragma("unroll") for (int j = 0; j < 8; ++j)                                       \
    {                                                                                   \
        const int i_ = (g).e0 + j * kIter + (tid) * 4;                                  \
        const float4 v_ = *reinterpret_cast<const float4*>((x) + min(i_, (g).v4end - 4)); \
        (xv)[4 * j] = v_.x;                                                             \
        (xv)[4 * j + 1] = v_.y;                                                         \
        (xv)[4 * j + 2] = v_.z;                                                         \
        (xv)[4 * j + 3] = v_.w;                                                         \
    }
#define SPD_MASK_SLICE(xv, g, tid)                                                      \
    _Pragma("unroll") for (int j = 0; j < 8; ++j)                                       \
    {                                                                                   \
        if (!((g).e0 + j * kIter + (tid) * 4 < (g).v4end)) {                            \
            (xv)[4 * j] = (xv)[4 * j + 1] = (xv)[4 * j + 2] = (xv)[4 * j + 3] = -INFINITY; \
        }                                                                               \
    }

// ---- kernel 1: slice maximum and histogram -----------------------------------------------------------
__global__ __launch_bounds__(kBlock) void sampler_hist_kernel(SamplerParams sp, char* ws, int slices,
                                                              int slice_elems)
{
    __shared__ unsigned hist[kPubBins];
    __shared__ float red_f[kWaves];
    __shared__ int red_i[kWaves];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long r = blockIdx.x / slices;
    const int slice = blockIdx.x % slices;
    const float* __restrict__ x = sp.logits + r * sp.stride;
    const SliceRange g = slice_range(slice, slice_elems, (int)sp.vocab);
    const RowWs W = row_ws(ws, r, slices);
    const float T = sp.temperature[r];
    const bool greedy = (T == 0.f);
    const bool cut = !greedy && sp.top_p[r] < 1.f;

    float xv[32];
    SPD_LOAD_SLICE(xv, x, g, tid)
    SPD_MASK_SLICE(xv, g, tid)
    if (slice == 0 && tid == 0) {
        W.ctl->arrived = 0u;
        W.ctl->cand_total = 0u;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int q = 0; q < 32; ++q)
        mx = fmaxf(mx, xv[q]);
    if (tid == 0)
        for (int k = 0; k < g.ntail; ++k)
            mx = fmaxf(mx, x[g.v4end + k]);
    for (int o = 32; o > 0; o >>= 1)
        mx = fmaxf(mx, __shfl_xor(mx, o));
    if (lane == 0)
        red_f[wave] = mx;
    for (int b = tid; b < kPubBins; b += kBlock)
        hist[b] = 0u;
    __syncthreads();
    mx = red_f[0];
    for (int w = 1; w < kWaves; ++w)
        mx = fmaxf(mx, red_f[w]);

    int mi = 0x7fffffff;
    if (greedy) {
#pragma unroll
        for (int q = 31; q >= 0; --q)
            if (xv[q] == mx)
                mi = g.e0 + (q >> 2) * kIter + tid * 4 + (q & 3);
        if (tid == 0)
            for (int k = g.ntail - 1; k >= 0; --k)
                if (x[g.v4end + k] == mx)
                    mi = min(mi, g.v4end + k);
        for (int o = 32; o > 0; o >>= 1)
            mi = min(mi, __shfl_xor(mi, o));
        if (lane == 0)
            red_i[wave] = mi;
        __syncthreads();
        for (int w = 0; w < kWaves; ++w)
            mi = min(mi, red_i[w]);
    }

    if (cut) {
        const RowConst rc = row_const(T);
        const float kf_loc = bin_coord(mx, rc.c16);
        auto add = [&](float xq) {
            const float t = xq * rc.c16;
            const float kf = floorf(t);
            const int b = min(bin_below(kf_loc, kf), kPubBins - 1);
            // mass relative to the bin's own reference 2^(kf/16): 2^(frac/16) in [1, 2^(1/16))
            const unsigned q = (unsigned)(__builtin_amdgcn_exp2f((t - kf) * 0.0625f) * 32768.f + 0.5f);
            atomicAdd(&hist[b], q);
        };
#pragma unroll
        for (int q = 0; q < 32; ++q)
            if (xv[q] != -INFINITY)
                add(xv[q]);
        if (tid == 0)
            for (int k = 0; k < g.ntail; ++k)
                add(x[g.v4end + k]);
        __syncthreads();  // histogram complete
        for (int b = tid; b < kPubBins; b += kBlock)
            W.hist[(size_t)slice * kPubBins + b] = hist[b];
    }
    if (tid == 0) {
        SliceStat* st = stat_at(W, slice);
        st->max_x = mx;
        st->argmax = mi;
    }
}

// ---- bin selection by one wavefront ----------------------------------------------------------------
// A histogram of kBins doubles in "rank order" (bin 0 = most probable) is kept transposed in
// LDS, bin b in slot (b & 31) * 64 + (b >> 5), so that lane l owns the 32 consecutive bins
// 32 l .. 32 l + 31 and the 64 lanes read consecutive slots.
__device__ __forceinline__ int rank_slot(int b) { return (b & 31) * 64 + (b >> 5); }

struct BinPick {
    int bin;        // first non-empty bin whose cumulative mass reaches `need`
    double above;   // mass strictly above it (including `above0`)
    double in_bin;  // its own mass
    double total;   // sum of the histogram
};

// Every lane of the calling wavefront returns the same result; no workgroup barrier is used, so
// all wavefronts of a workgroup may call it redundantly on a finished histogram.  With
// `relative`, `need` is a fraction of the histogram's total.  If rounding leaves even the total
// short of `need`, the last non-empty bin is taken (everything is kept).
__device__ __forceinline__ BinPick wave_pick(const double* H, double above0, double need, bool relative)
{
    const int lane = threadIdx.x & 63;
    double own = 0.0;
#pragma unroll 8
    for (int k = 0; k < 32; ++k)
        own += H[k * 64 + lane];
    double incl = own;
    for (int o = 1; o < 64; o <<= 1) {
        const double up = __shfl_up(incl, o);
        if (lane >= o)
            incl += up;
    }
    BinPick r;
    r.total = __shfl(incl, 63);
    if (relative)
        need *= r.total;
    const double before_lane = above0 + (incl - own);
    const unsigned long long nonempty = __ballot(own > 0.0);
    const unsigned long long hit = __ballot(own > 0.0 && before_lane + own >= need);
    r.bin = 0;
    r.above = above0;
    r.in_bin = 0.0;
    if (!nonempty)
        return r;
    const int hl = hit ? __ffsll((long long)hit) - 1 : 63 - __clzll((long long)nonempty);
    // the 32 bins of lane hl, one per lane (both halves of the wavefront hold the same), scanned
    const double h = H[(lane & 31) * 64 + hl];
    double cum = h;
    for (int o = 1; o < 32; o <<= 1) {
        const double up = __shfl_up(cum, o);
        if ((lane & 31) >= o)
            cum += up;
    }
    cum += __shfl(before_lane, hl);
    const unsigned ne32 = (unsigned)__ballot(h > 0.0);
    const unsigned hit32 = hit ? (unsigned)__ballot(h > 0.0 && cum >= need) : 0u;
    // first bin that reaches `need`; else (rounding, or nothing reaches it) the last non-empty one
    const int k = hit32 ? __ffs((int)hit32) - 1 : 31 - __clz((int)ne32);
    r.bin = 32 * hl + k;
    r.in_bin = __shfl(h, k);
    r.above = __shfl(cum, k) - r.in_bin;
    return r;
}

// Two block-wide fp64 sums at once (fixed reduction tree).
__device__ void block_sum2_f64(double& a, double& b, double* scratch /* 2 kWaves */)
{
    a = wave_sum_f64(a);
    b = wave_sum_f64(b);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        scratch[threadIdx.x >> 6] = a;
        scratch[kWaves + (threadIdx.x >> 6)] = b;
    }
    __syncthreads();
    a = 0.0;
    b = 0.0;
    for (int w = 0; w < kWaves; ++w) {
        a += scratch[w];
        b += scratch[kWaves + w];
    }
}

// ---- kernel 2: cut bins, exact masses, candidates; last workgroup of a row: threshold and walk ----------
struct SelectLds {
    RowLds row;                           // hist / scratch / seg_mass of the row routines
    unsigned long long cand[kCandCap];    // candidates of the row (last workgroup only)
    double smass[kMaxSlices];
    double sabove[kMaxSlices];
    float smax[kMaxSlices];
    int sarg[kMaxSlices];
    int shift[kMaxSlices];
    int wave_cnt[kWaves];
    unsigned cand_base;
    unsigned arrived_before;
    uint32_t kmin[kWaves], kmax[kWaves];
};

// Estimate of the nucleus cut from the slices' histograms: the candidate bins [lo, hi] of the
// row, counted down from the bin of the row maximum.  Called by a whole workgroup; L.smax
// holds the slice maxima.  The arithmetic depends only on the row's data, so every workgroup
// that evaluates it for a row gets the same bins.
struct CutBins {
    int lo, hi;
};

__device__ __forceinline__ CutBins estimate_cut(SelectLds& L, const RowWs& W, int slices, float kf_row, const RowConst& rc,
                                float top_p)
{
    const int tid = threadIdx.x;
    int lo, hi;
    if (tid < slices)
        L.shift[tid] = L.smax[tid] == -INFINITY
                           ? kBins
                           : (int)fminf(fmaxf(kf_row - bin_coord(L.smax[tid], rc.c16), 0.f), (float)kBins);
    __syncthreads();
    // Bin b of slice s is bin b + shift[s] of the row; its mass is q 2^-15 2^(-bin/16) relative
    // to the reference of the row maximum's bin.  Thread t gathers row bins 4 t .. 4 t + 3
    // (all loads of eight slices are requested before any is used).
    const int rb0 = kBinsPerThread * tid;
    unsigned long long qsum[kBinsPerThread];
#pragma unroll
    for (int k = 0; k < kBinsPerThread; ++k)
        qsum[k] = 0ull;
    for (int s0 = 0; s0 < slices; s0 += 8) {
        // unconditional loads from clamped positions (a guarded load would be waited for on
        // the spot); what lies outside a slice's published bins is masked afterwards
        unsigned qv[8][kBinsPerThread];
        int sh[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int sl = min(s0 + u, slices - 1);
            sh[u] = s0 + u < slices ? L.shift[sl] : kBins;
#pragma unroll
            for (int k = 0; k < kBinsPerThread; ++k) {
                const int b = min(max(rb0 + k - sh[u], 0), kPubBins - 1);
                qv[u][k] = W.hist[(size_t)sl * kPubBins + b];
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int k = 0; k < kBinsPerThread; ++k) {
                const int b = rb0 + k - sh[u];
                qsum[k] += (b >= 0 && b < kPubBins) ? qv[u][k] : 0u;
            }
    }
#pragma unroll
    for (int k = 0; k < kBinsPerThread; ++k) {
        const int rb = rb0 + k;
        // 2^(-(rb mod 16)/16) in fp32 (an estimate is all that is needed), 2^(-15 - rb/16) as
        // an exponent
        const double root = (double)__builtin_amdgcn_exp2f(-0.0625f * (float)(rb & 15));
        const double pow2 = __hiloint2double((1023 - 15 - (rb >> 4)) << 20, 0);
        L.row.hist[rank_slot(rb)] = (double)qsum[k] * root * pow2;
    }
    __syncthreads();
    const BinPick est = wave_pick(L.row.hist, 0.0, (double)top_p, true);
    // the estimate is good to about 1e-5 of the total; be generous
    const double need_est = (double)top_p * est.total, tol = 1e-3 * est.total;
    lo = hi = est.bin;
    if (need_est - est.above <= tol && lo > 0)
        --lo;
    if (est.above + est.in_bin - need_est <= tol && hi < kBins - 1)
        ++hi;
    __syncthreads();  // the histogram array is reused below
    CutBins c;
    c.lo = lo;
    c.hi = hi;
    return c;
}

// ---- optional kernel between the two: the row's cut bins, once per row ------------------------------
// Used when a launch has so many workgroups that recomputing the estimate in each of them
// would cost more than one more small kernel.
__global__ __launch_bounds__(kBlock) void sampler_cut_kernel(SamplerParams sp, char* ws, int slices)
{
    __shared__ SelectLds L;
    const int tid = threadIdx.x;
    const long long r = blockIdx.x;
    const RowWs W = row_ws(ws, r, slices);
    const float T = sp.temperature[r];
    const float top_p = sp.top_p[r];
    if (T == 0.f || !(top_p < 1.f))
        return;
    if (tid < slices)
        L.smax[tid] = stat_at(W, tid)->max_x;
    __syncthreads();
    float M = -INFINITY;
    for (int s = 0; s < slices; ++s)
        M = fmaxf(M, L.smax[s]);
    const RowConst rc = row_const(T);
    const CutBins cb = estimate_cut(L, W, slices, bin_coord(M, rc.c16), rc, top_p);
    if (tid == 0) {
        W.ctl->lo = cb.lo;
        W.ctl->hi = cb.hi;
    }
}

// ---- exact threshold among the candidates, CDF walk: one workgroup per row -----------------------------
// Runs in the workgroup of a row that finished last (select kernel) or in a kernel of its own.
__device__ __forceinline__ void finish_row(SelectLds& L, const SamplerParams& sp, long long r, const RowWs& W,
                                           int slices, int slice_elems, const RowScale& rs, const RowConst& rc,
                                           float kf_row, int lo, int hi, bool cut, float top_p)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* __restrict__ x = sp.logits + r * sp.stride;
    const int V = (int)sp.vocab;
    const unsigned cand_total = observe(&W.ctl->cand_total);
    const int C = (int)min(cand_total, (unsigned)kCandCap);
    const int nseg = slices * kSegPerSlice;
    double* seg_mass = L.row.seg_mass;
    if (tid < slices) {
        const SliceStat* st = stat_at(W, tid);
        L.smass[tid] = observe(&st->mass);
        L.sabove[tid] = observe(&st->above);
    }
    for (int i = tid; i < C; i += kBlock)
        L.cand[i] = observe(&W.cand[i]);
    for (int sidx = tid; sidx < nseg; sidx += kBlock)
        seg_mass[sidx] = observe(&W.seg[sidx]);
    __syncthreads();
    double S = 0.0, above_total = 0.0;
    for (int s = 0; s < slices; ++s) {
        S += L.smass[s];
        above_total += L.sabove[s];
    }
    const double need = (double)top_p * S;

    uint32_t key_tau = 0u;
    double Z = above_total;
    if (cut) {
        // Radix select over the candidates' order keys, taken relative to the largest one
        // (rel = kmax - key, 0 = most probable) so that only the bits in which the candidates
        // differ are resolved: 11 bits per level, usually two levels.
        uint32_t kmin = 0xffffffffu, kmax = 0u;
        for (int i = tid; i < C; i += kBlock) {
            const uint32_t key = order_key(__uint_as_float((unsigned)L.cand[i]));
            kmin = min(kmin, key);
            kmax = max(kmax, key);
        }
        for (int o = 32; o > 0; o >>= 1) {
            kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o));
            kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o));
        }
        if (lane == 0) {
            L.kmin[wave] = kmin;
            L.kmax[wave] = kmax;
        }
        double* H = L.row.hist;
        for (int b = tid; b < kBins; b += kBlock)
            H[b] = 0.0;
        __syncthreads();
        for (int w = 0; w < kWaves; ++w) {
            kmin = min(kmin, L.kmin[w]);
            kmax = max(kmax, L.kmax[w]);
        }
        const uint32_t span = C > 0 ? kmax - kmin : 0u;
        const int nbits = span ? 32 - __clz((int)span) : 1;
        uint32_t prefix = 0u;
        double abv = above_total;
        bool bad = cand_total > (unsigned)kCandCap || !(above_total < need);
        for (int shift = 11 * ((nbits - 1) / 11); shift >= 0 && !bad; shift -= 11) {
            for (int i = tid; i < C; i += kBlock) {
                const float xc = __uint_as_float((unsigned)L.cand[i]);
                const uint32_t rel = kmax - order_key(xc);
                if ((uint64_t)rel >> (shift + 11) == prefix)
                    atomicAdd(&H[rank_slot((rel >> shift) & 0x7ffu)], (double)prob(xc, rs));
            }
            __syncthreads();
            const BinPick pk = wave_pick(H, abv, need, false);
            // the cut must fall among the candidates
            if (shift == 11 * ((nbits - 1) / 11) && !(above_total + pk.total >= need))
                bad = true;
            prefix = (prefix << 11) | (uint32_t)pk.bin;
            abv = pk.above;
            Z = pk.above + pk.in_bin;
            __syncthreads();
            if (shift > 0) {
                for (int b = tid; b < kBins; b += kBlock)
                    H[b] = 0.0;
                __syncthreads();
            }
        }
        if (bad) {
            // candidate overflow or an estimate that missed the cut: redo the row the slow way
            sample_row_from_memory(sp, r, L.row);
            return;
        }
        key_tau = kmax - prefix;
    }

    // kept candidates join their segments (vocabulary order)
    for (int i = tid; i < C; i += kBlock) {
        const float xc = __uint_as_float((unsigned)L.cand[i]);
        if (order_key(xc) >= key_tau) {
            const int idx = (int)(L.cand[i] >> 32);
            const int s = idx / slice_elems;
            atomicAdd(&seg_mass[s * kSegPerSlice + (idx - s * slice_elems) / kSeg], (double)prob(xc, rs));
        }
    }
    __syncthreads();
    if (!cut) {
        // Nothing is cut: the normaliser is the sum of the segments as they stand now, i.e. with the
        // row's last one to three logits (which travel as candidates) included.
        double part = 0.0;
        for (int sidx = tid; sidx < nseg; sidx += kBlock)
            part += seg_mass[sidx];
        Z = block_sum_f64(part, L.row.scratch);
    }
    const double target = (double)sp.uniforms[r] * Z;

    if (wave == 0) {
        const int per = (nseg + 63) / 64;
        double mine = 0.0;
        for (int k = 0; k < per; ++k) {
            const int sidx = lane * per + k;
            if (sidx < nseg)
                mine += seg_mass[sidx];
        }
        double inc = mine;
        for (int o = 1; o < 64; o <<= 1) {
            const double up = __shfl_up(inc, o);
            if (lane >= o)
                inc += up;
        }
        const double before_lane = inc - mine;
        const unsigned long long hit = __ballot(inc > target);
        int seg = -1;
        double before = 0.0;
        bool take_last = false;
        if (hit) {
            const int hl = __ffsll((long long)hit) - 1;
            double run = __shfl(before_lane, hl);
            for (int k = 0; k < per; ++k) {
                const int sidx = hl * per + k;
                if (sidx >= nseg)
                    break;
                const double sm = seg_mass[sidx];
                if (run + sm > target) {
                    seg = sidx;
                    before = run;
                    break;
                }
                run += sm;
            }
        }
        if (seg < 0) {
            // rounding: the target is not below the total; take the last segment with mass
            int last = -1;
            for (int k = 0; k < per; ++k) {
                const int sidx = lane * per + k;
                if (sidx < nseg && seg_mass[sidx] > 0.0)
                    last = sidx;
            }
            for (int o = 32; o > 0; o >>= 1)
                last = max(last, __shfl_xor(last, o));
            seg = last;
            take_last = true;
        }
        int token = -1;
        if (seg >= 0) {
            const int s = seg / kSegPerSlice;
            const int base = s * slice_elems + (seg % kSegPerSlice) * kSeg + lane * 4;
            const int end = min(V, (s + 1) * slice_elems);
            float pk[4];
            bool keep[4];
            float s4 = 0.f;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int i = base + k;
                pk[k] = 0.f;
                keep[k] = false;
                if (i < end) {
                    const float xi = x[i];
                    const int b = bin_below(kf_row, bin_coord(xi, rc.c16));
                    if (b < lo || (b <= hi && order_key(xi) >= key_tau)) {
                        pk[k] = prob(xi, rs);
                        keep[k] = true;
                        s4 += pk[k];
                    }
                }
            }
            double inc2 = (double)s4;
            for (int o = 1; o < 64; o <<= 1) {
                const double up = __shfl_up(inc2, o);
                if (lane >= o)
                    inc2 += up;
            }
            double run = before + inc2 - (double)s4;
            int first = 0x7fffffff, lastk = -1;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (keep[k]) {
                    lastk = base + k;
                    run += (double)pk[k];
                    if (run > target && first == 0x7fffffff)
                        first = base + k;
                }
            for (int o = 32; o > 0; o >>= 1) {
                first = min(first, __shfl_xor(first, o));
                lastk = max(lastk, __shfl_xor(lastk, o));
            }
            token = (first != 0x7fffffff && !take_last) ? first : lastk;
        }
        if (lane == 0)
            sp.tokens[r] = token >= 0 ? token : 0;
    }
}

__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(4))) void sampler_select_kernel(SamplerParams sp, char* ws, int slices,
                                                                int slice_elems, int cut_ready)
{
    __shared__ SelectLds L;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long r = blockIdx.x / slices;
    const int slice = blockIdx.x % slices;
    const RowWs W = row_ws(ws, r, slices);
    const float* __restrict__ x = sp.logits + r * sp.stride;
    const int V = (int)sp.vocab;
    const SliceRange g = slice_range(slice, slice_elems, V);
    const float T = sp.temperature[r];
    const bool greedy = (T == 0.f);
    const float top_p = sp.top_p[r];
    const bool cut = !greedy && top_p < 1.f;

    // The slice statistics are requested first and the slice's logits right behind them (loads
    // return in order); the row's cut is worked out while the logits travel.
    float st_max = -INFINITY;
    int st_arg = 0x7fffffff;
    int lo = kBins, hi = kBins;  // candidate bins, counted down from the maximum's bin; kBins = no cut
    if (cut && cut_ready) {
        lo = W.ctl->lo;
        hi = W.ctl->hi;
    }
    if (tid < slices) {
        const SliceStat* st = stat_at(W, tid);
        st_max = st->max_x;
        st_arg = st->argmax;
    }
    float xv[32];
    {
        // a greedy row needs no second look: all its loads collapse onto one float4
        SliceRange gl = g;
        if (greedy)
            gl.v4end = gl.e0 + 4;
        SPD_LOAD_SLICE(xv, x, gl, tid)
    }
    if (tid < slices) {
        L.smax[tid] = st_max;
        L.sarg[tid] = st_arg;
    }
    __syncthreads();
    float M = -INFINITY;
    int arg = 0x7fffffff;
    for (int s = 0; s < slices; ++s) {
        if (L.smax[s] > M || (L.smax[s] == M && L.sarg[s] < arg)) {
            M = L.smax[s];
            arg = L.sarg[s];
        }
    }
    if (greedy) {
        if (slice == 0 && tid == 0)
            sp.tokens[r] = arg == 0x7fffffff ? 0 : arg;
        return;
    }
    const RowConst rc = row_const(T);
    const float kf_row = bin_coord(M, rc.c16);
    if (cut && !cut_ready) {
        const CutBins cb = estimate_cut(L, W, slices, kf_row, rc, top_p);
        lo = cb.lo;
        hi = cb.hi;
    }

    SPD_MASK_SLICE(xv, g, tid)
    RowScale rs;
    rs.max_x = M;
    rs.c_hi = rc.c_hi;
    rs.c_lo = rc.c_lo;
    // Bin tests without forming the bin: with t = x c16, bin(x) < lo  <=>  floor(t) > kf_row - lo
    // <=>  t >= kf_row - lo + 1 (both sides of the middle inequality are integers); likewise
    // bin(x) <= hi  <=>  t >= kf_row - hi.  The clamps of the bin only matter at the ends:
    // lo == kBins keeps everything, hi == kBins - 1 makes every remaining element a candidate.
    const float t_above = lo >= kBins ? -INFINITY : kf_row - (float)lo + 1.f;
    const float t_cand = hi >= kBins - 1 ? -INFINITY : kf_row - (float)hi;

    int ncand = 0;
    double above = 0.0;
    float all32 = 0.f;  // this thread's 32 probabilities; widened once
    float s_above[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        s_above[j] = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float xq = xv[4 * j + k];
            if (xq == -INFINITY)
                continue;
            const float pq = prob(xq, rs);
            all32 += pq;
            const float t = xq * rc.c16;
            if (t >= t_above)
                s_above[j] += pq;
            else if (t >= t_cand)
                ++ncand;
        }
    }
    // 256 fp32 terms per segment.  The eight wavefront reductions are folded: after the exchange
    // across 32 lanes each half keeps four segments, then two, then one, so that lane 8 s ends
    // up with the sum of segment s (10 exchanges instead of 48).
    {
        const bool up32 = (lane & 32) != 0, up16 = (lane & 16) != 0, up8 = (lane & 8) != 0;
        float a4[4], a2[2], a1;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float keep = up32 ? s_above[4 + j] : s_above[j];
            const float give = up32 ? s_above[j] : s_above[4 + j];
            a4[j] = keep + __shfl_xor(give, 32);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const float keep = up16 ? a4[2 + j] : a4[j];
            const float give = up16 ? a4[j] : a4[2 + j];
            a2[j] = keep + __shfl_xor(give, 16);
        }
        {
            const float keep = up8 ? a2[1] : a2[0];
            const float give = up8 ? a2[0] : a2[1];
            a1 = keep + __shfl_xor(give, 8);
        }
        a1 += __shfl_xor(a1, 4);
        a1 += __shfl_xor(a1, 2);
        a1 += __shfl_xor(a1, 1);
        // lane 8 s (and its seven neighbours) holds segment j = 4 (lane/32) + 2 (lane/16 % 2) + lane/8 % 2
        if ((lane & 7) == 0) {
            const int j = lane >> 3;
            publish(&W.seg[(size_t)slice * kSegPerSlice + j * kWaves + wave], (double)a1, cut_ready != 0);
            above = (double)a1;
        }
    }
    double mass = (double)all32;
    // tail logits (thread 0): counted in the slice mass, always sent as candidates when kept at all
    int tail_cand = 0;
    if (tid == 0)
        for (int k = 0; k < g.ntail; ++k) {
            const float xt = x[g.v4end + k];
            mass += (double)prob(xt, rs);
            if (bin_below(kf_row, bin_coord(xt, rc.c16)) <= hi || lo == kBins)
                ++tail_cand;
        }
    ncand += tail_cand;
    block_sum2_f64(mass, above, L.row.scratch);

    int incl = ncand;
    for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o);
        if (lane >= o)
            incl += up;
    }
    __syncthreads();
    if (lane == 63)
        L.wave_cnt[wave] = incl;
    __syncthreads();
    int wave_off = 0, block_total = 0;
    for (int w = 0; w < kWaves; ++w) {
        if (w < wave)
            wave_off += L.wave_cnt[w];
        block_total += L.wave_cnt[w];
    }
    if (tid == 0) {
        L.cand_base = block_total ? __hip_atomic_fetch_add(&W.ctl->cand_total, (unsigned)block_total,
                                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                  : 0u;
        SliceStat* st = stat_at(W, slice);
        publish(&st->mass, mass, cut_ready != 0);
        publish(&st->above, above, cut_ready != 0);
    }
    __syncthreads();
    if (ncand) {
        unsigned pos = L.cand_base + (unsigned)(wave_off + incl - ncand);
#pragma unroll
        for (int q = 0; q < 32; ++q) {
            const float xq = xv[q];
            if (xq == -INFINITY)
                continue;
            const float t = xq * rc.c16;
            if (t < t_above && t >= t_cand) {
                if (pos < (unsigned)kCandCap)
                    publish(&W.cand[pos],
                            (unsigned long long)__float_as_uint(xq) |
                                ((unsigned long long)(unsigned)(g.e0 + (q >> 2) * kIter + tid * 4 + (q & 3)) << 32),
                            cut_ready != 0);
                ++pos;
            }
        }
        if (tid == 0)
            for (int k = 0; k < g.ntail; ++k) {
                const float xt = x[g.v4end + k];
                if (bin_below(kf_row, bin_coord(xt, rc.c16)) <= hi || lo == kBins) {
                    if (pos < (unsigned)kCandCap)
                        publish(&W.cand[pos], (unsigned long long)__float_as_uint(xt) |
                                                  ((unsigned long long)(unsigned)(g.v4end + k) << 32),
                                cut_ready != 0);
                    ++pos;
                }
            }
    }

    if (cut_ready)
        return;  // many workgroups per launch: the pick kernel finishes the rows

    // ---- arrival: everything this workgroup published has been acknowledged before it counts ----
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (tid == 0)
        L.arrived_before = __hip_atomic_fetch_add(&W.ctl->arrived, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (L.arrived_before != (unsigned)(slices - 1))
        return;
    // last workgroup of the row
    finish_row(L, sp, r, W, slices, slice_elems, rs, rc, kf_row, lo, hi, cut, top_p);
}

// The finishing step as a kernel of its own, for launches with many workgroups: there the select
// kernel's workgroups neither wait for their stores to be acknowledged nor count arrivals.
__global__ __launch_bounds__(kBlock) void sampler_pick_kernel(SamplerParams sp, char* ws, int slices,
                                                              int slice_elems)
{
    __shared__ SelectLds L;
    const int tid = threadIdx.x;
    const long long r = blockIdx.x;
    const RowWs W = row_ws(ws, r, slices);
    const float T = sp.temperature[r];
    if (T == 0.f)
        return;  // greedy rows were answered by the select kernel
    const float top_p = sp.top_p[r];
    const bool cut = top_p < 1.f;
    if (tid < slices)
        L.smax[tid] = stat_at(W, tid)->max_x;
    __syncthreads();
    float M = -INFINITY;
    for (int s = 0; s < slices; ++s)
        M = fmaxf(M, L.smax[s]);
    const RowConst rc = row_const(T);
    RowScale rs;
    rs.max_x = M;
    rs.c_hi = rc.c_hi;
    rs.c_lo = rc.c_lo;
    const int lo = cut ? W.ctl->lo : kBins, hi = cut ? W.ctl->hi : kBins;
    finish_row(L, sp, r, W, slices, slice_elems, rs, rc, bin_coord(M, rc.c16), lo, hi, cut, top_p);
}


__global__ __launch_bounds__(kBlock) void sample_rows_kernel(SamplerParams sp)
{
    __shared__ RowLds lds;
    sample_row_from_memory(sp, blockIdx.x, lds);
}

}  // namespace

// Slices per row: enough workgroups to cover the chip, pieces that fit the registers.
int sampler_slices(long long rows, long long vocab)
{
    const long long smin = (vocab + kSliceMax - 1) / kSliceMax;
    if (smin > kMaxSlices)
        return 0;  // whole-row kernel
    // Two workgroups per CU, but no more than eight slices unless the vocabulary needs them (every
    // workgroup of a row re-reads all the row's slice histograms: measured 42 / 60 / 76 us with
    // 8 / 12 / 16 slices on 64 rows of 128256), and no slice shorter than 4096 logits.
    long long s = (512 + rows - 1) / rows;
    const long long smax_small = vocab / 4096 > 1 ? vocab / 4096 : 1;
    if (s > smax_small) s = smax_small;
    if (s > 8) s = 8;
    if (s < smin) s = smin;
    return (int)s;
}

size_t sampler_workspace_bytes(long long rows, long long vocab)
{
    const int s = sampler_slices(rows, vocab);
    return 256 + (s ? (size_t)rows * sliced_row_bytes(s) : 0);
}

hipError_t launch_sampler(const SamplerParams& p, void* ws, hipStream_t s)
{
    const int slices = sampler_slices(p.rows, p.vocab);
    const bool aligned = (p.stride % 4 == 0) && ((uintptr_t)p.logits % 16 == 0);
    if (slices == 0 || !aligned || p.vocab < 4 || p.top_k || p.min_p) {  // filters: whole-row kernel only
        hipLaunchKernelGGL(sample_rows_kernel, dim3((unsigned)p.rows), dim3(kBlock), 0, s, p);
        return hipGetLastError();
    }
    int slice_elems = (int)((p.vocab + slices - 1) / slices);
    slice_elems = (slice_elems + 3) / 4 * 4;
    const dim3 per_slice((unsigned)(p.rows * slices)), block(kBlock);
    hipLaunchKernelGGL(sampler_hist_kernel, per_slice, block, 0, s, p, (char*)ws, slices, slice_elems);
    // With many workgroups per launch the cut estimate is computed once per row instead of in
    // every workgroup of the row, and the rows are finished by a kernel of their own: four
    // kernels whose workgroups are short, instead of two whose workgroups wait on one another's
    // results.
    const int cut_ready = p.rows * slices > 2048 ? 1 : 0;
    if (cut_ready)
        hipLaunchKernelGGL(sampler_cut_kernel, dim3((unsigned)p.rows), block, 0, s, p, (char*)ws, slices);
    hipLaunchKernelGGL(sampler_select_kernel, per_slice, block, 0, s, p, (char*)ws, slices, slice_elems,
                       cut_ready);
    if (cut_ready)
        hipLaunchKernelGGL(sampler_pick_kernel, dim3((unsigned)p.rows), block, 0, s, p, (char*)ws, slices,
                           slice_elems);
    return hipGetLastError();
}

}  // namespace spd
