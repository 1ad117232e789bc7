// Temperature / nucleus / inverse-CDF token sampler.
//
// Two paths.  The sliced path (below: two stream-ordered kernels) reads a row from HBM once, leaves
// what the row-level step needs in the workspace, and finds the exact nucleus threshold without
// sorting.  The whole-row routine (one workgroup per row, every pass from memory) covers what the
// sliced path does not take: unaligned rows, vocabularies beyond 16 slices, the rare row whose
// candidate set overflows, and rows whose min-p or top-k filter reaches further down than the
// sliced path's windows.
//
// Probabilities are evaluated by one shared routine, p_i = 2^((x_i - max) c) with
// c = log2(e)/T carried as hi + lo floats, so every pass sees the same bits; every sum that
// decides something is carried in fp64; comparisons that define the kept set are on bit
// patterns, so all ties with the threshold are kept by construction.
#include "spd_internal.h"

#include <cstdlib>
#include <type_traits>

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
    double scratch[2 * kWaves];  // block sums and scans
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
// handled by two kernels in stream order; no workgroup ever waits for another and there are no
// cross-workgroup counters.
//
//   scan    (rows x slices)  the one pass over the logits.  A workgroup holds its slice in
//           registers and leaves behind everything the row-level step can need from it:
//           the slice maximum (and its lowest index), the slice mass relative to that maximum,
//           a histogram of mass over bins of width 1/16 in log2 p (the bin of a logit is
//           floor(x c 16), an integer function of x alone, so a slice histogram differs from
//           the row's by an integer shift; mass is accumulated in u32 fixed point relative to the
//           bin's own reference), and the elements the nucleus cut can fall among, written out as
//           (logit, index) pairs.  Which elements those are is a local guess: the slice finds its
//           own cut bin L from its own histogram; if the slice's elements down to a few bins
//           past L fit the budget it emits from the top (bins 0 .. L + margin, as far as the
//           budget goes), otherwise a window of bins centred on L, as wide as the budget allows,
//           and it sums the mass above the window per 256-element segment.  A slice whose cut bin
//           alone exceeds the budget emits nothing.
//   finish  (rows)  combines the slice maxima and histograms into the row's cut bins [lo, hi].
//           A slice is "covered" if its emitted bins contain [lo, hi] and everything it summed as
//           above its window really is above lo; its emitted elements are then classified with
//           p_i = 2^((x_i - row max) c) exactly as defined (kept for certain, candidate, dropped).
//           Slices that are not covered are read a second time by this workgroup.  The exact
//           threshold is found among the candidates by radix select on the logit's bit pattern
//           with fp64 masses; kept candidates join their segments; the segments are scanned and
//           the walk ends inside the segment that contains u * Z.
//           Rows with a min-p or top-k filter (a second instantiation of the kernel, launched
//           beside the first when filter arrays are given): the scan kernel writes such a row out
//           from the top as far as the budget goes, and the survivors of the filters, found among
//           the pairs, become the candidate list.
//
// With the row statistics exchanged through memory between two kernels, plain stores and loads do.
// =============================================================================================
constexpr int kIter = kBlock * 4;         // elements one float4 per thread covers
constexpr int kSliceMax = 8 * kIter;      // elements per workgroup: 8 float4 per thread
constexpr int kMaxSlices = 16;
constexpr int kSegPerSlice = kSliceMax / kSeg;  // 64
constexpr int kCandCap = 3072;
constexpr int kPubBins = 1024;    // histogram bins of a slice (64 octaves below its maximum)
constexpr int kEmitCap = 2048;    // (logit, index) pairs a slice may write out
constexpr int kTopProbe = 0;      // a slice emits from the top if its elements down to L + kTopProbe fit
constexpr int kTopMargin = 160;   // ... and then goes on down to L + kTopMargin at most (10 octaves)
static_assert(kMaxSlices * kSegPerSlice <= kMaxSegments, "segment table too small");

struct SliceStat {
    float max_x;
    int argmax;
    double rest;      // estimated mass of the slice's bins past win_hi, in units of 2^(bin_coord(max_x) / 16)
    int win_lo;       // emitted bins [win_lo, win_hi], counted down from the bin of max_x
    int win_hi;
    int count;        // emitted pairs; -1: the slice emitted nothing although the row has a cut
    int pad;
};
static_assert(sizeof(SliceStat) <= 64, "slice statistics are kept 64 bytes apart");

__host__ __device__ inline size_t sliced_row_bytes(int slices)
{
    return (size_t)slices * (64 + (size_t)kPubBins * 4 + (size_t)kSegPerSlice * 8 + (size_t)kEmitCap * 8);
}

struct RowWs {
    char* stat;                // [slices] SliceStat, 64 B apart
    unsigned* hist;            // [slices][kPubBins]
    double* seg;               // [slices][kSegPerSlice] mass above the window (whole mass when nothing is cut)
    unsigned long long* emit;  // [slices][kEmitCap] logit bits | index << 32
};

__device__ __forceinline__ RowWs row_ws(char* base, long long row, int slices)
{
    char* p = base + row * sliced_row_bytes(slices);
    RowWs w;
    w.stat = p;
    p += (size_t)slices * 64;
    w.hist = (unsigned*)p;
    p += (size_t)slices * kPubBins * 4;
    w.seg = (double*)p;
    p += (size_t)slices * kSegPerSlice * 8;
    w.emit = (unsigned long long*)p;
    return w;
}

__device__ __forceinline__ SliceStat* stat_at(const RowWs& w, int s) { return (SliceStat*)(w.stat + (size_t)s * 64); }

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

// Mass that one unit of a bin's fixed-point histogram stands for, relative to the reference of
// bin 0: 2^-15 2^(-bin/16) (the root in fp32: an estimate is all that is needed).
__device__ __forceinline__ double bin_unit(int bin)
{
    const double root = (double)__builtin_amdgcn_exp2f(-0.0625f * (float)(bin & 15));
    return root * __hiloint2double((1023 - 15 - (bin >> 4)) << 20, 0);
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

// Largest b in [lo_b, hi_b] with pred(b), where pred is true on a prefix of the range; lo_b - 1
// if it is false everywhere.
template <typename F> __device__ __forceinline__ int last_true(int lo_b, int hi_b, F pred)
{
    int lo = lo_b - 1, hi = hi_b;  // invariant: pred(lo) (or lo == lo_b - 1), answer <= hi
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (pred(mid))
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

// ---- kernel 1: the pass over the logits --------------------------------------------------------------
constexpr int kWaveStage = kEmitCap / kWaves * 2;  // pairs one wavefront may gather (twice its even share)

struct ScanLds {
    unsigned hist[kPubBins + 64];       // + one place per lane for what lies past the last bin
    unsigned cumq[kPubBins];            // inclusive running sum of hist
    unsigned long long stage[kWaves][kWaveStage + 1];  // each wavefront's pairs, copied out in one piece (+ one
                                                       // place that takes whatever does not fit)
    double wave_mass[kWaves];
    unsigned wave_q[kWaves];
    float red_f[kWaves];
    int red_i[kWaves];
    double rest;               // estimated mass of the bins past the window
    int cut_bin;               // the slice's own cut bin L
    int best;                  // scratch of the window search
    int emitted;               // places reserved in the slice's list so far
    int overflow;              // some wavefront gathered more pairs than it has room for
};

// Barrier between phases that exchange data through LDS only: waits for this wavefront's LDS
// traffic, not for its global loads and stores (a __syncthreads would drain those too, and the
// slice's logits and the published results are still in flight at most barriers of this kernel).
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Fixed-point mass of a logit inside its bin: 32768 2^(f/16) for f in [0, 1), as a quadratic in f:
// the series 32768 + a1 f + a2 f^2 + a3 f^3 with f^3 replaced by its best quadratic on [0, 1],
// (48 f^2 - 18 f + 1) / 32 (error a3 / 32 = 0.014 units; the next term of the series is below
// 0.005).  Values run from 32768 to 34219.  NaN (positions past the end of a slice) converts to 0.
// The scan kernel's pass over the logits is bound by its vector instructions (every instruction
// per logit costs it about 2 % of its time), hence the count of every one here and below.
__device__ __forceinline__ unsigned bin_units(float f)
{
    const float a1 = 1419.5653f, a2 = 30.749034f, a3 = 0.44403f;
    const float b0 = 32768.5f + a3 / 32.f, b1 = a1 - a3 * (18.f / 32.f), b2 = a2 + a3 * (48.f / 32.f);
    return (unsigned)__builtin_fmaf(__builtin_fmaf(b2, f, b1), f, b0);
}

__device__ __forceinline__ int wave_max_i32(int v)
{
    for (int o = 32; o > 0; o >>= 1)
        v = max(v, __shfl_xor(v, o));
    return v;
}

// Folds eight per-lane partial sums (one per 256-element segment j of the wavefront's pass) across the
// wavefront: after the exchange across 32 lanes each half keeps four segments, then two, then one,
// so that lane 8 s ends up with the sum of segment s (10 exchanges instead of 48).
__device__ __forceinline__ float fold_segments(const float (&s_seg)[8])
{
    const int lane = threadIdx.x & 63;
    const bool up32 = (lane & 32) != 0, up16 = (lane & 16) != 0, up8 = (lane & 8) != 0;
    float a4[4], a2[2], a1;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float keep = up32 ? s_seg[4 + j] : s_seg[j];
        const float give = up32 ? s_seg[j] : s_seg[4 + j];
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
    return a1;  // lanes 8 s .. 8 s + 7 hold segment j = 4 (lane/32) + 2 (lane/16 % 2) + lane/8 % 2 = lane >> 3
}

__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(4))) void sampler_scan_kernel(SamplerParams sp, char* ws, int slices, int slice_elems)
{
    __shared__ ScanLds L;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long r = blockIdx.x / slices;
    const int slice = blockIdx.x % slices;
    const float* __restrict__ x = sp.logits + r * sp.stride;
    const SliceRange g = slice_range(slice, slice_elems, (int)sp.vocab);
    const RowWs W = row_ws(ws, r, slices);
    const float T = sp.temperature[r];
    const bool greedy = (T == 0.f);
    const float top_p = sp.top_p[r];
    // rows with a min-p or top-k filter are finished from their pairs alone, whatever top_p is
    const bool filtered = (sp.top_k && sp.top_k[r] > 0) || (sp.min_p && sp.min_p[r] > 0.f);
    const bool cut = !greedy && (top_p < 1.f || filtered);

    float xv[32];
    SPD_LOAD_SLICE(xv, x, g, tid)
    float tail[3] = {-INFINITY, -INFINITY, -INFINITY};  // the row's last one to three logits (thread 0 of the last slice)
    if (tid == 0)
        for (int k = 0; k < 3; ++k)
            if (k < g.ntail)
                tail[k] = x[g.v4end + k];
    for (int b = tid; b < kPubBins + 64; b += kBlock)
        L.hist[b] = 0u;
    if (tid == 0) {
        L.cut_bin = kPubBins - 1;
        L.best = -1;
        L.emitted = 0;
        L.overflow = 0;
        L.rest = 0.0;
    }
    // wavefronts whose 32 x 64 x 4 logits all lie inside the slice skip the end-of-slice masking
    const bool whole = g.e0 + 7 * kIter + (tid | 63) * 4 + 4 <= g.v4end;
    if (!whole) {
        SPD_MASK_SLICE(xv, g, tid)
    }
    float mx = fmaxf(fmaxf(tail[0], tail[1]), tail[2]);
#pragma unroll
    for (int q = 0; q < 32; ++q)
        mx = fmaxf(mx, xv[q]);
    for (int o = 32; o > 0; o >>= 1)
        mx = fmaxf(mx, __shfl_xor(mx, o));
    if (lane == 0)
        L.red_f[wave] = mx;
    lds_barrier();
    mx = L.red_f[0];
    for (int w = 1; w < kWaves; ++w)
        mx = fmaxf(mx, L.red_f[w]);

    if (greedy) {
        int mi = 0x7fffffff;
#pragma unroll
        for (int q = 31; q >= 0; --q)
            if (xv[q] == mx)
                mi = g.e0 + (q >> 2) * kIter + tid * 4 + (q & 3);
        for (int k = 2; k >= 0; --k)
            if (tail[k] == mx)  // (-inf where there is no tail logit, and a slice maximum is finite)
                mi = min(mi, g.v4end + k);
        for (int o = 32; o > 0; o >>= 1)
            mi = min(mi, __shfl_xor(mi, o));
        if (lane == 0)
            L.red_i[wave] = mi;
        lds_barrier();
        if (tid == 0) {
            for (int w = 0; w < kWaves; ++w)
                mi = min(mi, L.red_i[w]);
            SliceStat* st = stat_at(W, slice);
            st->max_x = mx;
            st->argmax = mi;
        }
        return;
    }

    const RowConst rc = row_const(T);
    RowScale rs;
    rs.max_x = mx;
    rs.c_hi = rc.c_hi;
    rs.c_lo = rc.c_lo;
    const float kf_loc = bin_coord(mx, rc.c16);
    unsigned long long* out = W.emit + (size_t)slice * kEmitCap;
    double* seg_out = W.seg + (size_t)slice * kSegPerSlice;

    if (!cut) {
        // ---- nothing is cut: the mass of every 256-element segment, relative to the slice maximum; the
        // row's tail logits travel as pairs ----
        float s_seg[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            s_seg[j] = 0.f;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float xq = xv[4 * j + k];
                s_seg[j] += (whole || xq != -INFINITY) ? prob(xq, rs) : 0.f;
            }
        }
        const float a1 = fold_segments(s_seg);
        if ((lane & 7) == 0)
            seg_out[(lane >> 3) * kWaves + wave] = (double)a1;
        if (tid == 0) {
            int n = 0;
            for (int k = 0; k < 3; ++k)
                if (tail[k] != -INFINITY)
                    out[n++] = (unsigned long long)__float_as_uint(tail[k]) | ((unsigned long long)(unsigned)(g.v4end + k) << 32);
            SliceStat* st = stat_at(W, slice);
            st->max_x = mx;
            st->argmax = 0;
            st->rest = 0.0;
            st->win_lo = 0;
            st->win_hi = -1;
            st->count = n;
        }
        return;
    }

    // ---- histogram of mass over the slice's own bins.  Elements 64 octaves and more below the slice
    // maximum belong to the last bin; each lane collects them in a place of its own (they would
    // otherwise all meet at one LDS address) and the places are added to the last bin afterwards.
    // Positions past the end of the slice (-inf) land there too, with zero units. ----
    // (byte offsets: four times the bin, formed in floating point, so that one conversion gives
    // the LDS address; what lands between the last bin and the lane's own place belongs to the
    // last bin all the same)
    const float far4 = (float)(4 * (kPubBins + lane)), kf_loc4 = 4.f * kf_loc;
    auto bin_one = [&](float xq) __attribute__((always_inline)) {
        const float t = xq * rc.c16;
        const float kf = floorf(t);
        const float off = fminf(__builtin_fmaf(kf, -4.f, kf_loc4), far4);  // >= 0: kf_loc belongs to the maximum
        atomicAdd((unsigned*)((char*)L.hist + (unsigned)off), bin_units(t - kf));
    };
#pragma unroll
    for (int q = 0; q < 32; ++q)
        bin_one(xv[q]);
    for (int k = 0; k < 3; ++k)
        if (tail[k] != -INFINITY)
            bin_one(tail[k]);
    lds_barrier();  // histogram complete
    // what the lanes collected past the last bin belongs to the last bin (every wavefront adds the
    // places up for itself; only the owner of the last bin uses the sum)
    static_assert(kPubBins == 2 * kBlock, "thread t owns bins 2t and 2t+1; the last thread owns the last bin");
    unsigned far_units = L.hist[kPubBins + lane];
    for (int o = 32; o > 0; o >>= 1)
        far_units += __shfl_xor(far_units, o);

    // ---- running sums over the bins (thread t owns bins 2t, 2t+1): fixed-point units for the element
    // counts, estimated mass for the slice's own cut bin ----
    const unsigned q0 = L.hist[2 * tid], q1 = L.hist[2 * tid + 1] + (tid == kBlock - 1 ? far_units : 0u);
    const double m0 = (double)q0 * bin_unit(2 * tid), m1 = (double)q1 * bin_unit(2 * tid + 1);
    unsigned qi = q0 + q1;
    double mi = m0 + m1;
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned uq = __shfl_up(qi, o);
        const double um = __shfl_up(mi, o);
        if (lane >= o) {
            qi += uq;
            mi += um;
        }
    }
    if (lane == 63) {
        L.wave_q[wave] = qi;
        L.wave_mass[wave] = mi;
    }
    lds_barrier();
    unsigned qbefore = 0u;
    double mbefore = 0.0, mtotal = 0.0;
    for (int w = 0; w < kWaves; ++w) {
        if (w < wave) {
            qbefore += L.wave_q[w];
            mbefore += L.wave_mass[w];
        }
        mtotal += L.wave_mass[w];
    }
    qi += qbefore;   // inclusive through bin 2t+1
    mi += mbefore;
    L.cumq[2 * tid] = qi - q1;
    L.cumq[2 * tid + 1] = qi;
    // the one thread whose bins take the running mass across top_p of the total names the cut bin
    const double need = (double)top_p * mtotal;
    if (mi - m0 - m1 < need) {
        if (mi - m1 >= need)
            L.cut_bin = 2 * tid;
        else if (mi >= need)
            L.cut_bin = 2 * tid + 1;
    }
    lds_barrier();
    // ---- which bins to write out.  Element counts come from the fixed-point sums: every element adds
    // between 32768 and 34219 units, so (units >> 15) never undercounts.  Every thread tests two
    // places of the search range; the largest that fits wins. ----
    const int cap = kEmitCap - 3;  // room for the row's tail logits
    const int Lb = L.cut_bin;
    auto units = [&](int a, int z) { return L.cumq[z] - (a > 0 ? L.cumq[a - 1] : 0u); };
    auto fits = [&](int a, int z) { return (int)(units(a, z) >> 15) <= cap; };
    // (a row with a filter: always from the top, as many bins as fit; its filters decide later how
    // far down they reach)
    const bool from_top = filtered || fits(0, min(Lb + kTopProbe, kPubBins - 1));
    int mine = -1;
    if (from_top) {
        // bins 0 .. z, z as large as fits, at most L + kTopMargin
        const int zmax = filtered ? kPubBins - 1 : min(Lb + kTopMargin, kPubBins - 1);
        if (2 * tid + 1 <= zmax && (int)(qi >> 15) <= cap)
            mine = 2 * tid + 1;
        else if (2 * tid <= zmax && (int)((qi - q1) >> 15) <= cap)
            mine = 2 * tid;
    } else if (fits(Lb, Lb)) {
        // bins L - w .. L + w, w as large as fits
#pragma unroll
        for (int k = 1; k >= 0; --k) {
            const int w = tid + k * kBlock;
            if (mine < 0 && fits(max(Lb - w, 0), min(Lb + w, kPubBins - 1)))
                mine = w;
        }
    }
    mine = wave_max_i32(mine);
    if (lane == 0 && mine >= 0)
        atomicMax(&L.best, mine);
    lds_barrier();
    const int best = L.best;
    int win_lo = 0, win_hi = -1;   // bins written out; win_hi < 0: none
    if (best >= 0) {
        win_lo = from_top ? 0 : max(Lb - best, 0);
        win_hi = from_top ? best : min(Lb + best, kPubBins - 1);
    }
    // the thread that owns bin win_hi knows the estimated mass of everything past it
    if (win_hi >= 0 && (win_hi >> 1) == tid)
        L.rest = mtotal - ((win_hi & 1) ? mi : mi - m1);
    // Bin tests without forming the bin: with t = x c16, bin(x) < a  <=>  floor(t) > kf_loc - a
    // <=>  t >= kf_loc - a + 1 (both sides of the middle inequality are integers); likewise
    // bin(x) <= z  <=>  t >= kf_loc - z, and the last bin takes everything below it (every finite
    // logit: positions past the end of the slice hold -inf and fail the test).
    const float t_above = win_lo <= 0 ? INFINITY : kf_loc - (float)win_lo + 1.f;
    const float t_emit = win_hi < 0 ? INFINITY : (win_hi >= kPubBins - 1 ? -3.0e38f : kf_loc - (float)win_hi);

    // ---- the pairs: every wavefront gathers its own in LDS (the lanes that hold one take consecutive
    // places), reserves as many places in the slice's list and copies them out in one piece ----
    int have = 0;  // pairs this wavefront has gathered (uniform)
    // (one compare, two lane counts that also add the running total, a clamp, the index, the address;
    // logit and index go out of two registers with one two-dword write)
    const unsigned stage_base = (unsigned)(size_t)(__attribute__((address_space(3))) void*)&L.stage[wave][0];
    auto gather = [&](unsigned long long mask /* the wavefront's ballot of pred */, bool pred, float xq,
                      int idx) __attribute__((always_inline)) {
        if (pred) {
            const int pos = min((int)__builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),
                                                               __builtin_amdgcn_mbcnt_lo((unsigned)mask, (unsigned)have)),
                                kWaveStage);
            const unsigned addr = stage_base + 8u * (unsigned)pos;
            asm volatile("ds_write2_b32 %0, %1, %2 offset1:1" ::"v"(addr), "v"(xq), "v"(idx) : "memory");
        }
        have += __popcll(mask);
    };
    if (win_hi >= 0) {
        if (win_lo <= 0) {
#pragma unroll
            for (int q = 0; q < 32; ++q) {
                const bool in = xv[q] * rc.c16 >= t_emit;
                gather(__builtin_amdgcn_ballot_w64(in), in, xv[q], g.e0 + (q >> 2) * kIter + tid * 4 + (q & 3));
            }
        } else {
#pragma unroll
            for (int q = 0; q < 32; ++q) {
                const float t = xv[q] * rc.c16;
                const bool in = t >= t_emit, below = t < t_above;  // (two ballots and a scalar AND: no vector work)
                gather(__builtin_amdgcn_ballot_w64(in) & __builtin_amdgcn_ballot_w64(below), in && below, xv[q],
                       g.e0 + (q >> 2) * kIter + tid * 4 + (q & 3));
            }
        }
        for (int k = 0; k < 3; ++k) {
            const bool in = tail[k] * rc.c16 >= t_emit;  // (-inf where there is no tail logit)
            gather(__builtin_amdgcn_ballot_w64(in), in, tail[k], g.v4end + k);
        }
    }
    int base = 0;
    if (lane == 0 && have) {
        base = atomicAdd(&L.emitted, have);
        if (have > kWaveStage)
            L.overflow = 1;
    }
    base = __builtin_amdgcn_readfirstlane(base);
    lds_barrier();
    // A wavefront that ran out of room (sorted logits can put a slice's whole window into one
    // wavefront) makes the slice publish nothing: the row-level step then reads it a second time.
    const bool publish = win_hi >= 0 && !L.overflow;
    const int total = L.emitted;
    if (tid == 0) {
        SliceStat* st = stat_at(W, slice);
        st->max_x = mx;
        st->argmax = 0;
        st->rest = L.rest;
        st->win_lo = win_lo;
        st->win_hi = publish ? win_hi : -1;
        st->count = publish ? total : -1;
    }
    if (publish)
        for (int i = lane; i < min(have, kWaveStage); i += 64)
            if (base + i < kEmitCap)
                out[base + i] = L.stage[wave][i];
    *reinterpret_cast<uint2*>(&W.hist[(size_t)slice * kPubBins + 2 * tid]) = make_uint2(q0, q1);
    // ---- segment sums: what lies above the window (nothing when the window starts at the top) ----
    float a1 = 0.f;
    if (win_hi >= 0 && win_lo > 0) {
        float s_seg[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
            s_seg[j] = 0.f;
#pragma unroll
        for (int q = 0; q < 32; ++q)
            if (xv[q] * rc.c16 >= t_above)
                s_seg[q >> 2] += prob(xv[q], rs);
        a1 = fold_segments(s_seg);
    }
    if ((lane & 7) == 0)
        seg_out[(lane >> 3) * kWaves + wave] = (double)a1;
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

// ---- kernel 2: the row-level step ---------------------------------------------------------------------
struct FinishLds {
    RowLds row;                           // hist / scratch / seg_mass of the row routines
    unsigned long long cand[kCandCap];    // candidates: logit bits | index << 32
    double srest[kMaxSlices];             // estimated mass past the slice's window, relative to the row maximum
    double sfac[kMaxSlices];              // 2^((slice max - row max) c)
    float smax[kMaxSlices];
    int sarg[kMaxSlices];
    int shift[kMaxSlices];
    int swin_lo[kMaxSlices], swin_hi[kMaxSlices], scount[kMaxSlices];
    int covered[kMaxSlices];
    unsigned cand_total;
    uint32_t kmin[kWaves], kmax[kWaves];
};

// FILTERED = false takes the rows without a min-p / top-k filter, FILTERED = true the rows with one
// (a launch with filter arrays runs both; each leaves the other's rows alone).
// Three workgroups of the unfiltered kind share a CU (80 registers per lane, 50 KB of LDS each): the
// step is bound by the latency of its phases, so the third one is nearly free (1024 rows: 78 -> 67 us).
template <bool FILTERED>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(FILTERED ? 4 : 6))) void sampler_finish_kernel(SamplerParams sp, char* ws, int slices, int slice_elems)
{
    __shared__ FinishLds L;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long r = blockIdx.x;
    const RowWs W = row_ws(ws, r, slices);
    const float* __restrict__ x = sp.logits + r * sp.stride;
    const int V = (int)sp.vocab;
    const float T = sp.temperature[r];
    const float top_p = sp.top_p[r];
    const bool greedy = (T == 0.f);
    const int top_k = sp.top_k ? sp.top_k[r] : 0;
    const float min_p = sp.min_p ? sp.min_p[r] : 0.f;
    if (((top_k > 0 || min_p > 0.f) && !greedy) != FILTERED)
        return;
    const bool cut = !greedy && top_p < 1.f;
    const int nseg = slices * kSegPerSlice;
    double* seg_mass = L.row.seg_mass;

    if (tid < slices) {
        const SliceStat* st = stat_at(W, tid);
        L.smax[tid] = st->max_x;
        L.sarg[tid] = st->argmax;
        if (!greedy) {
            L.srest[tid] = st->rest;
            L.swin_lo[tid] = st->win_lo;
            L.swin_hi[tid] = st->win_hi;
            L.scount[tid] = st->count;
        }
    }
    if (tid == 0)
        L.cand_total = 0u;
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
        if (tid == 0)
            sp.tokens[r] = arg == 0x7fffffff ? 0 : arg;
        return;
    }
    const RowConst rc = row_const(T);
    RowScale rs;
    rs.max_x = M;
    rs.c_hi = rc.c_hi;
    rs.c_lo = rc.c_lo;
    const float kf_row = bin_coord(M, rc.c16);
    if (tid < slices) {
        const bool empty = L.smax[tid] == -INFINITY;
        L.shift[tid] = empty ? kBins : (int)fminf(fmaxf(kf_row - bin_coord(L.smax[tid], rc.c16), 0.f), (float)kBins);
        L.sfac[tid] = empty ? 0.0 : exp2(((double)L.smax[tid] - (double)M) * rc.cd);
        // the slice's histogram units refer to 2^(bin_coord(slice max) / 16); the row maximum is 2^(M c16 / 16)
        L.srest[tid] = empty ? 0.0
                             : L.srest[tid] * exp2(((double)bin_coord(L.smax[tid], rc.c16) - (double)M * (double)rc.c16) * 0.0625);
    }
    __syncthreads();

    int lo = kBins, hi = kBins;  // candidate bins, counted down from the maximum's bin; kBins = no cut
    // Units of the slices' histograms per row bin: bin b of slice s is bin b + shift[s] of the row;
    // thread t gathers row bins 4 t .. 4 t + 3 (all loads of four slices are requested before any
    // is used; loads are unconditional from clamped positions, what lies outside a slice's bins is
    // masked afterwards).
    const int rb0 = kBinsPerThread * tid;
    auto gather_units = [&](unsigned long long (&qsum)[kBinsPerThread]) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < kBinsPerThread; ++k)
            qsum[k] = 0ull;
        for (int s0 = 0; s0 < slices; s0 += 4) {
            unsigned qv[4][kBinsPerThread];
            int sh[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int sl = min(s0 + u, slices - 1);
                sh[u] = s0 + u < slices ? L.shift[sl] : kBins;
#pragma unroll
                for (int k = 0; k < kBinsPerThread; ++k) {
                    const int b = min(max(rb0 + k - sh[u], 0), kPubBins - 1);
                    qv[u][k] = W.hist[(size_t)sl * kPubBins + b];
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int k = 0; k < kBinsPerThread; ++k) {
                    const int b = rb0 + k - sh[u];
                    qsum[k] += (b >= 0 && b < kPubBins) ? qv[u][k] : 0u;
                }
        }
    };
    if (cut && !FILTERED) {
        // Estimate of the nucleus cut from the slices' histograms.
        unsigned long long qsum[kBinsPerThread];
        gather_units(qsum);
#pragma unroll
        for (int k = 0; k < kBinsPerThread; ++k)
            L.row.hist[rank_slot(rb0 + k)] = (double)qsum[k] * bin_unit(rb0 + k);
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
    }
    // A slice is covered when its emitted bins contain the row's cut bins and everything it summed
    // as above its window is above `lo` (bin b of the slice is bin b + shift of the row).
    if (tid < slices) {
        bool ok = !FILTERED;  // (a row with a filter is finished from its pairs further down)
        if (cut && !FILTERED) {
            const int a = L.swin_lo[tid], z = L.swin_hi[tid], sh = L.shift[tid];
            ok = L.scount[tid] >= 0 && z >= 0 && (a == 0 || a + sh <= lo) && (z >= kPubBins - 1 || hi <= z + sh);
        }
        L.covered[tid] = ok ? 1 : 0;
    }
    __syncthreads();
    // Bin tests without forming the bin (see the scan kernel): lo == kBins keeps everything,
    // hi == kBins - 1 makes every remaining element a candidate.
    const float t_above = lo >= kBins ? -INFINITY : kf_row - (float)lo + 1.f;
    const float t_cand = hi >= kBins - 1 ? -INFINITY : kf_row - (float)hi;

    // ---- mass kept for certain, per 256-element segment in vocabulary order; candidates ----------------
    // The row mass S is put together on the way: exact for every element this kernel sees (the pairs
    // of the covered slices, every logit of the others) and for what the covered slices summed above
    // their windows, estimated from the histograms for the bins past the windows.
    double s_part = 0.0;
    for (int sidx = tid; sidx < nseg; sidx += kBlock) {
        const int s = sidx / kSegPerSlice;
        const double v = L.covered[s] ? W.seg[sidx] * L.sfac[s] : 0.0;
        seg_mass[sidx] = v;
        s_part += v;
    }
    if (cut && tid < slices && L.covered[tid])
        s_part += L.srest[tid];
    __syncthreads();
    // One element: kept for certain -> its segment; inside the cut bins -> the candidate list (the
    // lanes of a wavefront take consecutive places reserved with one counter update); else dropped.
    // Called by whole wavefronts (`live` masks lanes that hold nothing).
    float f_part = 0.f;  // exact mass of the elements taken since the last widening
    // (the lane's place among the wavefront's candidates comes from the two lane-count instructions)
    auto append_masked = [&](unsigned long long mask, bool want, unsigned long long pair) __attribute__((always_inline)) {
        if (mask != 0ull) {
            unsigned base = 0u;
            if (lane == 0)
                base = atomicAdd(&L.cand_total, (unsigned)__popcll(mask));
            base = (unsigned)__builtin_amdgcn_readfirstlane((int)base);
            if (want) {
                const unsigned pos = __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, base));
                if (pos < (unsigned)kCandCap)
                    L.cand[pos] = pair;
            }
        }
    };
    auto take = [&](bool live, float xq, int idx, int s) __attribute__((always_inline)) {
        if (__builtin_amdgcn_ballot_w64(live) == 0ull)
            return;  // nothing in this wavefront's 64 places
        const float t = xq * rc.c16;
        const bool above = live && t >= t_above;
        const bool candq = live && !above && t >= t_cand;
        const float pq = live ? prob(xq, rs) : 0.f;
        f_part += pq;
        if (above)
            atomicAdd(&seg_mass[s * kSegPerSlice + (int)((unsigned)(idx - s * slice_elems) / (unsigned)kSeg)], (double)pq);
        append_masked(__builtin_amdgcn_ballot_w64(candq), candq,
                      (unsigned long long)__float_as_uint(xq) | ((unsigned long long)(unsigned)idx << 32));
    };
    // One wavefront-wide append to the candidate list.
    auto append = [&](bool want, unsigned long long pair) __attribute__((always_inline)) {
        append_masked(__builtin_amdgcn_ballot_w64(want), want, pair);
    };
    // Radix select over the order keys of the first C candidates, taken relative to the largest one
    // (rel = kmax - key, 0 = most probable) so that only the bits in which the candidates differ
    // are resolved: 11 bits per level, usually two levels.  Returns the key of the highest candidate
    // whose upper set (on top of `above0`) reaches `need`, counting candidates (`by_count`) or
    // summing their probabilities; `reached` is what that upper set amounts to, `bad` says that
    // the candidates do not reach `need` at all.
    auto radix_select = [&](int C, bool by_count, double above0, double need, bool& bad, double& reached) -> uint32_t {
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
        __syncthreads();  // an earlier call's readers of kmin / kmax are through
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
        double abv = above0;
        bad = !(above0 < need);
        for (int shift = 11 * ((nbits - 1) / 11); shift >= 0 && !bad; shift -= 11) {
            for (int i = tid; i < C; i += kBlock) {
                const float xc = __uint_as_float((unsigned)L.cand[i]);
                const uint32_t rel = kmax - order_key(xc);
                if ((uint64_t)rel >> (shift + 11) == prefix)
                    atomicAdd(&H[rank_slot((rel >> shift) & 0x7ffu)], by_count ? 1.0 : (double)prob(xc, rs));
            }
            __syncthreads();
            const BinPick pk = wave_pick(H, abv, need, false);
            // the threshold must fall among the candidates
            if (shift == 11 * ((nbits - 1) / 11) && !(above0 + pk.total >= need))
                bad = true;
            prefix = (prefix << 11) | (uint32_t)pk.bin;
            abv = pk.above;
            reached = pk.above + pk.in_bin;
            __syncthreads();
            if (shift > 0) {
                for (int b = tid; b < kBins; b += kBlock)
                    H[b] = 0.0;
                __syncthreads();
            }
        }
        return kmax - prefix;
    };
    // pairs written out by the covered slices: four consecutive ones per thread and slice, four slices
    // at a time, all requested before any is used (unconditional loads; what lies past a slice's count
    // is masked).  A wavefront of the scan kernel lists its pairs segment by segment, so a thread's
    // four pairs mostly belong to one 256-element segment: their kept mass is added up in the thread
    // and goes to the segment's sum with one LDS addition per run of equal segments (one addition
    // per pair would have most of a wavefront's lanes meet at one LDS address).
    static_assert(kEmitCap == 4 * kBlock, "four pairs per thread and slice");
    for (int s0 = 0; s0 < (FILTERED ? 0 : slices); s0 += 4) {
        unsigned long long ev[4][4];
        int cnt[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int s = min(s0 + u, slices - 1);
            cnt[u] = (s0 + u < slices && L.covered[s]) ? min(L.scount[s], kEmitCap) : 0;
            const ulonglong2* e = reinterpret_cast<const ulonglong2*>(W.emit + (size_t)s * kEmitCap) + 2 * tid;
            const ulonglong2 a = e[0], b = e[1];
            ev[u][0] = a.x;
            ev[u][1] = a.y;
            ev[u][2] = b.x;
            ev[u][3] = b.y;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int s = min(s0 + u, slices - 1);
            const int mine = min(max(cnt[u] - 4 * tid, 0), 4);  // how many of the four places hold a pair
            if (__builtin_amdgcn_ballot_w64(mine > 0) == 0ull)
                continue;  // nothing in this wavefront's 256 places
            double run = 0.0;   // kept mass of the present run of pairs of one segment
            int run_seg = -1;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool live = k < mine;
                const float xq = __uint_as_float((unsigned)ev[u][k]);
                const int idx = (int)(ev[u][k] >> 32);
                const float t = xq * rc.c16;
                const bool above = live && t >= t_above;
                const bool candq = live && !above && t >= t_cand;
                const float pq = live ? prob(xq, rs) : 0.f;
                f_part += pq;
                const int seg = s * kSegPerSlice + (int)((unsigned)(idx - s * slice_elems) / (unsigned)kSeg);
                if (above && seg != run_seg && run_seg >= 0) {
                    atomicAdd(&seg_mass[run_seg], run);
                    run = 0.0;
                }
                if (above) {
                    run_seg = seg;
                    run += (double)pq;
                }
                append_masked(__builtin_amdgcn_ballot_w64(candq), candq, ev[u][k]);
            }
            if (run_seg >= 0)
                atomicAdd(&seg_mass[run_seg], run);
        }
        s_part += (double)f_part;
        f_part = 0.f;
    }
    // slices that are not covered: a second look at their logits
    for (int s = 0; s < (FILTERED ? 0 : slices); ++s) {
        if (L.covered[s])
            continue;
        const SliceRange g = slice_range(s, slice_elems, V);
        float xv[32];
        SPD_LOAD_SLICE(xv, x, g, tid)
#pragma unroll
        for (int q = 0; q < 32; ++q) {
            const int i = g.e0 + (q >> 2) * kIter + tid * 4 + (q & 3);
            take(i < g.v4end, xv[q], i, s);
        }
        for (int k = 0; k < 3; ++k)
            take(tid == 0 && k < g.ntail, tid == 0 && k < g.ntail ? x[g.v4end + k] : 0.f, g.v4end + k, s);
        s_part += (double)f_part;
        f_part = 0.f;
    }
    uint32_t key_floor = 0u;  // rows with a filter: the lowest key that survives the filters
    if (FILTERED) {
        // ---- min-p and top-k ahead of the nucleus.  Both keep an upper set of the logits, and the scan
        // kernel wrote such a row's slices out from the top, so everything that survives is among the
        // pairs, provided every slice's window reaches as far down as the filters do; otherwise the
        // row goes to the whole-row routine.  Survivors become the candidate list. ----
        bool ok = slices <= 8;  // the pairs of a row stay in registers (four per thread and slice)
        // top-k: the k-th largest logit lies in row bins b1 .. b2, by the element-count bounds of the
        // histogram units (an element adds 32768 to 34219 units): the running units reach 32768 k no
        // later than the k-th element's bin and 34219 k no earlier
        int b1 = 0, b2 = 0;
        if (top_k > 0) {
            unsigned long long qsum[kBinsPerThread];
            gather_units(qsum);
#pragma unroll
            for (int k = 0; k < kBinsPerThread; ++k)
                L.row.hist[rank_slot(rb0 + k)] = (double)qsum[k];
            __syncthreads();
            const BinPick p1 = wave_pick(L.row.hist, 0.0, 32768.0 * (double)top_k, false);
            const BinPick p2 = wave_pick(L.row.hist, 0.0, 34219.0 * (double)top_k, false);
            b1 = p1.bin;
            b2 = p2.bin;
            // fewer than k elements inside the histogram's range: not a case for this path
            ok = ok && p2.total >= 34219.0 * (double)top_k && b2 < kBins - 1;
            __syncthreads();
        }
        // row bin that every slice's window has to reach: the k-th element's, else the last one that
        // can hold p >= min_p (bins are 1/16 octave; two bins of slack for the rounding of p)
        const int reach = top_k > 0 ? b2 : min(kBins - 1, (int)(-__log2f(min_p) * 16.f) + 2);
        if (tid < slices) {
            const int z = L.swin_hi[tid], sh = L.shift[tid];
            L.covered[tid] = sh >= kBins ||
                             (L.scount[tid] >= 0 && z >= 0 && L.swin_lo[tid] == 0 && (z >= kPubBins - 1 || z + sh >= reach));
        }
        __syncthreads();
        for (int s = 0; s < slices; ++s)
            ok = ok && L.covered[s];
        if (!ok) {
            sample_row_from_memory(sp, r, L.row);
            return;
        }
        unsigned long long ev[8][4];
        int cnt[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int s = min(u, slices - 1);
            cnt[u] = (u < slices && L.shift[s] < kBins) ? min(L.scount[s], kEmitCap) : 0;
            const unsigned long long* e = W.emit + (size_t)s * kEmitCap;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                ev[u][k] = e[tid + k * kBlock];
        }
        uint32_t key_k = 0u;
        if (top_k > 0) {
            // elements above bin b1 are counted, those in b1 .. b2 listed; the k-th largest is found
            // among the listed ones by rank
            const float t_b1 = b1 <= 0 ? INFINITY : kf_row - (float)b1 + 1.f;
            const float t_b2 = kf_row - (float)b2;
            int n_above = 0;
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const bool live = tid + k * kBlock < cnt[u];
                    const float t = __uint_as_float((unsigned)ev[u][k]) * rc.c16;
                    const bool above = live && t >= t_b1;
                    n_above += above ? 1 : 0;
                    append(live && !above && t >= t_b2, ev[u][k]);
                }
            double da = (double)n_above, db = 0.0;
            block_sum2_f64(da, db, L.row.scratch);  // (its barriers also complete the list)
            const unsigned listed = L.cand_total;
            const double rank = (double)top_k - da;
            bool bad = listed > (unsigned)kCandCap || rank < 1.0;
            double reached = 0.0;
            if (!bad)
                key_k = radix_select((int)listed, true, 0.0, rank, bad, reached);
            if (bad) {
                sample_row_from_memory(sp, r, L.row);
                return;
            }
            __syncthreads();
            if (tid == 0)
                L.cand_total = 0u;
            __syncthreads();
        }
        // survivors: at least as large as the k-th largest logit, and p >= min_p
        uint32_t kfl = 0xffffffffu;
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float xq = __uint_as_float((unsigned)ev[u][k]);
                const uint32_t key = order_key(xq);
                const float pq = prob(xq, rs);
                const bool keep = tid + k * kBlock < cnt[u] && key >= key_k && pq >= min_p;
                f_part += keep ? pq : 0.f;
                kfl = keep ? min(kfl, key) : kfl;
                append(keep, ev[u][k]);
            }
        s_part += (double)f_part;
        for (int o = 32; o > 0; o >>= 1)
            kfl = min(kfl, (uint32_t)__shfl_xor((int)kfl, o));
        if (lane == 0)
            L.kmin[wave] = kfl;
        __syncthreads();
        key_floor = 0xffffffffu;
        for (int w = 0; w < kWaves; ++w)
            key_floor = min(key_floor, L.kmin[w]);
        lo = 0;            // no bin is kept wholesale,
        hi = kBins - 1;    // every element is compared with the threshold
    }
    __syncthreads();
    const unsigned cand_total = L.cand_total;
    const int C = (int)min(cand_total, (unsigned)kCandCap);
    double above_total = 0.0;
    for (int sidx = tid; sidx < nseg; sidx += kBlock)
        above_total += seg_mass[sidx];
    block_sum2_f64(above_total, s_part, L.row.scratch);
    const double need = (double)top_p * s_part;  // s_part: the row mass S (of what the filters left)

    uint32_t key_tau = key_floor;
    double Z = FILTERED ? s_part : above_total;
    bool bad = cand_total > (unsigned)kCandCap;
    if (cut && !bad) {
        const uint32_t key_cut = radix_select(C, false, above_total, need, bad, Z);
        key_tau = max(key_tau, key_cut);
    }
    if (bad) {
        // candidate overflow or an estimate that missed the cut: redo the row the slow way
        sample_row_from_memory(sp, r, L.row);
        return;
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
    // Two workgroups per CU, at most eight slices unless the vocabulary needs more (the row-level
    // step reads every slice's histogram), and no slice shorter than 4096 logits.
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
    if (slices == 0 || !aligned || p.vocab < 4) {
        hipLaunchKernelGGL(sample_rows_kernel, dim3((unsigned)p.rows), dim3(kBlock), 0, s, p);
        return hipGetLastError();
    }
    int slice_elems = (int)((p.vocab + slices - 1) / slices);
    slice_elems = (slice_elems + 3) / 4 * 4;
    hipLaunchKernelGGL(sampler_scan_kernel, dim3((unsigned)(p.rows * slices)), dim3(kBlock), 0, s, p, (char*)ws, slices,
                       slice_elems);
    hipLaunchKernelGGL(sampler_finish_kernel<false>, dim3((unsigned)p.rows), dim3(kBlock), 0, s, p, (char*)ws, slices,
                       slice_elems);
    if (p.top_k || p.min_p)  // rows with a filter
        hipLaunchKernelGGL(sampler_finish_kernel<true>, dim3((unsigned)p.rows), dim3(kBlock), 0, s, p, (char*)ws,
                           slices, slice_elems);
    return hipGetLastError();
}

}  // namespace spd
