// Temperature / nucleus / inverse-CDF token sampler.
//
// Two paths.  The sliced path (below, four stream-ordered kernels) reads a row from HBM once,
// takes a second look that caches serve when the logits fit, and finds the exact nucleus
// threshold without sorting.  The whole-row routine (one workgroup per row, every pass from
// memory) covers rows the sliced path does not take: unaligned rows, vocabularies beyond
// 16 slices, and the rare row whose candidate set overflows.
//
// Probabilities are evaluated by one shared routine, p_i = 2^((x_i - max) c) with
// c = log2(e)/T carried as hi + lo floats, so every pass sees the same bits; every sum that
// decides something is carried in fp64; comparisons that define the kept set are on bit
// patterns, so all ties with the threshold are kept by construction.
#include "spd_internal.h"

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

    // ---- pass 2: total mass and top-level histogram -------------------------------------
    for (int b = tid; b < kBins; b += kBlock)
        hist[b] = 0.0;
    __syncthreads();
    const float top_p = sp.top_p[r];
    const bool cut = top_p < 1.f;
    double part = 0.0;
    {
        float acc = 0.f;
        int cnt = 0;
        for (int i = tid; i < V; i += kBlock) {
            const float pv = prob(x[i], rs);
            acc += pv;
            if (++cnt == 32) {  // bound the fp32 run length before widening
                part += (double)acc;
                acc = 0.f;
                cnt = 0;
            }
            if (cut)
                atomicAdd(&hist[(__float_as_uint(pv) >> 20) & 0x7ffu], (double)pv);
        }
        part += (double)acc;
    }
    const double S = block_sum_f64(part, scratch);

    uint32_t tau_bits = 0u;  // keep everything
    double Z = S;
    if (cut) {
        const double need = (double)top_p * S;
        // level 1: bits 30..20
        pick_bin(hist, 0.0, need, &sh_bin, &sh_low, &sh_above, scratch);
        const uint32_t b1 = (uint32_t)sh_bin;
        double above = sh_above;
        __syncthreads();
        // level 2: bits 19..9 of the patterns that share b1
        for (int b = tid; b < kBins; b += kBlock)
            hist[b] = 0.0;
        __syncthreads();
        for (int i = tid; i < V; i += kBlock) {
            const float pv = prob(x[i], rs);
            const uint32_t u = __float_as_uint(pv) & 0x7fffffffu;
            if ((u >> 20) == b1)
                atomicAdd(&hist[(u >> 9) & 0x7ffu], (double)pv);
        }
        __syncthreads();
        pick_bin(hist, above, need, &sh_bin, &sh_low, &sh_above, scratch);
        const uint32_t b2 = (uint32_t)sh_bin;
        above = sh_above;
        __syncthreads();
        // level 3: bits 8..0
        for (int b = tid; b < kBins; b += kBlock)
            hist[b] = 0.0;
        __syncthreads();
        const uint32_t prefix = (b1 << 11) | b2;
        for (int i = tid; i < V; i += kBlock) {
            const float pv = prob(x[i], rs);
            const uint32_t u = __float_as_uint(pv) & 0x7fffffffu;
            if ((u >> 9) == prefix)
                atomicAdd(&hist[u & 0x1ffu], (double)pv);
        }
        __syncthreads();
        pick_bin(hist, above, need, &sh_bin, &sh_low, &sh_above, scratch);
        tau_bits = (prefix << 9) | (uint32_t)sh_bin;
        __syncthreads();
    }

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
// handled by four small kernels in stream order (no workgroup ever waits for another):
//
//   hist   (rows x slices)  one HBM pass: slice maximum (and its lowest index) and a histogram
//          of scaled mass over bins of width 1/16 in log2 p.  The bin of a logit is
//          floor(x c 16), an integer function of x alone; a histogram built against the slice
//          maximum differs from one built against the row maximum by an integer shift.
//          Mass is accumulated in u32 fixed point relative to the bin's own reference
//          (q = 2^(frac/16) 2^15 in [32768, 34219]), which needs no maximum at all.
//   cut    (rows)           combines the slices' histograms and picks the bin that holds the
//          nucleus cut, plus a neighbour when the estimate cannot decide.
//   mass   (rows x slices)  second look at the slice (served by cache when the logits fit):
//          p_i = 2^((x_i - row max) c) exactly as defined, slice mass in fp64, mass of the
//          certainly-kept elements per 256-element segment in vocabulary order, and the
//          elements of the cut bins as candidates (logit, index).
//   pick   (rows)           exact threshold among the candidates by radix select on the logit's
//          bit pattern with fp64 masses, kept candidates added to their segments, scan of the
//          segments, walk inside the segment that contains u * Z.
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
    float kf_max;   // floor(max_x * c16)
    int nbins;      // histogram bins written
    double mass;    // sum of p over the slice (mass kernel)
    double above;   // mass of certainly-kept elements (mass kernel)
};

struct RowCut {
    float max_x;        // row maximum
    float kf_row;       // floor(max_x * c16)
    int lo, hi;         // candidate bins, counted down from the maximum's bin; kBins = no cut
    int done;           // 1 = token already written (greedy row)
    unsigned cand_total;
};

__host__ __device__ inline size_t sliced_row_bytes(int slices)
{
    return 256 + (size_t)slices * 64 + (size_t)slices * kBins * 4 + (size_t)slices * kSegPerSlice * 8 +
           (size_t)kCandCap * 8;
}

struct RowWs {
    RowCut* cut;
    SliceStat* stat;      // [slices], 64 B apart
    unsigned* hist;       // [slices][kBins]
    double* seg;          // [slices][kSegPerSlice]
    unsigned long long* cand;  // [kCandCap] logit bits | index << 32
};

__device__ __forceinline__ RowWs row_ws(char* base, long long row, int slices)
{
    char* p = base + row * sliced_row_bytes(slices);
    RowWs w;
    w.cut = (RowCut*)p;
    p += 256;
    w.stat = (SliceStat*)p;
    p += (size_t)slices * 64;
    w.hist = (unsigned*)p;
    p += (size_t)slices * kBins * 4;
    w.seg = (double*)p;
    p += (size_t)slices * kSegPerSlice * 8;
    w.cand = (unsigned long long*)p;
    return w;
}

__device__ __forceinline__ SliceStat* stat_at(const RowWs& w, int s)
{
    return (SliceStat*)((char*)w.stat + (size_t)s * 64);
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

#define SPD_LOAD_SLICE(xv, x, g, tid)                                                   \
    _Pragma("unroll") for (int j = 0; j < 8; ++j)                                       \
    {                                                                                   \
        const int i_ = (g).e0 + j * kIter + (tid) * 4;                                  \
        float4 v_ = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);            \
        if (i_ < (g).v4end)                                                             \
            v_ = *reinterpret_cast<const float4*>((x) + i_);                            \
        (xv)[4 * j] = v_.x;                                                             \
        (xv)[4 * j + 1] = v_.y;                                                         \
        (xv)[4 * j + 2] = v_.z;                                                         \
        (xv)[4 * j + 3] = v_.w;                                                         \
    }

// ---- kernel 1: slice maximum and histogram -----------------------------------------------------------
__global__ __launch_bounds__(kBlock) void sampler_hist_kernel(SamplerParams sp, char* ws, int slices,
                                                              int slice_elems)
{
    __shared__ unsigned hist[kBins];
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
    for (int b = tid; b < kBins; b += kBlock)
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

    const RowConst rc = row_const(greedy ? 1.f : T);
    const float kf_loc = bin_coord(mx, rc.c16);
    int nbins = 0;
    if (cut) {
        int bmax = -1;
        auto add = [&](float xq) {
            const float t = xq * rc.c16;
            const float kf = floorf(t);
            const int b = min(bin_below(kf_loc, kf), kPubBins - 1);
            // mass relative to the bin's own reference 2^(kf/16): 2^(frac/16) in [1, 2^(1/16))
            const unsigned q = (unsigned)(__builtin_amdgcn_exp2f((t - kf) * 0.0625f) * 32768.f + 0.5f);
            atomicAdd(&hist[b], q);
            bmax = max(bmax, b);
        };
#pragma unroll
        for (int q = 0; q < 32; ++q)
            if (xv[q] != -INFINITY)
                add(xv[q]);
        if (tid == 0)
            for (int k = 0; k < g.ntail; ++k)
                add(x[g.v4end + k]);
        (void)bmax;
        __syncthreads();  // histogram complete
        // a fixed number of bins is written so that the reader needs nothing else to fetch them
        nbins = kPubBins;
        for (int b = tid; b < kPubBins; b += kBlock)
            W.hist[(size_t)slice * kBins + b] = hist[b];
    }
    if (tid == 0) {
        SliceStat* st = stat_at(W, slice);
        st->max_x = mx;
        st->argmax = mi;
        st->kf_max = kf_loc;
        st->nbins = nbins;
    }
}

// 2^(-k/16), k = 0..15
__device__ const double kRoot16[16] = {
    1.0,                 0.95760328069857365, 0.91700404320467122, 0.87812608018664974,
    0.84089641525371454, 0.80524516597462716, 0.77110541270397041, 0.73841307296974966,
    0.70710678118654752, 0.67712777346844633, 0.64841977732550483, 0.62092890603674203,
    0.59460355750136054, 0.56939431737834583, 0.54525386633262883, 0.52213689121370692};

// ---- kernel 2: the row's cut bins --------------------------------------------------------------------
struct CutLds {
    double hist[kBins];
    double scratch[kWaves];
    float smax[kMaxSlices];
    int snb[kMaxSlices];
    int sarg[kMaxSlices];
    int shift[kMaxSlices];
    int sh_bin, sh_low;
    double sh_above;
};

__global__ __launch_bounds__(kBlock) void sampler_cut_kernel(SamplerParams sp, char* ws, int slices)
{
    __shared__ CutLds L;
    const int tid = threadIdx.x;
    const long long r = blockIdx.x;
    const RowWs W = row_ws(ws, r, slices);
    const float T = sp.temperature[r];
    const bool greedy = (T == 0.f);
    const float top_p = sp.top_p[r];
    const bool cut = !greedy && top_p < 1.f;
    // everything this kernel reads from memory is requested up front, in one round
    constexpr int kPerThread = kMaxSlices * kPubBins / kBlock;
    unsigned qv[kPerThread];
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) {
        const int it = tid + u * kBlock;
        const int sl = it / kPubBins, b = it % kPubBins;
        qv[u] = (cut && sl < slices) ? W.hist[(size_t)sl * kBins + b] : 0u;
    }
    if (tid < slices) {
        const SliceStat* st = stat_at(W, tid);
        L.smax[tid] = st->max_x;
        L.snb[tid] = st->nbins;
        L.sarg[tid] = st->argmax;
    }
    __syncthreads();
    float M = -INFINITY;
    int nb_max = 0, arg = 0x7fffffff;
    for (int s = 0; s < slices; ++s) {
        if (L.smax[s] > M || (L.smax[s] == M && L.sarg[s] < arg)) {
            M = L.smax[s];
            arg = L.sarg[s];
        }
        nb_max = max(nb_max, L.snb[s]);
    }
    const RowConst rc = row_const(greedy ? 1.f : T);
    const float kf_row = bin_coord(M, rc.c16);
    int lo = kBins, hi = kBins;
    if (cut) {
        if (tid < slices)
            L.shift[tid] = L.smax[tid] == -INFINITY
                               ? 0
                               : (int)fminf(fmaxf(kf_row - bin_coord(L.smax[tid], rc.c16), 0.f), (float)kBins);
        for (int b = tid; b < kBins; b += kBlock)
            L.hist[b] = 0.0;
        __syncthreads();
        // bin b of slice s is bin b + shift[s] of the row; mass = q 2^-15 2^(-bin/16) relative to
        // the reference of the row maximum's bin.  Stored mirrored (most probable bin last) for
        // pick_bin.
#pragma unroll
        for (int u = 0; u < kPerThread; ++u) {
            if (qv[u]) {
                const int it = tid + u * kBlock;
                const int sl = it / kPubBins, b = it % kPubBins;
                const int rb = min(b + L.shift[sl], kBins - 1);
                // q 2^-15 2^(-rb/16): sixteenth roots from a table, the rest is an exponent shift
                atomicAdd(&L.hist[kBins - 1 - rb], ldexp((double)qv[u] * kRoot16[rb & 15], -15 - (rb >> 4)));
            }
        }
        __syncthreads();
        double part = 0.0;
        for (int b = tid; b < kBins; b += kBlock)
            part += L.hist[b];
        const double S_est = block_sum_f64(part, L.scratch);
        const double need = (double)top_p * S_est;
        pick_bin(L.hist, 0.0, need, &L.sh_bin, &L.sh_low, &L.sh_above, L.scratch);
        const int bsel = kBins - 1 - L.sh_bin;
        const double above_est = L.sh_above, in_bin = L.hist[L.sh_bin];
        // the estimate is good to about 1e-5 of the total; be generous
        const double tol = 1e-3 * S_est;
        lo = hi = bsel;
        if (need - above_est <= tol && lo > 0)
            --lo;
        if (above_est + in_bin - need <= tol && hi < kBins - 1)
            ++hi;
    }
    if (tid == 0) {
        RowCut* c = W.cut;
        c->max_x = M;
        c->kf_row = kf_row;
        c->lo = lo;
        c->hi = hi;
        c->done = greedy ? 1 : 0;
        c->cand_total = 0u;
        if (greedy)
            sp.tokens[r] = arg == 0x7fffffff ? 0 : arg;
    }
}

// ---- kernel 3: exact masses, segments, candidates -------------------------------------------------------
__global__ __launch_bounds__(kBlock) void sampler_mass_kernel(SamplerParams sp, char* ws, int slices,
                                                              int slice_elems)
{
    __shared__ double scratch[kWaves];
    __shared__ int wave_cnt[kWaves];
    __shared__ unsigned cand_base;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long r = blockIdx.x / slices;
    const int slice = blockIdx.x % slices;
    const RowWs W = row_ws(ws, r, slices);
    const RowCut cutv = *W.cut;
    if (cutv.done)
        return;
    const float* __restrict__ x = sp.logits + r * sp.stride;
    const SliceRange g = slice_range(slice, slice_elems, (int)sp.vocab);
    const RowConst rc = row_const(sp.temperature[r]);
    RowScale rs;
    rs.max_x = cutv.max_x;
    rs.c_hi = rc.c_hi;
    rs.c_lo = rc.c_lo;
    const int lo = cutv.lo, hi = cutv.hi;
    // Bin tests without forming the bin: with t = x c16, bin(x) < lo  <=>  floor(t) > kf_row - lo
    // <=>  t >= kf_row - lo + 1 (both sides of the middle inequality are integers); likewise
    // bin(x) <= hi  <=>  t >= kf_row - hi.  The clamps of the bin only matter at the ends:
    // lo == kBins keeps everything, hi == kBins - 1 makes every remaining element a candidate.
    const float t_above = lo >= kBins ? -INFINITY : cutv.kf_row - (float)lo + 1.f;
    const float t_cand = hi >= kBins - 1 ? -INFINITY : cutv.kf_row - (float)hi;

    float xv[32];
    SPD_LOAD_SLICE(xv, x, g, tid)

    int ncand = 0;
    double above = 0.0;
    float all32 = 0.f;  // this thread's 32 probabilities; widened once
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float s_above = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float xq = xv[4 * j + k];
            if (xq == -INFINITY)
                continue;
            const float p = prob(xq, rs);
            all32 += p;
            const float t = xq * rc.c16;
            if (t >= t_above)
                s_above += p;
            else if (t >= t_cand)
                ++ncand;
        }
        // 256 fp32 terms per segment; the segment sums are widened before they are combined
        for (int o = 32; o > 0; o >>= 1)
            s_above += __shfl_xor(s_above, o);
        if (lane == 0) {
            W.seg[(size_t)slice * kSegPerSlice + j * kWaves + wave] = (double)s_above;
            above += (double)s_above;
        }
    }
    double mass = (double)all32;
    // tail logits (thread 0): counted in the slice mass, always sent as candidates when kept at all
    int tail_cand = 0;
    if (tid == 0)
        for (int k = 0; k < g.ntail; ++k) {
            const float xt = x[g.v4end + k];
            mass += (double)prob(xt, rs);
            if (bin_below(cutv.kf_row, bin_coord(xt, rc.c16)) <= hi || lo == kBins)
                ++tail_cand;
        }
    ncand += tail_cand;
    mass = block_sum_f64(mass, scratch);
    above = block_sum_f64(above, scratch);

    int incl = ncand;
    for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o);
        if (lane >= o)
            incl += up;
    }
    __syncthreads();
    if (lane == 63)
        wave_cnt[wave] = incl;
    __syncthreads();
    int wave_off = 0, block_total = 0;
    for (int w = 0; w < kWaves; ++w) {
        if (w < wave)
            wave_off += wave_cnt[w];
        block_total += wave_cnt[w];
    }
    if (tid == 0) {
        cand_base = block_total ? atomicAdd(&W.cut->cand_total, (unsigned)block_total) : 0u;
        SliceStat* st = stat_at(W, slice);
        st->mass = mass;
        st->above = above;
    }
    __syncthreads();
    if (ncand) {
        unsigned pos = cand_base + (unsigned)(wave_off + incl - ncand);
#pragma unroll
        for (int q = 0; q < 32; ++q) {
            const float xq = xv[q];
            if (xq == -INFINITY)
                continue;
            const float t = xq * rc.c16;
            if (t < t_above && t >= t_cand) {
                if (pos < (unsigned)kCandCap)
                    W.cand[pos] = (unsigned long long)__float_as_uint(xq) |
                                  ((unsigned long long)(unsigned)(g.e0 + (q >> 2) * kIter + tid * 4 + (q & 3)) << 32);
                ++pos;
            }
        }
        if (tid == 0)
            for (int k = 0; k < g.ntail; ++k) {
                const float xt = x[g.v4end + k];
                if (bin_below(cutv.kf_row, bin_coord(xt, rc.c16)) <= hi || lo == kBins) {
                    if (pos < (unsigned)kCandCap)
                        W.cand[pos] = (unsigned long long)__float_as_uint(xt) |
                                      ((unsigned long long)(unsigned)(g.v4end + k) << 32);
                    ++pos;
                }
            }
    }
}

// ---- kernel 4: exact threshold, CDF walk -----------------------------------------------------------------
struct PickLds {
    RowLds row;
    unsigned long long cand[kCandCap];
    double smass[kMaxSlices];
    double sabove[kMaxSlices];
};

__global__ __launch_bounds__(kBlock) void sampler_pick_kernel(SamplerParams sp, char* ws, int slices,
                                                              int slice_elems)
{
    __shared__ PickLds L;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long r = blockIdx.x;
    const RowWs W = row_ws(ws, r, slices);
    const RowCut cutv = *W.cut;
    if (cutv.done)
        return;
    const float* __restrict__ x = sp.logits + r * sp.stride;
    const int V = (int)sp.vocab;
    const RowConst rc = row_const(sp.temperature[r]);
    RowScale rs;
    rs.max_x = cutv.max_x;
    rs.c_hi = rc.c_hi;
    rs.c_lo = rc.c_lo;
    const int lo = cutv.lo, hi = cutv.hi;
    const bool cut = lo < kBins;
    const int C = (int)min(cutv.cand_total, (unsigned)kCandCap);
    const int nseg = slices * kSegPerSlice;
    double* seg_mass = L.row.seg_mass;

    // everything this kernel needs from memory, fetched in one round
    if (tid < slices) {
        const SliceStat* st = stat_at(W, tid);
        L.smass[tid] = st->mass;
        L.sabove[tid] = st->above;
    }
    for (int i = tid; i < C; i += kBlock)
        L.cand[i] = W.cand[i];
    for (int sidx = tid; sidx < nseg; sidx += kBlock)
        seg_mass[sidx] = W.seg[sidx];
    __syncthreads();
    double S = 0.0, above_total = 0.0;
    for (int s = 0; s < slices; ++s) {
        S += L.smass[s];
        above_total += L.sabove[s];
    }
    const double need = (double)sp.top_p[r] * S;

    // candidate masses by the definition of p_i (deterministic tree)
    double cm = 0.0;
    for (int i = tid; i < C; i += kBlock)
        cm += (double)prob(__uint_as_float((unsigned)L.cand[i]), rs);
    cm = block_sum_f64(cm, L.row.scratch);

    uint32_t key_tau = 0u;
    double Z = above_total + cm;
    if (cut) {
        // the cut must fall among the candidates; otherwise redo the row the slow way
        if (cutv.cand_total > (unsigned)kCandCap || !(above_total < need) || !(above_total + cm >= need)) {
            sample_row_from_memory(sp, r, L.row);
            return;
        }
        // radix select over the candidates' order keys: 11 + 11 + 10 bits
        double* H = L.row.hist;
        uint32_t prefix = 0u;
        double above = above_total;
        for (int level = 0; level < 3; ++level) {
            const int shift = level == 0 ? 21 : level == 1 ? 10 : 0;
            const int bits = level == 2 ? 10 : 11;
            for (int b = tid; b < kBins; b += kBlock)
                H[b] = 0.0;
            __syncthreads();
            for (int i = tid; i < C; i += kBlock) {
                const float xc = __uint_as_float((unsigned)L.cand[i]);
                const uint32_t key = order_key(xc);
                if (level == 0 || (key >> (shift + bits)) == prefix)
                    atomicAdd(&H[(key >> shift) & ((1u << bits) - 1u)], (double)prob(xc, rs));
            }
            __syncthreads();
            pick_bin(H, above, need, &L.row.sh_bin, &L.row.sh_low, &L.row.sh_above, L.row.scratch);
            prefix = (prefix << bits) | (uint32_t)L.row.sh_bin;
            above = L.row.sh_above;
            __syncthreads();
        }
        key_tau = prefix;
        double kept = 0.0;
        for (int i = tid; i < C; i += kBlock) {
            const float xc = __uint_as_float((unsigned)L.cand[i]);
            if (order_key(xc) >= key_tau)
                kept += (double)prob(xc, rs);
        }
        Z = above_total + block_sum_f64(kept, L.row.scratch);
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
                    const int b = bin_below(cutv.kf_row, bin_coord(xi, rc.c16));
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
    long long s = (512 + rows - 1) / rows;  // two workgroups per CU
    const long long smax_small = vocab / 2048 > 1 ? vocab / 2048 : 1;
    if (s > smax_small) s = smax_small;
    if (s > kMaxSlices) s = kMaxSlices;
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
    if (slices == 0 || !aligned) {
        hipLaunchKernelGGL(sample_rows_kernel, dim3((unsigned)p.rows), dim3(kBlock), 0, s, p);
        return hipGetLastError();
    }
    int slice_elems = (int)((p.vocab + slices - 1) / slices);
    slice_elems = (slice_elems + 3) / 4 * 4;
    const dim3 per_slice((unsigned)(p.rows * slices)), per_row((unsigned)p.rows), block(kBlock);
    hipLaunchKernelGGL(sampler_hist_kernel, per_slice, block, 0, s, p, (char*)ws, slices, slice_elems);
    hipLaunchKernelGGL(sampler_cut_kernel, per_row, block, 0, s, p, (char*)ws, slices);
    hipLaunchKernelGGL(sampler_mass_kernel, per_slice, block, 0, s, p, (char*)ws, slices, slice_elems);
    hipLaunchKernelGGL(sampler_pick_kernel, per_row, block, 0, s, p, (char*)ws, slices, slice_elems);
    return hipGetLastError();
}

}  // namespace spd
