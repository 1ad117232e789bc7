// Temperature / nucleus / inverse-CDF token sampler.  One workgroup per row.
//
// Passes over the row (the first comes from HBM, the rest hit cache):
//   1. row maximum (and, for T == 0, the lowest index attaining it);
//   2. p_i = 2^((x_i - max) * log2(e)/T) in fp32, total mass S in fp64, and a mass
//      histogram keyed on the top bits of p's bit pattern;
//   3. (only if the nucleus cuts anything) two refinement histograms on the lower
//      bits, which pin the threshold tau to one exact bit pattern: the largest
//      value t with mass{p >= t} >= top_p * S.  Comparisons are on bit patterns, so
//      the kept set {p_i >= tau} includes every tie by construction;
//   4. kept mass of 256-element segments in vocabulary order, a scan over the
//      segments, and a walk inside the segment that contains u * Z.
// Probabilities are evaluated by one shared routine so every pass sees the same
// bits; all sums that decide something are carried in fp64.
#include "spd_internal.h"

namespace spd {
namespace {

constexpr int kBlock = 1024;
constexpr int kWaves = kBlock / 64;
constexpr int kBins = 2048;
constexpr int kSeg = 256;           // elements per wave per tile (64 lanes x 4)
constexpr int kTile = kWaves * kSeg;  // 4096 elements per block iteration
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
__device__ void pick_bin(const double* hist, double above, double need, int* bin_out,
                         int* low_out, double* above_out, double* scratch /* kBlock */)
{
    const int tid = threadIdx.x;
    // thread 0 owns the two highest bins, thread 1 the next two, ...
    const int b_hi = kBins - 1 - 2 * tid, b_lo = b_hi - 1;
    const double h_hi = hist[b_hi], h_lo = hist[b_lo];
    const double own = h_hi + h_lo;
    double incl = own;
    if (tid == 0) {
        *bin_out = -1;
        *low_out = kBins;
    }
    __syncthreads();
    scratch[tid] = incl;
    __syncthreads();
    for (int o = 1; o < kBlock; o <<= 1) {
        const double add = tid >= o ? scratch[tid - o] : 0.0;
        __syncthreads();
        incl += add;
        scratch[tid] = incl;
        __syncthreads();
    }
    const double before = above + (incl - own);
    if (h_hi > 0.0) {
        atomicMin(low_out, b_hi);
        if (before + h_hi >= need)
            atomicMax(bin_out, b_hi);
    }
    if (h_lo > 0.0) {
        atomicMin(low_out, b_lo);
        if (before + own >= need)
            atomicMax(bin_out, b_lo);
    }
    __syncthreads();
    const int chosen = *bin_out >= 0 ? *bin_out : (*low_out < kBins ? *low_out : 0);
    __syncthreads();
    if (chosen == b_hi)
        *above_out = before;
    if (chosen == b_lo)
        *above_out = before + h_hi;
    if (tid == 0)
        *bin_out = chosen;
    __syncthreads();
}

__global__ __launch_bounds__(kBlock) void sample_rows_kernel(SamplerParams sp)
{
    __shared__ double hist[kBins];
    __shared__ double scratch[kBlock];
    __shared__ double seg_mass[kMaxSegments];
    __shared__ int sh_low;
    __shared__ float red_f[kWaves];
    __shared__ int red_i[kWaves];
    __shared__ int sh_bin;
    __shared__ double sh_above;
    __shared__ int sh_token;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long r = blockIdx.x;
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

}  // namespace

hipError_t launch_sampler(const SamplerParams& p, hipStream_t s)
{
    hipLaunchKernelGGL(sample_rows_kernel, dim3((unsigned)p.rows), dim3(kBlock), 0, s, p);
    return hipGetLastError();
}

}  // namespace spd
