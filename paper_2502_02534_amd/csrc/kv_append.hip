// Appends one token's K and V to every live sample's private suffix and bumps the sample's
// length on the device: the step between two decode steps of the sampling loop (the paper
// generates up to 1024 tokens per sample, App. "Experiment settings").  Lengths stay on the
// device, so a loop of steps needs no host synchronisation.
//
// One workgroup per sample; a thread moves 16 bytes.  A sample is finished once its last token
// was the end token; finished samples, and samples whose slot is full, are left alone.
#include "spd_internal.h"

namespace spd {
namespace {

__global__ __launch_bounds__(256) void kv_append_kernel(KvAppendParams a)
{
    const int n = blockIdx.x;
    __shared__ int s_pos;
    if (threadIdx.x == 0) {
        int pos = a.suffix_lens[n];
        bool live = pos < a.capacity;
        if (a.page_size != 0)  // and inside the sample's own page list
            live = live && pos / a.page_size < a.page_indptr[n + 1] - a.page_indptr[n];
        if (a.finished) {
            if (a.last_tokens && a.last_tokens[n] == a.end_token)
                a.finished[n] = 1;
            live = live && a.finished[n] == 0;
        }
        s_pos = live ? pos : -1;
    }
    __syncthreads();
    const int pos = s_pos;
    if (pos < 0)
        return;
    const int row_u4 = a.Hkv * a.D * a.elt / 16;   // 16-byte pieces of one token (all KV heads)
    const int head_u4 = a.D * a.elt / 16;
    const uint4* ks = (const uint4*)a.k_new + (long long)n * row_u4;
    const uint4* vs = (const uint4*)a.v_new + (long long)n * row_u4;
    for (int i = threadIdx.x; i < row_u4; i += blockDim.x) {
        long long dst;
        if (a.page_size == 0) {
            dst = ((long long)n * a.capacity + pos) * row_u4 + i;
        } else {
            const int j = i / head_u4, c = i % head_u4;
            const long long pg = a.pages[a.page_indptr[n] + pos / a.page_size];
            dst = ((pg * a.Hkv + j) * a.page_size + pos % a.page_size) * head_u4 + c;
        }
        ((uint4*)a.k_suffix)[dst] = ks[i];
        ((uint4*)a.v_suffix)[dst] = vs[i];
    }
    if (threadIdx.x == 0)
        a.suffix_lens[n] = pos + 1;
}

}  // namespace

hipError_t launch_kv_append(const KvAppendParams& a, hipStream_t s)
{
    hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)a.N), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace spd
