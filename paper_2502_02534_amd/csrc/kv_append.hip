// Appends one token's K and V to every live sample's private suffix and bumps the sample's
// length on the device: the step between two decode steps of the sampling loop (the paper
// generates up to 1024 tokens per sample, App. "Experiment settings").  Lengths stay on the
// device, so a loop of steps needs no host synchronisation.
//
// One workgroup per sample; a thread moves 16-byte pieces.  A sample is finished once its last token
// was the end token; finished samples, and samples whose slot is full, are left alone.
#include "step_bodies.h"

namespace spd {
namespace {

__global__ __launch_bounds__(256) void kv_append_kernel(KvAppendParams a)
{
    step_impl::append_sample(a, blockIdx.x, a.k_new, a.v_new, nullptr);
}

}  // namespace

hipError_t launch_kv_append(const KvAppendParams& a, hipStream_t s)
{
    hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)a.N), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace spd
