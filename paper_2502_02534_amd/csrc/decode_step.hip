// Rows of a decode loop chosen by a step counter that lives on the device: the inputs of step t
// (queries, the new token's K and V, the uniforms) are copied out of [steps, ...] tensors into the
// buffers the step's calls read, and the step's results (tokens, lengths, outputs) are copied
// into row t of [steps, ...] records, so that one captured step can be replayed for a whole loop
// of the paper's up-to-1024-token generations (App. "Experiment settings") without the host.
//
// The counter is a pair {current, next}.  The select kernel reads `current` in every workgroup
// and one thread stores next = current + 1; the record kernel reads `next` in every workgroup
// and one thread stores current = next.  No kernel reads a word that the same kernel writes.
#include "spd_internal.h"

namespace spd {
namespace {

constexpr int kCopyThreads = 256;
constexpr long long kBytesPerBlock = 16ll * kCopyThreads * 8;  // eight 16-byte pieces per thread

template <bool RECORD>
__global__ __launch_bounds__(kCopyThreads) void step_rows_kernel(StepRowsParams a)
{
    // which copy this workgroup belongs to
    int i = 0;
#pragma unroll
    for (int k = 1; k < kMaxStepCopies; ++k)
        if (k < a.count && (int)blockIdx.x >= a.first_block[k])
            i = k;
    const long long blk = (long long)blockIdx.x - a.first_block[i];
    const long long step = RECORD ? a.state[1] - 1 : a.state[0];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (RECORD)
            a.state[0] = step + 1;
        else
            a.state[1] = step + 1;
    }
    const long long nbytes = a.row_bytes[i];
    const char* src = (const char*)a.src[i];
    char* dst = (char*)a.dst[i];
    if (RECORD) {
        if (step < 0 || step >= a.num_steps)
            return;  // past the end of the records: nothing is kept
        dst += step * nbytes;
    } else {
        src += (step < 0 ? 0 : step >= a.num_steps ? a.num_steps - 1 : step) * nbytes;
    }
    const long long b0 = blk * kBytesPerBlock;
    if (a.wide[i]) {
        for (long long o = b0 + 16ll * threadIdx.x; o < min(b0 + kBytesPerBlock, nbytes); o += 16ll * kCopyThreads)
            *reinterpret_cast<uint4*>(dst + o) = *reinterpret_cast<const uint4*>(src + o);
    } else {
        for (long long o = b0 + 4ll * threadIdx.x; o < min(b0 + kBytesPerBlock, nbytes); o += 4ll * kCopyThreads)
            *reinterpret_cast<uint32_t*>(dst + o) = *reinterpret_cast<const uint32_t*>(src + o);
    }
}

}  // namespace

// Blocks a copy of `row_bytes` takes.
long long step_rows_blocks(long long row_bytes) { return (row_bytes + kBytesPerBlock - 1) / kBytesPerBlock; }

hipError_t launch_step_rows(const StepRowsParams& a, bool record, hipStream_t s)
{
    const dim3 grid((unsigned)a.first_block[a.count]);
    if (record)
        hipLaunchKernelGGL(step_rows_kernel<true>, grid, dim3(kCopyThreads), 0, s, a);
    else
        hipLaunchKernelGGL(step_rows_kernel<false>, grid, dim3(kCopyThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace spd
