// Rows of a decode loop chosen by a step counter that lives on the device: the inputs of step t
// (queries, the new token's K and V, the uniforms) are copied out of [steps, ...] tensors into the
// buffers the step's calls read, and the step's results (tokens, lengths, outputs) are copied
// into row t of [steps, ...] records, so that one captured step can be replayed for a whole loop
// of the paper's up-to-1024-token generations (App. "Experiment settings") without the host.
//
// The counter is a pair {current, next}.  The select kernel reads `current` in every workgroup
// and one thread stores next = current + 1; the record kernel reads `next` in every workgroup
// and one thread stores current = next.  Neither kernel reads a word that it writes.  The advance
// kernel does the work of record, select and append in one launch (see there).
#include "step_bodies.h"

namespace spd {
namespace {

using namespace step_impl;

// Which copy workgroup `b` belongs to (first_block is non-decreasing; unused entries repeat the end).
template <int MAX> __device__ __forceinline__ int copy_of_block(const int (&first_block)[MAX + 1], int count, int b)
{
    int i = 0;
#pragma unroll
    for (int k = 1; k < MAX; ++k)
        if (k < count && b >= first_block[k])
            i = k;
    return i;
}

template <bool RECORD>
__global__ __launch_bounds__(kCopyThreads) void step_rows_kernel(StepRowsParams a)
{
    const int i = copy_of_block<kMaxStepCopies>(a.first_block, a.count, (int)blockIdx.x);
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
    copy_block(src, dst, nbytes, blk, a.wide[i] != 0);
}

// Everything between two decode steps in one launch: with t = current, the results of step t - 1
// go to row t - 1 of their records, row t of the step inputs goes to the buffers the step's calls
// read, and row t of the new K and V is appended to the suffixes.  Every workgroup reads `current`
// when it starts; the one that finishes last (an arrival count in the third word of the state,
// left at zero again) stores current = next = t + 1, after every other workgroup has read the old
// value.  No workgroup waits for another.
__global__ __launch_bounds__(kCopyThreads) void step_advance_kernel(StepAdvanceParams a)
{
    const long long t = a.state[0];
    const long long row_in = t < 0 ? 0 : t >= a.num_steps ? a.num_steps - 1 : t;  // rows past the last repeat the last
    const bool have_prev = t >= 1 && t - 1 < a.num_steps;                          // a row to record into
    const int copy_blocks = a.first_block[kMaxAdvanceCopies];
    if ((int)blockIdx.x < copy_blocks) {
        const int i = copy_of_block<kMaxAdvanceCopies>(a.first_block, a.count, (int)blockIdx.x);
        const long long blk = (long long)blockIdx.x - a.first_block[i];
        const long long nbytes = a.row_bytes[i];
        const bool record = a.record[i] != 0;
        if (!record)
            copy_block((const char*)a.src[i] + row_in * nbytes, (char*)a.dst[i], nbytes, blk, a.wide[i] != 0);
        else if (have_prev)
            copy_block((const char*)a.src[i], (char*)a.dst[i] + (t - 1) * nbytes, nbytes, blk, a.wide[i] != 0);
    } else {
        const int n = (int)blockIdx.x - copy_blocks;
        const long long step_bytes = (long long)a.kv.N * a.kv.Hkv * a.kv.D * a.kv.elt;  // one step of k_steps / v_steps
        append_sample(a.kv, n, (const char*)a.kv.k_new + row_in * step_bytes, (const char*)a.kv.v_new + row_in * step_bytes,
                      a.lens_record && have_prev ? a.lens_record + (t - 1) * a.kv.N + n : nullptr);
    }
    __syncthreads();  // every thread of the workgroup has read what it needs of the state
    if (threadIdx.x == 0) {
        const unsigned long long arrived = atomicAdd((unsigned long long*)&a.state[2], 1ull);
        if (arrived == (unsigned long long)gridDim.x - 1ull) {
            a.state[2] = 0;
            a.state[0] = t + 1;
            a.state[1] = t + 1;
        }
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

hipError_t launch_step_advance(const StepAdvanceParams& a, hipStream_t s)
{
    const dim3 grid((unsigned)(a.first_block[kMaxAdvanceCopies] + a.kv.N));
    hipLaunchKernelGGL(step_advance_kernel, grid, dim3(kCopyThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace spd
