// Verdict of each candidate over all of its unit tests: a kernel is correct only if it satisfies
// every unit test (GEAK section 3.3), so candidate k's verdict is the AND of the pass flags of its
// (segment, candidate) records.  One block per candidate.
#include <hip/hip_runtime.h>
#include "geak_internal.hpp"

namespace geak {
namespace {

constexpr int kVerdictThreads = 256;

__global__ __launch_bounds__(kVerdictThreads) void verdict_kernel(const VerdictArgs p)
{
    __shared__ uint32_t failed;
    if (threadIdx.x == 0) failed = 0;
    __syncthreads();
    const uint32_t k = blockIdx.x;
    uint32_t mine = 0;
    for (uint32_t s = threadIdx.x; s < p.num_segments; s += kVerdictThreads)
        mine += p.results[(uint64_t)s * p.num_candidates + k].pass == 0;
    if (mine) atomicAdd(&failed, mine);
    __syncthreads();
    if (threadIdx.x == 0) {
        p.verdicts[k] = failed == 0;
        if (p.failed_tests) p.failed_tests[k] = failed;
    }
}

}  // namespace

int launch_verdicts(const VerdictArgs &args, void *stream)
{
    if (!args.num_candidates) return (int)hipSuccess;
    hipLaunchKernelGGL(verdict_kernel, dim3(args.num_candidates), dim3(kVerdictThreads), 0, (hipStream_t)stream, args);
    return (int)hipGetLastError();
}

}  // namespace geak
