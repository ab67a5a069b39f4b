// Latency measurement for the evaluator's performance test (GEAK section 4.1: code that passes the
// functionality test is timed; section 3.3: the speedup is built from the median latency of every unit
// test).  The paper does not say how a latency is taken; this harness takes it the way kernel
// benchmarks usually do: every repetition starts from cold caches -- a scratch buffer larger than the
// last-level cache is overwritten on the same stream first -- and is bracketed by two events on that
// stream.  The latencies go to geak_metrics_speedup.
#include <hip/hip_runtime.h>
#include <atomic>
#include "geak_internal.hpp"

namespace geak {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Overwrites the buffer with 16-byte stores: every line of it ends up in the caches in place of what
// was there, and what was there has to be fetched from memory again by the kernel that is timed next.
__global__ __launch_bounds__(256) void flush_kernel(u32x4 *p, unsigned long long vectors, uint32_t value)
{
    const unsigned long long stride = (unsigned long long)gridDim.x * blockDim.x;
    const u32x4 v = {value, value, value, value};
    for (unsigned long long i = (unsigned long long)blockIdx.x * blockDim.x + threadIdx.x; i < vectors; i += stride) p[i] = v;
}

}  // namespace
}  // namespace geak

extern "C" {

geak_status geak_timing_flush(void *scratch_dev, uint64_t scratch_bytes, void *hip_stream)
{
    if (!scratch_dev || scratch_bytes < 16) return GEAK_EINVAL;
    if ((uintptr_t)scratch_dev & 15u) return GEAK_EALIGN;
    static std::atomic<uint32_t> round{0};                   // a different value every time: the stores cannot be elided as silent
    hipLaunchKernelGGL(geak::flush_kernel, dim3(2048), dim3(256), 0, (hipStream_t)hip_stream, (geak::u32x4 *)scratch_dev,
                       (unsigned long long)(scratch_bytes / 16), round.fetch_add(1u) + 1u);
    return hipGetLastError() == hipSuccess ? GEAK_OK : GEAK_EHIP;
}

geak_status geak_timing_measure(geak_launch_fn launch, void *user, uint32_t warmup, uint32_t repetitions, void *flush_scratch_dev,
                                uint64_t flush_bytes, void *hip_stream, double *latency_ms_out)
{
    if (!launch || !latency_ms_out || repetitions == 0) return GEAK_EINVAL;
    if (flush_scratch_dev && (flush_bytes < 16 || ((uintptr_t)flush_scratch_dev & 15u))) return GEAK_EINVAL;
    hipStream_t stream = (hipStream_t)hip_stream;
    hipEvent_t start, stop;
    if (hipEventCreate(&start) != hipSuccess) return GEAK_EHIP;
    if (hipEventCreate(&stop) != hipSuccess) { (void)hipEventDestroy(start); return GEAK_EHIP; }
    geak_status st = GEAK_OK;
    for (uint64_t r = 0; r < (uint64_t)warmup + repetitions && st == GEAK_OK; ++r) {
        if (flush_scratch_dev) st = geak_timing_flush(flush_scratch_dev, flush_bytes, hip_stream);
        if (st != GEAK_OK) break;
        if (hipEventRecord(start, stream) != hipSuccess) { st = GEAK_EHIP; break; }
        if (launch(user, hip_stream) != 0) { st = GEAK_EINVAL; break; }       // the kernel under test, enqueued by the caller
        if (hipEventRecord(stop, stream) != hipSuccess || hipEventSynchronize(stop) != hipSuccess) { st = GEAK_EHIP; break; }
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, start, stop) != hipSuccess) { st = GEAK_EHIP; break; }
        if (r >= warmup) latency_ms_out[r - warmup] = (double)ms;
    }
    (void)hipEventDestroy(start);
    (void)hipEventDestroy(stop);
    return st;
}

}  // extern "C"
