// geak_check_run_static: the check for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  The workspace that
// geak_check_run takes from its caller -- candidate pointer table, board of running maxima,
// per-(wave, segment run, candidate) partials -- lives in a device array of fixed size that is part
// of the library's code object instead.  Every GPU the library runs on holds its own copy of the
// array, at its own address, until the process ends.
#include <hip/hip_runtime.h>
#include <mutex>
#include "geak_internal.hpp"

// In host code this name is only a handle for hipGetSymbolAddress, never a device address.  (No
// `used` attribute: the compiler gives a static device variable that host code refers to external
// linkage in the code object, which the runtime's look-up by name needs, and that attribute stops it.)
static __device__ __align__(256) unsigned char scratch[GEAK_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void *g_scratch_ptr[kMaxDevices];        // device d's copy of the array; null until resolved

}  // namespace

namespace geak {

// Address of `device`'s copy of the scratch array, resolved once per device with that device
// current.  Called when a plan is built for the device (a set-up call, where the runtime may load
// the code object), so that geak_check_run_static itself finds the address already there.
int static_scratch_address(int device, void **out)
{
    if (device < 0 || device >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_ptr[device]) {
        int prev = -1;
        hipError_t e = hipGetDevice(&prev);
        if (e != hipSuccess) return (int)e;
        if (prev != device && (e = hipSetDevice(device)) != hipSuccess) return (int)e;
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (prev != device) (void)hipSetDevice(prev);
        if (e != hipSuccess) return (int)e;
        if (!ptr) return (int)hipErrorInvalidSymbol;
        g_scratch_ptr[device] = ptr;
    }
    if (out) *out = g_scratch_ptr[device];
    return (int)hipSuccess;
}

}  // namespace geak

extern "C" geak_status geak_check_run_static(const geak_plan *plan, const void *ref_dev, const void *const *cand_dev,
                                             geak_result *results_dev, void *hip_stream)
{
    if (!plan) return GEAK_EINVAL;
    geak_plan_info info;
    if (geak_check_plan_info(plan, &info) != GEAK_OK || info.device < 0) return GEAK_EINVAL;
    if (geak_check_workspace_bytes(plan) > (uint64_t)GEAK_STATIC_SCRATCH_BYTES) return GEAK_EWORKSPACE;
    void *ptr = nullptr;
    if (geak::static_scratch_address(info.device, &ptr) != (int)hipSuccess) return GEAK_EHIP;
    // Everything the kernels read from the workspace is written by this run before it is read: the
    // pointer table and the zeroed board by the init kernel, every partial by the wave that owns it.
    return geak_check_run(plan, ref_dev, cand_dev, ptr, results_dev, hip_stream);
}
