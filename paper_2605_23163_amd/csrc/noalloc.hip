// fdd_unmask_step_static: the unmask step for callers that cannot allocate
// device memory (code under HIP graph capture, tight serving loops, harnesses
// that forbid hipMalloc) and do not want to carry a workspace either.  It is
// fdd_unmask_step with the per-piece partial results of the vocabulary
// reduction kept in a fixed array that lives in the library's device image.
//
// Every GPU the library runs on holds its own copy of the array, at its own
// address, from the moment the code object is loaded there until the process
// ends.  The array's name below is a host-side stand-in for it: device code
// may use it, host code may only hand it to hipGetSymbolAddress, which returns
// the address on the current device.  That address is looked up once per
// device and is what the kernels receive, exactly as they receive the
// caller's workspace pointer in fdd_unmask_step.
#include <mutex>

#include "fdd_internal.h"

namespace fdd {
namespace {

constexpr size_t kScratchBytes = FDD_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on device d, once looked up

// Device address of the array on the current device (nullptr + error code on failure).
hipError_t scratch_on_current_device(void** out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace
}  // namespace fdd

using namespace fdd;

extern "C" fdd_status fdd_unmask_step_static(const fdd_unmask_params* p)
{
    fdd_status st = check_unmask_args(p, "fdd_unmask_step_static");
    if (st != FDD_OK) return st;
    UnmaskPlan plan;
    make_unmask_plan(*p, &plan);
    if (plan.ws_bytes > kScratchBytes)
        return set_error(FDD_ERR_WORKSPACE,
                         "fdd_unmask_step_static: this shape needs %zu bytes of scratch, the built-in array holds %zu "
                         "(N*B*pieces <= %zu); use fdd_unmask_step with a workspace",
                         plan.ws_bytes, kScratchBytes, kScratchBytes / 16);
    void* ptr = nullptr;
    hipError_t e = scratch_on_current_device(&ptr);
    if (e != hipSuccess)
        return set_error(FDD_ERR_LAUNCH, "fdd_unmask_step_static: cannot locate the scratch array on this device: %s",
                         hipGetErrorString(e));
    fdd_unmask_params q = *p;
    q.workspace = ptr;               // from here on only the looked-up address is used, never the array's name
    q.workspace_bytes = kScratchBytes;
    e = launch_unmask(q, plan, static_cast<hipStream_t>(p->stream));
    if (e != hipSuccess) return set_error(FDD_ERR_LAUNCH, "fdd_unmask_step_static: launch failed: %s", hipGetErrorString(e));
    return FDD_OK;
}
