// ccdc_pipeline_fused_noalloc: the one-pass pipeline for callers that cannot have
// device memory allocated on their behalf (code under HIP graph capture, tight
// serving loops, harnesses that forbid hipMalloc).  The partial outputs of the
// round chunks, which ccdc_pipeline_fused keeps in the plan's workspace, go to a
// fixed array in device memory instead.
#include <mutex>

#include "common.hpp"

namespace {
using namespace ccdc;

// The scratch: one copy per device, there from the moment the library's code is
// loaded on that device until the process ends.  In host code this name is only
// a handle for hipGetSymbolAddress, never an address: the kernels get the device
// address that scratch_address() returns.
constexpr size_t kScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_ptr[kMaxDevices] = {};

}  // namespace

namespace ccdc {

// Device address of the scratch array on the CURRENT device; the runtime is asked
// once per device.  Called by ccdc_plan_upload (set-up) and, for a device no plan
// was uploaded on through this path yet, by the entry point's first call there.
int scratch_address(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return CCDC_EHIP;
    }
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return CCDC_EHIP;
        }
        scratch_ptr[dev] = ptr;
    }
    if (out) *out = scratch_ptr[dev];
    return CCDC_OK;
}

}  // namespace ccdc

extern "C" int ccdc_pipeline_fused_noalloc(const ccdc_plan_t *plan, const void *V, void *X, void *Phi, void *stream)
{
    const int rc = ready(plan);                       // also: the plan's device is the current one
    if (rc != CCDC_OK) return rc;
    void *ptr = nullptr;
    const int rs = scratch_address(&ptr);
    if (rs != CCDC_OK) return rs;
    // every chunk overwrites its whole slice of the scratch before the second kernel
    // reads it, so nothing has to be cleared between calls
    return pipeline_entry(plan, V, X, Phi, stream, ptr, kScratchBytes);
}
