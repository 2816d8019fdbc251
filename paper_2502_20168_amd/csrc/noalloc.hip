// ssm_scan_states without any allocation: the scratch of the scan (status header, ticket counters,
// look-back descriptors) is a device array inside the library image instead of a caller's workspace.
// For callers that cannot call hipMalloc or hand over a workspace (graph capture, serving loops).
#include "../../include/ssm.h"
#include "ssm_internal.h"

#include <atomic>

namespace {

// One copy per GPU that loads the library, held until the process ends.  In host code this name is
// only a handle for hipGetSymbolAddress: the device address differs per GPU and is looked up once
// per device below; kernels and copies only ever see that looked-up pointer.
static __device__ __align__(256) unsigned char scratch[SSM_NOALLOC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::atomic<void *> g_scratch_ptr[MAX_DEVICES];

// device address of the current device's copy of the array (nullptr on failure)
void *scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // two racing threads store the same address
    return p;
}

}  // namespace

extern "C" {

ssm_status ssm_scan_states_noalloc(const ssm_c64 *A_bar, ssm_c64 *v, const uint8_t *is_first,
                                   const ssm_c64 *x0, int64_t Bt, int64_t L, int64_t P, ssm_c64 *x_last,
                                   void *stream)
{
    if (!A_bar || !v) return SSM_ERR_INVALID_ARG;
    ssm::ScanOnlyLayout lo;
    const int st = ssm::make_scan_layout(Bt, L, P, false, lo);
    if (st != SSM_OK) return (ssm_status)st;
    if (lo.total > SSM_NOALLOC_SCRATCH_BYTES) return SSM_ERR_SCRATCH_LIMIT;
    void *ptr = scratch_of_current_device();
    if (!ptr) return SSM_ERR_HIP;
    return (ssm_status)ssm::scan_states_forward(A_bar, v, is_first, x0, Bt, L, P, x_last, ptr, SSM_NOALLOC_SCRATCH_BYTES,
                                                static_cast<hipStream_t>(stream));
}

ssm_status ssm_scan_states_noalloc_status(void *stream)
{
    void *ptr = scratch_of_current_device();
    if (!ptr) return SSM_ERR_HIP;
    return ssm_workspace_status(ptr, stream);
}

}  // extern "C"
