// psd_sync_fc_sfb_static: psd_sync_fc_sfb for callers that cannot hand over (or allocate) a workspace.
// The partial dW tiles of a split reconstruction go to a fixed array in device memory that is part of
// the library's code object: every GPU the library runs on holds its own copy from the moment the code
// object is loaded until the process ends, and this entry point allocates nothing.
#include <atomic>
#include "psd_internal.h"

namespace {

// The array's name is a host-side stand-in, not a device address: host code only ever uses the pointer
// that hipGetSymbolAddress returns for the current device (one per device, each GPU has its own copy).
static __device__ __align__(256) unsigned char scratch[PSD_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];       // nullptr = not looked up yet on that device

// Address of this device's copy of `scratch`; looked up once per device with that device current.
psd_status scratch_for_current_device(void** out)
{
    int dev = -1;
    PSD_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return PSD_E_UNSUPPORTED;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        PSD_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return PSD_E_HIP;
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // a second first caller stores the same value
    }
    *out = p;
    return PSD_OK;
}

}  // namespace

extern "C" psd_status psd_sync_fc_sfb_static(const psd_plan* plan, int32_t factor_dtype, const void* U, int64_t ldu,
                                             const void* V, int64_t ldv, float* W, float* Mom, float lr, float mu,
                                             float wd, void* stream)
{
    if (!plan) return PSD_E_NULL;
    // how much scratch the split of this layer takes (0: it is not split and needs none)
    const size_t need = psd_sfb_workspace_bytes(plan, factor_dtype);
    if (need > PSD_STATIC_SCRATCH_BYTES) return PSD_E_WORKSPACE;
    if (need == 0)
        return psd_sync_fc_sfb(plan, factor_dtype, U, ldu, V, ldv, W, Mom, lr, mu, wd, nullptr, 0, stream);
    void* ptr = nullptr;
    const psd_status r = scratch_for_current_device(&ptr);
    if (r != PSD_OK) return r;
    // Every split writes its whole partial before the sum reads it, so nothing in the array has to be
    // cleared between calls.
    return psd_sync_fc_sfb(plan, factor_dtype, U, ldu, V, ldv, W, Mom, lr, mu, wd, ptr, need, stream);
}
