// sc_execute_static: the execute entry point for callers that cannot allocate device memory
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  It runs
// the same kernels as sc_execute, with the workspace (temporaries of a FISSIONED schedule, pieces
// and segment sums of a deterministic one) taken from a fixed array in the library's own device
// image instead of a caller buffer.
//
// The array exists once per GPU the library runs on, from the moment the code object is loaded
// there until the process ends.  Its name is a host-side stand-in, not a device address: the
// address on a device is looked up once per device with hipGetSymbolAddress (with that device
// current) and only that pointer is handed to kernels.
#include <mutex>

#include "plan.h"

namespace {

constexpr size_t kScratchBytes = SC_STATIC_WORKSPACE_BYTES;
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_lock;
void *g_scratch_ptr[kMaxDevices];   // per device: address of that device's copy of `scratch`, null until looked up

}  // namespace

// Address of the current device's scratch array (looked up on first use on that device), or
// null with *st set when there is no device or the lookup fails.
void *sck::static_scratch(sc_status *st)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        *st = SC_ERR_DEVICE;
        return nullptr;
    }
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            *st = SC_ERR_DEVICE;
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *st = SC_OK;
    return g_scratch_ptr[dev];
}

extern "C" sc_status sc_execute_static(const sc_plan *plan, const sc_csf_view *sparse, const sc_dense_view *factors, int32_t nfactors,
                                       void *out, void *hip_stream)
{
    if (!plan) return SC_ERR_NULL;
    if (plan->ws_bytes > kScratchBytes) return SC_ERR_WORKSPACE_SMALL;   // the plan needs more than the fixed array holds
    try {
        sc_status st = SC_OK;
        void *ws = sck::static_scratch(&st);
        if (!ws) return st;
        return sck::execute_checked(plan, sparse, factors, nfactors, out, ws, kScratchBytes, (hipStream_t)hip_stream);
    } catch (...) {
        return SC_ERR_DEVICE;
    }
}
