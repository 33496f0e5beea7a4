// sbn_pointwise_chain_static: the chain run call for callers that cannot allocate device
// memory (code under HIP graph capture, serving loops, harnesses that forbid hipMalloc).  The
// intermediate activations ping-pong inside a fixed array that is part of the library's code
// object instead of a caller-provided workspace.
#include <hip/hip_runtime.h>

#include <mutex>

#include "sbn_internal.h"

namespace {

// Every GPU the library runs on holds its own copy of this array, at its own address, until
// the process ends.  In host code the name is only a handle for hipGetSymbolAddress: the
// address kernels receive is the one looked up below, per device.
static __device__ __align__(256) unsigned char scratch[SBN_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices] = {};          // device address of `scratch` on each device, once looked up

// Address of the array on `device`, which must be the current device.  The first call per
// device asks the runtime (and may load the code object); later calls read the table.
int scratch_address(int device, void** out)
{
    if (device < 0 || device >= kMaxDevices) return sbn::fail(SBN_EINVAL, "device %d is out of range", device);
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return sbn::fail(SBN_EHIP, "hipGetSymbolAddress(static workspace) on device %d: %s", device, hipGetErrorString(e));
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return SBN_OK;
}

}  // namespace

namespace sbn {

// Set-up hook, called by sbn_chain_create with the chain's device current: looks the array up
// once so that no later run call has to (a run call may sit inside a stream capture).
int static_workspace_init(int device)
{
    void* p = nullptr;
    return scratch_address(device, &p);
}

}  // namespace sbn

extern "C" int sbn_pointwise_chain_static(const sbn_chain_t* c, const float* x, float* y, int n, int h, int w,
                                          float* const* layer_outputs, void* stream)
{
    sbn::clear_error();
    if (!c) return sbn::fail(SBN_EINVAL, "sbn_pointwise_chain_static: chain is NULL");
    if (n < 0 || h < 0 || w < 0) return sbn::fail(SBN_EINVAL, "sbn_pointwise_chain_static: negative extent");
    if ((long long)n * h * w == 0) return SBN_OK;
    const size_t need = sbn::chain_workspace_bytes(c, n, h, w);
    if (need > (size_t)SBN_STATIC_WORKSPACE_BYTES)
        return sbn::fail(SBN_EINVAL,
                         "sbn_pointwise_chain_static: an input of %d x %d x %d needs %zu bytes of intermediate "
                         "activations, the built-in workspace holds %zu (use sbn_pointwise_chain with a workspace of "
                         "your own)", n, h, w, need, (size_t)SBN_STATIC_WORKSPACE_BYTES);
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return sbn::fail(SBN_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (cur != sbn::chain_device(c))
        return sbn::fail(SBN_EINVAL, "sbn_pointwise_chain_static: current device is %d, chain lives on %d", cur,
                         sbn::chain_device(c));
    void* ws = nullptr;                                       // this device's copy of the array
    if (int rc = scratch_address(cur, &ws)) return rc;
    // Every item writes the whole of its output before the next item reads it, so nothing in the
    // array has to start at zero and what an earlier call left there is never read.
    return sbn::run_chain(c, x, y, n, h, w, ws, (size_t)SBN_STATIC_WORKSPACE_BYTES, layer_outputs, stream,
                          "sbn_pointwise_chain_static");
}
