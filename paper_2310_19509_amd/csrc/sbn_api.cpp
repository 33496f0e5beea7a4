// Run-time entry points of libsbn: argument checks and kernel dispatch.
#include <hip/hip_runtime_api.h>

#include "sbn_internal.h"

using namespace sbn;

static int check_run(const sbn_packed_t* p, int kind, const float* x, const float* y, int n, int h, int w,
                     const char* who)
{
    if (!p) return fail(SBN_EINVAL, "%s: packed layer is NULL", who);
    if (p->kind != kind) return fail(SBN_EINVAL, "%s: packed layer is of kind %d", who, p->kind);
    if (n < 0 || h < 0 || w < 0) return fail(SBN_EINVAL, "%s: negative extent (%d,%d,%d)", who, n, h, w);
    if (p->device < 0 || !p->dev.d_blob) return fail(SBN_ENODEV, "%s: layer was packed without a device copy", who);
    const long long m = (long long)n * h * w;
    if (m > 0 && (!x || !y)) return fail(SBN_EINVAL, "%s: activation pointer is NULL", who);
    if (m > 0 && x == y) return fail(SBN_EINVAL, "%s: x and y must not overlap", who);
    // the kernels move activations with 16-byte loads and stores
    if (m > 0 && (((uintptr_t)x | (uintptr_t)y) & 15u))
        return fail(SBN_EINVAL, "%s: x and y must be 16-byte aligned", who);
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return fail(SBN_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (cur != p->device)
        return fail(SBN_EINVAL, "%s: current device is %d but the layer lives on device %d", who, cur, p->device);
    return SBN_OK;
}

extern "C" {

int sbn_conv1x1_sparse(const sbn_packed_t* p, const float* x, float* y, int n, int h, int w, void* stream)
{
    clear_error();
    if (int rc = check_run(p, SBN_CONV1X1, x, y, n, h, w, "sbn_conv1x1_sparse")) return rc;
    const long long m = (long long)n * h * w;
    if (m == 0) return SBN_OK;
    return launch_conv1x1(p, x, y, m, stream);
}

int sbn_conv3x3_sparse(const sbn_packed_t* p, const float* x, float* y, int n, int h, int w, void* stream)
{
    clear_error();
    if (int rc = check_run(p, SBN_CONV3X3, x, y, n, h, w, "sbn_conv3x3_sparse")) return rc;
    if ((long long)n * h * w == 0) return SBN_OK;
    return launch_conv3x3(p, x, y, n, h, w, stream);
}

int sbn_copy_bytes(const void* src, void* dst, size_t bytes, void* stream)
{
    clear_error();
    if (bytes == 0) return SBN_OK;
    if (!src || !dst) return fail(SBN_EINVAL, "sbn_copy_bytes: NULL pointer");
    if (bytes % 16) return fail(SBN_EINVAL, "sbn_copy_bytes: size must be a multiple of 16");
    return launch_copy(src, dst, bytes, stream);
}

}  // extern "C"
