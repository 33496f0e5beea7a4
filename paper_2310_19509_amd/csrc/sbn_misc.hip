// Small dense helper kernels: device copy (counter calibration / HBM rate),
// dense depthwise 3x3 + bias + activation and global average pool, which sit
// between the sparse pointwise layers when a whole network is chained.
#include <hip/hip_runtime.h>

#include "sbn_internal.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void copy_kernel(const v4f* __restrict__ src, v4f* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// One thread: 4 channels of one output pixel.  x [n][h][w][c], wt [9][c], y [n][oh][ow][c].
__global__ __launch_bounds__(256) void dw3x3_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                   const float* __restrict__ wt, const float* __restrict__ bias,
                                                   int h, int w, int c, int oh, int ow, int stride, int act,
                                                   long long total)
{
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int c4n = c >> 2;
    const int c4 = (int)(t % c4n) * 4;
    long long pix = t / c4n;
    const int ox = (int)(pix % ow);
    pix /= ow;
    const int oy = (int)(pix % oh);
    const long long b = pix / oh;
    v4f acc = *(const v4f*)(bias + c4);
#pragma unroll
    for (int ky = 0; ky < 3; ++ky) {
        const int iy = oy * stride + ky - 1;
        if (iy < 0 || iy >= h) continue;
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) {
            const int ix = ox * stride + kx - 1;
            if (ix < 0 || ix >= w) continue;
            const v4f xv = *(const v4f*)(x + ((b * h + iy) * w + ix) * c + c4);
            const v4f wv = *(const v4f*)(wt + (ky * 3 + kx) * c + c4);
            acc += xv * wv;
        }
    }
    if (act == SBN_ACT_RELU) {
        acc.x = fmaxf(acc.x, 0.f);
        acc.y = fmaxf(acc.y, 0.f);
        acc.z = fmaxf(acc.z, 0.f);
        acc.w = fmaxf(acc.w, 0.f);
    }
    *(v4f*)(y + ((b * oh + oy) * (long long)ow + ox) * c + c4) = acc;
}

// x [n][hw][c] -> y [n][c]; one thread per (image, channel).
__global__ __launch_bounds__(256) void avgpool_kernel(const float* __restrict__ x, float* __restrict__ y, int hw,
                                                     int c, long long total)
{
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const long long b = t / c;
    const int ch = (int)(t % c);
    float s = 0.f;
    for (int p = 0; p < hw; ++p) s += x[(b * hw + p) * c + ch];
    y[t] = s / (float)hw;
}

int check_launch(const char* who)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return sbn::fail(SBN_EHIP, "%s launch: %s", who, hipGetErrorString(e));
    return SBN_OK;
}

}  // namespace

namespace sbn {

int launch_copy(const void* src, void* dst, size_t bytes, void* stream)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return SBN_OK;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;      // grid-stride, 32 workgroups per CU
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (const v4f*)src,
                       (v4f*)dst, n16);
    return check_launch("copy");
}

int launch_dw3x3(const float* x, float* y, const float* w_dev, const float* b_dev, int n, int h, int w, int c,
                 int stride, int act, void* stream)
{
    const int oh = (h - 1) / stride + 1, ow = (w - 1) / stride + 1;
    const long long total = (long long)n * oh * ow * (c / 4);
    if (total == 0) return SBN_OK;
    const long long blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return fail(SBN_EINVAL, "depthwise layer too large for one launch");
    hipLaunchKernelGGL(dw3x3_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, x, y, w_dev, b_dev, h,
                       w, c, oh, ow, stride, act, total);
    return check_launch("dw3x3");
}

int launch_avgpool(const float* x, float* y, int n, int hw, int c, void* stream)
{
    const long long total = (long long)n * c;
    if (total == 0) return SBN_OK;
    hipLaunchKernelGGL(avgpool_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream, x, y,
                       hw, c, total);
    return check_launch("avgpool");
}

}  // namespace sbn
