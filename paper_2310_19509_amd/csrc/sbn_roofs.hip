// Stand-alone loops that measure what this machine's units deliver, to set beside the datasheet
// roofs in the benchmark: the matrix pipe on the instruction the sparse kernels are built from
// (v_mfma_f32_4x4x1 with a broadcast operand), LDS reads of the kernels' width, and a read-only
// stream from device memory.  Measurement helpers only: nothing of the method runs here.
#include <hip/hip_runtime.h>

#include "sbn_internal.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

// 16 independent accumulators per wave: no multiply waits for an earlier one's result.
__global__ __launch_bounds__(256) void mfma_roof_kernel(float* __restrict__ sink, int iters)
{
    v4f acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = (v4f){0.f, 0.f, 0.f, 0.f};
    const float a = (float)threadIdx.x * 1e-3f, b = (float)blockIdx.x * 1e-3f;
    for (int it = 0; it < iters; ++it) {
#define SBN_M(i) acc[i] = __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, acc[i], 4, i, 0);
        SBN_M(0) SBN_M(1) SBN_M(2) SBN_M(3) SBN_M(4) SBN_M(5) SBN_M(6) SBN_M(7)
        SBN_M(8) SBN_M(9) SBN_M(10) SBN_M(11) SBN_M(12) SBN_M(13) SBN_M(14) SBN_M(15)
#undef SBN_M
    }
    v4f s = acc[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) s += acc[i];
    if (s.x + s.y + s.z + s.w == 123456.789f) sink[0] = s.x;          // keeps the loop alive, never true
}

// Every lane reads 16 bytes at its own 16-byte slot of a 68-float row (the 1x1 kernel's pattern).
__global__ __launch_bounds__(256) void lds_roof_kernel(float* __restrict__ sink, int iters)
{
    __shared__ __attribute__((aligned(16))) float tile[64 * 68 * 2];
    for (int i = threadIdx.x; i < 64 * 68 * 2; i += 256) tile[i] = (float)i;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const char* base = (const char*)tile + lane * (68 * 4);
    v4f s = {0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            v4f v = *(const v4f*)(base + q * 16 + (it & 1) * (64 * 68 * 4));
            asm volatile("" : "+v"(v));                                // one LDS instruction per read
            s += v;
        }
    }
    if (s.x + s.y + s.z + s.w == 123456.789f) sink[0] = s.x;
}

__global__ __launch_bounds__(256) void read_roof_kernel(const v4f* __restrict__ src, float* __restrict__ sink, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    v4f s = {0.f, 0.f, 0.f, 0.f};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) s += src[i];
    if (s.x + s.y + s.z + s.w == 123456.789f) sink[0] = s.x;
}

int check(const char* what)
{
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? SBN_OK : sbn::fail(SBN_EHIP, "%s launch: %s", what, hipGetErrorString(e));
}

int device_cus()
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return 256;
    return cus;
}

}  // namespace

extern "C" {

int sbn_roof_mfma(int iters, float* sink, void* stream, double* flops_out)
{
    sbn::clear_error();
    if (iters <= 0 || !sink) return sbn::fail(SBN_EINVAL, "sbn_roof_mfma: bad argument");
    const int blocks = device_cus() * 4;                 // four waves per SIMD
    hipLaunchKernelGGL(mfma_roof_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, sink, iters);
    // a 4x4x1 MFMA with 16 blocks: 16 * 4 * 4 multiply-adds
    if (flops_out) *flops_out = 2.0 * 256.0 * 16.0 * (double)iters * 4.0 * (double)blocks;
    return check("mfma roof");
}

int sbn_roof_lds(int iters, float* sink, void* stream, double* bytes_out)
{
    sbn::clear_error();
    if (iters <= 0 || !sink) return sbn::fail(SBN_EINVAL, "sbn_roof_lds: bad argument");
    const int blocks = device_cus() * 4;
    hipLaunchKernelGGL(lds_roof_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, sink, iters);
    if (bytes_out) *bytes_out = 16.0 * 16.0 * (double)iters * 256.0 * (double)blocks;
    return check("lds roof");
}

int sbn_roof_read(const void* src, size_t bytes, float* sink, void* stream)
{
    sbn::clear_error();
    if (!src || !sink || bytes % 16) return sbn::fail(SBN_EINVAL, "sbn_roof_read: bad argument");
    if (bytes == 0) return SBN_OK;
    const int blocks = device_cus() * 16;
    hipLaunchKernelGGL(read_roof_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const v4f*)src, sink, bytes / 16);
    return check("read roof");
}

}  // extern "C"
