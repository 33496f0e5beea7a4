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

// Dense depthwise 3x3, pad 1.  One thread: 4 channels of R vertically adjacent output pixels;
// the input rows slide through registers so that every loaded row serves up to three outputs,
// and the nine weight vectors are loaded once per thread.  Consecutive threads take consecutive
// channel quads, then consecutive columns: all loads and stores are 16-byte and coalesced.
// x [n][h][w][c], wt [9][c], y [n][oh][ow][c].
template <int STRIDE, int R>
__global__ __launch_bounds__(256) void dw3x3_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                   const float* __restrict__ wt, const float* __restrict__ bias,
                                                   int h, int w, int c, int oh, int ow, int act, long long total)
{
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int c4n = c >> 2;
    const int c4 = (int)(t % c4n) * 4;
    long long r = t / c4n;
    const int ox = (int)(r % ow);
    r /= ow;
    const int strips = (oh + R - 1) / R;
    const int oy0 = (int)(r % strips) * R;
    const long long b = r / strips;

    v4f wv[9];
#pragma unroll
    for (int k = 0; k < 9; ++k) wv[k] = *(const v4f*)(wt + k * c + c4);
    const v4f bv = *(const v4f*)(bias + c4);
    v4f acc[R];
#pragma unroll
    for (int i = 0; i < R; ++i) acc[i] = bv;

    constexpr int ROWS = (R - 1) * STRIDE + 3;              // input rows touched by the strip
    const int iy0 = oy0 * STRIDE - 1, ix0 = ox * STRIDE - 1;
    const float* xb = x + b * h * w * c + c4;
#pragma unroll
    for (int ir = 0; ir < ROWS; ++ir) {
        const int iy = iy0 + ir;
        v4f row[3];
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) {
            const int ix = ix0 + kx;
            const bool ok = iy >= 0 && iy < h && ix >= 0 && ix < w;
            const v4f v = *(const v4f*)(xb + ((long long)(ok ? iy : 0) * w + (ok ? ix : 0)) * c);
            row[kx] = ok ? v : (v4f){0.f, 0.f, 0.f, 0.f};
        }
        // input row ir is tap row ky of output i when ir == i*STRIDE + ky
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int ky = ir - i * STRIDE;
            if (ky >= 0 && ky < 3) {
#pragma unroll
                for (int kx = 0; kx < 3; ++kx) acc[i] += row[kx] * wv[ky * 3 + kx];
            }
        }
    }
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int oy = oy0 + i;
        if (oy >= oh) break;
        v4f o = acc[i];
        if (act == SBN_ACT_RELU) {
            o.x = fmaxf(o.x, 0.f);
            o.y = fmaxf(o.y, 0.f);
            o.z = fmaxf(o.z, 0.f);
            o.w = fmaxf(o.w, 0.f);
        }
        *(v4f*)(y + ((b * oh + oy) * (long long)ow + ox) * c + c4) = o;
    }
}

// Dense 3x3 convolution of a few input channels (network stem), pad 1.  One thread: 4 output
// channels of one output pixel; the (c_out x 9 x c_in) weights sit in LDS as [tap][ci][c_out].
// x [n][h][w][c_in], y [n][oh][ow][c_out].
__global__ __launch_bounds__(256) void stem3x3_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                     const float* __restrict__ wt, const float* __restrict__ bias,
                                                     int h, int w, int c_in, int c_out, int oh, int ow, int stride,
                                                     int act, long long total)
{
    __shared__ __attribute__((aligned(16))) float ws[9 * 4 * 64];
    for (int i = threadIdx.x; i < 9 * c_in * c_out; i += 256) ws[i] = wt[i];
    __syncthreads();
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int c4n = c_out >> 2;
    const int co = (int)(t % c4n) * 4;
    long long pix = t / c4n;
    const int ox = (int)(pix % ow);
    pix /= ow;
    const int oy = (int)(pix % oh);
    const long long b = pix / oh;
    v4f acc = *(const v4f*)(bias + co);
#pragma unroll
    for (int ky = 0; ky < 3; ++ky) {
        const int iy = oy * stride + ky - 1;
        if (iy < 0 || iy >= h) continue;
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) {
            const int ix = ox * stride + kx - 1;
            if (ix < 0 || ix >= w) continue;
            const float* xp = x + ((b * h + iy) * w + ix) * c_in;
            for (int ci = 0; ci < c_in; ++ci)
                acc += xp[ci] * *(const v4f*)(ws + ((ky * 3 + kx) * c_in + ci) * c_out + co);
        }
    }
    if (act == SBN_ACT_RELU) {
        acc.x = fmaxf(acc.x, 0.f);
        acc.y = fmaxf(acc.y, 0.f);
        acc.z = fmaxf(acc.z, 0.f);
        acc.w = fmaxf(acc.w, 0.f);
    }
    *(v4f*)(y + ((b * oh + oy) * (long long)ow + ox) * c_out + co) = acc;
}

// The usual stem (3 -> 32 channels): one lane computes all 32 output channels of one output pixel
// on the matrix pipe.  The 27 inputs of the window sit in registers; the 27 x 32 weights fill 14
// registers of the wave ([k][c_out] in memory order: lane l of register r holds element 64 r + l),
// and one v_mfma_f32_4x4x1 per (input k, group of 4 output channels) broadcasts the four weights
// from lanes 4b..4b+3 of their register to all 16 blocks: 216 MFMAs per 64 pixels instead of 864
// multiply-adds per lane, which leaves the kernel bound by its memory traffic.
template <int ABID>
__device__ __forceinline__ v4f stem_mfma(float w, float x, v4f c)
{
    return __builtin_amdgcn_mfma_f32_4x4x1f32(w, x, c, 4, ABID, 0);
}

template <int CIN, int COUT, int P>
__device__ __forceinline__ void stem_pairs(const float (&wreg)[(9 * CIN * COUT + 63) / 64], const float (&xin)[9 * CIN],
                                           v4f (&acc)[COUT / 4])
{
    // pair P = k * (COUT/4) + g lives in block P % 16 of register P / 16
    if constexpr (P < 9 * CIN * (COUT / 4)) {
        constexpr int G = P % (COUT / 4), KI = P / (COUT / 4);
        acc[G] = stem_mfma<P % 16>(wreg[P / 16], xin[KI], acc[G]);
        stem_pairs<CIN, COUT, P + 1>(wreg, xin, acc);
    }
}

template <int CIN, int COUT>
__global__ __launch_bounds__(256) void stem3x3_fixed_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                           const float* __restrict__ wt,
                                                           const float* __restrict__ bias, int h, int w, int oh,
                                                           int ow, int stride, int act, long long total)
{
    constexpr int LS = COUT + 4;                           // LDS row stride (floats)
    constexpr int NWR = (9 * CIN * COUT + 63) / 64;        // weight registers
    __shared__ __attribute__((aligned(16))) float tile[256 * LS];
    const int lane = threadIdx.x & 63;
    const long long t0 = (long long)blockIdx.x * 256;
    const long long t = t0 + threadIdx.x;
    float wreg[NWR];
#pragma unroll
    for (int r = 0; r < NWR; ++r) wreg[r] = r * 64 + lane < 9 * CIN * COUT ? wt[r * 64 + lane] : 0.f;
    // every lane takes part in the MFMAs; lanes past the last pixel compute pixel total-1 again
    const long long tc = t < total ? t : total - 1;
    const int ox = (int)(tc % ow);
    const int oy = (int)((tc / ow) % oh);
    const long long b = tc / ((long long)ow * oh);
    float xin[9 * CIN];
#pragma unroll
    for (int k = 0; k < 9; ++k) {
        const int iy = oy * stride + k / 3 - 1, ix = ox * stride + k % 3 - 1;
        const bool ok = iy >= 0 && iy < h && ix >= 0 && ix < w;
        const float* xp = x + ((b * h + (ok ? iy : 0)) * w + (ok ? ix : 0)) * CIN;
#pragma unroll
        for (int ci = 0; ci < CIN; ++ci) {
            const float v = xp[ci];
            xin[k * CIN + ci] = ok ? v : 0.f;
        }
    }
    v4f acc[COUT / 4];
#pragma unroll
    for (int g = 0; g < COUT / 4; ++g) acc[g] = *(const v4f*)(bias + g * 4);
    stem_pairs<CIN, COUT, 0>(wreg, xin, acc);
#pragma unroll
    for (int g = 0; g < COUT / 4; ++g) {
        v4f o = acc[g];
        if (act == SBN_ACT_RELU) {
            o.x = fmaxf(o.x, 0.f);
            o.y = fmaxf(o.y, 0.f);
            o.z = fmaxf(o.z, 0.f);
            o.w = fmaxf(o.w, 0.f);
        }
        *(v4f*)(tile + threadIdx.x * LS + g * 4) = o;
    }
    // the workgroup's 256 pixels are contiguous in y: store them as full rows
    __syncthreads();
#pragma unroll
    for (int i = 0; i < COUT / 4; ++i) {
        const int slot = i * 256 + threadIdx.x;
        const int pl = slot / (COUT / 4), c0 = (slot % (COUT / 4)) * 4;
        if (t0 + pl < total) *(v4f*)(y + (t0 + pl) * COUT + c0) = *(const v4f*)(tile + pl * LS + c0);
    }
}

// x [n][hw][c] -> y [n][c].  A workgroup takes one image x 256 channels: thread t owns channels
// 4*(t%64)..+3 and every fourth pixel starting at t/64 (16-byte loads, all of them independent);
// the four partial sums meet in LDS and are added in a fixed order.
__global__ __launch_bounds__(256) void avgpool_kernel(const float* __restrict__ x, float* __restrict__ y, int hw,
                                                     int c, int c_tiles)
{
    __shared__ __attribute__((aligned(16))) float part[3 * 256];
    const long long b = blockIdx.x / c_tiles;
    const int ch = (blockIdx.x % c_tiles) * 256 + (threadIdx.x & 63) * 4;
    const int q = threadIdx.x >> 6;
    v4f s = {0.f, 0.f, 0.f, 0.f};
    if (ch < c)
        for (int p = q; p < hw; p += 4) s += *(const v4f*)(x + (b * hw + p) * c + ch);
    if (q) *(v4f*)(part + (q - 1) * 256 + (threadIdx.x & 63) * 4) = s;
    __syncthreads();
    if (q == 0 && ch < c) {
#pragma unroll
        for (int k = 0; k < 3; ++k) s += *(const v4f*)(part + k * 256 + threadIdx.x * 4);
        const float r = 1.0f / (float)hw;
        *(v4f*)(y + b * c + ch) = s * r;
    }
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
    constexpr int R = 4;
    const int oh = (h - 1) / stride + 1, ow = (w - 1) / stride + 1;
    const long long total = (long long)n * ((oh + R - 1) / R) * ow * (c / 4);
    if (total == 0) return SBN_OK;
    const long long blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return fail(SBN_EINVAL, "depthwise layer too large for one launch");
    if (stride == 1)
        hipLaunchKernelGGL((dw3x3_kernel<1, R>), dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, x, y, w_dev,
                           b_dev, h, w, c, oh, ow, act, total);
    else
        hipLaunchKernelGGL((dw3x3_kernel<2, R>), dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, x, y, w_dev,
                           b_dev, h, w, c, oh, ow, act, total);
    return check_launch("dw3x3");
}

int launch_stem3x3(const float* x, float* y, const float* w_dev, const float* b_dev, int n, int h, int w, int c_in,
                   int c_out, int stride, int act, void* stream)
{
    const int oh = (h - 1) / stride + 1, ow = (w - 1) / stride + 1;
    if (c_in == 3 && c_out == 32) {
        const long long pixels = (long long)n * oh * ow;
        if (pixels == 0) return SBN_OK;
        if ((pixels + 255) / 256 > 0x7FFFFFFFll) return fail(SBN_EINVAL, "stem layer too large for one launch");
        hipLaunchKernelGGL((stem3x3_fixed_kernel<3, 32>), dim3((unsigned)((pixels + 255) / 256)), dim3(256), 0,
                           (hipStream_t)stream, x, y, w_dev, b_dev, h, w, oh, ow, stride, act, pixels);
        return check_launch("stem3x3");
    }
    const long long total = (long long)n * oh * ow * (c_out / 4);
    if (total == 0) return SBN_OK;
    const long long blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return fail(SBN_EINVAL, "stem layer too large for one launch");
    hipLaunchKernelGGL(stem3x3_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, x, y, w_dev, b_dev, h,
                       w, c_in, c_out, oh, ow, stride, act, total);
    return check_launch("stem3x3");
}

int launch_avgpool(const float* x, float* y, int n, int hw, int c, void* stream)
{
    if ((long long)n * c * hw == 0) return SBN_OK;
    if (c % 4) return fail(SBN_ESHAPE, "the average pool needs a multiple of 4 channels (got %d)", c);
    const int c_tiles = (c + 255) / 256;
    hipLaunchKernelGGL(avgpool_kernel, dim3((unsigned)((long long)n * c_tiles)), dim3(256), 0, (hipStream_t)stream, x, y,
                       hw, c, c_tiles);
    return check_launch("avgpool");
}

}  // namespace sbn
