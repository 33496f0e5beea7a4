// Kernel-level group-sparse 3x3 convolution for gfx950 (Section 3.2, Conv3x3
// connectivity pruning: whole 3x3 kernels are kept or removed in groups).
//
// Same engine as the 1x1 kernel, with every kept piece carrying nine taps.
// One lane owns one output pixel of an 8x8 spatial tile; a wave owns one
// bundle of four 4-filter groups; the four waves of a workgroup share the
// input tile ((8-1)*stride+3)^2 pixels x 32 channels, staged in LDS (pixel
// stride 36 floats) through registers.  Input positions outside the image are
// staged as zeros, which realises the zero padding.  For stride 1 the tile is
// double buffered: the next 32 channels are fetched while the current ones are
// multiplied and published with one barrier per sub-chunk.
//
// Per entry (a 4-channel piece kept by at least one group of the bundle) the
// lane reads the nine shifted 16-byte activation vectors of its window, the
// wave loads the entry's 9 x 64 weights ([tap][group][ci][co], one float per
// lane and tap), and for every present group issues 36 v_mfma_f32_4x4x1 with
// the weight column broadcast from lanes 4*abid..4*abid+3.  Descriptors of a
// 64-channel record are held one per lane and broadcast with v_readlane.
#include <hip/hip_runtime.h>

#include "sbn_internal.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int TW = 8, TH = 8;          // output tile
constexpr int KC = 32;                 // channels staged at a time
constexpr int RS = 9;                  // 16-byte slots per staged pixel (8 + padding)
constexpr int XS = RS * 4;             // staged pixel stride in floats
constexpr int OS = 68;                 // output tile row stride in floats

template <int ABID>
__device__ __forceinline__ v4f mfma_bcast(float w, float x, v4f c)
{
    return __builtin_amdgcn_mfma_f32_4x4x1f32(w, x, c, 4, ABID, 0);
}

struct Entry {
    float w[9];      // weights of the nine taps, lane l = [g][ci][co]
    v4f x[9];        // this lane's activations under the nine taps
};

template <int G>
__device__ __forceinline__ void group_fma(const Entry& s, v4f (&acc)[4][2])
{
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        acc[G][0] = mfma_bcast<G * 4 + 0>(s.w[t], s.x[t].x, acc[G][0]);
        acc[G][1] = mfma_bcast<G * 4 + 1>(s.w[t], s.x[t].y, acc[G][1]);
        acc[G][0] = mfma_bcast<G * 4 + 2>(s.w[t], s.x[t].z, acc[G][0]);
        acc[G][1] = mfma_bcast<G * 4 + 3>(s.w[t], s.x[t].w, acc[G][1]);
    }
}

template <int STRIDE>
__global__ __launch_bounds__(256) void conv3x3_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                      const uint32_t* __restrict__ records,
                                                      const uint32_t* __restrict__ woff,
                                                      const float* __restrict__ wts, const float* __restrict__ bias,
                                                      const float* __restrict__ zeros, int H, int W, int OH, int OW,
                                                      int K, int N, int n_bundles, int n_chunks, int n_col_tiles,
                                                      int tiles_x, int tiles_y, int n_pix_tiles, int act)
{
    constexpr int IW = (TW - 1) * STRIDE + 3;          // input tile width
    constexpr int IH = (TH - 1) * STRIDE + 3;
    constexpr int NPIX = IW * IH;                      // staged input pixels
    constexpr int NSLOT = NPIX * (KC / 4);             // 16-byte slots of a staged tile
    constexpr int NL = (NSLOT + 255) / 256;            // slots per thread
    constexpr int XBUF = NPIX * XS;                    // floats per activation buffer
    constexpr bool DB = STRIDE == 1;
    constexpr int OBUF = 64 * OS;
    __shared__ __attribute__((aligned(16))) float lds[XBUF > OBUF ? XBUF : OBUF];
    __shared__ __attribute__((aligned(16))) float lds_b[DB ? XBUF : 4];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // workgroup -> (pixel tile, column tile): column tiles of one pixel tile run on one XCD
    const int id = blockIdx.x;
    const int xcd = id & 7, j = id >> 3;
    const int pix_tile = (j / n_col_tiles) * 8 + xcd;
    const int col_tile = j % n_col_tiles;
    if (pix_tile >= n_pix_tiles) return;
    const int tx = pix_tile % tiles_x, ty = (pix_tile / tiles_x) % tiles_y;
    const long long img = pix_tile / (tiles_x * tiles_y);
    const int oy0 = ty * TH, ox0 = tx * TW;
    const int iy0 = oy0 * STRIDE - 1, ix0 = ox0 * STRIDE - 1;
    const int bundle = col_tile * 4 + wave;
    const bool active = bundle < n_bundles;
    const int bsafe = active ? bundle : 0;

    v4f acc[4][2];
#pragma unroll
    for (int g = 0; g < 4; ++g) acc[g][0] = acc[g][1] = (v4f){0.f, 0.f, 0.f, 0.f};

    // ---- staging: thread t moves slots t, t+256, ...; slot = pixel * 8 + col
    const float* xi = x + img * H * W * K;
    const float* gpix[NL];        // channel 0 of the slot's input pixel (any valid address when outside)
    int gcol[NL];
    bool ginside[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        int s = i * 256 + threadIdx.x;
        s = s < NSLOT ? s : NSLOT - 1;
        const int pix = s / (KC / 4), col = s % (KC / 4);
        const int iy = iy0 + pix / IW, ix = ix0 + pix % IW;
        ginside[i] = iy >= 0 && iy < H && ix >= 0 && ix < W;
        gpix[i] = ginside[i] ? xi + ((long long)iy * W + ix) * K : zeros;
        gcol[i] = col * 4;
    }
    v4f stage_reg[NL];
    auto issue_x = [&](int sc) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            // keep the 16-byte read inside the pixel's channels; outside the image read zeros
            const int ch = ginside[i] ? min(gcol[i] + sc * KC, K - 4) : 0;
            stage_reg[i] = *(const v4f*)(gpix[i] + ch);
        }
    };
    auto write_x = [&](float* buf) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int s = i * 256 + threadIdx.x;
            if (s < NSLOT) *(v4f*)(buf + (s / (KC / 4)) * XS + (s % (KC / 4)) * 4) = stage_reg[i];
        }
    };

    // this lane's window origin inside the staged tile
    const int oyl = lane / TW, oxl = lane % TW;
    const int lane_off = ((oyl * STRIDE) * IW + oxl * STRIDE) * (XS * 4);      // bytes

    const uint32_t* wo = woff + (size_t)bsafe * (n_chunks + 1);
    const uint32_t* recs = records + (size_t)bsafe * n_chunks * 16;
    const int n_sub = (K + KC - 1) / KC;

    uint32_t dv = 0;          // descriptors of the current 64-channel record, one per lane (lanes 0..15)
    uint32_t q = 0, e = 0;
    // One sub-chunk of 32 channels: fetch the next one, multiply this one, publish the next.
    auto sub_chunk = [&](int sc, const float* xbuf, float* xnext) {
        if (DB) issue_x(sc + 1 < n_sub ? sc + 1 : sc);      // unconditional: see the 1x1 kernel
        const uint32_t h = sc & 1;
        if (h == 0) {
            dv = recs[(sc >> 1) * 16 + (lane & 15)];
            q = 0;
            e = __builtin_amdgcn_readfirstlane(wo[sc >> 1]);
        }

        if (active) {
            const char* xl = (const char*)xbuf + lane_off;
            auto desc = [&](uint32_t qq) -> uint32_t {
                return qq < 16 ? (uint32_t)__builtin_amdgcn_readlane((int)dv, (int)qq) : 0u;
            };
            auto mine = [&](uint32_t d) { return d != 0 && ((d >> 11) & 1u) == h; };
            auto load = [&](uint32_t en, uint32_t d, Entry& s) {
                const float* wp = wts + (size_t)en * 576 + lane;
                const char* xp = xl + ((d >> 8) & 7u) * 16;
#pragma unroll
                for (int t = 0; t < 9; ++t) {
                    s.w[t] = wp[t * 64];
                    s.x[t] = *(const v4f*)(xp + ((t / 3) * IW + (t % 3)) * (XS * 4));
                }
            };
            auto compute = [&](const Entry& s, uint32_t m) {
                if (__builtin_expect((m & 1u) != 0, 1)) group_fma<0>(s, acc);
                if (__builtin_expect((m & 2u) != 0, 1)) group_fma<1>(s, acc);
                if (__builtin_expect((m & 4u) != 0, 1)) group_fma<2>(s, acc);
                if (__builtin_expect((m & 8u) != 0, 1)) group_fma<3>(s, acc);
            };
            // Data run one entry ahead of the arithmetic.  A prefetch past the
            // sub-chunk's last entry reads the weight array's slack or the next
            // entry's weights and some in-tile activations; it is never used.
            uint32_t d_cur = desc(q);
            if (mine(d_cur)) {
                Entry a, b;
                load(e, d_cur, a);
                for (;;) {
                    uint32_t d_nxt = desc(q + 1);
                    load(e + 1, d_nxt, b);
                    compute(a, d_cur);
                    ++q, ++e;
                    d_cur = d_nxt;
                    if (!mine(d_cur)) break;
                    d_nxt = desc(q + 1);
                    load(e + 1, d_nxt, a);
                    compute(b, d_cur);
                    ++q, ++e;
                    d_cur = d_nxt;
                    if (!mine(d_cur)) break;
                }
            }
        }
        if (!DB) {                       // single buffer: fetch after everyone has finished reading it
            __syncthreads();
            issue_x(sc + 1 < n_sub ? sc + 1 : sc);
        }
        write_x(xnext);
        __syncthreads();
    };

    issue_x(0);
    write_x(lds);
    __syncthreads();
    for (int sc = 0; sc < n_sub; sc += 2) {
        sub_chunk(sc, lds, DB ? lds_b : lds);
        if (sc + 1 < n_sub) sub_chunk(sc + 1, DB ? lds_b : lds, lds);
    }

    // ---- epilogue: bias, activation, transpose through LDS, full 256-byte rows per pixel
    if (active) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            v4f o = acc[g][0] + acc[g][1] + *(const v4f*)(bias + bundle * 16 + g * 4);
            if (act == SBN_ACT_RELU) {
                o.x = fmaxf(o.x, 0.f);
                o.y = fmaxf(o.y, 0.f);
                o.z = fmaxf(o.z, 0.f);
                o.w = fmaxf(o.w, 0.f);
            }
            *(v4f*)(lds + lane * OS + wave * 16 + g * 4) = o;
        }
    }
    __syncthreads();
    const int ch_base = col_tile * 64;
    float* yi = y + img * OH * OW * N;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int slot = i * 256 + threadIdx.x;
        const int pl = slot >> 4, col = (slot & 15) * 4;
        const int oy = oy0 + pl / TW, ox = ox0 + pl % TW;
        if (oy < OH && ox < OW && ch_base + col < N)
            *(v4f*)(yi + ((long long)oy * OW + ox) * N + ch_base + col) = *(const v4f*)(lds + pl * OS + col);
    }
}

template <int STRIDE>
int launch(const sbn_packed* p, const float* x, float* y, int n, int h, int w, hipStream_t st)
{
    const sbn::DeviceLayout& L = p->dev;
    const int oh = (h - 1) / STRIDE + 1, ow = (w - 1) / STRIDE + 1;
    const int tiles_x = (ow + TW - 1) / TW, tiles_y = (oh + TH - 1) / TH;
    const long long n_pix_tiles = (long long)n * tiles_x * tiles_y;
    const int n_col_tiles = (L.n_bundles + 3) / 4;
    const long long grid = ((n_pix_tiles + 7) / 8) * 8 * n_col_tiles;
    if (grid > 0x7FFFFFFFll || n_pix_tiles > 0x7FFFFFFFll)
        return sbn::fail(SBN_EINVAL, "too many output tiles for one launch (%lld)", n_pix_tiles);
    hipLaunchKernelGGL((conv3x3_kernel<STRIDE>), dim3((unsigned)grid), dim3(256), 0, st, x, y, L.d_records, L.d_woff,
                       L.d_wts, L.d_bias, L.d_zeros, h, w, oh, ow, p->c_in, p->c_out, L.n_bundles, L.n_chunks,
                       n_col_tiles, tiles_x, tiles_y, (int)n_pix_tiles, p->act);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return sbn::fail(SBN_EHIP, "conv3x3 launch: %s", hipGetErrorString(e));
    return SBN_OK;
}

}  // namespace

namespace sbn {

int launch_conv3x3(const sbn_packed* p, const float* x, float* y, int n, int h, int w, void* stream)
{
    if (p->c_in % 4)
        return fail(SBN_ESHAPE, "3x3 layers need c_in to be a multiple of 4 on the device (got %d)", p->c_in);
    return p->stride == 1 ? launch<1>(p, x, y, n, h, w, (hipStream_t)stream)
                          : launch<2>(p, x, y, n, h, w, (hipStream_t)stream);
}

}  // namespace sbn
