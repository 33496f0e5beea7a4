// Depthwise 3x3 (+ bias, ReLU) computed inside the staging of the group-sparse 1x1 layer that
// consumes it, for gfx950: the depthwise output never goes to HBM.  (Section 3.2 treats the
// depthwise and the pointwise layer of a separable block as separate operators; on this machine
// the early blocks of MobileNet-v1 are bound by HBM traffic, and the intermediate tensor is
// half of it.)
//
// One workgroup = an 8x8 tile of output pixels (one per lane) x ALL output channels: four waves
// (64 channels) or eight (128), a wave per bundle, so that the depthwise result of a tile is
// computed once.  Per sub-chunk of 32 channels:
//   1. the depthwise layer's input tile with its halo, (7s+3)^2 pixels x 32 channels, goes
//      global -> registers -> LDS (zeros outside the image = the padding); the loads are issued
//      before the previous sub-chunk is multiplied;
//   2. every thread computes the depthwise outputs of one or two vertically adjacent pixels x 4
//      channels (weights and bias of the whole layer sit in LDS) and writes them to the activation tile
//      X[64 pixels][32 channels] that the 1x1 arithmetic reads.  For a layer with 3:9 pattern
//      groups of 16 channels (Section 3.2, DwConv3x3; Algorithm 2's per-group pattern information;
//      template parameter PAT) a wave works on ONE 16-channel half of the sub-chunk, which is one
//      pattern group: the group's kept taps are a wave-uniform word, and one scalar branch picks
//      the body that loads and multiplies only those six taps;
//   3. the wave walks the bundle's entries of the sub-chunk exactly as the 1x1 kernel does: a
//      16-byte LDS read per entry, 4 v_mfma_f32_4x4x1 per present group.
// Used when the 1x1 layer has at most 128 input and 128 output channels; wider layers are bound by
// the matrix pipe, not by memory traffic, and keep the two launches.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "sbn_internal.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int TH = 8, TW = 8;          // output tile: 64 pixels, lane = oy * 8 + ox
constexpr int KC = 32;                 // channels per sub-chunk
constexpr int XS = KC + 4;             // row stride of the activation tile in floats (no bank conflicts)
constexpr int KMAX = 128;              // most input channels (depthwise parameters held in LDS)

template <int ABID>
__device__ __forceinline__ v4f mfma_bcast(float w, float x, v4f c)
{
    return __builtin_amdgcn_mfma_f32_4x4x1f32(w, x, c, 4, ABID, 0);
}

// group G of entry Q: lanes 4*AB..4*AB+3 of w hold [co 0..3], the components the four input channels
template <int Q, int G>
__device__ __forceinline__ void group_fma(const v4f& w, const v4f& xv, v4f (&acc)[4][2])
{
    constexpr int AB = (Q & 3) * 4 + G;
    acc[G][0] = mfma_bcast<AB>(w.x, xv.x, acc[G][0]);
    acc[G][1] = mfma_bcast<AB>(w.y, xv.y, acc[G][1]);
    acc[G][0] = mfma_bcast<AB>(w.z, xv.z, acc[G][0]);
    acc[G][1] = mfma_bcast<AB>(w.w, xv.w, acc[G][1]);
}

template <int Q>
__device__ __forceinline__ void entry_fma(uint32_t m, const v4f& w, const v4f& xv, v4f (&acc)[4][2])
{
    if (__builtin_expect((m & 1u) != 0, 1)) group_fma<Q, 0>(w, xv, acc);
    if (__builtin_expect((m & 2u) != 0, 1)) group_fma<Q, 1>(w, xv, acc);
    if (__builtin_expect((m & 4u) != 0, 1)) group_fma<Q, 2>(w, xv, acc);
    if (__builtin_expect((m & 8u) != 0, 1)) group_fma<Q, 3>(w, xv, acc);
}

struct Record8 {
    uint32_t d[8];
};

template <int STRIDE, int NWV, bool PAT>
__global__ __launch_bounds__(64 * NWV) void dwpw_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                   const float* __restrict__ dw_w, const float* __restrict__ dw_b,
                                                   const uint32_t* __restrict__ dw_taps, int dw_act,
                                                   const uint32_t* __restrict__ records,
                                                   const uint32_t* __restrict__ woff, const float* __restrict__ wts,
                                                   const float* __restrict__ bias, int H, int W, int OH, int OW, int K,
                                                   int N, int n_bundles, int n_sub, int n_col_tiles, int tiles_x,
                                                   int tiles_y, int n_pix_tiles, int act)
{
    constexpr int IW = (TW - 1) * STRIDE + 3, IH = (TH - 1) * STRIDE + 3;     // input tile
    constexpr int NPIX = IW * IH;
    constexpr int NPIXP = NPIX + (6 - NPIX % 4) % 4;           // = 2 mod 4: the two halves of a pixel pair fill all banks
    constexpr int NSLOT = NPIX * (KC / 4);
    constexpr int NT = 64 * NWV;                               // threads
    constexpr int NL = (NSLOT + NT - 1) / NT;
    constexpr int OS = 16 * NWV + 4;                           // row stride of the output tile in floats
    constexpr int NO = 8 / NWV;                                // depthwise output pixels per thread
    constexpr int ABUF = PAT ? 2 * NPIXP * 16 : NPIX * KC, OBUF = 64 * OS;
    __shared__ __attribute__((aligned(16))) float lds_a[ABUF > OBUF ? ABUF : OBUF];   // input tile [pixel][32], PAT: [16-channel half][pixel][16]; output tile at the end
    __shared__ __attribute__((aligned(16))) float lds_x[64 * XS];                     // depthwise result
    __shared__ __attribute__((aligned(16))) float lds_p[10 * KMAX];                   // depthwise weights [9][K], bias [K]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int id = blockIdx.x;
    const int xcd = id & 7, j = id >> 3;
    const int pix_tile = (j / n_col_tiles) * 8 + xcd;
    const int col_tile = j % n_col_tiles;
    if (pix_tile >= n_pix_tiles) return;
    const int tx = pix_tile % tiles_x, ty = (pix_tile / tiles_x) % tiles_y;
    const long long img = pix_tile / (tiles_x * tiles_y);
    const int oy0 = ty * TH, ox0 = tx * TW;
    const int iy0 = oy0 * STRIDE - 1, ix0 = ox0 * STRIDE - 1;
    const int bundle = col_tile * NWV + wave;
    const bool active = bundle < n_bundles;
    const int bsafe = active ? bundle : 0;

    v4f acc[4][2];
#pragma unroll
    for (int g = 0; g < 4; ++g) acc[g][0] = acc[g][1] = (v4f){0.f, 0.f, 0.f, 0.f};

    // ---- depthwise parameters of the whole layer
    for (int i = threadIdx.x; i < 9 * K; i += NT) lds_p[i] = dw_w[i];
    for (int i = threadIdx.x; i < K; i += NT) lds_p[9 * KMAX + i] = dw_b[i];

    // ---- input tile staging: thread t moves 16-byte slots t, t+NT, ...; slot = pixel * 8 + column
    const float* xi = x + img * H * W * K;
    const int col4 = (threadIdx.x & 7) * 4;
    int goff[NL];
    uint32_t inside = 0;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        int pix = i * (NT / 8) + (threadIdx.x >> 3);
        pix = pix < NPIX ? pix : NPIX - 1;
        const int iy = iy0 + pix / IW, ix = ix0 + pix % IW;
        if (iy >= 0 && iy < H && ix >= 0 && ix < W) inside |= 1u << i;
        goff[i] = (min(max(iy, 0), H - 1) * W + min(max(ix, 0), W - 1)) * K;
    }
    v4f stage_reg[NL];
    auto issue_a = [&](int sc) {
        const int ch = sc * KC + col4;                       // K is a multiple of 32: always inside
#pragma unroll
        for (int i = 0; i < NL; ++i) stage_reg[i] = *(const v4f*)(xi + goff[i] + ch);
    };
    auto write_a = [&]() {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int pix = i * (NT / 8) + (threadIdx.x >> 3);
            const v4f v = (inside >> i) & 1u ? stage_reg[i] : (v4f){0.f, 0.f, 0.f, 0.f};
            if (pix < NPIX) {
                if (PAT)
                    *(v4f*)(lds_a + ((col4 >> 4) * NPIXP + pix) * 16 + (col4 & 15)) = v;
                else
                    *(v4f*)(lds_a + pix * KC + col4) = v;
            }
        }
    };

    // ---- depthwise: thread t -> channels col4..col4+3 of the sub-chunk, output pixels (oyp .. oyp +
    //      NO - 1, oxp) of the tile; the (NO - 1) * STRIDE + 3 input rows under them are read once
    const int oxp = (threadIdx.x >> 3) & 7, oyp = (threadIdx.x >> 6) * NO;
    auto dw_dense = [&](int sc) {
        const int ch = sc * KC + col4;
        v4f wt[9];
#pragma unroll
        for (int t = 0; t < 9; ++t) wt[t] = *(const v4f*)(lds_p + t * K + ch);
        const v4f b = *(const v4f*)(lds_p + 9 * KMAX + ch);
        v4f o[NO];
#pragma unroll
        for (int jo = 0; jo < NO; ++jo) o[jo] = b;
        const float* a0 = lds_a + ((oyp * STRIDE) * IW + oxp * STRIDE) * KC + col4;
#pragma unroll
        for (int r = 0; r < (NO - 1) * STRIDE + 3; ++r) {
            v4f a[3];
#pragma unroll
            for (int kx = 0; kx < 3; ++kx) a[kx] = *(const v4f*)(a0 + (r * IW + kx) * KC);
#pragma unroll
            for (int jo = 0; jo < NO; ++jo) {
                const int ky = r - jo * STRIDE;
                if (ky >= 0 && ky < 3) {
#pragma unroll
                    for (int kx = 0; kx < 3; ++kx) o[jo] += wt[ky * 3 + kx] * a[kx];
                }
            }
        }
#pragma unroll
        for (int jo = 0; jo < NO; ++jo) {
            v4f v = o[jo];
            if (dw_act == SBN_ACT_RELU) {
                v.x = fmaxf(v.x, 0.f);
                v.y = fmaxf(v.y, 0.f);
                v.z = fmaxf(v.z, 0.f);
                v.w = fmaxf(v.w, 0.f);
            }
            *(v4f*)(lds_x + ((oyp + jo) * TW + oxp) * XS + col4) = v;
        }
    };

    // ---- depthwise with pattern groups: a wave takes one 16-channel half of the sub-chunk (one group) and
    //      2 * NO rows of the tile; lane -> channel quad, column, row pair.  Output pixels (oyp ..
    //      oyp + NO - 1, oxp); the (NO - 1) * STRIDE + 3 input rows under them are read once.
    const int half = wave & 1, quad4 = (lane & 3) * 4;
    const int oxq = (lane >> 2) & 7, oyq = (wave >> 1) * (2 * NO) + (lane >> 5) * NO;
    const float* aq = lds_a + (half * NPIXP + (oyq * STRIDE) * IW + oxq * STRIDE) * 16 + quad4;
    float* xo = lds_x + (oyq * TW + oxq) * XS + half * 16 + quad4;
    // TAPS: bit ky * 3 + kx set = the tap is kept by every channel of the group (removed taps hold
    // zeros in dw_w, so a body that multiplies more taps than needed is still right)
    auto dw_body = [&](int sc, auto taps_c) {
        constexpr uint32_t TAPS = decltype(taps_c)::value;
        const int ch = sc * KC + half * 16 + quad4;
        const float* wp = lds_p + ch;                          // weights are read where they are used: few live registers
        const v4f b = *(const v4f*)(lds_p + 9 * KMAX + ch);
        v4f o[NO];
#pragma unroll
        for (int jo = 0; jo < NO; ++jo) o[jo] = b;
#pragma unroll
        for (int r = 0; r < (NO - 1) * STRIDE + 3; ++r) {
            v4f a[3];
#pragma unroll
            for (int kx = 0; kx < 3; ++kx) {
                bool needed = false;
#pragma unroll
                for (int jo = 0; jo < NO; ++jo) {
                    const int ky = r - jo * STRIDE;
                    if (ky >= 0 && ky < 3 && ((TAPS >> (ky * 3 + kx)) & 1u)) needed = true;
                }
                if (needed) a[kx] = *(const v4f*)(aq + (r * IW + kx) * 16);
            }
#pragma unroll
            for (int jo = 0; jo < NO; ++jo) {
                const int ky = r - jo * STRIDE;
                if (ky >= 0 && ky < 3) {
#pragma unroll
                    for (int kx = 0; kx < 3; ++kx)
                        if ((TAPS >> (ky * 3 + kx)) & 1u) o[jo] += *(const v4f*)(wp + (ky * 3 + kx) * K) * a[kx];
                }
            }
        }
#pragma unroll
        for (int jo = 0; jo < NO; ++jo) {
            v4f v = o[jo];
            if (dw_act == SBN_ACT_RELU) {
                v.x = fmaxf(v.x, 0.f);
                v.y = fmaxf(v.y, 0.f);
                v.z = fmaxf(v.z, 0.f);
                v.w = fmaxf(v.w, 0.f);
            }
            *(v4f*)(xo + jo * TW * XS) = v;
        }
    };
    // the 3:9 family: row r keeps columns {0, 1} (mask 3) or {1, 2} (mask 6)
#define SBN_TAPS(R0, R1, R2) std::integral_constant<uint32_t, (R0) | ((R1) << 3) | ((R2) << 6)>()
    auto dw_pattern = [&](int sc) {
        const uint32_t taps = dw_taps ? __builtin_amdgcn_readfirstlane(dw_taps[sc * (KC / 16) + half]) : 0x1FFu;
        switch (taps) {
        case 6 | (6 << 3) | (6 << 6): dw_body(sc, SBN_TAPS(6, 6, 6)); break;
        case 3 | (6 << 3) | (6 << 6): dw_body(sc, SBN_TAPS(3, 6, 6)); break;
        case 6 | (3 << 3) | (6 << 6): dw_body(sc, SBN_TAPS(6, 3, 6)); break;
        case 3 | (3 << 3) | (6 << 6): dw_body(sc, SBN_TAPS(3, 3, 6)); break;
        case 6 | (6 << 3) | (3 << 6): dw_body(sc, SBN_TAPS(6, 6, 3)); break;
        case 3 | (6 << 3) | (3 << 6): dw_body(sc, SBN_TAPS(3, 6, 3)); break;
        case 6 | (3 << 3) | (3 << 6): dw_body(sc, SBN_TAPS(6, 3, 3)); break;
        case 3 | (3 << 3) | (3 << 6): dw_body(sc, SBN_TAPS(3, 3, 3)); break;
        default: dw_body(sc, SBN_TAPS(7, 7, 7)); break;
        }
    };
#undef SBN_TAPS

    auto dw_compute = [&](int sc) {
        if constexpr (PAT)
            dw_pattern(sc);
        else
            dw_dense(sc);
    };

    // ---- the 1x1 layer's tables: one record of 8 descriptors and one first-entry index per sub-chunk;
    //      a 16-byte weight load per lane covers four entries
    const uint32_t* wo = woff + (size_t)bsafe * (n_sub + 1);
    const Record8* recs = (const Record8*)__builtin_assume_aligned(records, 32) + (size_t)bsafe * n_sub;
    auto load_weights = [&](int sc, v4f (&w)[2]) {
        const uint32_t e0 = __builtin_amdgcn_readfirstlane(wo[sc]);
        const v4f* src = (const v4f*)(wts + (size_t)e0 * 64) + lane;
        w[0] = src[0];
        w[1] = src[64];
    };
    auto multiply = [&](const Record8& r, const v4f (&w)[2]) {
        const char* xl = (const char*)lds_x + lane * (XS * 4);
        v4f xa, xb;
#define SBN_ENTRY(Q, XC, XN)                                             \
    if (__builtin_expect(r.d[Q] == 0, 0)) goto sub_chunk_done;           \
    if (Q + 1 < 8) XN = *(const v4f*)(xl + (r.d[(Q + 1) & 7] >> 8));      \
    entry_fma<Q>(r.d[Q], w[Q / 4], XC, acc);
        xa = *(const v4f*)(xl + (r.d[0] >> 8));
        SBN_ENTRY(0, xa, xb)
        SBN_ENTRY(1, xb, xa)
        SBN_ENTRY(2, xa, xb)
        SBN_ENTRY(3, xb, xa)
        SBN_ENTRY(4, xa, xb)
        SBN_ENTRY(5, xb, xa)
        SBN_ENTRY(6, xa, xb)
        SBN_ENTRY(7, xb, xa)
#undef SBN_ENTRY
    sub_chunk_done:;
    };

    v4f w_cur[2], w_nxt[2];
    Record8 r_cur, r_nxt;
    issue_a(0);
    load_weights(0, w_cur);
    r_cur = recs[0];
    write_a();
    __syncthreads();                                   // input tile and depthwise parameters visible
    dw_compute(0);
    __syncthreads();
    for (int sc = 0; sc < n_sub; ++sc) {
        const bool more = sc + 1 < n_sub;              // uniform over the workgroup
        const int scn = more ? sc + 1 : sc;
        issue_a(scn);                                  // in flight while this sub-chunk is multiplied
        load_weights(scn, w_nxt);
        r_nxt = recs[scn];
        if (active) multiply(r_cur, w_cur);
        if (more) write_a();                           // the input tile was consumed before the multiply
        __syncthreads();                               // X released, next input tile visible
        if (more) {
            dw_compute(sc + 1);
            __syncthreads();
        }
        w_cur[0] = w_nxt[0];
        w_cur[1] = w_nxt[1];
        r_cur = r_nxt;
    }

    // ---- epilogue: bias, activation, transpose through LDS (the input tile's memory), 256-byte rows
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
            *(v4f*)(lds_a + lane * OS + wave * 16 + g * 4) = o;
        }
    }
    __syncthreads();
    const int ch_base = col_tile * (16 * NWV);
    float* yi = y + img * OH * OW * N;
#pragma unroll
    for (int i = 0; i < 4; ++i) {                      // 64 pixels x 4 * NWV 16-byte columns = 4 * NT slots
        const int slot = i * NT + threadIdx.x;
        const int pl = slot / (4 * NWV), col = (slot % (4 * NWV)) * 4;
        const int oy = oy0 + pl / 8, ox = ox0 + pl % 8;
        if (oy < OH && ox < OW && ch_base + col < N)
            *(v4f*)(yi + ((long long)oy * OW + ox) * N + ch_base + col) = *(const v4f*)(lds_a + pl * OS + col);
    }
}

template <int STRIDE, int NWV, bool PAT>
int launch(const sbn_packed* p, const float* x, float* y, const float* dw_w, const float* dw_b, const uint32_t* dw_taps,
           int dw_act, int n, int h, int w, hipStream_t st)
{
    const sbn::DeviceLayout& L = p->dev;
    const int oh = (h - 1) / STRIDE + 1, ow = (w - 1) / STRIDE + 1;
    const int tiles_x = (ow + TW - 1) / TW, tiles_y = (oh + TH - 1) / TH;
    const long long n_pix_tiles = (long long)n * tiles_x * tiles_y;
    const int n_col_tiles = (L.n_bundles + NWV - 1) / NWV;
    const long long grid = ((n_pix_tiles + 7) / 8) * 8 * n_col_tiles;
    if ((long long)h * w * p->c_in > 0x7FFFFFFFll)
        return sbn::fail(SBN_EINVAL, "one image of %d x %d x %d elements is too large for 32-bit offsets", h, w, p->c_in);
    if (grid > 0x7FFFFFFFll || n_pix_tiles > 0x7FFFFFFFll)
        return sbn::fail(SBN_EINVAL, "too many output tiles for one launch (%lld)", n_pix_tiles);
    hipLaunchKernelGGL((dwpw_kernel<STRIDE, NWV, PAT>), dim3((unsigned)grid), dim3(64 * NWV), 0, st, x, y, dw_w, dw_b, dw_taps, dw_act, L.d_records32,
                       L.d_woff32, L.d_wts, L.d_bias, h, w, oh, ow, p->c_in, p->c_out, L.n_bundles, L.n_chunks32, n_col_tiles,
                       tiles_x, tiles_y, (int)n_pix_tiles, p->act);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return sbn::fail(SBN_EHIP, "fused depthwise + 1x1 launch: %s", hipGetErrorString(e));
    return SBN_OK;
}

}  // namespace

namespace sbn {

bool dwpw_fusable(const sbn_packed* p, int channels, int stride)
{
    return p->kind == SBN_CONV1X1 && p->c_in == channels && channels % KC == 0 && channels <= KMAX && p->c_out <= 128 &&
           (stride == 1 || stride == 2);
}

int launch_dwpw(const sbn_packed* p, const float* x, float* y, const float* dw_w, const float* dw_b,
                const uint32_t* dw_taps, int dw_stride, int dw_act, int n, int h, int w, void* stream)
{
    if (!dwpw_fusable(p, p->c_in, dw_stride))
        return fail(SBN_EINVAL, "internal error: fused depthwise + 1x1 launch for a layer it does not cover");
    hipStream_t st = (hipStream_t)stream;
    const bool wide = p->dev.n_bundles > 4;      // more than 64 output channels: eight waves cover up to 128
#define SBN_DWPW(S, NWV, PAT) launch<S, NWV, PAT>(p, x, y, dw_w, dw_b, dw_taps, dw_act, n, h, w, st)
    // Pattern bodies everywhere but in the eight-wave stride-2 form: there they need 134 registers,
    // one workgroup per CU instead of two (109 us against 79 us for MobileNet-v1's second block at
    // batch 64), so that form multiplies the stored zeros of the removed taps instead.
    if (dw_taps && !(wide && dw_stride == 2)) {
        if (wide) return SBN_DWPW(1, 8, true);
        return dw_stride == 2 ? SBN_DWPW(2, 4, true) : SBN_DWPW(1, 4, true);
    }
    if (wide) return dw_stride == 2 ? SBN_DWPW(2, 8, false) : SBN_DWPW(1, 8, false);
    return dw_stride == 2 ? SBN_DWPW(2, 4, false) : SBN_DWPW(1, 4, false);
#undef SBN_DWPW
}

}  // namespace sbn
