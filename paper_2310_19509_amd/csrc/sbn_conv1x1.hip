// Group-sparse 1x1 convolution for gfx950 (Algorithm 1 re-tiled for CDNA4).
//
// Mapping.  One lane owns one pixel (a wave owns 64*P pixels); a wave owns one
// bundle of four 4-filter output groups, a workgroup of four waves owns four
// bundles (64 output channels) over the same pixels.  The activation tile
// X[64*P pixels][KC channels] is staged once per workgroup in LDS, row stride
// KC+4 floats so that the per-lane 16-byte row reads are bank-conflict free.
//
// Inner step (one ENTRY = one 4-channel piece kept by at least one group of
// the bundle): each lane reads its pixel's 4 channels from LDS (one
// ds_read_b128 per pixel set), the wave loads the 64 weights of the entry
// ([group][ci][co], one float per lane), and for every group whose bit is
// set issues 4 x v_mfma_f32_4x4x1 (16 blocks): block b multiplies the weight
// column w[ci][0..3] -- broadcast from lanes 4*abid..4*abid+3 of the weight
// register to all 16 blocks -- with the activations of pixels 4b..4b+3.  The
// accumulator register i of lane L then holds output channel i of pixel L.
// The staged activation is reused by every group of the bundle that keeps the
// piece; the weight register is reused by every pixel set.
#include <hip/hip_runtime.h>

#include "sbn_internal.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

template <int ABID>
__device__ __forceinline__ v4f mfma_bcast(float w, float x, v4f c)
{
    // cbsz = 4: the A operand of block ABID is used by all 16 blocks
    return __builtin_amdgcn_mfma_f32_4x4x1f32(w, x, c, 4, ABID, 0);
}

template <int P>
struct Stage {
    float wv;
    v4f xv[P];
};

template <int P, int G>
__device__ __forceinline__ void group_fma(const Stage<P>& s, v4f (&acc)[P][4])
{
#pragma unroll
    for (int p = 0; p < P; ++p) acc[p][G] = mfma_bcast<4 * G + 0>(s.wv, s.xv[p].x, acc[p][G]);
#pragma unroll
    for (int p = 0; p < P; ++p) acc[p][G] = mfma_bcast<4 * G + 1>(s.wv, s.xv[p].y, acc[p][G]);
#pragma unroll
    for (int p = 0; p < P; ++p) acc[p][G] = mfma_bcast<4 * G + 2>(s.wv, s.xv[p].z, acc[p][G]);
#pragma unroll
    for (int p = 0; p < P; ++p) acc[p][G] = mfma_bcast<4 * G + 3>(s.wv, s.xv[p].w, acc[p][G]);
}

// P: pixel sets of 64 per wave.  KC: channels per LDS chunk (32 or 64).
// VEC: c_in % 4 == 0 (16-byte activation loads); otherwise scalar loads.
template <int P, int KC, bool VEC>
__global__ __launch_bounds__(256) void conv1x1_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                      const uint32_t* __restrict__ entries,
                                                      const float* __restrict__ wts,
                                                      const uint32_t* __restrict__ chunk_ptr32,
                                                      const float* __restrict__ bias, long long M, int K, int N,
                                                      int n_bundles, int n_chunks32, int n_col_tiles,
                                                      int n_pix_tiles, int act)
{
    constexpr int T = 64 * P;          // pixels per workgroup
    constexpr int S = KC + 4;          // LDS row stride in floats
    constexpr int C4 = KC / 4;         // float4 slots per row
    __shared__ __attribute__((aligned(16))) float lds[T * S];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // Workgroup -> (pixel tile, column tile).  Consecutive workgroup ids go to
    // different XCDs (8 of them, each with its own L2); the column tiles of
    // one pixel tile are given ids that differ by multiples of 8 so that they
    // run on the same XCD and share the activation tile in its L2.
    const int id = blockIdx.x;
    const int xcd = id & 7, j = id >> 3;
    const int pix_tile = (j / n_col_tiles) * 8 + xcd;
    const int col_tile = j % n_col_tiles;
    if (pix_tile >= n_pix_tiles) return;
    const long long pix0 = (long long)pix_tile * T;
    const int bundle = col_tile * 4 + wave;
    const bool active = bundle < n_bundles;

    v4f acc[P][4];
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
        for (int g = 0; g < 4; ++g) acc[p][g] = (v4f){0.f, 0.f, 0.f, 0.f};

    const uint32_t* cp = chunk_ptr32 + (size_t)(active ? bundle : 0) * (n_chunks32 + 1);
    const char* lds_lane = (const char*)lds + lane * (S * 4);
    const int n_chunks = (K + KC - 1) / KC;

    // Global -> register loads of one chunk (issued together so that their
    // latencies overlap), then register -> LDS.  Rows past the last pixel and
    // channels past c_in are staged as zeros.
    constexpr int NL = T * C4 / 256;
    v4f stage_reg[NL];
    auto issue_loads = [&](int c) {
        const int ch0 = c * KC;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int slot = i * 256 + threadIdx.x;
            const int row = slot / C4, col = (slot % C4) * 4;
            const long long pix = pix0 + row;
            const long long pixc = pix < M ? pix : M - 1;
            if (VEC) {
                const int chc = ch0 + col < K ? ch0 + col : 0;
                const v4f v = *(const v4f*)(x + pixc * K + chc);
                const bool ok = pix < M && ch0 + col < K;
                stage_reg[i] = ok ? v : (v4f){0.f, 0.f, 0.f, 0.f};
            } else {
                v4f v;
                for (int q = 0; q < 4; ++q) {
                    const int ch = ch0 + col + q;
                    const float t = x[pixc * K + (ch < K ? ch : 0)];
                    v[q] = (pix < M && ch < K) ? t : 0.f;
                }
                stage_reg[i] = v;
            }
        }
    };
    auto write_lds = [&]() {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int slot = i * 256 + threadIdx.x;
            const int row = slot / C4, col = (slot % C4) * 4;
            *(v4f*)(lds + row * S + col) = stage_reg[i];
        }
    };

    issue_loads(0);
    for (int c = 0; c < n_chunks; ++c) {
        if (c) __syncthreads();          // every wave has finished reading the previous chunk
        write_lds();
        __syncthreads();
        if (c + 1 < n_chunks) issue_loads(c + 1);   // in flight while this chunk is consumed

        if (active) {
            const int c32 = c * (KC / 32);
            const int c32e = min(c32 + KC / 32, n_chunks32);
            uint32_t e = __builtin_amdgcn_readfirstlane(cp[c32]);
            const uint32_t e1 = __builtin_amdgcn_readfirstlane(cp[c32e]);

            // Data of entry `en` whose descriptor `ent` is already in a scalar register.
            auto load = [&](uint32_t en, uint32_t ent, Stage<P>& s) {
                s.wv = wts[(size_t)en * 64 + lane];
                const int off = ((ent >> 8) & (C4 - 1)) * 16;
#pragma unroll
                for (int p = 0; p < P; ++p) s.xv[p] = *(const v4f*)(lds_lane + off + p * (64 * S * 4));
            };
            auto compute = [&](const Stage<P>& s, uint32_t m) {
                if (m & 1u) group_fma<P, 0>(s, acc);
                if (m & 2u) group_fma<P, 1>(s, acc);
                if (m & 4u) group_fma<P, 2>(s, acc);
                if (m & 8u) group_fma<P, 3>(s, acc);
            };

            if (e < e1) {
                // Descriptors run two entries ahead and data one entry ahead of
                // the arithmetic.  Reads past e1 stay inside the buffers' slack
                // and inside the LDS tile; their values are never used.
                uint32_t ent_cur = entries[e], ent_nxt = entries[e + 1];
                Stage<P> a, b;
                load(e, ent_cur, a);
                for (;;) {
                    uint32_t ent_nn = entries[e + 2];
                    load(e + 1, ent_nxt, b);
                    compute(a, ent_cur);
                    ent_cur = ent_nxt;
                    ent_nxt = ent_nn;
                    if (++e >= e1) break;
                    ent_nn = entries[e + 2];
                    load(e + 1, ent_nxt, a);
                    compute(b, ent_cur);
                    ent_cur = ent_nxt;
                    ent_nxt = ent_nn;
                    if (++e >= e1) break;
                }
            }
        }
    }

    // ---- epilogue: bias, activation, store 4 channels (16 bytes) per group
    if (!active) return;
    const int ch_base = bundle * 16;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int ch = ch_base + g * 4;
        if (ch >= N) break;
        const v4f b = *(const v4f*)(bias + ch);
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const long long pix = pix0 + p * 64 + lane;
            if (pix < M) {
                v4f o = acc[p][g] + b;
                if (act == SBN_ACT_RELU) {
                    o.x = fmaxf(o.x, 0.f);
                    o.y = fmaxf(o.y, 0.f);
                    o.z = fmaxf(o.z, 0.f);
                    o.w = fmaxf(o.w, 0.f);
                }
                *(v4f*)(y + pix * N + ch) = o;
            }
        }
    }
}

template <int P, int KC, bool VEC>
int launch(const sbn_packed* p, const float* x, float* y, long long M, hipStream_t st)
{
    const sbn::DeviceLayout& L = p->dev;
    const long long n_pix_tiles = (M + 64 * P - 1) / (64 * P);
    const int n_col_tiles = (L.n_bundles + 3) / 4;
    const long long grid = ((n_pix_tiles + 7) / 8) * 8 * n_col_tiles;
    if (grid > 0x7FFFFFFFll) return sbn::fail(SBN_EINVAL, "too many pixels for one launch (%lld)", M);
    hipLaunchKernelGGL((conv1x1_kernel<P, KC, VEC>), dim3((unsigned)grid), dim3(256), 0, st, x, y, L.d_entries,
                       L.d_wts, L.d_chunk_ptr32, L.d_bias, M, p->c_in, p->c_out, L.n_bundles, L.n_chunks32,
                       n_col_tiles, (int)n_pix_tiles, p->act);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return sbn::fail(SBN_EHIP, "conv1x1 launch: %s", hipGetErrorString(e));
    return SBN_OK;
}

}  // namespace

namespace sbn {

int launch_conv1x1(const sbn_packed* p, const float* x, float* y, long long M, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    const bool vec = p->c_in % 4 == 0;
    const bool kc32 = p->c_in <= 32;
    // pixel sets per wave: two when there are enough pixel tiles to fill the chip
    const int n_col_tiles = (p->dev.n_bundles + 3) / 4;
    const long long wgs_p2 = ((M + 127) / 128) * n_col_tiles;
    const bool p2 = wgs_p2 >= 1024;
    if (!vec) return kc32 ? launch<1, 32, false>(p, x, y, M, st) : launch<1, 64, false>(p, x, y, M, st);
    if (kc32) return p2 ? launch<2, 32, true>(p, x, y, M, st) : launch<1, 32, true>(p, x, y, M, st);
    return p2 ? launch<2, 64, true>(p, x, y, M, st) : launch<1, 64, true>(p, x, y, M, st);
}

}  // namespace sbn
