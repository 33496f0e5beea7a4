// Kernel-level group-sparse 3x3 convolution for gfx950 (Section 3.2, Conv3x3
// connectivity pruning: whole 3x3 kernels are kept or removed in groups).
//
// Same engine as the 1x1 kernel, with every kept piece carrying nine taps.
// One lane owns PX horizontally adjacent output pixels of an (8*PX)x8 spatial
// tile; a wave owns one bundle of four 4-filter groups (16 output channels);
// the four waves of a workgroup share the input tile, 32 channels at a time,
// staged in LDS through registers.  Input positions outside the image are
// staged as zeros, which realises the zero padding.  For stride 1 the tile is
// double buffered: the next 32 channels are fetched while the current ones
// are multiplied and are published with one barrier per sub-chunk.
//
// Every multiply consumes one activation scalar per lane, so the LDS read
// rate is what saturates first: with PX = 2 the two pixels share two of their
// three window columns, and all present groups of an entry share the window.
// The LDS image is swizzled so that these 16-byte reads are free of bank
// conflicts (see the kernel).
//
// Per entry (a 4-channel piece kept by at least one group of the bundle) the
// wave holds the entry's 9 x 64 weights ([tap][group][ci][co], one register
// per tap, fetched one entry ahead; with PX = 2 one row of taps at a time,
// fetched a row ahead) and walks the three rows of taps: the
// lane reads the row's shifted 16-byte activation vectors (one row ahead of
// the arithmetic) and, for every present group, issues 12 v_mfma_f32_4x4x1
// per pixel: the weight column [co 0..3] of (group, ci) is broadcast from
// lanes 4*abid..4*abid+3 to all 16 blocks and meets the activations of pixels
// 4b..4b+3, so accumulator register i of lane L is output channel i of pixel
// L.  The (up to 8) descriptors of a sub-chunk's record are held one per lane
// and broadcast with v_readlane.
//
// Launches too small to give every SIMD several waves use a workgroup of
// eight waves instead: two slices of four, each multiplying every second
// sub-chunk out of its own buffers, partial sums added through LDS at the end.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "sbn_internal.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

constexpr int TH = 8;                  // output tile height (width: 8 * PX)
constexpr int KC = 32;                 // channels staged at a time
constexpr int OS = 68;                 // output tile row stride in floats

template <int ABID>
__device__ __forceinline__ v4f mfma_bcast(float w, float x, v4f c)
{
    return __builtin_amdgcn_mfma_f32_4x4x1f32(w, x, c, 4, ABID, 0);
}

// One row of taps (ky = KY, kx = 0..2) of group G over the lane's PX pixels.  w holds the entry's
// nine taps (WT = 9) or just this row's three (WT = 3), lane l = [g][ci][co]; x holds the
// (PX-1)*STRIDE+3 input columns under the pixels.
// PX = 1: acc[G][0/1] are two partial sums of the one pixel (a dependent MFMA issues later than an
// independent one, which shows when a SIMD holds one or two waves: a single sum was measured 8-20 %
// slower there); PX = 2: acc[G][p] is pixel p.
template <int G, int KY, int PX, int STRIDE, int NX, int WT>
__device__ __forceinline__ void row_fma(const float (&w)[WT], const v4f (&x)[NX], v4f (&acc)[4][2])
{
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) {
        const float wt = w[WT == 9 ? KY * 3 + kx : kx];
        if constexpr (PX == 1) {
            acc[G][0] = mfma_bcast<G * 4 + 0>(wt, x[kx].x, acc[G][0]);
            acc[G][1] = mfma_bcast<G * 4 + 1>(wt, x[kx].y, acc[G][1]);
            acc[G][0] = mfma_bcast<G * 4 + 2>(wt, x[kx].z, acc[G][0]);
            acc[G][1] = mfma_bcast<G * 4 + 3>(wt, x[kx].w, acc[G][1]);
        } else {
            const v4f x0 = x[kx], x1 = x[STRIDE + kx];
            acc[G][0] = mfma_bcast<G * 4 + 0>(wt, x0.x, acc[G][0]);
            acc[G][1] = mfma_bcast<G * 4 + 0>(wt, x1.x, acc[G][1]);
            acc[G][0] = mfma_bcast<G * 4 + 1>(wt, x0.y, acc[G][0]);
            acc[G][1] = mfma_bcast<G * 4 + 1>(wt, x1.y, acc[G][1]);
            acc[G][0] = mfma_bcast<G * 4 + 2>(wt, x0.z, acc[G][0]);
            acc[G][1] = mfma_bcast<G * 4 + 2>(wt, x1.z, acc[G][1]);
            acc[G][0] = mfma_bcast<G * 4 + 3>(wt, x0.w, acc[G][0]);
            acc[G][1] = mfma_bcast<G * 4 + 3>(wt, x1.w, acc[G][1]);
        }
    }
}

template <int STRIDE, int PX, bool DEEP, int SPLIT>
__global__ __launch_bounds__(256 * SPLIT) void conv3x3_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                      const uint32_t* __restrict__ records,
                                                      const uint32_t* __restrict__ woff,
                                                      const float* __restrict__ wts, const float* __restrict__ bias,
                                                      int H, int W, int OH, int OW,
                                                      int K, int N, int n_bundles, int n_sub, int n_col_tiles,
                                                      int tiles_x, int tiles_y, int n_pix_tiles, int act)
{
    constexpr int TW = 8 * PX;                         // output tile width
    constexpr int NX = (PX - 1) * STRIDE + 3;          // input columns under a lane's pixels
    constexpr int IW = (TW - 1) * STRIDE + 3;          // input tile width
    constexpr int IH = (TH - 1) * STRIDE + 3;
    constexpr int NPIX = IW * IH;                      // staged input pixels
    constexpr int NSLOT = NPIX * (KC / 4);             // 16-byte slots of a staged tile
    constexpr int NL = (NSLOT + 255) / 256;            // slots per thread
    // LDS image of the tile: one 128-byte block per input pixel at block index
    // row * IWP + col (+ 1 for stride 2 when row/2 is odd); inside the block the 16-byte slot of
    // channels 4s..4s+3 sits at position s ^ g(col), g = col % 8 (PX = 1, stride 1) or
    // (col / 2) % 8.  With an odd row pitch (stride 1) or the row shift (stride 2) the 16 lanes
    // that a ds_read_b128 serves per cycle, two tile rows of 8 lanes, then hit 16 different
    // 16-byte bank groups for every tap and piece.
    constexpr int IWP = STRIDE == 2 ? IW + 1 : (IW | 1) == IW ? IW : IW + 1;
    constexpr int XBUF = IH * IWP * 32;                // floats per activation buffer
    constexpr bool DB = STRIDE == 1;
    struct XW {
        v4f r[DEEP ? 3 : 1][NX];
    };
    // SPLIT > 1: the workgroup has SPLIT slices of four waves; slice s multiplies the sub-chunks
    // s, s + SPLIT, ... out of its own pair of buffers and the partial sums are added through LDS
    // at the end.  For launches of at most one workgroup per CU, where the waves of a plain
    // workgroup would have a SIMD each to themselves and nothing to hide their waits behind.
    static_assert(SPLIT == 1 || (PX == 1 && STRIDE == 1), "the input channels are split for the one-pixel stride-1 form only");
    constexpr int OBUF = 64 * OS;                      // epilogue: 64 pixels x 64 channels
    constexpr int RBUF = (SPLIT - 1) * 4 * 64 * 16;    // partial sums of the slices above 0
    constexpr int NBUF = DB ? 2 : 1;
    constexpr int LDSF = SPLIT * NBUF * XBUF > OBUF + RBUF ? SPLIT * NBUF * XBUF : OBUF + RBUF;
    __shared__ __attribute__((aligned(16))) float lds_all[LDSF];

    const int lane = threadIdx.x & 63;
    const int tid = SPLIT == 1 ? threadIdx.x : threadIdx.x & 255;                     // thread within the slice
    const int slice = SPLIT == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x >> 8);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6) & 3;
    float* const lds = lds_all + slice * NBUF * XBUF;
    float* const lds_b = DB ? lds + XBUF : lds;

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

    // ---- staging: thread t moves 16-byte slots t, t+256, ...; slot = pixel * 8 + column, so a
    //      thread keeps its column and walks pixels t/8, t/8 + 32, ...  Positions outside the
    //      image load some inside position and are replaced by zeros on the way to LDS.
    // Addresses stay out of the VALU (plain vector instructions share the matrix pipe's issue
    // port): the image is a buffer, a slot's byte offset in it is computed once, positions outside
    // the image get an offset outside the buffer and are returned as zeros by the bounds check,
    // and the sub-chunk advances a scalar offset.
    const float* xi = x + img * H * W * K;
    const __amdgpu_buffer_rsrc_t xres =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(xi), 0, (int)((uint32_t)H * (uint32_t)W * (uint32_t)K * 4u), 0x00020000);
    const int col4 = (tid & 7) * 4;
    uint32_t goff[NL];            // byte offset of the slot's input position in the image; outside: 2^31, past any
                                  // image the launcher admits, and far enough from 2^32 not to wrap with the scalar offset
    int loff[NL];                 // float offset of the slot in the LDS image, -1: no such slot
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int pix = i * 32 + (tid >> 3);
        const int r = pix / IW, c = pix % IW;
        const int iy = iy0 + r, ix = ix0 + c;
        const bool in_image = pix < NPIX && iy >= 0 && iy < H && ix >= 0 && ix < W;
        goff[i] = in_image ? (uint32_t)((iy * W + ix) * K + col4) * 4u : 0x80000000u;
        const int g = PX == 1 && STRIDE == 1 ? c & 7 : (c >> 1) & 7;
        const int blk = r * IWP + c + (STRIDE == 2 ? (r >> 1) & 1 : 0);
        loff[i] = pix < NPIX ? blk * 32 + (((col4 >> 2) ^ g) << 2) : -1;
    }
    v4f stage_reg[NL];
    // (a ragged last sub-chunk reads channels past c_in: the next position's first channels, or
    // zeros at the image's very end; no entry ever uses them)
    auto issue_x = [&](int sc) {
#pragma unroll
        for (int i = 0; i < NL; ++i)
            stage_reg[i] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(xres, (int)goff[i], sc * (KC * 4), 0));
    };
    auto write_x = [&](float* buf) {
#pragma unroll
        for (int i = 0; i < NL; ++i)
            if (i + 1 < NL || loff[i] >= 0) *(v4f*)(buf + loff[i]) = stage_reg[i];
    };

    // this lane's window origin inside the staged tile
    const int oyl = lane / 8, oxl = (lane % 8) * PX;       // first of the lane's PX pixels
    const int row0 = oyl * STRIDE, col0 = oxl * STRIDE;
    constexpr int NG = PX == 1 && STRIDE == 1 ? 3 : 2;     // distinct g among the lane's columns
    int xrow[3], g16[NG];           // byte offsets of the window's rows relative to row 0's pitch; g << 4
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)      // stride 1: all three equal, the row pitch becomes an immediate
        xrow[ky] = (row0 * IWP + col0 + (STRIDE == 2 ? ((row0 + ky) >> 1) & 1 : 0)) * 128;
#pragma unroll
    for (int j = 0; j < NG; ++j) g16[j] = ((PX == 1 && STRIDE == 1 ? col0 + j : (col0 >> 1) + j) & 7) << 4;

    // the bundle's tables: one record of 8 descriptors and one first-entry index per 32 channels
    const uint32_t* wo = woff + (size_t)bsafe * (n_sub + 1);
    const uint32_t* recs = records + (size_t)bsafe * n_sub * 8;

    // Weights: one register per tap, lane l = [g][ci][co].  Fetched an entry ahead (WT = 9), or, with
    // two pixels per lane, a row of taps ahead (WT = 3): that form needs the registers for the
    // second pixel's window, and a row already carries 24 multiplies per present group.
    constexpr int WT = PX == 2 ? 3 : 9;
    auto load_w = [&](uint32_t en, int ky, float (&w)[WT]) {
        const float* wp = wts + (size_t)en * 576 + (WT == 3 ? ky * 192 : 0) + lane;
#pragma unroll
        for (int t = 0; t < WT; ++t) w[t] = wp[t * 64];
    };
    float wa[WT], wb[WT];     // weights in use and weights on their way
    float wn[SPLIT > 1 ? WT : 1];   // SPLIT > 1: first weights of the slice's next sub-chunk
    // dv: descriptors of the sub-chunk being multiplied, one per lane (lanes 0..7); e: the entry
    // whose first weights are in wa.  A bundle's entries are numbered in channel order, so with
    // SPLIT = 1 the entry after a sub-chunk's last is the next sub-chunk's first and e just counts
    // on.  With SPLIT > 1 the first weights of the slice's next sub-chunk (entry e1, read from the
    // table a round earlier) are fetched separately while this one is multiplied.
    uint32_t dv = 0, e = 0, e1 = 0;
    auto clamp_sc = [&](int sc) { return sc < n_sub ? sc : n_sub - 1; };

    // One sub-chunk of 32 channels: fetch the slice's next one, multiply this one, publish the next.
    auto sub_chunk = [&](int sc, const float* xbuf, float* xnext) {
        const int sc_nxt = clamp_sc(sc + SPLIT);
        uint32_t dv_nxt = 0;
        if (DB) {                                           // unconditional: loads under a branch
            issue_x(sc_nxt);                                // would be waited for before the arithmetic
            dv_nxt = recs[sc_nxt * 8 + (lane & 7)];
        }
        uint32_t e2 = 0;
        if constexpr (SPLIT > 1) {
            e2 = wo[clamp_sc(sc + 2 * SPLIT)];
            load_w(e1, 0, wn);
        }

        if (active && sc < n_sub) {
            const char* xl = (const char*)xbuf;
            uint32_t q = 0;                                 // position in the record
            auto desc = [&](uint32_t qq) -> uint32_t {
                return qq < 8 ? (uint32_t)__builtin_amdgcn_readlane((int)dv, (int)qq) : 0u;
            };
            auto mine = [&](uint32_t d) { return d != 0; };
            // activations under one row of taps of the piece named by descriptor d
            auto load_x = [&](uint32_t d, int ky, v4f (&xr)[NX]) {
                const int s16 = (int)((d >> 8) & 0x70u);     // 16 * (piece within the 32-channel sub-chunk)
#pragma unroll
                for (int c = 0; c < NX; ++c) {
                    const int j = PX == 1 && STRIDE == 1 ? c : c >> 1;
                    xr[c] = *(const v4f*)(xl + (xrow[ky] + (s16 ^ g16[j])) + (ky * IWP + c) * 128);
                }
            };
            auto row = [&](auto kytag, uint32_t m, const float (&w)[WT], const v4f (&xr)[NX]) {
                constexpr int KY = decltype(kytag)::value;
                // Each row tests its own copy of the mask with scalar instructions: were the three
                // rows' tests recognised as the same, the compiler would keep their results in
                // vector registers and pay VALU instructions (which share the matrix pipe's issue
                // port) to get them back.
                asm volatile("" : "+s"(m));
                // a taken branch costs the wave tens of cycles: keep "present" the fall-through path
                if (__builtin_expect((m & 1u) != 0, 1)) row_fma<0, KY, PX, STRIDE, NX, WT>(w, xr, acc);
                if (__builtin_expect((m & 2u) != 0, 1)) row_fma<1, KY, PX, STRIDE, NX, WT>(w, xr, acc);
                if (__builtin_expect((m & 4u) != 0, 1)) row_fma<2, KY, PX, STRIDE, NX, WT>(w, xr, acc);
                if (__builtin_expect((m & 8u) != 0, 1)) row_fma<3, KY, PX, STRIDE, NX, WT>(w, xr, acc);
            };
            // One entry.  Its weights are in w; the next entry's are fetched into w_nxt meanwhile.
            // Row-ahead (!DEEP): on entry p holds the activations under its first row of taps, on exit
            // r holds those of the next entry's first row.  Entry-ahead (DEEP, for launches with so
            // few waves per SIMD that latency counts): p holds the whole window and r receives the
            // next entry's.  Either way consecutive entries swap the two register sets.  A fetch past
            // the sub-chunk's last entry reads some in-tile activations that are not used, and the
            // weights of the first entry of the slice's next sub-chunk (past the last sub-chunk:
            // of some entry, or the array's slack).
            // e_cur: this entry's index, e_fetch: the entry whose first weights are fetched meanwhile
            // (SPLIT > 1: not used after the sub-chunk's last entry).
            auto entry = [&](uint32_t d, uint32_t d_nxt, uint32_t e_cur, uint32_t e_fetch, float (&w)[WT],
                             float (&w_nxt)[WT], XW& p, XW& r) {
                if constexpr (WT == 3) {
                    // weights and activations both run one row ahead; on exit w_nxt and r hold the
                    // first row of the next entry
                    load_w(e_cur, 1, w_nxt);
                    load_x(d, 1, r.r[0]);
                    row(std::integral_constant<int, 0>{}, d, w, p.r[0]);
                    load_w(e_cur, 2, w);
                    load_x(d, 2, p.r[0]);
                    row(std::integral_constant<int, 1>{}, d, w_nxt, r.r[0]);
                    load_w(e_fetch, 0, w_nxt);
                    load_x(d_nxt, 0, r.r[0]);
                    row(std::integral_constant<int, 2>{}, d, w, p.r[0]);
                    return;
                }
                load_w(e_fetch, 0, w_nxt);
                if constexpr (DEEP) {
                    load_x(d_nxt, 0, r.r[0]);
                    load_x(d_nxt, 1, r.r[1]);
                    load_x(d_nxt, 2, r.r[2]);
                    auto group = [&](auto gtag) {
                        constexpr int G = decltype(gtag)::value;
                        row_fma<G, 0, PX, STRIDE, NX, WT>(w, p.r[0], acc);
                        row_fma<G, 1, PX, STRIDE, NX, WT>(w, p.r[1], acc);
                        row_fma<G, 2, PX, STRIDE, NX, WT>(w, p.r[2], acc);
                    };
                    if (__builtin_expect((d & 1u) != 0, 1)) group(std::integral_constant<int, 0>{});
                    if (__builtin_expect((d & 2u) != 0, 1)) group(std::integral_constant<int, 1>{});
                    if (__builtin_expect((d & 4u) != 0, 1)) group(std::integral_constant<int, 2>{});
                    if (__builtin_expect((d & 8u) != 0, 1)) group(std::integral_constant<int, 3>{});
                } else {
                    load_x(d, 1, r.r[0]);
                    row(std::integral_constant<int, 0>{}, d, w, p.r[0]);
                    load_x(d, 2, p.r[0]);
                    row(std::integral_constant<int, 1>{}, d, w, r.r[0]);
                    load_x(d_nxt, 0, r.r[0]);
                    row(std::integral_constant<int, 2>{}, d, w, p.r[0]);
                }
            };
            uint32_t d_cur = desc(q);
            if (mine(d_cur)) {
                XW xa, xb;
                load_x(d_cur, 0, xa.r[0]);
                if constexpr (DEEP) {
                    load_x(d_cur, 1, xa.r[1]);
                    load_x(d_cur, 2, xa.r[2]);
                }
                // Entries go in pairs, the second with the two register sets (weights and window in
                // use / on their way) in exchanged roles, so that nothing is ever copied: plain
                // moves are VALU instructions and share the matrix pipe's issue port (the one-entry
                // loop with an exchange by name cost up to 27 moves per entry).  After an odd
                // number of entries the pair's second half runs on the record's terminator: it
                // multiplies nothing (no group bit is set) and fetches the same next weights again,
                // which leaves them where the next sub-chunk expects them.
                while (true) {
                    const uint32_t d1 = desc(q + 1);
                    entry(d_cur, d1, e, e + 1, wa, wb, xa, xb);
                    const uint32_t d2 = desc(q + 2);
                    const uint32_t two = mine(d1) ? 1u : 0u;
                    entry(d1, d2, e + 1, e + 1 + two, wb, wa, xb, xa);
                    q += 1 + two, e += 1 + two;
                    d_cur = d2;
                    if (!(mine(d1) && mine(d2))) break;
                }
            }
        }
        if constexpr (SPLIT > 1) {
#pragma unroll
            for (int t = 0; t < WT; ++t) wa[t] = wn[t];
            e = e1;
            e1 = __builtin_amdgcn_readfirstlane(e2);
        }
        if (!DB) {                       // single buffer: fetch after everyone has finished reading it
            __syncthreads();
            issue_x(sc_nxt);
            dv_nxt = recs[sc_nxt * 8 + (lane & 7)];
        }
        write_x(xnext);
        dv = dv_nxt;
        __syncthreads();
    };

    {
        const int sc0 = clamp_sc(slice), sc1 = clamp_sc(slice + SPLIT);
        issue_x(sc0);
        dv = recs[sc0 * 8 + (lane & 7)];
        e = __builtin_amdgcn_readfirstlane(wo[sc0]);
        e1 = __builtin_amdgcn_readfirstlane(wo[sc1]);
        load_w(e, 0, wa);
        write_x(lds);
        __syncthreads();
    }
    // every slice runs the same number of rounds (and barriers); a slice whose turn lies past the
    // last sub-chunk stages the last one again and multiplies nothing
    const int n_rounds = (n_sub + SPLIT - 1) / SPLIT;
    for (int i = 0; i < n_rounds; i += 2) {
        sub_chunk(slice + i * SPLIT, lds, lds_b);
        if (i + 1 < n_rounds) sub_chunk(slice + (i + 1) * SPLIT, lds_b, lds);
    }

    // ---- SPLIT > 1: add the slices' partial sums into slice 0.  The staging buffers are dead after
    //      the last barrier above; [0, OBUF) is the epilogue's transpose area, the sums go behind it.
    if constexpr (SPLIT > 1) {
        float* red = lds_all + OBUF;
        if (slice > 0 && active) {
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *(v4f*)(red + ((((slice - 1) * 4 + wave) * 4 + g) * 64 + lane) * 4) = acc[g][0] + acc[g][1];
        }
        __syncthreads();
        if (slice == 0 && active) {
#pragma unroll
            for (int sl = 1; sl < SPLIT; ++sl)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    acc[g][0] += *(const v4f*)(red + ((((sl - 1) * 4 + wave) * 4 + g) * 64 + lane) * 4);
        }
    }

    // ---- epilogue: bias, activation, transpose through LDS, full 256-byte rows per pixel;
    //      one pass per pixel of the lane
    const int ch_base = col_tile * 64;
    float* yi = y + img * OH * OW * N;
#pragma unroll
    for (int p = 0; p < PX; ++p) {
        if (p) __syncthreads();
        if (active && slice == 0) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                v4f o = (PX == 1 ? acc[g][0] + acc[g][1] : acc[g][p]) + *(const v4f*)(bias + bundle * 16 + g * 4);
                if (act == SBN_ACT_RELU) {
                    o.x = fmaxf(o.x, 0.f);
                    o.y = fmaxf(o.y, 0.f);
                    o.z = fmaxf(o.z, 0.f);
                    o.w = fmaxf(o.w, 0.f);
                }
                *(v4f*)(lds_all + lane * OS + wave * 16 + g * 4) = o;
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4 / SPLIT; ++i) {
            const int slot = i * 256 * SPLIT + threadIdx.x;
            const int pl = slot >> 4, col = (slot & 15) * 4;             // pl: the lane that owned the pixel
            const int oy = oy0 + pl / 8, ox = ox0 + (pl % 8) * PX + p;
            if (oy < OH && ox < OW && ch_base + col < N)
                *(v4f*)(yi + ((long long)oy * OW + ox) * N + ch_base + col) = *(const v4f*)(lds_all + pl * OS + col);
        }
    }
}

template <int STRIDE, int PX, bool DEEP, int SPLIT = 1>
int launch(const sbn_packed* p, const float* x, float* y, int n, int h, int w, hipStream_t st)
{
    const sbn::DeviceLayout& L = p->dev;
    const int oh = (h - 1) / STRIDE + 1, ow = (w - 1) / STRIDE + 1;
    const int tiles_x = (ow + 8 * PX - 1) / (8 * PX), tiles_y = (oh + TH - 1) / TH;
    const long long n_pix_tiles = (long long)n * tiles_x * tiles_y;
    const int n_col_tiles = (L.n_bundles + 3) / 4;
    const long long grid = ((n_pix_tiles + 7) / 8) * 8 * n_col_tiles;
    if ((long long)h * w * p->c_in > 0x1FFFFFFFll)     // 2 GiB per image: byte offsets and the out-of-image mark fit 32 bits
        return sbn::fail(SBN_EINVAL, "one image of %d x %d x %d elements is too large for 32-bit byte offsets", h, w, p->c_in);
    if (grid > 0x7FFFFFFFll || n_pix_tiles > 0x7FFFFFFFll)
        return sbn::fail(SBN_EINVAL, "too many output tiles for one launch (%lld)", n_pix_tiles);
    hipLaunchKernelGGL((conv3x3_kernel<STRIDE, PX, DEEP, SPLIT>), dim3((unsigned)grid), dim3(256 * SPLIT), 0, st, x, y,
                       L.d_records32, L.d_woff32, L.d_wts, L.d_bias, h, w, oh, ow, p->c_in, p->c_out, L.n_bundles, L.n_chunks32,
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
    hipStream_t st = (hipStream_t)stream;
    if (p->stride == 2) return launch<2, 1, false>(p, x, y, n, h, w, st);
    // Form, from timings of ResNet-50-shaped layers at batches 4..128 (thresholds in workgroups per
    // compute unit of the device the layer lives on): up to one
    // plain workgroup per CU the waves would sit alone on their SIMDs, so the input channels are
    // split over two slices (entry-ahead fetch); up to two per CU the entry-ahead form; above that
    // two pixels per lane when 16-wide tiles waste no more lanes than 8-wide ones (they need 7 %
    // less time per pixel), else one pixel per lane, row-ahead (four workgroups per CU).
    int form = forced_kernel_form(SBN_CONV3X3);         // testing / benchmarking override
    if (!form) {
        const long long col_tiles = (p->dev.n_bundles + 3) / 4;
        const long long tiles1 = (long long)((w + 7) / 8) * ((h + 7) / 8), tiles2 = (long long)((w + 15) / 16) * ((h + 7) / 8);
        const long long wg1 = n * tiles1 * col_tiles;
        const long long cus = p->dev.cus;
        form = wg1 <= cus ? 32 : wg1 <= 2 * cus ? 3 : w > 8 && tiles2 * 2 * 93 < tiles1 * 100 ? 2 : 1;
    }
    switch (form) {
    case 2: return launch<1, 2, false>(p, x, y, n, h, w, st);
    case 3: return launch<1, 1, true>(p, x, y, n, h, w, st);
    case 32: return launch<1, 1, true, 2>(p, x, y, n, h, w, st);
    default: return launch<1, 1, false>(p, x, y, n, h, w, st);
    }
}

}  // namespace sbn
