// Group-sparse 1x1 convolution for gfx950 (Algorithm 1 re-tiled for CDNA4).
//
// Mapping.  One lane owns one pixel (a wave owns 64*P pixels); a wave owns one
// bundle of four 4-filter output groups (16 output channels); a workgroup of
// four waves owns four bundles over the same pixels.  The activation tile
// X[64*P pixels][KC channels] of a chunk is staged once per workgroup in LDS,
// row stride KC+4 floats so that the per-lane 16-byte row reads are free of
// bank conflicts.
//
// Inner step (one ENTRY = one 4-channel piece kept by at least one group of
// the bundle): each lane reads its pixel's 4 channels from LDS (ds_read_b128
// per pixel set) and, for every group whose bit is set, the wave issues
// 4*P v_mfma_f32_4x4x1 (16 blocks each): block b multiplies the weight column
// w[co 0..3][ci] -- broadcast from lanes 4*abid..4*abid+3 of a weight register
// to all 16 blocks -- with the activations of pixels 4b..4b+3, so accumulator
// register i of lane L holds output channel i of pixel L.  That MFMA shape is
// exactly one row of a 4x4 block: no padding, no idle lanes.  The staged
// activation is reused by every group of the bundle that keeps the piece, a
// weight register by every pixel set.  Group bits are tested with scalar
// instructions on the wave-uniform descriptor.  The weights of a whole chunk
// (16-byte loads per lane, four entries each) and the chunk's record of
// descriptors (one scalar load) are fetched one chunk ahead.
//
// Epilogue: partial sums are added (the first one started from the bias), the
// activation applied, the output tile is transposed through LDS and written as
// full rows of 16-byte stores.
//
// Forms (launch_conv1x1 picks one per launch): the workgroup form above with 64 or
// 128 pixels per tile (plain_tile); the few-pixel form, one bundle per workgroup with
// the input channels split over its waves (splitk_tile); the mixed launch, whole
// rounds of workgroup tiles plus the remaining pixels as few-pixel workgroups in one
// grid; and, for layers that keep most of their pieces, the walk over the
// every-piece tables, where entry q of a chunk is piece q and its activations sit
// at a compile-time offset.  chain_tail_kernel runs several small chain items as
// phases of one launch.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "sbn_internal.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

// max(v, 0) per component as ONE instruction each: a signed integer maximum on the bit patterns
// (a float with its sign bit set is a negative integer; -0.0 and negative NaNs become +0.0).
// fmaxf() costs two (the compiler first re-quiets its operand), and every VALU instruction takes
// matrix-pipe issue time.
__device__ __forceinline__ v4f relu4(v4f v)
{
    typedef int v4i __attribute__((ext_vector_type(4)));
    const v4i b = __builtin_bit_cast(v4i, v);
    return __builtin_bit_cast(v4f, (v4i){b.x > 0 ? b.x : 0, b.y > 0 ? b.y : 0, b.z > 0 ? b.z : 0, b.w > 0 ? b.w : 0});
}
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// Vector instructions share their issue port with the matrix instructions: a plain VALU
// instruction costs a SIMD about half of a 4x4x1 MFMA (measured: 32 extra v_add per chunk and
// wave make a 512 x 512 layer 5 % slower).  So the kernels keep address arithmetic out of the
// VALU.  Tiles are addressed through buffer descriptors: a scalar base and size (the tile's own
// bytes, so accesses past the tile's last row return zero / are dropped), a per-lane 32-bit
// offset that never changes, and a scalar offset that advances from chunk to chunk.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);   // raw, 32-bit words
}
__device__ __forceinline__ v4f buf_load(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t scalar_off)
{
    return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, (int)scalar_off, 0));
}

template <int ABID>
__device__ __forceinline__ v4f mfma_bcast(float w, float x, v4f c)
{
    // cbsz = 4: the A operand of block ABID is used by all 16 blocks
    return __builtin_amdgcn_mfma_f32_4x4x1f32(w, x, c, 4, ABID, 0);
}

// acc[p][g][a]: pixel set p, group g, partial sum a.  An MFMA that adds to the result of
// the MFMA issued just before it has to wait for that result, so the four input channels
// of a piece alternate over NA partial sums (with NA = 3 the rotation also advances with the
// entry slot Q so that the distance stays three across entries).
template <int P, int NA, int Q, int G>
__device__ __forceinline__ void group_fma(const v4f& w, const v4f (&xv)[P], v4f (&acc)[P][4][NA])
{
    constexpr int R = NA == 3 ? Q % 3 : 0;
    constexpr int AB = (Q & 3) * 4 + G;           // lanes 4*AB..4*AB+3 of w hold [co 0..3] of entry Q, group G
#pragma unroll
    for (int p = 0; p < P; ++p) acc[p][G][(0 + R) % NA] = mfma_bcast<AB>(w.x, xv[p].x, acc[p][G][(0 + R) % NA]);
#pragma unroll
    for (int p = 0; p < P; ++p) acc[p][G][(1 + R) % NA] = mfma_bcast<AB>(w.y, xv[p].y, acc[p][G][(1 + R) % NA]);
#pragma unroll
    for (int p = 0; p < P; ++p) acc[p][G][(2 + R) % NA] = mfma_bcast<AB>(w.z, xv[p].z, acc[p][G][(2 + R) % NA]);
#pragma unroll
    for (int p = 0; p < P; ++p) acc[p][G][(3 + R) % NA] = mfma_bcast<AB>(w.w, xv[p].w, acc[p][G][(3 + R) % NA]);
}

template <int P, int NA, int Q>
__device__ __forceinline__ void entry_fma(uint32_t m, const v4f& w, const v4f (&xv)[P], v4f (&acc)[P][4][NA])
{
    // a taken branch costs the wave tens of cycles: keep "present" the fall-through path
    if (__builtin_expect((m & 1u) != 0, 1)) group_fma<P, NA, Q, 0>(w, xv, acc);
    if (__builtin_expect((m & 2u) != 0, 1)) group_fma<P, NA, Q, 1>(w, xv, acc);
    if (__builtin_expect((m & 4u) != 0, 1)) group_fma<P, NA, Q, 2>(w, xv, acc);
    if (__builtin_expect((m & 8u) != 0, 1)) group_fma<P, NA, Q, 3>(w, xv, acc);
}

// Lanes of one wave exchange data through LDS without a workgroup barrier (the hardware executes
// a wave's LDS operations in order).  This keeps the compiler from moving LDS accesses across
// the exchange point; it emits no instruction.
__device__ __forceinline__ void wave_lds_order()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int NS>
struct Record {
    uint32_t d[NS];
};

// P: pixel sets of 64 per wave.  NA: partial sums per (pixel set, group).
// KC: channels staged per chunk, 64, or 32 for layers with c_in <= 32.
// MULTI: c_in > KC, more than one chunk.  VEC: c_in % 4 == 0 (16-byte
// activation loads); otherwise scalar loads with zero fill.
//
// Activations go global -> registers -> LDS.  (global_load_lds would save the
// registers, but the compiler then drains the whole vector-memory counter
// before every LDS read, which serialises the prefetch with the arithmetic.)
// Two LDS buffers alternate: the loads of chunk c+1 are issued before chunk c
// is multiplied, land in registers meanwhile, are written to the other buffer
// afterwards, and one barrier per chunk publishes them.  The prefetch is
// unconditional (the last chunk fetches itself again): loads issued under a
// branch would make the compiler wait for them before the first multiply.
// One tile of the workgroup form: 64*P pixels x 64 output channels (four bundles, one per wave),
// all input channels.  lds / lds_b: the workgroup's two activation buffers of 64*P x (KC+4)
// floats each (lds_b unused when !MULTI).  Called by all 256 threads of the workgroup.
//
// STATIC: the layer's every-piece tables (layers that keep most of their pieces).  Entry q of a
// chunk is piece q, present or not: `records` is then the array of present masks (s_stride per
// bundle), `wts` the every-piece weights, `woff` is not used; the activations of entry q sit at a
// compile-time offset of the lane's row, which takes the one VALU instruction per entry (the
// address add) out of the loop -- it shares the issue port with the MFMAs.
template <int P, int NA, int KC, bool MULTI, bool VEC, bool STATIC = false>
__device__ __forceinline__ void plain_tile(float* __restrict__ lds, float* __restrict__ lds_b,
                                           const float* __restrict__ x, float* __restrict__ y,
                                           const uint32_t* __restrict__ records, const uint32_t* __restrict__ woff,
                                           const float* __restrict__ wts, const float* __restrict__ bias, long long M,
                                           int K, int N, int n_bundles, int n_chunks, int pix_tile, int col_tile, int act,
                                           int s_stride = 0)
{
    static_assert(!STATIC || (MULTI && VEC), "every-piece tables exist for multi-chunk layers with c_in % 4 == 0");
    constexpr int T = 64 * P;                  // pixels per workgroup
    constexpr int NS = KC / 4;                 // descriptors per record (one record per KC channels)
    constexpr int NW = NS / 4;                 // 16-byte weight loads per lane and chunk
    constexpr int XS = KC + 4;                 // staged row stride in floats

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long pix0 = (long long)pix_tile * T;
    const int bundle = col_tile * 4 + wave;
    const bool active = bundle < n_bundles;
    const int bsafe = active ? bundle : 0;

    // the first partial sum of every group starts from the bias (a lane's four accumulator
    // components are four output channels): the epilogue then has no bias add
    v4f acc[P][4][NA];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const v4f b = *(const v4f*)(bias + bsafe * 16 + g * 4);
#pragma unroll
        for (int p = 0; p < P; ++p)
#pragma unroll
            for (int a = 0; a < NA; ++a) acc[p][g][a] = a == 0 ? b : (v4f){0.f, 0.f, 0.f, 0.f};
    }
    // (Setting the accumulators with MFMAs instead -- bias x 1 + 0 and 0 x 0 + 0, eight MFMAs for
    // 32 register writes -- was measured 1.5 % slower over the 13-layer pass.)

    // ---- activation staging.  Thread t moves slots t, t+256, ... of the tile's
    // T x (KC/4) 16-byte slots.  Rows past the last pixel repeat the last pixel
    // (a lane only ever reads its own pixel's row); channels past c_in are never
    // read by any entry (VEC) or are zero filled (!VEC).
    constexpr int C4 = KC / 4;
    constexpr int NL = T * C4 / 256;
    const float* xtile = x + pix0 * K;
    const int rows_valid = (int)(M - pix0 < T ? M - pix0 : T);
    v4f stage_reg[NL];
    // VEC: the tile as a buffer of rows_valid rows; a slot's offset is row * K + column (bytes),
    // the chunk advances the scalar offset.  Rows past the last pixel and, in a ragged last chunk,
    // channels past the end of the last row lie outside the buffer and read as zero; channels past
    // c_in of other rows read the next row's first channels, which no entry ever uses.
    const __amdgpu_buffer_rsrc_t xres = make_rsrc(xtile, (uint32_t)rows_valid * (uint32_t)K * 4u);
    uint32_t xoff[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int slot = i * 256 + threadIdx.x;
        xoff[i] = ((uint32_t)(slot / C4) * (uint32_t)K + (uint32_t)(slot % C4) * 4u) * 4u;
    }
    auto issue_x = [&](int c) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            if (VEC) {
                stage_reg[i] = buf_load(xres, xoff[i], (uint32_t)c * (KC * 4));
            } else {
                const int slot = i * 256 + threadIdx.x;
                const int row = slot / C4, col = (slot % C4) * 4;
                const float* rp = xtile + (size_t)(row < rows_valid ? row : rows_valid - 1) * K;
                v4f v;
                for (int q = 0; q < 4; ++q) {
                    const int ch = c * KC + col + q;
                    const float t = rp[ch < K ? ch : 0];
                    v[q] = ch < K ? t : 0.f;
                }
                stage_reg[i] = v;
            }
        }
    };
    auto write_x = [&](float* buf) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int slot = i * 256 + threadIdx.x;
            const int row = slot / C4, col = (slot % C4) * 4;
            *(v4f*)(buf + row * XS + col) = stage_reg[i];
        }
    };

    // ---- weights and descriptors of one chunk.  NW 16-byte loads per lane cover
    // NS entries; entries past the chunk's own belong to later chunks or to the
    // array's slack and are never used.
    const uint32_t* wo = STATIC ? nullptr : woff + (size_t)bsafe * (n_chunks + 1);
    const Record<NS>* recs = STATIC ? (const Record<NS>*)__builtin_assume_aligned(records + (size_t)bsafe * s_stride, 4 * NS)
                                    : (const Record<NS>*)__builtin_assume_aligned(records, 4 * NS) + (size_t)bsafe * n_chunks;
    const __amdgpu_buffer_rsrc_t wres = make_rsrc(wts, 0xFFFFFFFFu);     // (the launcher checks the array is below 4 GiB)
    auto load_weights = [&](int c, v4f (&w)[NW]) {
        const uint32_t e0 = STATIC ? (uint32_t)bsafe * (uint32_t)s_stride + (uint32_t)c * NS
                                   : __builtin_amdgcn_readfirstlane(wo[c]);
#pragma unroll
        for (int q4 = 0; q4 < NW; ++q4) w[q4] = buf_load(wres, (uint32_t)lane * 16u + q4 * 1024u, e0 * 256u);
    };

    // One chunk: start the loads of the next chunk, multiply the current one out
    // of `xbuf`, then store the arrived activations to `xnext` and synchronise.
    auto chunk = [&](int c, const float* xbuf, float* xnext, const v4f (&w_cur)[NW], v4f (&w_nxt)[NW],
                     const Record<NS>& r_cur, Record<NS>& r_nxt) {
        if (MULTI) {                         // in flight while this chunk is multiplied
            const int cn = c + 1 < n_chunks ? c + 1 : c;
            issue_x(cn);
            load_weights(cn, w_nxt);
            r_nxt = recs[cn];
            // This chunk's weights were fetched a chunk ago: everything but the loads just issued
            // has to be complete.  Saying so once here spares a wait in front of every group's
            // multiplies (the compiler cannot carry that knowledge across the group branches).
            constexpr int NEW = (VEC ? NL : 4 * NL) + NW;
            static_assert(NEW < 64, "vmcnt is a 6-bit counter");
            __builtin_amdgcn_s_waitcnt((NEW & 15) | ((NEW >> 4) << 14) | (7 << 4) | (15 << 8));
        }

        if (active) {
            const char* lds_lane = (const char*)xbuf + lane * (XS * 4);
            v4f xa[P], xb[P];
            auto read_x = [&](uint32_t d, v4f (&xv)[P]) {
                const int off = d >> 8;                  // 16 * kb4 within the chunk
#pragma unroll
                for (int p = 0; p < P; ++p) xv[p] = *(const v4f*)(lds_lane + off + p * (64 * XS * 4));
            };
            // Entries are compacted at the front of the record; the first zero
            // descriptor ends the chunk.  Activations run one entry ahead.
            // One wait per entry, in front of the group tests: LDS reads return in order, so with
            // at most the P reads of the next entry outstanding this entry's activations have
            // arrived (the first entry also waits for the record, a scalar load).  Without it the
            // compiler puts a wait in front of every group's multiplies.
#define SBN_ENTRY(Q, XC, XN)                                                   \
    if (Q < NS) {                                                              \
        if (__builtin_expect(r_cur.d[Q % NS] == 0, 0)) goto chunk_done;        \
        if (Q + 1 < NS) read_x(r_cur.d[(Q + 1) % NS], XN);                     \
        __builtin_amdgcn_s_waitcnt(0xC07F | ((Q == 0 || Q + 1 >= NS ? 0 : P) << 8)); \
        entry_fma<P, NA, Q>(r_cur.d[Q % NS], w_cur[(Q / 4) % NW], XC, acc);    \
    }
            // every-piece walk: no terminator, the row offset of entry Q is 16 * Q; a piece that no
            // group keeps (rare where these tables are built) is skipped with one test
            auto read_s = [&](auto q_c, v4f (&xv)[P]) {
                constexpr int QQ = decltype(q_c)::value;
#pragma unroll
                for (int p = 0; p < P; ++p) xv[p] = *(const v4f*)(lds_lane + QQ * 16 + p * (64 * XS * 4));
            };
#define SBN_ENTRY_S(Q, XC, XN)                                                 \
    if (Q < NS) {                                                              \
        if (Q + 1 < NS) read_s(std::integral_constant<int, (Q + 1) % NS>(), XN); \
        __builtin_amdgcn_s_waitcnt(0xC07F | ((Q == 0 || Q + 1 >= NS ? 0 : P) << 8)); \
        if (__builtin_expect(r_cur.d[Q % NS] != 0, 1))                         \
            entry_fma<P, NA, Q>(r_cur.d[Q % NS], w_cur[(Q / 4) % NW], XC, acc); \
    }
            if (STATIC) {
                read_s(std::integral_constant<int, 0>(), xa);
                SBN_ENTRY_S(0, xa, xb)
                SBN_ENTRY_S(1, xb, xa)
                SBN_ENTRY_S(2, xa, xb)
                SBN_ENTRY_S(3, xb, xa)
                SBN_ENTRY_S(4, xa, xb)
                SBN_ENTRY_S(5, xb, xa)
                SBN_ENTRY_S(6, xa, xb)
                SBN_ENTRY_S(7, xb, xa)
                SBN_ENTRY_S(8, xa, xb)
                SBN_ENTRY_S(9, xb, xa)
                SBN_ENTRY_S(10, xa, xb)
                SBN_ENTRY_S(11, xb, xa)
                SBN_ENTRY_S(12, xa, xb)
                SBN_ENTRY_S(13, xb, xa)
                SBN_ENTRY_S(14, xa, xb)
                SBN_ENTRY_S(15, xb, xa)
                goto chunk_done;
            }
#undef SBN_ENTRY_S
            read_x(r_cur.d[0], xa);
            SBN_ENTRY(0, xa, xb)
            SBN_ENTRY(1, xb, xa)
            SBN_ENTRY(2, xa, xb)
            SBN_ENTRY(3, xb, xa)
            SBN_ENTRY(4, xa, xb)
            SBN_ENTRY(5, xb, xa)
            SBN_ENTRY(6, xa, xb)
            SBN_ENTRY(7, xb, xa)
            SBN_ENTRY(8, xa, xb)
            SBN_ENTRY(9, xb, xa)
            SBN_ENTRY(10, xa, xb)
            SBN_ENTRY(11, xb, xa)
            SBN_ENTRY(12, xa, xb)
            SBN_ENTRY(13, xb, xa)
            SBN_ENTRY(14, xa, xb)
            SBN_ENTRY(15, xb, xa)
#undef SBN_ENTRY
        chunk_done:;
        }
        if (MULTI) write_x(xnext);
        __syncthreads();                     // tile of the next chunk published / this one released
    };

    v4f w_a[NW], w_b[NW];
    Record<NS> r_a, r_b;
    issue_x(0);
    load_weights(0, w_a);
    r_a = recs[0];
    write_x(lds);
    __syncthreads();
    if (MULTI) {
        for (int c = 0; c < n_chunks; c += 2) {
            chunk(c, lds, lds_b, w_a, w_b, r_a, r_b);
            if (c + 1 < n_chunks) chunk(c + 1, lds_b, lds, w_b, w_a, r_b, r_a);
        }
    } else {
        chunk(0, lds, lds, w_a, w_b, r_a, r_b);
    }

    // ---- epilogue: the output tile is transposed through LDS in passes of KC channels (KC/16
    // waves each) and stored as full rows.  The accumulators go to LDS as they are (the store
    // takes them straight from the accumulator registers: no copy, no VALU instruction); with two
    // partial sums per group and two activation buffers the second sums go through the second
    // buffer, and the threads that store a row add the two, apply the activation and store.
    // (The bias is in the first partial sum.  The barrier that ended the last chunk makes the
    // tile memory reusable.)
    constexpr bool TWO = MULTI && NA == 2;
#pragma unroll
    for (int h = 0; h < 64 / KC; ++h) {
        if (h) __syncthreads();
        if (active && wave / (KC / 16) == h) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    const int at = (p * 64 + lane) * XS + (wave % (KC / 16)) * 16 + g * 4;
                    if (TWO) {
                        *(v4f*)(lds + at) = acc[p][g][0];
                        *(v4f*)(lds_b + at) = acc[p][g][1];
                    } else {
                        v4f o = acc[p][g][0];
#pragma unroll
                        for (int a = 1; a < NA; ++a) o += acc[p][g][a];
                        *(v4f*)(lds + at) = o;
                    }
                }
            }
        }
        __syncthreads();
        // The tile's rows of y as a buffer: rows past the last pixel are dropped by the bounds
        // check, a thread whose column lies past c_out gets an offset outside the buffer.
        // (Streaming stores: the output is not read again by this launch; measured 3 % of a
        // 13-layer pass whose buffers do not fit the last-level cache.)
        const int ch_base = col_tile * 64 + h * KC;
        const __amdgpu_buffer_rsrc_t yres = make_rsrc(y + pix0 * N, (uint32_t)rows_valid * (uint32_t)N * 4u);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int slot = i * 256 + threadIdx.x;
            const int row = slot / C4, col = (slot % C4) * 4;
            const uint32_t off = ch_base + col < N ? ((uint32_t)row * (uint32_t)N + (uint32_t)(ch_base + col)) * 4u : 0xFFFFFFF0u;
            v4f o = *(const v4f*)(lds + row * XS + col);
            if (TWO) o += *(const v4f*)(lds_b + row * XS + col);
            if (act == SBN_ACT_RELU) o = relu4(o);
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, o), yres, (int)off, 0, 2 /* slc: streaming */);
        }
    }
}

// Workgroup -> (pixel tile, column tile).  Consecutive workgroup ids go to different XCDs (8 of
// them, each with its own L2); the column tiles of one pixel tile get ids that differ by
// multiples of 8 so that they run on the same XCD and share the activation tile in its L2.
__device__ __forceinline__ void xcd_tile(int id, int n_col_tiles, int& pix_tile, int& col_tile)
{
    const int xcd = id & 7, j = id >> 3;
    pix_tile = (j / n_col_tiles) * 8 + xcd;
    col_tile = j % n_col_tiles;
}

template <int P, int NA, int KC, bool MULTI, bool VEC, bool STATIC = false>
__global__ __launch_bounds__(256) void conv1x1_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                      const uint32_t* __restrict__ records,
                                                      const uint32_t* __restrict__ woff,
                                                      const float* __restrict__ wts, const float* __restrict__ bias,
                                                      long long M, int K, int N, int n_bundles, int n_chunks,
                                                      int n_col_tiles, int n_pix_tiles, int act, int s_stride)
{
    constexpr int XBUF = 64 * P * (KC + 4);    // floats per activation buffer
    __shared__ __attribute__((aligned(16))) float lds[XBUF];
    __shared__ __attribute__((aligned(16))) float lds_b[MULTI ? XBUF : 4];
    int pix_tile, col_tile;
    xcd_tile(blockIdx.x, n_col_tiles, pix_tile, col_tile);
    if (pix_tile >= n_pix_tiles) return;
    plain_tile<P, NA, KC, MULTI, VEC, STATIC>(lds, lds_b, x, y, records, woff, wts, bias, M, K, N, n_bundles, n_chunks,
                                              pix_tile, col_tile, act, s_stride);
}

// Few-pixel form.  With few pixels (batch 1, deep layers) the workgroup kernel above leaves most
// of the chip idle: pixel tiles x column tiles is far below the number of CUs while every wave walks
// all of c_in serially.  Here a workgroup owns 64 pixels x ONE bundle and its NW waves split the
// input channels: wave s takes the 32-channel sub-chunks s, s + NW, ...  A wave shares nothing while
// it works (own activation tile in its own LDS slice, staged through registers one sub-chunk ahead;
// LDS operations of one wave execute in order, so no barrier is needed); at the end the NW partial
// results meet in LDS and are added in wave order, which keeps the sum deterministic.
// Needs c_in % 4 == 0.
// lds_pool: NW tiles of 64 x 36 floats, one per wave.  Called by all 64*NW threads of the workgroup.
template <int NW>
__device__ __forceinline__ void splitk_tile(float* __restrict__ lds_pool, const float* __restrict__ x,
                                            float* __restrict__ y, const uint32_t* __restrict__ records,
                                            const uint32_t* __restrict__ woff, const float* __restrict__ wts,
                                            const float* __restrict__ bias, long long M, int K, int N, int n_chunks,
                                            long long pix0, int bundle, int act)
{
    constexpr int KC = 32, NS = KC / 4, NWL = NS / 4, XS = KC + 4, NA = 2;
    constexpr int NL = 8;                                // 16-byte slots per lane and tile
    float(*lds_all)[64 * XS] = (float(*)[64 * XS])lds_pool;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float* lds = lds_all[wave];

    v4f acc[1][4][NA];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int a = 0; a < NA; ++a) acc[0][g][a] = (v4f){0.f, 0.f, 0.f, 0.f};

    // ---- activation staging: 8 lanes fetch the 128 bytes of one row, 8 rows per instruction
    const float* xtile = x + pix0 * K;
    const int rows_valid = (int)(M - pix0 < 64 ? M - pix0 : 64);
    const int scol = (lane & 7) * 4;
    v4f stage_reg[NL];
    // (addresses as in the workgroup form: the tile is a buffer of rows_valid rows, a per-lane
    // offset that never changes, the sub-chunk in the scalar offset)
    const __amdgpu_buffer_rsrc_t xres = make_rsrc(xtile, (uint32_t)rows_valid * (uint32_t)K * 4u);
    uint32_t xoff[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) xoff[i] = ((uint32_t)(i * 8 + (lane >> 3)) * (uint32_t)K + (uint32_t)scol) * 4u;
    auto issue_x = [&](int c) {
#pragma unroll
        for (int i = 0; i < NL; ++i) stage_reg[i] = buf_load(xres, xoff[i], (uint32_t)c * (KC * 4));
    };
    auto write_x = [&]() {
#pragma unroll
        for (int i = 0; i < NL; ++i) *(v4f*)(lds + (i * 8 + (lane >> 3)) * XS + scol) = stage_reg[i];
    };
    const uint32_t* wo = woff + (size_t)bundle * (n_chunks + 1);
    const Record<NS>* recs = (const Record<NS>*)__builtin_assume_aligned(records, 4 * NS) + (size_t)bundle * n_chunks;
    const __amdgpu_buffer_rsrc_t wres = make_rsrc(wts, 0xFFFFFFFFu);
    auto load_weights = [&](int c, v4f (&w)[NWL]) {
        const uint32_t e0 = __builtin_amdgcn_readfirstlane(wo[c]);
#pragma unroll
        for (int q4 = 0; q4 < NWL; ++q4) w[q4] = buf_load(wres, (uint32_t)lane * 16u + q4 * 1024u, e0 * 256u);
    };
    const char* lds_lane = (const char*)lds + lane * (XS * 4);
    auto read_x = [&](uint32_t d, v4f (&xv)[1]) { xv[0] = *(const v4f*)(lds_lane + (d >> 8)); };
    auto walk = [&](const Record<NS>& r, const v4f (&w)[NWL]) {
        v4f xa[1], xb[1];
#define SBN_ENTRY(Q, XC, XN)                                            \
    if (__builtin_expect(r.d[Q] == 0, 0)) goto walk_done;               \
    if (Q + 1 < NS) read_x(r.d[(Q + 1) % NS], XN);                      \
    entry_fma<1, NA, Q>(r.d[Q], w[Q / 4], XC, acc);
        read_x(r.d[0], xa);
        SBN_ENTRY(0, xa, xb)
        SBN_ENTRY(1, xb, xa)
        SBN_ENTRY(2, xa, xb)
        SBN_ENTRY(3, xb, xa)
        SBN_ENTRY(4, xa, xb)
        SBN_ENTRY(5, xb, xa)
        SBN_ENTRY(6, xa, xb)
        SBN_ENTRY(7, xb, xa)
#undef SBN_ENTRY
    walk_done:;
    };

    // this wave's sub-chunks: wave, wave + NW, ...; the next one's loads are in flight while the
    // current one is multiplied (the last one fetches itself again: loads stay unconditional)
    if (wave < n_chunks) {
        v4f w_cur[NWL], w_nxt[NWL];
        Record<NS> r_cur, r_nxt;
        issue_x(wave);
        load_weights(wave, w_cur);
        r_cur = recs[wave];
        write_x();
        for (int c = wave; c < n_chunks; c += NW) {
            const int cn = c + NW < n_chunks ? c + NW : c;
            issue_x(cn);
            load_weights(cn, w_nxt);
            r_nxt = recs[cn];
            wave_lds_order();                  // rows written by other lanes are read below
            walk(r_cur, w_cur);
            wave_lds_order();                  // all reads of the tile precede its overwrite
            write_x();
#pragma unroll
            for (int q4 = 0; q4 < NWL; ++q4) w_cur[q4] = w_nxt[q4];
            r_cur = r_nxt;
        }
    }

    // ---- the NW partial results meet in LDS and are added in wave order
    wave_lds_order();                          // the last staged tile is dead before it is reused
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        v4f o = acc[0][g][0];
#pragma unroll
        for (int a = 1; a < NA; ++a) o += acc[0][g][a];
        *(v4f*)(lds + lane * XS + g * 4) = o;
    }
    __syncthreads();
    if (threadIdx.x < 256) {
        const int row = threadIdx.x >> 2, col = (threadIdx.x & 3) * 4;
        v4f o = *(const v4f*)(lds_all[0] + row * XS + col);
#pragma unroll
        for (int s = 1; s < NW; ++s) o += *(const v4f*)(lds_all[s] + row * XS + col);
        o += *(const v4f*)(bias + bundle * 16 + col);
        if (act == SBN_ACT_RELU) o = relu4(o);
        const long long pix = pix0 + row;
        if (pix < M && bundle * 16 + col < N) *(v4f*)(y + pix * N + bundle * 16 + col) = o;
    }
}

template <int NW>
__global__ __launch_bounds__(64 * NW) void conv1x1_splitk_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                                 const uint32_t* __restrict__ records,
                                                                 const uint32_t* __restrict__ woff,
                                                                 const float* __restrict__ wts,
                                                                 const float* __restrict__ bias, long long M, int K,
                                                                 int N, int n_bundles, int n_chunks, int act)
{
    __shared__ __attribute__((aligned(16))) float lds_pool[NW * 64 * 36];
    const int bundle = blockIdx.x % n_bundles;           // neighbouring workgroups share the pixels
    const long long pix0 = (long long)(blockIdx.x / n_bundles) * 64;
    splitk_tile<NW>(lds_pool, x, y, records, woff, wts, bias, M, K, N, n_chunks, pix0, bundle, act);
}

// Mixed form for launches of a few rounds of workgroups.  A launch of W workgroup tiles on C
// compute units finishes when the busiest unit does: ceil(W / C) tiles, although the work is
// only W / C.  Here the first n_plain workgroups (a whole number of tiles per compute unit) run
// the workgroup form on pixel tiles [0, tail_tile0); the pixels after that are covered by
// workgroups of the few-pixel form (one bundle, input channels split over the four waves), each
// a quarter of a tile's work per SIMD, which the dispatcher spreads evenly at the end.
// (STATIC: the workgroup-form part walks the every-piece tables -- records = the masks, wts_plain =
// the every-piece weights; the few-pixel part always uses the compact tables.)
template <int P, int NA, int KC, bool STATIC = false>
__global__ __launch_bounds__(256) void conv1x1_mixed_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                            const uint32_t* __restrict__ records,
                                                            const uint32_t* __restrict__ woff,
                                                            const float* __restrict__ wts_plain,
                                                            const uint32_t* __restrict__ records32,
                                                            const uint32_t* __restrict__ woff32,
                                                            const float* __restrict__ wts,
                                                            const float* __restrict__ bias, long long M, int K, int N,
                                                            int n_bundles, int n_chunks, int n_chunks32, int n_col_tiles,
                                                            int n_plain, long long tail_pix0, int n_tail_tiles, int act,
                                                            int s_stride)
{
    constexpr int XBUF = 64 * P * (KC + 4);
    constexpr int POOL = 2 * XBUF > 4 * 64 * 36 ? 2 * XBUF : 4 * 64 * 36;
    __shared__ __attribute__((aligned(16))) float pool[POOL];
    if ((int)blockIdx.x < n_plain) {
        int pix_tile, col_tile;
        xcd_tile(blockIdx.x, n_col_tiles, pix_tile, col_tile);      // n_plain covers whole groups of 8 pixel tiles
        plain_tile<P, NA, KC, true, true, STATIC>(pool, pool + XBUF, x, y, records, woff, wts_plain, bias, M, K, N, n_bundles,
                                                  n_chunks, pix_tile, col_tile, act, s_stride);
    } else {
        // the bundles of one pixel tile get ids that differ by multiples of 8: same XCD, shared L2
        const int id = blockIdx.x - n_plain;
        const int xcd = id & 7, j = id >> 3;
        const int tile = (j / n_bundles) * 8 + xcd;
        if (tile >= n_tail_tiles) return;
        splitk_tile<4>(pool, x, y, records32, woff32, wts, bias, M, K, N, n_chunks32, tail_pix0 + (long long)tile * 64,
                       j % n_bundles, act);
    }
}

// ---- several chain items in one launch (few pixels) ---------------------------------------
// Grid-wide barrier for a grid whose workgroups are all resident.  Sense reversal: the last
// workgroup to arrive clears the arrival count and advances the generation the others wait
// for, so the two words need no reset between barriers or launches.  Waits are bounded: after
// spin_limit polls a workgroup sets the status word and the whole grid leaves (every wave
// reaches an exit whatever happens to the others).  Returns false if the grid is to leave.
__device__ __forceinline__ bool grid_barrier(unsigned* sync, unsigned n_wg, unsigned spin_limit, int* flag_lds)
{
    // The workgroup barrier orders every thread's stores before thread 0, whose device-scope
    // release then writes this XCD's L2 back; after the wait its device-scope acquire drops the
    // stale lines of this CU's vector cache and of the L2 before the second workgroup barrier
    // lets the other threads read what the other workgroups wrote.
    __syncthreads();
    if (threadIdx.x == 0) {
        int ok = 1;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        const unsigned gen = __hip_atomic_load(&sync[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned prev = __hip_atomic_fetch_add(&sync[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (prev + 1 == n_wg) {
            __hip_atomic_store(&sync[0], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_fetch_add(&sync[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            unsigned spins = 0;
            while (__hip_atomic_load(&sync[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gen) {
                __builtin_amdgcn_s_sleep(2);
                if (++spins > spin_limit || __hip_atomic_load(&sync[2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                    __hip_atomic_store(&sync[2], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    ok = 0;
                    break;
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        *flag_lds = ok;
    }
    __syncthreads();
    return *flag_lds != 0;
}

// Dense depthwise 3x3 (+ bias, activation), pad 1, as a phase: a thread per four channels of
// one output pixel, grid-stride.  w [9][c], b [c].
__device__ __forceinline__ void tail_depthwise(const sbn::TailPhase& ph)
{
    const int c4n = ph.c >> 2;
    const long long total = (long long)ph.n * ph.oh * ph.ow * c4n;
    for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (long long)gridDim.x * blockDim.x) {
        const int c4 = (int)(t % c4n) * 4;
        long long pix = t / c4n;
        const int ox = (int)(pix % ph.ow);
        pix /= ph.ow;
        const int oy = (int)(pix % ph.oh);
        const long long b = pix / ph.oh;
        v4f acc = *(const v4f*)(ph.dw_b + c4);
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
            const int iy = oy * ph.stride + ky - 1;
            if (iy < 0 || iy >= ph.h) continue;
#pragma unroll
            for (int kx = 0; kx < 3; ++kx) {
                const int ix = ox * ph.stride + kx - 1;
                if (ix < 0 || ix >= ph.w) continue;
                acc += *(const v4f*)(ph.src + ((b * ph.h + iy) * ph.w + ix) * ph.c + c4) *
                       *(const v4f*)(ph.dw_w + (ky * 3 + kx) * ph.c + c4);
            }
        }
        if (ph.act == SBN_ACT_RELU) {
            acc.x = fmaxf(acc.x, 0.f);
            acc.y = fmaxf(acc.y, 0.f);
            acc.z = fmaxf(acc.z, 0.f);
            acc.w = fmaxf(acc.w, 0.f);
        }
        *(v4f*)(ph.dst + ((b * ph.oh + oy) * (long long)ph.ow + ox) * ph.c + c4) = acc;
    }
}

constexpr int kTailWaves = 8;       // waves per workgroup: a 1x1 task is 64 pixels x one bundle, channels split eight ways

__global__ __launch_bounds__(64 * kTailWaves) void chain_tail_kernel(sbn::TailArgs a, unsigned* sync, unsigned spin_limit)
{
    __shared__ __attribute__((aligned(16))) float pool[kTailWaves * 64 * 36];
    __shared__ int flag;
    if (__hip_atomic_load(&sync[2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;   // an earlier launch gave up
    for (int p = 0; p < a.n_phases; ++p) {
        const sbn::TailPhase& ph = a.ph[p];
        if (ph.kind == 1) {
            const long long n_tasks = ((ph.M + 63) / 64) * ph.n_bundles;
            for (long long t = blockIdx.x; t < n_tasks; t += gridDim.x) {
                splitk_tile<kTailWaves>(pool, ph.src, ph.dst, ph.rec32, ph.woff32, ph.wts, ph.bias, ph.M, ph.K, ph.N,
                                        ph.n_chunks32, (t / ph.n_bundles) * 64, (int)(t % ph.n_bundles), ph.act);
                __syncthreads();                       // the tile memory is free for the next task
            }
        } else if (ph.kind == 0) {
            tail_depthwise(ph);
        } else {
            const v4f* s4 = (const v4f*)ph.src;
            v4f* d4 = (v4f*)ph.dst;
            for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < ph.M; i += (long long)gridDim.x * blockDim.x)
                d4[i] = s4[i];
        }
        if (p + 1 < a.n_phases && !grid_barrier(sync, gridDim.x, spin_limit, &flag)) return;
    }
}

template <int NW>
int launch_splitk(const sbn_packed* p, const float* x, float* y, long long M, hipStream_t st)
{
    const sbn::DeviceLayout& L = p->dev;
    const long long n_pix_tiles = (M + 63) / 64;
    const long long grid = n_pix_tiles * L.n_bundles;
    if (grid > 0x7FFFFFFFll) return sbn::fail(SBN_EINVAL, "too many pixels for one launch (%lld)", M);
    hipLaunchKernelGGL((conv1x1_splitk_kernel<NW>), dim3((unsigned)grid), dim3(64 * NW), 0, st, x, y, L.d_records32,
                       L.d_woff32, L.d_wts, L.d_bias, M, p->c_in, p->c_out, L.n_bundles, L.n_chunks32, p->act);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return sbn::fail(SBN_EHIP, "conv1x1 launch: %s", hipGetErrorString(e));
    return SBN_OK;
}

template <int P, int NA, int KC, bool MULTI, bool VEC, bool STATIC = false>
int launch(const sbn_packed* p, const float* x, float* y, long long M, hipStream_t st)
{
    const sbn::DeviceLayout& L = p->dev;
    const long long n_pix_tiles = (M + 64 * P - 1) / (64 * P);
    const int n_col_tiles = (L.n_bundles + 3) / 4;
    const long long grid = ((n_pix_tiles + 7) / 8) * 8 * n_col_tiles;
    if (grid > 0x7FFFFFFFll) return sbn::fail(SBN_EINVAL, "too many pixels for one launch (%lld)", M);
    if (STATIC && !L.d_desc_s) return sbn::fail(SBN_EINVAL, "internal error: the layer has no every-piece tables");
    hipLaunchKernelGGL((conv1x1_kernel<P, NA, KC, MULTI, VEC, STATIC>), dim3((unsigned)grid), dim3(256), 0, st, x, y,
                       STATIC ? L.d_desc_s : KC == 64 ? L.d_records : L.d_records32, KC == 64 ? L.d_woff : L.d_woff32,
                       STATIC ? L.d_wts_s : L.d_wts, L.d_bias, M,
                       p->c_in, p->c_out, L.n_bundles, KC == 64 ? L.n_chunks : L.n_chunks32, n_col_tiles,
                       (int)n_pix_tiles, p->act, L.n_chunks * sbn::kSlots);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return sbn::fail(SBN_EHIP, "conv1x1 launch: %s", hipGetErrorString(e));
    return SBN_OK;
}

// Mixed launch: pixel tiles [0, plain_tiles) (a multiple of 8) in the workgroup form, the pixels
// after them in the few-pixel form.
template <int P, int NA, int KC, bool STATIC = false>
int launch_mixed(const sbn_packed* p, const float* x, float* y, long long M, long long plain_tiles, hipStream_t st)
{
    const sbn::DeviceLayout& L = p->dev;
    const int n_col_tiles = (L.n_bundles + 3) / 4;
    const long long tail_pix0 = plain_tiles * 64 * P;
    const long long n_tail_tiles = (M - tail_pix0 + 63) / 64;
    const long long n_plain = plain_tiles * n_col_tiles;
    const long long grid = n_plain + ((n_tail_tiles + 7) / 8) * 8 * L.n_bundles;
    if (plain_tiles % 8 || tail_pix0 > M) return sbn::fail(SBN_EINVAL, "internal error: bad split of a mixed launch");
    if (grid > 0x7FFFFFFFll) return sbn::fail(SBN_EINVAL, "too many pixels for one launch (%lld)", M);
    if (STATIC && !L.d_desc_s) return sbn::fail(SBN_EINVAL, "internal error: the layer has no every-piece tables");
    hipLaunchKernelGGL((conv1x1_mixed_kernel<P, NA, KC, STATIC>), dim3((unsigned)grid), dim3(256), 0, st, x, y,
                       STATIC ? L.d_desc_s : KC == 64 ? L.d_records : L.d_records32, KC == 64 ? L.d_woff : L.d_woff32,
                       STATIC ? L.d_wts_s : L.d_wts, L.d_records32,
                       L.d_woff32, L.d_wts, L.d_bias, M, p->c_in, p->c_out, L.n_bundles,
                       KC == 64 ? L.n_chunks : L.n_chunks32, L.n_chunks32, n_col_tiles, (int)n_plain, tail_pix0,
                       (int)n_tail_tiles, p->act, L.n_chunks * sbn::kSlots);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return sbn::fail(SBN_EHIP, "conv1x1 launch: %s", hipGetErrorString(e));
    return SBN_OK;
}

}  // namespace

namespace sbn {

int launch_chain_tail(const TailArgs& a, unsigned* sync, int cus, void* stream)
{
    if (a.n_phases <= 0 || a.n_phases > kTailMaxPhases || !sync) return fail(SBN_EINVAL, "internal error: bad multi-layer launch");
    // as many workgroups as the largest phase has tasks, and never more than are resident at once
    // (two of these workgroups fit a compute unit; one per unit is asked for)
    long long want = 1;
    for (int p = 0; p < a.n_phases; ++p) {
        const TailPhase& ph = a.ph[p];
        long long tasks;
        if (ph.kind == 1)
            tasks = ((ph.M + 63) / 64) * ph.n_bundles;
        else if (ph.kind == 0)
            tasks = ((long long)ph.n * ph.oh * ph.ow * (ph.c / 4) + 64 * kTailWaves - 1) / (64 * kTailWaves);
        else
            tasks = (ph.M + 64 * kTailWaves - 1) / (64 * kTailWaves);
        want = std::max(want, tasks);
    }
    const int grid = (int)std::min<long long>(want, cus);
    hipLaunchKernelGGL(chain_tail_kernel, dim3(grid), dim3(64 * kTailWaves), 0, (hipStream_t)stream, a, sync, 1u << 20);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SBN_EHIP, "multi-layer launch: %s", hipGetErrorString(e));
    return SBN_OK;
}

int launch_conv1x1(const sbn_packed* p, const float* x, float* y, long long M, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    const int K = p->c_in;
    // the kernels address the weights with 32-bit byte offsets
    if ((p->dev.wts.size() + (size_t)kSlots * 64) * sizeof(float) >= 0xFFFFFFFFull ||
        p->dev.wts_s.size() * sizeof(float) >= 0xFFFFFFFFull)
        return fail(SBN_EINVAL, "the layer's device weights exceed 4 GiB");
    const int force = forced_kernel_form(SBN_CONV1X1);  // testing / benchmarking override
    if (K % 4) {
        if (K <= 32) return launch<1, 2, 32, false, false>(p, x, y, M, st);
        if (K <= 64) return launch<1, 2, 64, false, false>(p, x, y, M, st);
        return launch<1, 2, 64, true, false>(p, x, y, M, st);
    }
    // one chunk (HBM-bound layers): 64-pixel tiles keep more workgroups, hence more loads, in flight
    const bool p2 = (force % 1000) / 10 == 2 && force != 1;
    if (K <= 32) return p2 ? launch<2, 1, 32, false, true>(p, x, y, M, st) : launch<1, 2, 32, false, true>(p, x, y, M, st);
    if (K <= 64) return p2 ? launch<2, 1, 64, false, true>(p, x, y, M, st) : launch<1, 2, 64, false, true>(p, x, y, M, st);
    const int cus = p->dev.cus;
    // forms 1000 + f: form f on the every-piece tables (f where the layer has none); the automatic
    // choice uses them whenever the layer has them
    const bool have_s = p->dev.d_desc_s != nullptr;
    const bool stat = force ? force >= 1000 && have_s : have_s;
    int variant = force == 1 ? 0 : force % 1000;        // 1: the automatic choice, but never the every-piece tables
    // few pixels (at most four 64-pixel x one-bundle workgroups per CU) and at least 256 input
    // channels -> one bundle per workgroup, input channels split over its waves: as many waves as
    // keep the launch within about four waves per SIMD and leave every wave at least two
    // sub-chunks (timed on the deep MobileNet layers at batches 1..32)
    const int n_sub = p->dev.n_chunks32;
    const long long wg_split = ((M + 63) / 64) * p->dev.n_bundles;
    if (!variant && n_sub >= 8 && wg_split <= 4ll * cus)
        variant = n_sub >= 32 && wg_split <= cus ? 516 : n_sub >= 16 && wg_split <= 2ll * cus ? 508 : 504;
    const int n_col_tiles = (p->dev.n_bundles + 3) / 4;
    if (!variant) {
        // 128-pixel tiles with 32-channel chunks halve the per-entry overhead; they pay off
        // from three such tiles per CU on (timed with every form forced on every layer of the
        // MobileNet stack at batch 64: 5-9 % over 64-pixel tiles at 3.06 tiles per CU, 15-20 %
        // behind them at 1.6)
        variant = ((M + 127) / 128) * n_col_tiles >= 3ll * cus ? 21 : 12;
        // Whole rounds of workgroups only: when the last round would occupy at most half of
        // the compute units, the pixels of that round go to few-pixel workgroups instead.
        const int px = variant == 21 ? 128 : 64;
        const long long tiles = (M + px - 1) / px, w = tiles * n_col_tiles, rem = w % cus;
        if (rem && 2 * rem <= cus && w > cus && n_sub >= 4) {
            const long long plain_tiles = (w - rem) / n_col_tiles / 8 * 8;
            if (stat)
                return variant == 21 ? launch_mixed<2, 1, 32, true>(p, x, y, M, plain_tiles, st)
                                     : launch_mixed<1, 2, 64, true>(p, x, y, M, plain_tiles, st);
            return variant == 21 ? launch_mixed<2, 1, 32>(p, x, y, M, plain_tiles, st)
                                 : launch_mixed<1, 2, 64>(p, x, y, M, plain_tiles, st);
        }
    }
    if (variant == 112 || variant == 121) {             // forced mixed forms: all but the last pixel tiles plain
        const int px = variant == 121 ? 128 : 64;
        const long long plain_tiles = ((M + px - 1) / px - 1) / 8 * 8;
        if (stat)
            return variant == 121 ? launch_mixed<2, 1, 32, true>(p, x, y, M, plain_tiles, st)
                                  : launch_mixed<1, 2, 64, true>(p, x, y, M, plain_tiles, st);
        return variant == 121 ? launch_mixed<2, 1, 32>(p, x, y, M, plain_tiles, st)
                              : launch_mixed<1, 2, 64>(p, x, y, M, plain_tiles, st);
    }
    if (stat && (variant == 21 || variant == 12 || variant == 0))
        return variant == 21 ? launch<2, 1, 32, true, true, true>(p, x, y, M, st) : launch<1, 2, 64, true, true, true>(p, x, y, M, st);
    switch (variant) {
    case 11: return launch<1, 1, 64, true, true>(p, x, y, M, st);
    case 14: return launch<1, 4, 64, true, true>(p, x, y, M, st);
    case 21: return launch<2, 1, 32, true, true>(p, x, y, M, st);
    case 22: return launch<2, 2, 32, true, true>(p, x, y, M, st);
    case 504: return launch_splitk<4>(p, x, y, M, st);
    case 508: return launch_splitk<8>(p, x, y, M, st);
    case 516: return launch_splitk<16>(p, x, y, M, st);
    default: return launch<1, 2, 64, true, true>(p, x, y, M, st);
    }
}

}  // namespace sbn
