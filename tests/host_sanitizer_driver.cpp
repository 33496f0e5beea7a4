// Driver for the AddressSanitizer / UndefinedBehaviorSanitizer build of libsbn's host side
// (tests/test_host_sanitizers.py compiles it together with the library's .cpp files).  It walks
// the offline calls -- pruning, rearrangement, packing, unpacking, export, the pattern
// selectors -- and their error paths on small seeded layers, with no device (device = -1), and
// checks the round trips.  The kernel launchers live in the .hip files and are stubbed here:
// nothing in this program may reach them.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <utility>
#include <vector>

#include "sbn_internal.h"

namespace sbn {
static int unreachable(const char* what)
{
    std::fprintf(stderr, "launcher %s reached in a host-only program\n", what);
    std::abort();
}
int launch_conv1x1(const sbn_packed*, const float*, float*, long long, void*) { return unreachable("conv1x1"); }
int launch_conv3x3(const sbn_packed*, const float*, float*, int, int, int, void*) { return unreachable("conv3x3"); }
int launch_dw3x3(const float*, float*, const float*, const float*, int, int, int, int, int, int, void*) { return unreachable("dw3x3"); }
int launch_stem3x3(const float*, float*, const float*, const float*, int, int, int, int, int, int, int, void*) { return unreachable("stem3x3"); }
int launch_avgpool(const float*, float*, int, int, int, void*) { return unreachable("avgpool"); }
int launch_copy(const void*, void*, size_t, void*) { return unreachable("copy"); }
int static_workspace_init(int) { return SBN_OK; }
int launch_chain_tail(const TailArgs&, unsigned*, int, void*) { return unreachable("chain tail"); }
bool dwpw_fusable(const sbn_packed*, int, int) { return false; }
int launch_dwpw(const sbn_packed*, const float*, float*, const float*, const float*, const uint32_t*, int, int, int, int, int, void*) { return unreachable("dwpw"); }
}  // namespace sbn

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static float rnd()
{
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((double)(g_state >> 40) / (double)(1ull << 24)) * 2.0f - 1.0f;
}

static void shuffle(std::vector<int32_t>& v)
{
    for (size_t i = v.size(); i > 1; --i) {
        const size_t j = (size_t)((rnd() * 0.5f + 0.5f) * (float)i) % i;
        std::swap(v[i - 1], v[j]);
    }
}

#define CHECK(cond)                                                                              \
    do {                                                                                         \
        if (!(cond)) {                                                                           \
            std::fprintf(stderr, "%s:%d: check failed: %s (last error: %s)\n", __FILE__, __LINE__, #cond, \
                         sbn_last_error());                                                      \
            return 1;                                                                            \
        }                                                                                        \
    } while (0)

static int one_layer(int kind, int c_in, int c_out, int go, int gi, int pct, bool perms)
{
    const int k = kind == SBN_CONV3X3 ? 3 : 1;
    const size_t nw = (size_t)c_out * k * k * c_in;
    std::vector<float> w(nw), bias((size_t)c_out);
    for (auto& v : w) v = rnd();
    for (auto& v : bias) v = rnd();
    w[0] = -0.0f;
    std::vector<int32_t> po((size_t)c_out), pi((size_t)c_in);
    for (int i = 0; i < c_out; ++i) po[(size_t)i] = i;
    for (int i = 0; i < c_in; ++i) pi[(size_t)i] = i;
    if (perms) {
        shuffle(po);
        shuffle(pi);
    }
    // weights in packed order for the pruning call
    std::vector<float> wp(nw);
    for (int r = 0; r < c_out; ++r)
        for (int t = 0; t < k * k; ++t)
            for (int c = 0; c < c_in; ++c)
                wp[((size_t)r * k * k + t) * c_in + c] = w[((size_t)po[(size_t)r] * k * k + t) * c_in + pi[(size_t)c]];
    std::vector<uint8_t> mask((size_t)(c_out / go) * (c_in / gi));
    CHECK(sbn_prune_magnitude(wp.data(), kind, c_in, c_out, go, gi, pct, mask.data()) == SBN_OK);
    double obj = 0;
    CHECK(sbn_retained_l1(wp.data(), kind, c_in, c_out, go, gi, pct, &obj) == SBN_OK && obj >= 0);

    sbn_layer_desc_t d;
    std::memset(&d, 0, sizeof d);
    d.kind = kind, d.c_in = c_in, d.c_out = c_out, d.go = go, d.gi = gi, d.stride = 1, d.pad = k / 2;
    d.w = w.data(), d.mask = mask.data(), d.bias = bias.data(), d.perm_out = po.data(), d.perm_in = pi.data();
    d.act = SBN_ACT_RELU;
    sbn_packed_t* p = nullptr;
    CHECK(sbn_pack(&d, -1, &p) == SBN_OK && p);
    size_t nnz = 0, nnz2 = 0, macs = 0;
    CHECK(sbn_export(p, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, &nnz) == SBN_OK);
    std::vector<uint32_t> row_ptr((size_t)c_out / go + 1);
    std::vector<uint16_t> kidx(nnz + 1);
    std::vector<float> vals(nnz * k * k * gi * go + 1), b2((size_t)c_out);
    std::vector<int32_t> po2((size_t)c_out), pi2((size_t)c_in);
    CHECK(sbn_export(p, row_ptr.data(), kidx.data(), vals.data(), po2.data(), pi2.data(), b2.data(), &nnz2) == SBN_OK);
    CHECK(nnz2 == nnz && row_ptr.back() == nnz && po2 == po && pi2 == pi);
    CHECK(sbn_packed_work(p, &nnz2, &macs) == SBN_OK && nnz2 == nnz && macs == nnz * go * gi * k * k);
    std::vector<float> back(nw);
    std::vector<uint8_t> mask2(mask.size());
    CHECK(sbn_unpack(p, back.data(), mask2.data()) == SBN_OK && mask2 == mask);
    for (int r = 0; r < c_out; ++r)          // unpack(pack(W)) = W (.) M bit for bit, pruned blocks +0.0
        for (int t = 0; t < k * k; ++t)
            for (int c = 0; c < c_in; ++c) {
                const size_t i = ((size_t)po[(size_t)r] * k * k + t) * c_in + pi[(size_t)c];
                const bool kept = mask[(size_t)(r / go) * (c_in / gi) + c / gi] != 0;
                uint32_t a, e = 0;
                std::memcpy(&a, &back[i], 4);
                if (kept) std::memcpy(&e, &w[i], 4);
                CHECK(a == e);
            }
    int kind2 = 0, dev = 0;
    CHECK(sbn_packed_info(p, &kind2, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, &dev) == SBN_OK && kind2 == kind && dev == -1);
    // run calls on a layer without a device copy are refused before anything is launched
    float dummy[4];
    CHECK((kind == SBN_CONV1X1 ? sbn_conv1x1_sparse(p, dummy, dummy + 1, 1, 1, 1, nullptr)
                               : sbn_conv3x3_sparse(p, dummy, dummy + 1, 1, 1, 1, nullptr)) == SBN_ENODEV);
    sbn_chain_item_t it;
    std::memset(&it, 0, sizeof it);
    it.item = SBN_ITEM_SPARSE, it.packed = p;
    sbn_chain_t* ch = nullptr;
    CHECK(sbn_chain_create(&it, 1, 0, &ch) != SBN_OK && ch == nullptr);     // layer lives on no device
    // implied mask (mask = NULL) and no permutations
    d.mask = nullptr, d.perm_out = nullptr, d.perm_in = nullptr, d.bias = nullptr;
    sbn_packed_t* q = nullptr;
    CHECK(sbn_pack(&d, -1, &q) == SBN_OK && q);
    sbn_free(q);
    sbn_free(p);
    return 0;
}

static int error_paths()
{
    std::vector<float> w(8 * 8, 1.0f);
    std::vector<uint8_t> mask(4);
    CHECK(sbn_prune_magnitude(nullptr, SBN_CONV1X1, 8, 8, 4, 4, 50, mask.data()) == SBN_EINVAL);
    CHECK(sbn_prune_magnitude(w.data(), SBN_CONV1X1, 8, 8, 4, 4, 101, mask.data()) == SBN_EINVAL);
    CHECK(sbn_prune_magnitude(w.data(), SBN_CONV1X1, 6, 8, 4, 4, 50, mask.data()) == SBN_ESHAPE);
    CHECK(sbn_prune_magnitude(w.data(), SBN_CONV1X1, 8, 8, 3, 4, 50, mask.data()) != SBN_OK);
    sbn_layer_desc_t d;
    std::memset(&d, 0, sizeof d);
    d.kind = SBN_CONV1X1, d.c_in = 8, d.c_out = 8, d.go = 4, d.gi = 4, d.stride = 1, d.w = w.data();
    sbn_packed_t* p = nullptr;
    int32_t bad[8] = {0, 1, 2, 3, 4, 5, 6, 6};
    d.perm_out = bad;
    CHECK(sbn_pack(&d, -1, &p) == SBN_EPERM && p == nullptr);
    d.perm_out = nullptr;
    CHECK(sbn_pack(nullptr, -1, &p) == SBN_EINVAL);
    CHECK(sbn_pack(&d, -1, nullptr) == SBN_EINVAL);
    CHECK(sbn_unpack(nullptr, w.data(), nullptr) == SBN_EINVAL);
    CHECK(sbn_force_kernel_form(SBN_CONV1X1, 13) == SBN_EINVAL && sbn_force_kernel_form(SBN_CONV3X3, 32) == SBN_OK &&
          sbn_force_kernel_form(SBN_CONV3X3, 0) == SBN_OK);
    CHECK(std::strlen(sbn_last_error()) == 0);
    CHECK(sbn_chain_set_fusion(nullptr, 1) == SBN_EINVAL);
    sbn_free(nullptr);
    sbn_chain_free(nullptr);
    return 0;
}

static int patterns()
{
    const int c = 28;
    std::vector<float> w((size_t)c * 9), out((size_t)c * 9);
    for (auto& v : w) v = rnd();
    int n_groups = 0;
    std::vector<int> start((size_t)c / 4 + 2);
    CHECK(sbn_dw_pattern_groups(c, 16, &n_groups, start.data()) == SBN_OK && n_groups == 3);
    std::vector<uint8_t> ids((size_t)n_groups), keep((size_t)n_groups, 0);
    keep[1] = 1;
    CHECK(sbn_dw_pattern_select(w.data(), c, 16, keep.data(), ids.data()) == SBN_OK && ids[1] == SBN_DW_PATTERN_DENSE);
    CHECK(sbn_dw_pattern_apply(w.data(), c, 16, ids.data(), out.data()) == SBN_OK);
    CHECK(sbn_dw_pattern_apply(w.data(), c, 16, ids.data(), w.data()) == SBN_OK);      // in place
    ids[0] = 9;
    CHECK(sbn_dw_pattern_apply(w.data(), c, 16, ids.data(), out.data()) == SBN_EINVAL);
    CHECK(sbn_dw_pattern_groups(6, 16, &n_groups, nullptr) == SBN_ESHAPE);

    const int co = 8, ci = 5;
    std::vector<float> w3((size_t)co * 9 * ci), o3(w3.size());
    for (auto& v : w3) v = rnd();
    for (int share : {1, 2, 4}) {
        std::vector<uint8_t> pid((size_t)(co / share) * ci);
        CHECK(sbn_conv3x3_pattern_select(w3.data(), co, ci, share, pid.data()) == SBN_OK);
        CHECK(sbn_conv3x3_pattern_apply(w3.data(), co, ci, share, pid.data(), o3.data()) == SBN_OK);
        size_t kept = 0;
        for (float v : o3) kept += v != 0.0f;
        CHECK(kept == (size_t)co * ci * 4);
        pid[0] = 57;
        CHECK(sbn_conv3x3_pattern_apply(w3.data(), co, ci, share, pid.data(), o3.data()) == SBN_EINVAL);
    }
    uint32_t taps = 0;
    CHECK(sbn_conv3x3_pattern_taps(0, &taps) == SBN_OK && taps == 0x17u);
    CHECK(sbn_conv3x3_pattern_taps(56, &taps) == SBN_OK && taps == 0x1FFu);
    CHECK(sbn_conv3x3_pattern_taps(-1, &taps) == SBN_EINVAL);
    CHECK(sbn_conv3x3_pattern_select(w3.data(), 6, ci, 4, nullptr) == SBN_EINVAL);
    return 0;
}

static int rearrangement()
{
    // three chained 1x1 layers 16 -> 8 -> 24 -> 16; the middle one small enough for the exhaustive search
    const int cin[3] = {16, 8, 24}, cout[3] = {8, 24, 16};
    std::vector<std::vector<float>> w(3);
    sbn_layer_desc_t d[3];
    std::memset(d, 0, sizeof d);
    std::vector<std::vector<int32_t>> perm(3);
    int32_t* out[3];
    for (int l = 0; l < 3; ++l) {
        w[(size_t)l].resize((size_t)cin[l] * cout[l]);
        for (auto& v : w[(size_t)l]) v = rnd();
        d[l].kind = SBN_CONV1X1, d[l].c_in = cin[l], d[l].c_out = cout[l], d[l].go = 4, d[l].gi = 4, d[l].stride = 1;
        d[l].w = w[(size_t)l].data();
        perm[(size_t)l].assign((size_t)cout[l], -1);
        out[l] = perm[(size_t)l].data();
    }
    const int parent[3] = {-1, 0, 1}, keep[3] = {0, 0, 1};
    CHECK(sbn_rearrange(d, 3, parent, keep, 50, 42, 200, out) == SBN_OK);
    for (int l = 0; l < 3; ++l) {
        std::vector<int> seen((size_t)cout[l], 0);
        for (int32_t v : perm[(size_t)l]) {
            CHECK(v >= 0 && v < cout[l]);
            ++seen[(size_t)v];
        }
        for (int s : seen) CHECK(s == 1);
    }
    for (int i = 0; i < cout[2]; ++i) CHECK(perm[2][(size_t)i] == i);          // kept output order
    CHECK(sbn_order_groups(d, 3, parent, keep, 50, out) == SBN_OK);
    for (int l = 0; l < 3; ++l) {
        std::vector<int> seen((size_t)cout[l], 0);
        for (int32_t v : perm[(size_t)l]) {
            CHECK(v >= 0 && v < cout[l]);
            ++seen[(size_t)v];
        }
        for (int s : seen) CHECK(s == 1);
    }
    for (int i = 0; i < cout[2]; ++i) CHECK(perm[2][(size_t)i] == i);
    const int bad_parent[3] = {-1, 2, 1};
    CHECK(sbn_rearrange(d, 3, bad_parent, keep, 50, 42, 10, out) != SBN_OK);   // parents must come first
    CHECK(sbn_rearrange(d, 3, parent, keep, 50, 42, 10, nullptr) == SBN_EINVAL);
    return 0;
}

int main()
{
    const int cases[][7] = {
        // kind, c_in, c_out, go, gi, pct, perms
        {SBN_CONV1X1, 64, 32, 4, 4, 50, 1}, {SBN_CONV1X1, 72, 40, 8, 4, 30, 1}, {SBN_CONV1X1, 9, 8, 4, 1, 70, 0},
        {SBN_CONV1X1, 96, 16, 4, 8, 90, 1}, {SBN_CONV1X1, 16, 16, 4, 2, 100, 0}, {SBN_CONV1X1, 200, 24, 4, 4, 0, 1},
        {SBN_CONV3X3, 32, 16, 4, 4, 70, 1}, {SBN_CONV3X3, 24, 8, 8, 4, 50, 0}, {SBN_CONV3X3, 40, 24, 4, 1, 60, 1},
    };
    for (const auto& c : cases)
        if (one_layer(c[0], c[1], c[2], c[3], c[4], c[5], c[6] != 0)) return 1;
    if (error_paths() || patterns() || rearrangement()) return 1;
    std::puts("host sanitizer driver: ok");
    return 0;
}
