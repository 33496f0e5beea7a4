// Device layout of a packed layer: regroups the canonical rows (Algorithm 1's
// per-output-group block lists) into bundles of four 4-filter groups whose
// kept 4-channel pieces are walked together, so that one staged activation
// read serves every group of the bundle that keeps the piece.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstring>
#include <map>

#include "sbn_internal.h"

namespace sbn {

void build_device_layout(sbn_packed* p)
{
    DeviceLayout& L = p->dev;
    const int taps = p->kh * p->kw, go = p->go, gi = p->gi;
    const int n_groups4 = p->c_out / 4;                              // go is 4 or 8
    L.n_bundles = (n_groups4 + kBundleGroups - 1) / kBundleGroups;
    L.n_chunks = (p->c_in + kChunk - 1) / kChunk;
    const size_t wstride = (size_t)taps * kBundleGroups * 16;        // floats per entry
    const size_t blk = (size_t)taps * gi * go;

    L.n_chunks32 = (p->c_in + 31) / 32;
    L.records.assign((size_t)L.n_bundles * L.n_chunks * kSlots, 0u);
    L.woff.assign((size_t)L.n_bundles * (L.n_chunks + 1), 0u);
    L.records32.assign((size_t)L.n_bundles * L.n_chunks32 * 8, 0u);
    L.woff32.assign((size_t)L.n_bundles * (L.n_chunks32 + 1), 0u);
    L.wts.clear();
    size_t n_entries = 0;

    const int sub = go / 4;                                          // 4-filter groups per canonical row
    for (int b = 0; b < L.n_bundles; ++b) {
        // kb4 -> (entry index, present mask); std::map keeps channels ascending
        std::map<int, std::pair<size_t, uint32_t>> pos;
        const int g_lo = b * kBundleGroups, g_hi = std::min(n_groups4, g_lo + kBundleGroups);
        for (int g4 = g_lo; g4 < g_hi; ++g4) {
            const int row = g4 / sub;
            for (uint32_t e = p->row_ptr[(size_t)row]; e < p->row_ptr[(size_t)row + 1]; ++e)
                for (int c = 0; c < gi; ++c) pos[(p->kidx[e] + c) / 4].second |= 1u << (g4 - g_lo);
        }
        const size_t first = n_entries;
        for (auto& kv : pos) kv.second.first = n_entries++;
        L.wts.resize(n_entries * wstride, 0.0f);
        for (int g4 = g_lo; g4 < g_hi; ++g4) {
            const int row = g4 / sub, s = g4 % sub, g = g4 - g_lo;
            for (uint32_t e = p->row_ptr[(size_t)row]; e < p->row_ptr[(size_t)row + 1]; ++e)
                for (int c = 0; c < gi; ++c) {
                    const int ch = p->kidx[e] + c;
                    const size_t en = pos[ch / 4].first;
                    for (int t = 0; t < taps; ++t)
                        for (int co = 0; co < 4; ++co) {
                            // 1x1: [g][co][ci] (16-byte loads per lane); 3x3: [tap][g][ci][co] (4-byte loads)
                            const size_t inner = taps == 1 ? (size_t)co * 4 + (ch % 4) : (size_t)(ch % 4) * 4 + co;
                            L.wts[en * wstride + ((size_t)t * kBundleGroups + g) * 16 + inner] =
                                p->vals[e * blk + ((size_t)t * gi + c) * go + (size_t)s * 4 + co];
                        }
                }
        }
        // records and chunk offsets
        uint32_t* wo = &L.woff[(size_t)b * (L.n_chunks + 1)];
        std::vector<int> fill((size_t)L.n_chunks, 0);
        for (int c = 0; c <= L.n_chunks; ++c) wo[c] = (uint32_t)n_entries;
        for (const auto& kv : pos) {
            const int c = kv.first / kSlots, q = fill[(size_t)c]++;
            L.records[((size_t)b * L.n_chunks + c) * kSlots + q] = ((uint32_t)(kv.first % kSlots) << 12) | kv.second.second;
            wo[c] = std::min(wo[c], (uint32_t)kv.second.first);
        }
        // empty chunks start where the next non-empty one does
        for (int c = L.n_chunks - 1; c >= 0; --c) wo[c] = std::min(wo[c], wo[c + 1]);
        // the same entries, one record of 8 descriptors per 32 channels
        uint32_t* wo32 = &L.woff32[(size_t)b * (L.n_chunks32 + 1)];
        std::vector<int> fill32((size_t)L.n_chunks32, 0);
        for (int c = 0; c <= L.n_chunks32; ++c) wo32[c] = (uint32_t)n_entries;
        for (const auto& kv : pos) {
            const int c = kv.first / 8, q = fill32[(size_t)c]++;
            L.records32[((size_t)b * L.n_chunks32 + c) * 8 + q] = ((uint32_t)(kv.first % 8) << 12) | kv.second.second;
            wo32[c] = std::min(wo32[c], (uint32_t)kv.second.first);
        }
        for (int c = L.n_chunks32 - 1; c >= 0; --c) wo32[c] = std::min(wo32[c], wo32[c + 1]);
        (void)first;
    }
    L.n_entries = n_entries;
    // every-piece tables for 1x1 layers of more than one chunk that keep most of their pieces
    L.desc_s.clear();
    L.wts_s.clear();
    const size_t n_pieces = (size_t)(p->c_in + 3) / 4;
    if (taps == 1 && p->c_in > kChunk && p->c_in % 4 == 0 &&
        (double)n_entries >= kStaticWalkMinFill * (double)((size_t)L.n_bundles * n_pieces)) {
        const size_t per_bundle = (size_t)L.n_chunks * kSlots;
        L.desc_s.assign((size_t)L.n_bundles * per_bundle, 0u);
        L.wts_s.assign((size_t)L.n_bundles * per_bundle * 64, 0.0f);
        for (int b = 0; b < L.n_bundles; ++b)
            for (int c = 0; c < L.n_chunks; ++c) {
                const uint32_t* r = &L.records[((size_t)b * L.n_chunks + c) * kSlots];
                const size_t e0 = L.woff[(size_t)b * (L.n_chunks + 1) + c];
                for (int q = 0; q < kSlots && r[q] != 0; ++q) {
                    const size_t piece = (size_t)c * kSlots + (r[q] >> 12);
                    L.desc_s[(size_t)b * per_bundle + piece] = r[q] & 0xFu;
                    std::copy(L.wts.begin() + (e0 + q) * 64, L.wts.begin() + (e0 + q + 1) * 64,
                              L.wts_s.begin() + ((size_t)b * per_bundle + piece) * 64);
                }
            }
    }
    L.bias_padded.assign((size_t)L.n_bundles * kBundleChannels, 0.0f);
    std::copy(p->bias.begin(), p->bias.end(), L.bias_padded.begin());
}

// What the kernels take for granted about the tables: checked once per packed layer, on the
// host, so that no kernel ever walks a malformed record.  Returns NULL or what is wrong.
static const char* check_tables(const std::vector<uint32_t>& rec, const std::vector<uint32_t>& wo, int n_bundles,
                                int n_chunks, int slots, size_t n_entries)
{
    if (rec.size() != (size_t)n_bundles * n_chunks * slots || wo.size() != (size_t)n_bundles * (n_chunks + 1))
        return "table sizes";
    size_t next = 0;                                   // entries are numbered bundle by bundle, chunk by chunk
    for (int b = 0; b < n_bundles; ++b)
        for (int c = 0; c < n_chunks; ++c) {
            const uint32_t* r = &rec[((size_t)b * n_chunks + c) * slots];
            int n = 0;
            while (n < slots && r[n] != 0) ++n;
            for (int q = n; q < slots; ++q)
                if (r[q] != 0) return "descriptor after the terminator";
            for (int q = 0; q < n; ++q) {
                const uint32_t kb4 = r[q] >> 12, m = r[q] & 0xFFFu;
                if (kb4 >= (uint32_t)slots || m == 0 || m > 15u) return "descriptor out of range";
                if (q && kb4 <= (r[q - 1] >> 12)) return "pieces of a record not ascending";
            }
            if (wo[(size_t)b * (n_chunks + 1) + c] != next) return "first-entry index";
            next += (size_t)n;
            if (wo[(size_t)b * (n_chunks + 1) + c + 1] != next) return "first-entry index of the next chunk";
        }
    return next == n_entries ? nullptr : "entry count";
}

const char* check_device_layout(const sbn_packed* p)
{
    const DeviceLayout& L = p->dev;
    if (L.n_bundles != (p->c_out / 4 + kBundleGroups - 1) / kBundleGroups || L.n_chunks != (p->c_in + kChunk - 1) / kChunk ||
        L.n_chunks32 != (p->c_in + 31) / 32)
        return "bundle or chunk count";
    if (const char* e = check_tables(L.records, L.woff, L.n_bundles, L.n_chunks, kSlots, L.n_entries)) return e;
    if (const char* e = check_tables(L.records32, L.woff32, L.n_bundles, L.n_chunks32, 8, L.n_entries)) return e;
    if (L.wts.size() != L.n_entries * (size_t)p->kh * p->kw * kBundleGroups * 16) return "weight array size";
    if (L.bias_padded.size() != (size_t)L.n_bundles * kBundleChannels) return "bias array size";
    if (!L.desc_s.empty()) {
        const size_t per_bundle = (size_t)L.n_chunks * kSlots;
        if (p->kh != 1 || L.desc_s.size() != (size_t)L.n_bundles * per_bundle || L.wts_s.size() != L.desc_s.size() * 64)
            return "every-piece table sizes";
        size_t present = 0;
        for (size_t i = 0; i < L.desc_s.size(); ++i) {
            if (L.desc_s[i] > 15u) return "every-piece mask out of range";
            if ((i % per_bundle) * 4 >= (size_t)p->c_in && L.desc_s[i] != 0) return "every-piece mask past the last channel";
            present += L.desc_s[i] != 0;
        }
        if (present != L.n_entries) return "every-piece entry count";
    } else if (!L.wts_s.empty()) {
        return "every-piece weights without masks";
    }
    return nullptr;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

int upload_device_layout(sbn_packed* p)
{
    DeviceLayout& L = p->dev;
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess) return fail(SBN_EHIP, "hipGetDeviceCount: %s", hipGetErrorString(e));
    if (p->device >= ndev) return fail(SBN_EINVAL, "device %d does not exist (%d visible)", p->device, ndev);
    int prev = 0;
    (void)hipGetDevice(&prev);
    if ((e = hipSetDevice(p->device)) != hipSuccess) return fail(SBN_EHIP, "hipSetDevice: %s", hipGetErrorString(e));
    int cus = 0;                           // the launchers size their grids by it
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, p->device) == hipSuccess && cus > 0) L.cus = cus;

    // One allocation.  The kernels fetch the weights of a whole record (up to
    // 16 entries) at once, so the weight array carries 16 entries of slack.
    const size_t wstride = (size_t)p->kh * p->kw * kBundleGroups * 16;
    const size_t b_rec = align256(L.records.size() * sizeof(uint32_t));
    const size_t b_woff = align256(L.woff.size() * sizeof(uint32_t));
    const size_t b_rec32 = align256(L.records32.size() * sizeof(uint32_t));
    const size_t b_woff32 = align256(L.woff32.size() * sizeof(uint32_t));
    const size_t b_wts = align256((L.wts.size() + kSlots * wstride) * sizeof(float));
    const size_t b_bias = align256(L.bias_padded.size() * sizeof(float));
    const size_t b_desc_s = align256(L.desc_s.size() * sizeof(uint32_t));
    const size_t b_wts_s = align256(L.wts_s.size() * sizeof(float));
    const size_t total = b_rec + b_woff + b_rec32 + b_woff32 + b_wts + b_bias + b_desc_s + b_wts_s;
    char* blob = nullptr;
    if ((e = hipMalloc((void**)&blob, total)) != hipSuccess) {
        (void)hipSetDevice(prev);
        return fail(e == hipErrorOutOfMemory ? SBN_ENOMEM : SBN_EHIP, "hipMalloc(%zu): %s", total, hipGetErrorString(e));
    }
    std::vector<char> host(total, 0);
    size_t off = 0;
    std::memcpy(host.data() + off, L.records.data(), L.records.size() * sizeof(uint32_t));
    L.d_records = (uint32_t*)(blob + off);
    off += b_rec;
    std::memcpy(host.data() + off, L.woff.data(), L.woff.size() * sizeof(uint32_t));
    L.d_woff = (uint32_t*)(blob + off);
    off += b_woff;
    std::memcpy(host.data() + off, L.records32.data(), L.records32.size() * sizeof(uint32_t));
    L.d_records32 = (uint32_t*)(blob + off);
    off += b_rec32;
    std::memcpy(host.data() + off, L.woff32.data(), L.woff32.size() * sizeof(uint32_t));
    L.d_woff32 = (uint32_t*)(blob + off);
    off += b_woff32;
    std::memcpy(host.data() + off, L.wts.data(), L.wts.size() * sizeof(float));
    L.d_wts = (float*)(blob + off);
    off += b_wts;
    std::memcpy(host.data() + off, L.bias_padded.data(), L.bias_padded.size() * sizeof(float));
    L.d_bias = (float*)(blob + off);
    off += b_bias;
    L.d_desc_s = nullptr;
    L.d_wts_s = nullptr;
    if (!L.desc_s.empty()) {
        std::memcpy(host.data() + off, L.desc_s.data(), L.desc_s.size() * sizeof(uint32_t));
        L.d_desc_s = (uint32_t*)(blob + off);
        off += b_desc_s;
        std::memcpy(host.data() + off, L.wts_s.data(), L.wts_s.size() * sizeof(float));
        L.d_wts_s = (float*)(blob + off);
    }
    e = hipMemcpy(blob, host.data(), total, hipMemcpyHostToDevice);
    (void)hipSetDevice(prev);
    if (e != hipSuccess) {
        (void)hipFree(blob);
        return fail(SBN_EHIP, "hipMemcpy of packed layer: %s", hipGetErrorString(e));
    }
    L.d_blob = blob;
    return SBN_OK;
}

void release_device_layout(sbn_packed* p)
{
    if (p->dev.d_blob) {
        (void)hipFree(p->dev.d_blob);
        p->dev.d_blob = nullptr;
    }
}

}  // namespace sbn
