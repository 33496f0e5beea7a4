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
    L.n_chunks32 = (p->c_in + 31) / 32;
    const size_t wstride = (size_t)taps * kBundleGroups * 16;        // floats per entry
    const size_t blk = (size_t)taps * gi * go;

    L.entries.clear();
    L.wts.clear();
    L.chunk_ptr32.assign((size_t)L.n_bundles * (L.n_chunks32 + 1), 0u);

    const int sub = go / 4;                                          // 4-filter groups per canonical row
    for (int b = 0; b < L.n_bundles; ++b) {
        // kb4 -> entry position (within this bundle), ascending by construction of std::map
        std::map<int, size_t> pos;
        const int g_lo = b * kBundleGroups, g_hi = std::min(n_groups4, g_lo + kBundleGroups);
        for (int g4 = g_lo; g4 < g_hi; ++g4) {
            const int row = g4 / sub;
            for (uint32_t e = p->row_ptr[(size_t)row]; e < p->row_ptr[(size_t)row + 1]; ++e)
                for (int c = 0; c < gi; ++c) pos[(p->kidx[e] + c) / 4] = 0;
        }
        const size_t first = L.entries.size();
        size_t n = 0;
        for (auto& kv : pos) {
            kv.second = first + n++;
            L.entries.push_back((uint32_t)kv.first << 8);
        }
        L.wts.resize((first + n) * wstride, 0.0f);
        for (int g4 = g_lo; g4 < g_hi; ++g4) {
            const int row = g4 / sub, s = g4 % sub, g = g4 - g_lo;
            for (uint32_t e = p->row_ptr[(size_t)row]; e < p->row_ptr[(size_t)row + 1]; ++e)
                for (int c = 0; c < gi; ++c) {
                    const int ch = p->kidx[e] + c;
                    const size_t en = pos[ch / 4];
                    L.entries[en] |= 1u << g;
                    for (int t = 0; t < taps; ++t)
                        for (int co = 0; co < 4; ++co)
                            L.wts[en * wstride + (((size_t)t * kBundleGroups + g) * 4 + (ch % 4)) * 4 + co] =
                                p->vals[e * blk + ((size_t)t * gi + c) * go + (size_t)s * 4 + co];
                }
        }
        // chunk pointers: first entry with channel >= 32*c
        uint32_t* cp = &L.chunk_ptr32[(size_t)b * (L.n_chunks32 + 1)];
        size_t en = first;
        for (int c = 0; c <= L.n_chunks32; ++c) {
            while (en < first + n && (int)(L.entries[en] >> 8) * 4 < 32 * c) ++en;
            cp[c] = (uint32_t)en;
        }
        cp[L.n_chunks32] = (uint32_t)(first + n);
    }
    L.n_entries = L.entries.size();
    L.bias_padded.assign((size_t)L.n_bundles * kBundleChannels, 0.0f);
    std::copy(p->bias.begin(), p->bias.end(), L.bias_padded.begin());
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

    // one allocation; +256 floats of slack after the weights so that the
    // kernels' one-entry-ahead prefetch never leaves the buffer
    const size_t b_entries = align256((L.entries.size() + 64) * sizeof(uint32_t));
    const size_t b_wts = align256((L.wts.size() + 9 * 64) * sizeof(float));
    const size_t b_cp = align256(L.chunk_ptr32.size() * sizeof(uint32_t));
    const size_t b_bias = align256(L.bias_padded.size() * sizeof(float));
    const size_t total = b_entries + b_wts + b_cp + b_bias;
    char* blob = nullptr;
    if ((e = hipMalloc((void**)&blob, total)) != hipSuccess) {
        (void)hipSetDevice(prev);
        return fail(e == hipErrorOutOfMemory ? SBN_ENOMEM : SBN_EHIP, "hipMalloc(%zu): %s", total, hipGetErrorString(e));
    }
    std::vector<char> host(total, 0);
    size_t off = 0;
    std::memcpy(host.data() + off, L.entries.data(), L.entries.size() * sizeof(uint32_t));
    L.d_entries = (uint32_t*)(blob + off);
    off += b_entries;
    std::memcpy(host.data() + off, L.wts.data(), L.wts.size() * sizeof(float));
    L.d_wts = (float*)(blob + off);
    off += b_wts;
    std::memcpy(host.data() + off, L.chunk_ptr32.data(), L.chunk_ptr32.size() * sizeof(uint32_t));
    L.d_chunk_ptr32 = (uint32_t*)(blob + off);
    off += b_cp;
    std::memcpy(host.data() + off, L.bias_padded.data(), L.bias_padded.size() * sizeof(float));
    L.d_bias = (float*)(blob + off);
    e = hipMemcpy(blob, host.data(), total, hipMemcpyHostToDevice);
    (void)hipSetDevice(prev);
    if (e != hipSuccess) {
        (void)hipFree(blob);
        L.d_entries = nullptr;
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
