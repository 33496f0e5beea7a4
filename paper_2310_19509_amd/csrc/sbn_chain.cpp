// Layer chaining: a stack of packed sparse layers, optionally interleaved with
// dense depthwise 3x3 layers and a global average pool, run back to back on
// one stream with activations kept in rearranged channel order (Section 3.4).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstring>
#include <memory>
#include <new>

#include "sbn_internal.h"

using namespace sbn;

struct sbn_chain {
    struct Item {
        int item = 0;
        const sbn_packed* packed = nullptr;
        int channels = 0, stride = 1, act = 0, c_out = 0;
        float* d_w = nullptr;      // depthwise: [9][channels] in the arriving channel order
        float* d_b = nullptr;      // depthwise: [channels]
        uint32_t* d_taps = nullptr;  // depthwise with 3:9 patterns in groups of 16: kept taps (9 bits) per group
    };
    std::vector<Item> items;
    int device = 0;
    int c_in = 0;
    void* d_blob = nullptr;
    bool fuse_dw = true;           // run a depthwise item and the small 1x1 layer after it as one launch
    bool multi_layer = false;      // few pixels: consecutive depthwise / 1x1 items as phases of one launch (opt-in)
    unsigned* d_sync = nullptr;    // its grid barrier's words (in d_blob)
    int cus = 256;                 // compute units of the device
    ~sbn_chain()
    {
        if (d_blob) (void)hipFree(d_blob);
    }
};

namespace {

struct Shape {
    long long n;
    int h, w, c;
    size_t bytes() const { return (size_t)n * h * w * c * sizeof(float); }
};

Shape next_shape(const sbn_chain::Item& it, Shape s)
{
    switch (it.item) {
    case SBN_ITEM_SPARSE:
        if (it.packed->kind == SBN_CONV3X3) {
            s.h = (s.h - 1) / it.packed->stride + 1;
            s.w = (s.w - 1) / it.packed->stride + 1;
        }
        s.c = it.packed->c_out;
        break;
    case SBN_ITEM_DW3X3:
        s.h = (s.h - 1) / it.stride + 1;
        s.w = (s.w - 1) / it.stride + 1;
        break;
    case SBN_ITEM_AVGPOOL:
        s.h = s.w = 1;
        break;
    case SBN_ITEM_STEM3X3:
        s.h = (s.h - 1) / it.stride + 1;
        s.w = (s.w - 1) / it.stride + 1;
        s.c = it.c_out;
        break;
    }
    return s;
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

size_t max_intermediate(const sbn_chain* c, int n, int h, int w)
{
    Shape s{n, h, w, c->c_in};
    size_t mx = 0;
    for (size_t i = 0; i + 1 < c->items.size(); ++i) {
        s = next_shape(c->items[i], s);
        mx = std::max(mx, s.bytes());
    }
    return align256(mx);
}

}  // namespace

namespace sbn {

size_t chain_workspace_bytes(const sbn_chain* c, int n, int h, int w) { return c->items.size() > 1 ? 2 * max_intermediate(c, n, h, w) : 0; }
int chain_device(const sbn_chain* c) { return c->device; }

// Checks the arguments and queues every item of the chain on `stream`; the intermediate
// activations alternate between the two halves of `workspace`.  Allocates nothing.
int run_chain(const sbn_chain* c, const float* x, float* y, int n, int h, int w, void* workspace,
              size_t workspace_bytes, float* const* layer_outputs, void* stream, const char* who)
{
    if (!c) return fail(SBN_EINVAL, "%s: chain is NULL", who);
    if (n < 0 || h < 0 || w < 0) return fail(SBN_EINVAL, "%s: negative extent", who);
    if ((long long)n * h * w == 0) return SBN_OK;
    if (!x || !y) return fail(SBN_EINVAL, "%s: activation pointer is NULL", who);
    if (((uintptr_t)x | (uintptr_t)y) & 15u) return fail(SBN_EINVAL, "%s: x and y must be 16-byte aligned", who);
    const size_t half = max_intermediate(c, n, h, w);
    if (c->items.size() > 1) {
        if (!workspace || workspace_bytes < 2 * half)
            return fail(SBN_EINVAL, "%s: workspace of %zu bytes needed, %zu given", who, 2 * half, workspace_bytes);
        if ((uintptr_t)workspace % 256) return fail(SBN_EINVAL, "%s: workspace must be 256-byte aligned", who);
    }
    {
        // x, y and the workspace are three separate buffers: a launch reads one and writes another
        Shape so{n, h, w, c->c_in};
        for (const auto& it : c->items) so = next_shape(it, so);
        const Shape si{n, h, w, c->c_in};
        auto overlap = [](const void* a, size_t na, const void* b, size_t nb) {
            return (uintptr_t)a < (uintptr_t)b + nb && (uintptr_t)b < (uintptr_t)a + na;
        };
        if (overlap(x, si.bytes(), y, so.bytes())) return fail(SBN_EINVAL, "%s: x and y overlap", who);
        if (c->items.size() > 1 && (overlap(x, si.bytes(), workspace, 2 * half) || overlap(y, so.bytes(), workspace, 2 * half)))
            return fail(SBN_EINVAL, "%s: x or y overlaps the workspace", who);
        if (layer_outputs)
            for (size_t i = 0; i < c->items.size(); ++i)
                if ((uintptr_t)layer_outputs[i] & 15u)
                    return fail(SBN_EINVAL, "%s: layer_outputs[%zu] is not 16-byte aligned", who, i);
    }
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return fail(SBN_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (cur != c->device) return fail(SBN_EINVAL, "%s: current device is %d, chain lives on %d", who, cur, c->device);

    float* buf[2] = {(float*)workspace, (float*)((char*)workspace + half)};
    const float* src = x;
    Shape s{n, h, w, c->c_in};
    int which = 0;                   // half of the workspace the next launch writes
    // Items that qualify as phases of a multi-layer launch: a depthwise layer, or a 1x1 layer
    // whose input channels are a multiple of 4, with at most 1024 output pixels (every such launch
    // would sit at the launch-latency floor).
    auto tail_item = [&](const sbn_chain::Item& it, const Shape& in) {
        const Shape o = next_shape(it, in);
        if (o.n * o.h * o.w > 1024) return false;
        if (it.item == SBN_ITEM_DW3X3) return true;
        return it.item == SBN_ITEM_SPARSE && it.packed->kind == SBN_CONV1X1 && it.packed->c_in % 4 == 0 &&
               it.packed->c_in >= 128;
    };
    for (size_t i = 0; i < c->items.size(); ++i) {
        const sbn_chain::Item& it = c->items[i];
        if (c->multi_layer && tail_item(it, s)) {
            // the longest run of such items from here (each with its optional copy) that fits one launch
            size_t j = i;
            int phases = 0;
            Shape sj = s;
            while (j < c->items.size() && tail_item(c->items[j], sj)) {
                const int need = 1 + (layer_outputs && layer_outputs[j] ? 1 : 0);
                if (phases + need > kTailMaxPhases) break;
                phases += need;
                sj = next_shape(c->items[j], sj);
                ++j;
            }
            if (j - i >= 3) {
                TailArgs a;
                a.n_phases = 0;
                for (size_t k = i; k < j; ++k) {
                    const sbn_chain::Item& ik = c->items[k];
                    const Shape o = next_shape(ik, s);
                    float* dst = k + 1 == c->items.size() ? y : buf[which];
                    TailPhase& ph = a.ph[a.n_phases++];
                    ph = TailPhase{};
                    ph.src = src;
                    ph.dst = dst;
                    if (ik.item == SBN_ITEM_DW3X3) {
                        ph.kind = 0;
                        ph.n = (int)s.n, ph.h = s.h, ph.w = s.w, ph.c = s.c, ph.stride = ik.stride, ph.act = ik.act;
                        ph.oh = o.h, ph.ow = o.w;
                        ph.dw_w = ik.d_w, ph.dw_b = ik.d_b;
                    } else {
                        const sbn::DeviceLayout& L = ik.packed->dev;
                        ph.kind = 1;
                        ph.rec32 = L.d_records32, ph.woff32 = L.d_woff32, ph.wts = L.d_wts, ph.bias = L.d_bias;
                        ph.K = ik.packed->c_in, ph.N = ik.packed->c_out, ph.n_bundles = L.n_bundles, ph.n_chunks32 = L.n_chunks32;
                        ph.M = s.n * s.h * s.w;
                        ph.act = ik.packed->act;
                    }
                    if (layer_outputs && layer_outputs[k]) {
                        if (o.bytes() % 16) return fail(SBN_EINVAL, "output of item %zu is not a multiple of 16 bytes", k);
                        TailPhase& cp = a.ph[a.n_phases++];
                        cp = TailPhase{};
                        cp.kind = 2;
                        cp.src = dst, cp.dst = layer_outputs[k], cp.M = (long long)(o.bytes() / 16);
                    }
                    src = dst;
                    s = o;
                    which ^= 1;
                }
                if (int rc = launch_chain_tail(a, c->d_sync, c->cus, stream)) return rc;
                i = j - 1;
                continue;
            }
        }
        // A depthwise layer in front of a small 1x1 layer runs inside that layer's launch (its
        // output never exists in memory), unless the caller asked for a copy of it.
        if (c->fuse_dw && it.item == SBN_ITEM_DW3X3 && i + 1 < c->items.size() &&
            c->items[i + 1].item == SBN_ITEM_SPARSE && dwpw_fusable(c->items[i + 1].packed, it.channels, it.stride) &&
            !(layer_outputs && layer_outputs[i])) {
            const sbn_chain::Item& pw = c->items[i + 1];
            const bool last2 = i + 2 == c->items.size();
            float* dst2 = last2 ? y : buf[which];
            const Shape o2 = next_shape(pw, next_shape(it, s));
            int rc2 = launch_dwpw(pw.packed, src, dst2, it.d_w, it.d_b, it.d_taps, it.stride, it.act, (int)s.n, s.h, s.w, stream);
            if (rc2) return rc2;
            if (layer_outputs && layer_outputs[i + 1]) {
                if (o2.bytes() % 16) return fail(SBN_EINVAL, "output of item %zu is not a multiple of 16 bytes", i + 1);
                rc2 = launch_copy(dst2, layer_outputs[i + 1], o2.bytes(), stream);
                if (rc2) return rc2;
            }
            src = dst2;
            s = o2;
            which ^= 1;
            ++i;
            continue;
        }
        const bool last = i + 1 == c->items.size();
        float* dst = last ? y : buf[which];
        const Shape o = next_shape(it, s);
        int rc = SBN_OK;
        switch (it.item) {
        case SBN_ITEM_SPARSE:
            if (it.packed->kind == SBN_CONV1X1)
                rc = launch_conv1x1(it.packed, src, dst, s.n * s.h * s.w, stream);
            else
                rc = launch_conv3x3(it.packed, src, dst, (int)s.n, s.h, s.w, stream);
            break;
        case SBN_ITEM_DW3X3:
            rc = launch_dw3x3(src, dst, it.d_w, it.d_b, (int)s.n, s.h, s.w, s.c, it.stride, it.act, stream);
            break;
        case SBN_ITEM_AVGPOOL:
            rc = launch_avgpool(src, dst, (int)s.n, s.h * s.w, s.c, stream);
            break;
        case SBN_ITEM_STEM3X3:
            rc = launch_stem3x3(src, dst, it.d_w, it.d_b, (int)s.n, s.h, s.w, it.channels, it.c_out, it.stride, it.act,
                                stream);
            break;
        }
        if (rc) return rc;
        if (layer_outputs && layer_outputs[i]) {
            if (o.bytes() % 16) return fail(SBN_EINVAL, "output of item %zu is not a multiple of 16 bytes", i);
            rc = launch_copy(dst, layer_outputs[i], o.bytes(), stream);
            if (rc) return rc;
        }
        src = dst;
        s = o;
        which ^= 1;
    }
    return SBN_OK;
}

}  // namespace sbn

extern "C" {

static int chain_create_impl(const sbn_chain_item_t* items, int n_items, int device, sbn_chain_t** out)
{
    clear_error();
    if (!items || !out || n_items <= 0) return fail(SBN_EINVAL, "sbn_chain_create: NULL pointer or empty chain");
    *out = nullptr;
    if (device < 0) return fail(SBN_EINVAL, "sbn_chain_create: device must be >= 0");
    std::unique_ptr<sbn_chain> holder(new (std::nothrow) sbn_chain);     // freed on every early return
    sbn_chain* c = holder.get();
    if (!c) return fail(SBN_ENOMEM, "out of host memory");
    c->device = device;

    std::vector<int32_t> order;      // order[ch] = original channel carried at position ch; empty = identity
    int cur_c = -1;
    size_t dw_floats = 64;           // the first 64 words stay zero: the multi-layer launch's barrier state
    for (int i = 0; i < n_items; ++i) {
        const sbn_chain_item_t& s = items[i];
        sbn_chain::Item it;
        it.item = s.item;
        if (s.item == SBN_ITEM_SPARSE) {
            const sbn_packed* p = s.packed;
            if (!p) { return fail(SBN_EINVAL, "chain item %d: packed layer is NULL", i); }
            if (p->device != device) { return fail(SBN_EINVAL, "chain item %d lives on device %d, chain on %d", i, p->device, device); }
            if (cur_c >= 0 && p->c_in != cur_c) { return fail(SBN_ESHAPE, "chain item %d reads %d channels, previous item writes %d", i, p->c_in, cur_c); }
            for (int ch = 0; ch < p->c_in; ++ch) {
                const int32_t want = order.empty() ? ch : order[(size_t)ch];
                if (p->perm_in[(size_t)ch] != want) {
                    return fail(SBN_ESHAPE, "chain item %d: perm_in[%d] = %d but its input arrives with channel %d there", i, ch, p->perm_in[(size_t)ch], want);
                }
            }
            if (cur_c < 0) c->c_in = p->c_in;
            it.packed = p;
            cur_c = p->c_out;
            order = p->perm_out;
        } else if (s.item == SBN_ITEM_DW3X3) {
            if (s.channels <= 0 || s.channels % 4 || !s.dw_w || (s.stride != 1 && s.stride != 2) ||
                (s.act != SBN_ACT_NONE && s.act != SBN_ACT_RELU)) {
                return fail(SBN_EINVAL, "chain item %d: bad depthwise description (channels must be a positive multiple of 4, stride 1 or 2)", i);
            }
            if (cur_c >= 0 && s.channels != cur_c) { return fail(SBN_ESHAPE, "chain item %d has %d channels, previous item writes %d", i, s.channels, cur_c); }
            if (s.dw_pattern) {
                std::vector<int> st;
                if (int rc = dw_group_starts(s.channels, s.dw_go, st)) { return rc; }
                for (size_t g = 0; g + 1 < st.size(); ++g)
                    if (s.dw_pattern[g] > SBN_DW_PATTERN_DENSE) {
                            return fail(SBN_EINVAL, "chain item %d: pattern id %d of group %zu is not in 0..8", i, s.dw_pattern[g], g);
                    }
            }
            if (cur_c < 0) c->c_in = s.channels;
            it.channels = s.channels;
            it.stride = s.stride;
            it.act = s.act;
            cur_c = s.channels;
            dw_floats += (size_t)10 * s.channels;
            if (s.dw_pattern && s.dw_go == 16 && s.channels % 16 == 0) dw_floats += (size_t)(s.channels / 16 + 3) / 4 * 4;
        } else if (s.item == SBN_ITEM_STEM3X3) {
            if (i != 0) { return fail(SBN_ESHAPE, "the stem convolution must be the first item of a chain"); }
            if (s.channels < 1 || s.channels > 4 || s.c_out <= 0 || s.c_out % 4 || s.c_out > 64 || !s.dw_w ||
                (s.stride != 1 && s.stride != 2) || (s.act != SBN_ACT_NONE && s.act != SBN_ACT_RELU)) {
                return fail(SBN_EINVAL, "chain item %d: bad stem description (c_in 1..4, c_out multiple of 4 and <= 64, stride 1 or 2)", i);
            }
            c->c_in = s.channels;
            it.channels = s.channels;
            it.c_out = s.c_out;
            it.stride = s.stride;
            it.act = s.act;
            cur_c = s.c_out;
            dw_floats += (size_t)s.c_out * (9 * s.channels + 1);
        } else if (s.item == SBN_ITEM_AVGPOOL) {
            if (cur_c < 0) { return fail(SBN_ESHAPE, "a chain cannot start with the average pool"); }
            it.channels = cur_c;
        } else {
            return fail(SBN_EINVAL, "chain item %d: unknown item kind %d", i, s.item);
        }
        c->items.push_back(it);
    }

    {
        int prev = 0;
        (void)hipGetDevice(&prev);
        hipError_t e = hipSetDevice(device);
        float* blob = nullptr;
        if (e == hipSuccess) e = hipMalloc((void**)&blob, dw_floats * sizeof(float));
        if (e != hipSuccess) {
            (void)hipSetDevice(prev);
            return fail(e == hipErrorOutOfMemory ? SBN_ENOMEM : SBN_EHIP, "chain parameters: %s", hipGetErrorString(e));
        }
        c->d_blob = blob;                      // owned by the chain from here on
        std::vector<float> host(dw_floats, 0.0f);
        size_t off = 64;
        std::vector<int32_t> ord;
        c->d_sync = (unsigned*)blob;
        for (int i = 0; i < n_items; ++i) {
            sbn_chain::Item& it = c->items[(size_t)i];
            if (it.item == SBN_ITEM_SPARSE) ord = it.packed->perm_out;
            if (it.item == SBN_ITEM_STEM3X3) {
                // [tap][ci][c_out] and bias, original order (nothing precedes the stem)
                const int ci_n = it.channels, co_n = it.c_out;
                for (int o = 0; o < co_n; ++o) {
                    for (int t = 0; t < 9; ++t)
                        for (int ci = 0; ci < ci_n; ++ci)
                            host[off + ((size_t)t * ci_n + ci) * co_n + o] = items[i].dw_w[((size_t)o * 9 + t) * ci_n + ci];
                    host[off + (size_t)9 * ci_n * co_n + o] = items[i].dw_bias ? items[i].dw_bias[o] : 0.0f;
                }
                it.d_w = blob + off;
                it.d_b = blob + off + (size_t)9 * ci_n * co_n;
                off += (size_t)co_n * (9 * ci_n + 1);
                continue;
            }
            if (it.item != SBN_ITEM_DW3X3) continue;
            const int ch_n = it.channels;
            // 3:9 pattern groups are formed over the channels in the order the layer runs in.  The
            // weights are masked here, so every kernel is right whatever it does with the pattern:
            // the stand-alone depthwise kernel multiplies the zeros (it is bound by HBM, not by its
            // taps); the kernel that computes the depthwise layer inside a 1x1 launch skips the
            // removed taps of groups of 16, from the per-group tap masks built below.
            std::vector<uint8_t> pat_of_channel((size_t)ch_n, (uint8_t)SBN_DW_PATTERN_DENSE);
            if (items[i].dw_pattern) {
                std::vector<int> st;
                (void)dw_group_starts(ch_n, items[i].dw_go, st);
                for (size_t g = 0; g + 1 < st.size(); ++g)
                    for (int ch = st[g]; ch < st[g + 1]; ++ch) pat_of_channel[(size_t)ch] = items[i].dw_pattern[g];
            }
            for (int ch = 0; ch < ch_n; ++ch) {
                const int src = ord.empty() ? ch : ord[(size_t)ch];
                const int pid = pat_of_channel[(size_t)ch];
                for (int t = 0; t < 9; ++t) {
                    const bool gone = pid != SBN_DW_PATTERN_DENSE && t % 3 == ((pid >> (t / 3)) & 1 ? 2 : 0);
                    host[off + (size_t)t * ch_n + ch] = gone ? 0.0f : items[i].dw_w[(size_t)src * 9 + t];
                }
                host[off + (size_t)9 * ch_n + ch] = items[i].dw_bias ? items[i].dw_bias[src] : 0.0f;
            }
            it.d_w = blob + off;
            it.d_b = blob + off + (size_t)9 * ch_n;
            off += (size_t)10 * ch_n;
            if (items[i].dw_pattern && items[i].dw_go == 16 && ch_n % 16 == 0) {
                static_assert(sizeof(uint32_t) == sizeof(float), "tap masks live in the float blob");
                for (int g = 0; g < ch_n / 16; ++g) {
                    const int pid = items[i].dw_pattern[g];
                    uint32_t taps = 0x1FFu;
                    if (pid != SBN_DW_PATTERN_DENSE) {
                        taps = 0;
                        for (int r = 0; r < 3; ++r) taps |= ((pid >> r) & 1 ? 3u : 6u) << (3 * r);   // loses column 2 : loses column 0
                    }
                    std::memcpy(&host[off + (size_t)g], &taps, sizeof taps);
                }
                it.d_taps = (uint32_t*)(blob + off);
                off += (size_t)(ch_n / 16 + 3) / 4 * 4;
            }
        }
        e = hipMemcpy(blob, host.data(), dw_floats * sizeof(float), hipMemcpyHostToDevice);
        (void)hipSetDevice(prev);
        if (e != hipSuccess) return fail(SBN_EHIP, "chain parameters upload: %s", hipGetErrorString(e));
    }
    {
        // set-up for sbn_pointwise_chain_static: the built-in workspace's address on this device
        int prev = 0;
        (void)hipGetDevice(&prev);
        hipError_t e = hipSetDevice(device);
        if (e != hipSuccess) return fail(SBN_EHIP, "hipSetDevice(%d): %s", device, hipGetErrorString(e));
        const int rc = static_workspace_init(device);
        (void)hipSetDevice(prev);
        if (rc) return rc;
    }
    {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && cus > 0) c->cus = cus;
    }
    *out = holder.release();
    return SBN_OK;
}

int sbn_chain_create(const sbn_chain_item_t* items, int n_items, int device, sbn_chain_t** out)
{
    return guarded("sbn_chain_create", [&]() -> int { return chain_create_impl(items, n_items, device, out); });
}

int sbn_chain_workspace(const sbn_chain_t* c, int n, int h, int w, size_t* bytes_out)
{
    clear_error();
    if (!c || !bytes_out || n < 0 || h < 0 || w < 0) return fail(SBN_EINVAL, "sbn_chain_workspace: bad argument");
    *bytes_out = 2 * max_intermediate(c, n, h, w);
    return SBN_OK;
}

int sbn_chain_output_shape(const sbn_chain_t* c, int n, int h, int w, int* oh, int* ow, int* oc)
{
    clear_error();
    if (!c || n < 0 || h < 0 || w < 0) return fail(SBN_EINVAL, "sbn_chain_output_shape: bad argument");
    Shape s{n, h, w, c->c_in};
    for (const auto& it : c->items) s = next_shape(it, s);
    if (oh) *oh = s.h;
    if (ow) *ow = s.w;
    if (oc) *oc = s.c;
    return SBN_OK;
}

int sbn_pointwise_chain(const sbn_chain_t* c, const float* x, float* y, int n, int h, int w, void* workspace,
                        size_t workspace_bytes, float* const* layer_outputs, void* stream)
{
    clear_error();
    return run_chain(c, x, y, n, h, w, workspace, workspace_bytes, layer_outputs, stream, "sbn_pointwise_chain");
}

int sbn_chain_set_fusion(sbn_chain_t* c, int enable)
{
    clear_error();
    if (!c) return fail(SBN_EINVAL, "sbn_chain_set_fusion: chain is NULL");
    c->fuse_dw = enable != 0;
    return SBN_OK;
}

int sbn_chain_set_multi_layer(sbn_chain_t* c, int enable)
{
    clear_error();
    if (!c) return fail(SBN_EINVAL, "sbn_chain_set_multi_layer: chain is NULL");
    c->multi_layer = enable != 0;
    return SBN_OK;
}

int sbn_chain_check(const sbn_chain_t* c)
{
    clear_error();
    if (!c) return fail(SBN_EINVAL, "sbn_chain_check: chain is NULL");
    unsigned words[3] = {0, 0, 0};
    hipError_t e = hipMemcpy(words, c->d_sync, sizeof words, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(SBN_EHIP, "sbn_chain_check: %s", hipGetErrorString(e));
    if (words[2] != 0)
        return fail(SBN_EHIP, "a multi-layer launch of this chain gave up waiting at a grid barrier; its outputs are not valid");
    return SBN_OK;
}

void sbn_chain_free(sbn_chain_t* c)
{
    delete c;
}

}  // extern "C"
