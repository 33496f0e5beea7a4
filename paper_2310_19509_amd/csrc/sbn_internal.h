// Internal declarations shared by the host runtime and the kernel launchers of
// libsbn.  Nothing here is part of the public ABI (see include/sbn.h).
#pragma once

#include <cstdarg>
#include <cstddef>
#include <cstdint>
#include <exception>
#include <new>
#include <string>
#include <vector>

#include "sbn.h"

namespace sbn {

// ---- error reporting -------------------------------------------------------
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();
// Runs the body of an extern "C" entry point: no C++ exception may cross the C ABI.
template <class F>
int guarded(const char* who, F&& body)
{
    try {
        return body();
    } catch (const std::bad_alloc&) {
        return fail(SBN_ENOMEM, "%s: out of host memory", who);
    } catch (const std::exception& e) {
        return fail(SBN_EINVAL, "%s: %s", who, e.what());
    } catch (...) {
        return fail(SBN_EINVAL, "%s: unexpected failure", who);
    }
}
int dw_group_starts(int c, int go, std::vector<int>& start);   // pattern groups of a depthwise layer (+ c at the end)
int forced_kernel_form(int kind);                              // sbn_force_kernel_form's value, 0 = automatic

// ---- device-side layout ----------------------------------------------------
// The canonical rows (one per output group of `go` filters) are regrouped for
// the kernels into BUNDLES of kBundleGroups consecutive groups of 4 filters.
// A bundle walks the union of its groups' kept 4-channel pieces in ascending
// channel order; an ENTRY is one such piece.  Per bundle and per chunk of 64
// input channels there is one fixed-size RECORD of 16 descriptors (64 bytes):
//     records[bundle][chunk][q] = (kb4_in_chunk << 12) | present_mask  q < n   (so that
//                                 descriptor >> 8 is the piece's byte offset in a staged row)
//                               = 0                                    q >= n
// kb4_in_chunk = (first channel of the piece - 64*chunk) / 4; bit g of
// present_mask says that group g of the bundle keeps the piece; n <= 16 is
// the number of entries of the bundle inside the chunk.  woff[bundle][chunk]
// is the global index of the chunk's first entry (woff[bundle][n_chunks] its
// end).  The weights of an entry are stored for all groups of the bundle
// (zeros where absent), transposed so that a 16-byte load per lane yields the
// four input channels of one output channel:
//     1x1:  wts[entry][g][co][ci]                 64 floats per entry
//     3x3:  wts[entry][tap][g][ci][co]            9*64 floats per entry (4-byte loads per lane)
constexpr int kBundleGroups = 4;                       // groups of 4 filters per bundle
constexpr int kBundleChannels = 4 * kBundleGroups;     // 16 output channels per bundle
constexpr int kChunk = 64;                             // input channels per record
constexpr int kSlots = kChunk / 4;                     // descriptors per record
constexpr double kStaticWalkMinFill = 0.60;            // share of (bundle, piece) pairs kept, from which the every-piece tables are built

struct DeviceLayout {
    int n_bundles = 0;
    int n_chunks = 0;                     // ceil(c_in / 64)
    size_t n_entries = 0;
    int n_chunks32 = 0;                   // ceil(c_in / 32)
    int cus = 256;                        // compute units of the device the layer lives on (set at upload)
    // host staging
    std::vector<uint32_t> records;        // [n_bundles][n_chunks][16]
    std::vector<uint32_t> woff;           // [n_bundles][n_chunks + 1]
    std::vector<uint32_t> records32;      // [n_bundles][n_chunks32][8]: the same entries per 32 channels,
    std::vector<uint32_t> woff32;         // [n_bundles][n_chunks32 + 1]   kb4_in_chunk < 8
    std::vector<float> wts;
    std::vector<float> bias_padded;       // [n_bundles * 16], zeros when no bias
    // 1x1 layers that keep most of their pieces (see kStaticWalkMinFill) also get the tables with an
    // entry for EVERY piece, present or not: entry q of chunk c is piece q, so the kernel reads its
    // activations at an offset known at compile time.  desc_s[bundle][n_chunks * 16]: the present
    // mask of the piece (0 = no group keeps it); wts_s[bundle][n_chunks * 16][64]: as wts, zeros
    // for absent pieces.  Empty when the layer does not qualify.
    std::vector<uint32_t> desc_s;
    std::vector<float> wts_s;
    // device copies (one allocation)
    void* d_blob = nullptr;
    uint32_t* d_records = nullptr;
    uint32_t* d_woff = nullptr;
    uint32_t* d_records32 = nullptr;
    uint32_t* d_woff32 = nullptr;
    float* d_wts = nullptr;
    float* d_bias = nullptr;
    uint32_t* d_desc_s = nullptr;         // NULL when the layer has no every-piece tables
    float* d_wts_s = nullptr;
};

}  // namespace sbn

struct sbn_packed {
    int kind = 0, c_in = 0, c_out = 0, go = 0, gi = 0, stride = 1, pad = 0, act = 0;
    int kh = 1, kw = 1;
    int device = -1;
    bool has_bias = false;
    // canonical format
    std::vector<uint32_t> row_ptr;    // [c_out/go + 1]
    std::vector<uint16_t> kidx;       // [nnz]
    std::vector<float> vals;          // [nnz][kh][kw][gi][go]
    std::vector<int32_t> perm_out;    // [c_out]
    std::vector<int32_t> perm_in;     // [c_in]
    std::vector<float> bias;          // [c_out] packed order (zeros if !has_bias)
    sbn::DeviceLayout dev;
};

namespace sbn {

// Builds p->dev host arrays from the canonical arrays (no HIP calls).
void build_device_layout(sbn_packed* p);
// Invariants of p->dev that the kernels rely on; NULL if they hold, else what is violated.
const char* check_device_layout(const sbn_packed* p);
// Uploads p->dev to p->device.  Returns SBN_OK or an error code.
int upload_device_layout(sbn_packed* p);
void release_device_layout(sbn_packed* p);

// Kernel launchers (defined in the .hip files).
int launch_conv1x1(const sbn_packed* p, const float* x, float* y, long long m, void* stream);
int launch_conv3x3(const sbn_packed* p, const float* x, float* y, int n, int h, int w, void* stream);
int launch_dw3x3(const float* x, float* y, const float* w_dev, const float* b_dev, int n, int h, int w,
                 int c, int stride, int act, void* stream);
int launch_stem3x3(const float* x, float* y, const float* w_dev, const float* b_dev, int n, int h, int w, int c_in,
                   int c_out, int stride, int act, void* stream);
// depthwise 3x3 fused into the 1x1 layer that consumes it (small layers only: see dwpw_fusable)
bool dwpw_fusable(const sbn_packed* p, int channels, int stride);
// dw_taps: NULL, or per 16 channels (in running order) the 9-bit mask of the taps the group keeps
int launch_dwpw(const sbn_packed* p, const float* x, float* y, const float* dw_w, const float* dw_b,
                const uint32_t* dw_taps, int dw_stride, int dw_act, int n, int h, int w, void* stream);
int launch_avgpool(const float* x, float* y, int n, int hw, int c, void* stream);
int launch_copy(const void* src, void* dst, size_t bytes, void* stream);

// Looks up this device's copy of the built-in chain workspace (sbn_chain_static.hip); the
// device must be current.
int static_workspace_init(int device);

// Chain internals shared by the two run entry points (sbn_chain.cpp).
size_t chain_workspace_bytes(const sbn_chain* c, int n, int h, int w);   // 0 for a one-item chain
int chain_device(const sbn_chain* c);
int run_chain(const sbn_chain* c, const float* x, float* y, int n, int h, int w, void* workspace,
              size_t workspace_bytes, float* const* layer_outputs, void* stream, const char* who);

// Several consecutive chain items in ONE launch, for inputs of few pixels where every launch
// sits at the launch-latency floor: a grid of persistent workgroups runs the items as phases
// with a grid-wide barrier between them (sbn_conv1x1.hip).  The phases travel by value as kernel
// arguments.
struct TailPhase {
    int kind;                      // 0: depthwise 3x3, 1: group-sparse 1x1 (few-pixel form), 2: copy
    int n, h, w, c, stride, act, oh, ow;         // depthwise: input extents and channels
    const float* src;
    float* dst;
    const float* dw_w;             // depthwise [9][c], [c]
    const float* dw_b;
    const uint32_t* rec32;         // 1x1: the packed layer's tables per 32 channels
    const uint32_t* woff32;
    const float* wts;
    const float* bias;
    int K, N, n_bundles, n_chunks32;
    long long M;                   // 1x1: pixels; copy: 16-byte words
};
constexpr int kTailMaxPhases = 24;
struct TailArgs {
    int n_phases;
    TailPhase ph[kTailMaxPhases];
};
// sync: three device words {arrivals, generation, status}, zero when allocated; status != 0 after
// a barrier wait ran into its spin limit (the launch then ends early and later ones do nothing).
int launch_chain_tail(const TailArgs& a, unsigned* sync, int cus, void* stream);

// Block l1 norms in the exact summation order the pruning rule is defined with.
void block_norms(const float* w, int c_out, int kh, int kw, int c_in, int go, int gi, std::vector<double>& out);
bool is_permutation(const int32_t* p, int n);

}  // namespace sbn
