/*
 * sbn.h -- C ABI of libsbn: convolution with fine-grained group-sparse
 * weights on AMD MI355X (gfx950).
 *
 * The method (Section 3.1): a layer's weights W [oc][kh][kw][ic] are replaced
 * by W~ = W (.) M, where the 0/1 mask M is constant over blocks of `go` output
 * channels x `gi` input channels (all kh*kw taps of a block share its bit;
 * Eq. 2).  The sparse kernels skip removed blocks and are otherwise exact
 * (Algorithm 1).  Before pruning, filters and channels may be rearranged so
 * that a parent's filter order is its children's channel order (Section 3.4).
 *
 * Conventions for every call
 *   - Return value: 0 on success, a negative SBN_E* code otherwise.  The text
 *     of the last failure on the calling thread is kept for sbn_last_error().
 *   - "host" pointers are ordinary CPU memory, borrowed for the call only.
 *     "device" pointers are HIP device memory on the device the packed layer
 *     was created for; they stay owned by the caller.
 *   - Activations are NHWC fp32, contiguous: x[n][h][w][c].  Weights are OHWI
 *     fp32: w[oc][kh][kw][ic] (Section 3.1; Algorithm 1 "Data").  Device
 *     activation pointers (x, y, layer_outputs entries) must be 16-byte aligned
 *     (the kernels use 16-byte loads and stores): SBN_EINVAL otherwise.
 *   - No C++ exception leaves the library: running out of host memory inside
 *     any call is reported as SBN_ENOMEM.
 *   - Run calls (sbn_conv*_sparse, sbn_pointwise_chain) launch kernels on the
 *     stream given (a hipStream_t passed as void*; NULL = the null stream),
 *     never allocate, never synchronise and return right after the launch.
 *   - sbn_packed_t / sbn_chain_t are opaque, created by the library and
 *     released by sbn_free / sbn_chain_free.  A chain borrows its packed
 *     layers: free the chain first.
 *   - Removed blocks are skipped, not multiplied by zero: with finite activations the result is
 *     that of the dense convolution with W~ (up to fp32 summation order); a NaN or infinity in a
 *     channel that only removed blocks read may or may not reach the output.
 *   - Single-layer run calls work in PERMUTED channel space: x carries its
 *     channels in perm_in order and y comes out in perm_out order.  That is
 *     what makes the rearrangement free at run time (Section 3.4).
 */
#ifndef SBN_H
#define SBN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* error codes */
#define SBN_OK      0
#define SBN_EINVAL (-1)  /* NULL pointer or value out of range            */
#define SBN_ESHAPE (-2)  /* channels not divisible by go/gi, bad chain    */
#define SBN_EPERM  (-3)  /* an index array is not a permutation           */
#define SBN_ENOMEM (-4)  /* host or device allocation failed              */
#define SBN_EHIP   (-5)  /* a HIP call failed; text in sbn_last_error()   */
#define SBN_ENODEV (-6)  /* packed layer has no device copy (device = -1) */

/* layer kinds */
#define SBN_CONV1X1 1
#define SBN_CONV3X3 3

/* activations applied after bias */
#define SBN_ACT_NONE 0
#define SBN_ACT_RELU 1

typedef struct sbn_packed sbn_packed_t;
typedef struct sbn_chain  sbn_chain_t;

/*
 * One layer to pack.  Blocks are go output channels x gi input channels
 * (Section 3.2: 4x4 for Conv1x1 and for whole 3x3 kernels of Conv3x3).
 * Supported: go in {4, 8}; gi in {1, 2, 4, 8}; c_out % go == 0; c_in % gi == 0.
 */
typedef struct {
    int kind;                 /* SBN_CONV1X1 or SBN_CONV3X3                                     */
    int c_in, c_out;          /* ic, oc                                                          */
    int go, gi;               /* block = go filters x gi channels                                */
    int stride, pad;          /* 3x3: stride in {1,2}, pad must be 1.  1x1: must be 1 and 0      */
    const float*   w;         /* host, OHWI, ORIGINAL channel order                              */
    const uint8_t* mask;      /* host [c_out/go][c_in/gi] in PERMUTED block coordinates, 1=kept;
                                 NULL: a block is kept iff one of its weights has nonzero magnitude */
    const float*   bias;      /* host [c_out], original order; NULL = no bias                    */
    const int32_t* perm_out;  /* packed filter r is original filter perm_out[r]; NULL = identity */
    const int32_t* perm_in;   /* packed channel c is original channel perm_in[c]; NULL = identity*/
    int act;                  /* SBN_ACT_NONE or SBN_ACT_RELU                                    */
} sbn_layer_desc_t;

/* Text of the last error on this thread ("" if none).  Never NULL. */
const char* sbn_last_error(void);

/* ------------------------------------------------------------------ offline, host side */

/*
 * Block importance and magnitude pruning (Section 3.2: l1 norm per block, the
 * (oc/go)(ic/gi)*rho least important blocks of the layer are removed; Eq. 2).
 * w_permuted: host OHWI weights already in packed (permuted) order.
 * kh = kw = 1 for SBN_CONV1X1, 3 for SBN_CONV3X3.
 * Removed count = floor(n_blocks * sparsity_percent / 100); norms are summed
 * in fp64 in (filter, ky, kx, channel) order; ties remove the lower
 * (row-major) block index first.  mask_out: host uint8 [c_out/go][c_in/gi].
 * Weights holding NaN or infinity have no order of importance: SBN_EINVAL
 * (the same holds for sbn_retained_l1).
 */
int sbn_prune_magnitude(const float* w_permuted, int kind, int c_in, int c_out, int go, int gi,
                        int sparsity_percent, uint8_t* mask_out);

/*
 * Retained importance of a layer after pruning: the sum of the block norms
 * that survive sbn_prune_magnitude at this sparsity -- the quantity the
 * rearrangement of Section 3.4 tries to raise.  Written to *objective_out.
 */
int sbn_retained_l1(const float* w_permuted, int kind, int c_in, int c_out, int go, int gi,
                    int sparsity_percent, double* objective_out);

/*
 * 3:9 pattern group pruning of a depthwise 3x3 layer (Section 3.2, DwConv3x3;
 * Algorithm 2's PatternInfo).  Every kernel loses three weights, one per row,
 * each from the first or the third column: pattern id = 3 bits, bit r set
 * means row r loses its THIRD column, clear its FIRST.  `go` consecutive
 * channels (4, 8 or 16; the paper uses 16) share a pattern; channels left over
 * form groups of 8 and then 4 (Section 3.3).  SBN_DW_PATTERN_DENSE marks a
 * group that keeps all nine weights (the "full-1" pattern).
 *
 * sbn_dw_pattern_groups: number of groups for c channels (c % 4 == 0) and,
 * if group_start is not NULL, the first channel of every group plus c at the
 * end (int [*n_groups_out + 1], caller-allocated; c/4 + 1 entries always fit).
 *
 * sbn_dw_pattern_select: for w (host [c][3][3], in the channel order the layer
 * runs in) writes to pattern_out (uint8 [n_groups]) the pattern that keeps
 * the largest l1-norm over each group's kernels (fp64 sums in channel, row,
 * column order; ties -> the lowest id).  keep_dense (uint8 [n_groups] or NULL):
 * nonzero leaves that group dense.
 *
 * sbn_dw_pattern_apply: w_out = W (.) M as a select (removed weights +0.0,
 * kept ones bit for bit); w_out may equal w.
 */
#define SBN_DW_PATTERN_DENSE 8
int sbn_dw_pattern_groups(int c, int go, int* n_groups_out, int* group_start);
int sbn_dw_pattern_select(const float* w, int c, int go, const uint8_t* keep_dense, uint8_t* pattern_out);
int sbn_dw_pattern_apply(const float* w, int c, int go, const uint8_t* pattern, float* w_out);

/*
 * Pattern pruning inside the kept kernels of a 3x3 layer (Section 3.2, Conv3x3;
 * Section 3.3's closing remarks).  Every 3x3 kernel (one filter x one input
 * channel) keeps 4 of its 9 weights, the centre among them: C(8,3) = 56
 * patterns.  `share` adjacent filters (4, 2 or 1, in the order the layer
 * runs in) use the same pattern for a given input channel.  Whole kernels are
 * removed by the block mask of sbn_prune_magnitude / sbn_pack as before; the
 * usual order is select -> apply -> prune -> pack.
 *
 * Taps are numbered ky*3 + kx; the centre is tap 4.  Pattern id p in 0..55 is
 * the p-th 3-element subset {a < b < c} of the other taps (0,1,2,3,5,6,7,8) in
 * lexicographic order of (a, b, c); the kernel keeps a, b, c and the centre.
 * SBN_K3_PATTERN_DENSE keeps all nine.
 *
 * sbn_conv3x3_pattern_taps: bit t of *tap_mask_out set = tap t is kept.
 *
 * sbn_conv3x3_pattern_select: w host OHWI [c_out][3][3][c_in], c_out a multiple
 * of share.  Writes pattern_out (uint8 [c_out/share][c_in]): for filter group f
 * and channel c the pattern with the largest kept l1-norm.  Per tap the
 * magnitudes of the group's filters are summed in filter order (fp64); a
 * pattern's score is the sum of its three taps in ascending tap order; ties ->
 * the lowest id.
 *
 * sbn_conv3x3_pattern_apply: w_out = W (.) M as a select (removed weights +0.0,
 * kept ones bit for bit); w_out may equal w.  Ids above SBN_K3_PATTERN_DENSE
 * are SBN_EINVAL.
 *
 * The device kernel runs pattern-pruned layers through the same path as any
 * other packed 3x3 layer (zeros inside kept blocks are multiplied): see the
 * design notes for why the matrix pipe cannot skip single taps here.
 */
#define SBN_K3_PATTERNS 56
#define SBN_K3_PATTERN_DENSE 56
int sbn_conv3x3_pattern_taps(int pattern, uint32_t* tap_mask_out);
int sbn_conv3x3_pattern_select(const float* w, int c_out, int c_in, int share, uint8_t* pattern_out);
int sbn_conv3x3_pattern_apply(const float* w, int c_out, int c_in, int share, const uint8_t* pattern,
                              float* w_out);

/*
 * Whole-network rearrangement for a chain of layers (Section 3.4).
 * layers[l].w / c_in / c_out / go / gi / kind are read (mask, bias, perms are
 * ignored).  parent[l] is the index of the layer whose output feeds layer l,
 * or -1 if layer l reads the network input; a layer has at most one parent
 * and layers must be listed parents first.  For every layer l the call
 * searches a filter permutation perm[l] (int32 [c_out], caller-allocated,
 * perm_per_layer_out[l]) that raises the retained block importance at
 * `sparsity_percent`, with the layer's channels already ordered by its
 * parent's result.  The channel permutation of layer l is perm[parent[l]]
 * (identity for parent -1).  Layers with keep_output_order[l] != 0 get the
 * identity (use it for the network's last layer unless its consumer absorbs
 * the order).  keep_output_order may be NULL (= all zero).
 *
 * The search is deterministic, seeded and bounded: swaps of two filters of
 * different groups, at most max_iters candidates per tensor; a swap is kept only
 * if the objective strictly increases; after c_out rejected candidates in a row
 * the search restarts from the best order so far with two random swaps applied;
 * the best order seen is returned, so the result is never worse than the
 * identity.  Layers with at most 20 000 canonical groupings (12 filters in
 * groups of 4, 16 in groups of 8) are searched exhaustively instead.  Results
 * are in canonical form: filters ascending inside each group, groups ordered by
 * first filter.
 */
int sbn_rearrange(const sbn_layer_desc_t* layers, int n_layers, const int* parent,
                  const int* keep_output_order, int sparsity_percent, uint64_t seed, int max_iters,
                  int32_t* const* perm_per_layer_out);

/*
 * The same for any graph (Section 3.4: the rearrangement is propagated through
 * the whole network).  Channel orders belong to TENSORS: layer l reads tensor
 * in_tensor[l] and writes tensor out_tensor[l] (numbers in 0..n_tensors-1).
 * Several layers may write the same tensor -- the branches of a residual sum,
 * or a skip connection, which makes a block's output share the order of its
 * input -- and then share one filter order, found by maximising the SUM of
 * their retained importances.  Tensors are decided in increasing number; a
 * layer's channels count in the order of its input tensor if that tensor has a
 * lower number than the one being decided, in original order otherwise.  A
 * tensor no layer writes (a network input) and every tensor with
 * tensor_fixed[t] != 0 (network outputs; tensor_fixed may be NULL) keep the
 * identity.  perm_per_tensor_out[t]: int32 [channels of tensor t], caller-
 * allocated; pack layer l with perm_in = order of in_tensor[l], perm_out = order
 * of out_tensor[l].  All layers that write a tensor must agree on c_out and go.
 */
int sbn_rearrange_graph(const sbn_layer_desc_t* layers, int n_layers, const int* in_tensor, const int* out_tensor,
                        int n_tensors, const int* tensor_fixed, int sparsity_percent, uint64_t seed, int max_iters,
                        int32_t* const* perm_per_tensor_out);

/*
 * Order of the filter groups (Section 3.4: which filters share a group is what
 * the rearrangement decides; the order of the groups makes no difference to
 * the method, so it is chosen for the machine).  The device kernels walk 16
 * consecutive filters together over the union of the 4-channel input pieces
 * that any of them keeps at `sparsity_percent` (magnitude pruning, as
 * sbn_prune_magnitude); this call reorders whole groups so that groups that
 * keep the same pieces sit in the same 16.  Greedy and deterministic; the
 * grouping, hence every mask, the retained importance and the network's
 * function, is unchanged.  Whole units of max(go of the writers, gi of the
 * readers) filters are moved so that the readers' blocks stay whole.
 * The perms are read and rewritten in place: pass the result of sbn_rearrange /
 * sbn_rearrange_graph (or identities); arguments as in those calls.
 * SBN_EPERM if an order passed in is not a permutation.
 */
int sbn_order_groups(const sbn_layer_desc_t* layers, int n_layers, const int* parent,
                     const int* keep_output_order, int sparsity_percent, int32_t* const* perm_per_layer_inout);
int sbn_order_groups_graph(const sbn_layer_desc_t* layers, int n_layers, const int* in_tensor, const int* out_tensor,
                           int n_tensors, const int* tensor_fixed, int sparsity_percent,
                           int32_t* const* perm_per_tensor_inout);

/*
 * Pack one layer into the group-sparse format (Algorithm 1's "sparse info":
 * per output group the first input channel of every kept block) and, when
 * device >= 0, build the device copy on that HIP device.  device = -1 packs on
 * the host only (sbn_unpack / sbn_export work, run calls return SBN_ENODEV).
 * Steps: validate -> permute filters/channels/bias -> mask (given or implied)
 * -> gather kept blocks row by row.  Pruned weights are dropped; kept blocks
 * are copied bit for bit (signed zeros and denormals included).
 * A 3x3 layer packed for a device (device >= 0) needs c_in % 4 == 0 (its kernel
 * stages four channels at a time): SBN_ESHAPE otherwise; host-only packing
 * (device = -1) has no such limit.
 */
int sbn_pack(const sbn_layer_desc_t* desc, int device, sbn_packed_t** out);

/*
 * Exact inverse of sbn_pack: writes the masked weights W~ in ORIGINAL channel
 * order (host OHWI [c_out][kh][kw][c_in]; removed blocks are +0.0) and, if
 * mask_out != NULL, the mask in permuted block coordinates.
 */
int sbn_unpack(const sbn_packed_t* p, float* w_out, uint8_t* mask_out);

/*
 * Canonical arrays of the packed format.  Rows are output groups of `go`
 * filters in packed order; a row's kept blocks are listed by ascending
 * channel.  Any output pointer may be NULL (skipped).  *nnz_out receives the
 * number of kept blocks; call once with NULL arrays to size them.
 *   row_ptr  uint32 [c_out/go + 1]
 *   kidx     uint16 [nnz]                   first input channel of the block
 *   vals     float  [nnz][kh][kw][gi][go]
 *   perm_out int32  [c_out],  perm_in int32 [c_in],  bias float [c_out] (packed order)
 */
int sbn_export(const sbn_packed_t* p, uint32_t* row_ptr, uint16_t* kidx, float* vals,
               int32_t* perm_out, int32_t* perm_in, float* bias, size_t* nnz_out);

/* Shape of a packed layer; any output pointer may be NULL. */
int sbn_packed_info(const sbn_packed_t* p, int* kind, int* c_in, int* c_out, int* go, int* gi,
                    int* stride, int* act, int* device);

void sbn_free(sbn_packed_t* p);

/* ------------------------------------------------------------------ on the GPU */

/*
 * Group-sparse 1x1 convolution (Algorithm 1): for every pixel p and output
 * group j,  y[p, j*go:(j+1)*go] = act(bias + sum over kept blocks kb of row j
 * of x[p, kb:kb+gi] . Wblk[j, kb]).  x: device [n][h][w][c_in], y: device
 * [n][h][w][c_out], both in packed channel order; x and y must not overlap.
 * n*h*w may be 0 (nothing is launched).  fp32 multiply-add, fp32 accumulate.
 */
int sbn_conv1x1_sparse(const sbn_packed_t* p, const float* x, float* y,
                       int n, int h, int w, void* stream);

/*
 * Kernel-level group-sparse 3x3 convolution (Section 3.2, Conv3x3
 * connectivity pruning with gi x go kernels per group): as above with every
 * kept block carrying its 9 taps; zero padding 1, stride from the descriptor.
 * x: device [n][h][w][c_in]; y: device [n][oh][ow][c_out], oh = (h-1)/stride+1.
 */
int sbn_conv3x3_sparse(const sbn_packed_t* p, const float* x, float* y,
                       int n, int h, int w, void* stream);

/*
 * Testing and benchmarking hook: both run calls pick, per launch, one of
 * several forms of their kernel from the shape (tile size, channels staged at
 * a time, input channels split over waves).  This call forces one form for all
 * later launches of that kind in the process (0 = back to automatic), so that
 * every form can be checked on every shape; results never depend on the form
 * beyond summation order.  kind: SBN_CONV1X1 (forms 11, 12, 14, 21, 22: pixels
 * per lane and accumulator sets; 504, 508, 516: 4, 8, 16 waves splitting the
 * input channels; 112, 121: forms 12 / 21 with the last pixel tiles run as
 * four-wave channel-splitting workgroups inside the same launch; 1012, 1021,
 * 1112, 1121: forms 12, 21, 112, 121 on the every-piece tables of layers that
 * have them (sbn_packed_layout), the plain form otherwise -- forms below 1000
 * never use those tables, the automatic choice always does; 1: the automatic
 * choice without those tables) or SBN_CONV3X3 (1, 2, 3: one pixel per lane, two pixels per
 * lane, entry-ahead fetch; 32: entry-ahead with the input channels split over
 * two halves of an eight-wave workgroup).  Layers whose shape leaves no choice (c_in <= 64,
 * c_in not a multiple of 4, stride 2) ignore it.  Unknown values: SBN_EINVAL.
 * Not synchronised with launches in flight on other threads.
 */
int sbn_force_kernel_form(int kind, int form);

/*
 * A stack of layers run back to back on one stream (Section 3.4: activations
 * stay in rearranged channel order between layers; Section 3.5 engine).
 */
#define SBN_ITEM_SPARSE  1   /* a packed 1x1 or 3x3 layer                                 */
#define SBN_ITEM_DW3X3   2   /* depthwise 3x3, pad 1, + bias + act; dense or 3:9 pattern  */
#define SBN_ITEM_AVGPOOL 3   /* global average over h*w -> 1x1 spatial                    */
#define SBN_ITEM_STEM3X3 4   /* dense 3x3 conv of a few input channels (network stem),
                                pad 1, + bias + act; only as the first item of a chain    */

typedef struct {
    int item;                   /* SBN_ITEM_*                                              */
    const sbn_packed_t* packed; /* SBN_ITEM_SPARSE: the layer (borrowed)                   */
    int channels;               /* SBN_ITEM_DW3X3: channel count; SBN_ITEM_STEM3X3: c_in (1..4) */
    int stride;                 /* SBN_ITEM_DW3X3 / SBN_ITEM_STEM3X3: 1 or 2                */
    int act;                    /* SBN_ITEM_DW3X3 / SBN_ITEM_STEM3X3: SBN_ACT_*             */
    const float* dw_w;          /* SBN_ITEM_DW3X3: host [channels][3][3], ORIGINAL order;
                                   SBN_ITEM_STEM3X3: host OHWI [c_out][3][3][c_in]          */
    const float* dw_bias;       /* host [channels] (DW3X3) / [c_out] (STEM3X3) or NULL      */
    int c_out;                  /* SBN_ITEM_STEM3X3: output channels, multiple of 4, <= 64  */
    const uint8_t* dw_pattern;  /* SBN_ITEM_DW3X3: NULL (dense) or one 3:9 pattern id per
                                   group of the layer's channels IN THE ORDER IT RUNS IN (the
                                   rearranged order); the weights are masked accordingly.
                                   With groups of 16 the per-group kept taps also go to the
                                   device: where the layer runs inside the 1x1 launch that
                                   consumes it, a wave works on one group and loads and
                                   multiplies only the six kept taps (Algorithm 2's dispatch
                                   on the pattern); the stand-alone depthwise kernel is bound
                                   by memory traffic and multiplies the stored zeros         */
    int dw_go;                  /* SBN_ITEM_DW3X3 with dw_pattern: group size (4, 8 or 16)   */
} sbn_chain_item_t;

/*
 * Build a chain on `device`.  Checks that channel counts chain and that each
 * sparse layer's perm_in equals the order its input arrives in (the perm_out
 * of the nearest sparse layer before it; depthwise and pooling items keep the
 * order and have their per-channel parameters permuted to match); the first
 * item must expect the identity order.  SBN_ESHAPE otherwise.
 */
int sbn_chain_create(const sbn_chain_item_t* items, int n_items, int device, sbn_chain_t** out);

/* Bytes of device workspace the chain needs for an input of n x h x w. */
int sbn_chain_workspace(const sbn_chain_t* c, int n, int h, int w, size_t* bytes_out);

/* Output shape of the chain for an input of n x h x w (any pointer may be NULL). */
int sbn_chain_output_shape(const sbn_chain_t* c, int n, int h, int w, int* oh, int* ow, int* oc);

/*
 * Run the chain: x device [n][h][w][c_in of first item], y device
 * [n][oh][ow][oc] in the last item's channel order.  workspace: device
 * memory of at least sbn_chain_workspace bytes, 256-byte aligned, used for
 * the intermediate activations (ping-pong).  x, y and the workspace must be
 * three non-overlapping buffers (SBN_EINVAL otherwise).  If layer_outputs !=
 * NULL it is a host array of EXACTLY n_items device pointers (one per item of
 * the chain; the call reads all of them); a non-NULL entry i receives a copy
 * of item i's output (for per-layer checks), queued on the same stream.
 */
int sbn_pointwise_chain(const sbn_chain_t* c, const float* x, float* y, int n, int h, int w,
                        void* workspace, size_t workspace_bytes, float* const* layer_outputs,
                        void* stream);

/*
 * The same run for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * intermediate activations live in a fixed array of SBN_STATIC_WORKSPACE_BYTES
 * inside the library's code object (one copy per GPU, held until the process
 * ends) instead of a caller's workspace; x, y and layer_outputs are as above.
 * The call allocates nothing and frees nothing.  An input whose intermediates
 * (sbn_chain_workspace) exceed SBN_STATIC_WORKSPACE_BYTES is refused with
 * SBN_EINVAL before anything is launched.  All calls on one GPU share that
 * GPU's array: two calls whose kernels may overlap in time (different streams,
 * different threads) race -- order them on one stream or with events.  The
 * array needs no clearing between calls (every item overwrites what it later
 * reads).  The array's address is looked up when a chain is created on the
 * device, so a run call under stream capture queries nothing.
 */
#define SBN_STATIC_WORKSPACE_BYTES (32u << 20)
int sbn_pointwise_chain_static(const sbn_chain_t* c, const float* x, float* y, int n, int h, int w,
                               float* const* layer_outputs, void* stream);

/*
 * By default a depthwise item directly in front of a 1x1 layer with at most
 * 128 input and 128 output channels (input channels a multiple of 32) runs
 * inside that layer's launch: the depthwise result is computed tile by tile in
 * on-chip memory and never written out (those layers are bound by memory
 * traffic).  Results agree with the separate launches up to fp32 summation
 * order inside the depthwise layer.  enable = 0 switches this off for the
 * chain (every item its own launch); a copy of the depthwise output requested
 * through layer_outputs switches it off for that pair.
 */
int sbn_chain_set_fusion(sbn_chain_t* c, int enable);

/*
 * Inputs of few pixels (batch 1 of the deep layers: the paper's own setting is
 * single-image latency, Section 4.3).  Off by default, enable = 1 switches it
 * on for the chain: runs of at least three consecutive depthwise / 1x1 items
 * with at most 1024 output pixels each (1x1 layers: input channels a multiple
 * of 4 and at least 128) are queued as ONE launch: a grid of resident
 * workgroups walks the items as phases with a grid-wide barrier in between.
 * On MI355X this is SLOWER than one launch per item (whole MobileNet-v1 on one
 * image: 0.36 ms against 0.15 ms): a grid-wide barrier has to write one XCD's
 * L2 back and invalidate the others', about 14 us, where the boundary between
 * two launches costs about 6 us.  The path is kept for callers that must bound
 * the number of launches.  Results agree with the separate launches up to fp32
 * summation order.  The barrier's state lives in the chain: two runs of the
 * SAME chain must not overlap in time when they use this path (one stream, or
 * events between them).  Waits at the barrier are bounded; a launch that runs
 * into the bound ends early, later multi-layer launches of the chain return at
 * once (their outputs are not written), and sbn_chain_check reports it: call it
 * after synchronising when this path is on.
 * sbn_chain_check: synchronous (copies three words back): SBN_OK, or SBN_EHIP
 * if a multi-layer launch of the chain ever gave up.
 */
int sbn_chain_set_multi_layer(sbn_chain_t* c, int enable);
int sbn_chain_check(const sbn_chain_t* c);

void sbn_chain_free(sbn_chain_t* c);

/* ------------------------------------------------------------------ measurement helpers */

/*
 * Number of kept blocks and the multiply-adds per output pixel they imply
 * (go*gi*kh*kw per kept block): the "nonzero FLOPs" of the throughput metric
 * are 2 * macs_per_pixel * output pixels.
 */
int sbn_packed_work(const sbn_packed_t* p, size_t* nnz_blocks_out, size_t* macs_per_pixel_out);

/*
 * What the kernels walk: the number of entries (a 4-channel input piece kept by
 * at least one group of a bundle of 16 filters), the bytes of all tables and
 * weights built for the device, and whether the layer also has the tables with
 * an entry for every piece (1x1 layers of more than 64 input channels that keep
 * at least 60 % of their (bundle, piece) pairs: the kernel then reads an entry's
 * activations at a fixed offset).  Any output pointer may be NULL.
 */
int sbn_packed_layout(const sbn_packed_t* p, size_t* entries_out, size_t* table_bytes_out, int* every_piece_out);

/*
 * Plain device-to-device copy kernel of `bytes` bytes (multiple of 16), used
 * to calibrate hardware counters and to measure the attainable HBM rate.
 */
int sbn_copy_bytes(const void* src, void* dst, size_t bytes, void* stream);

/*
 * What this machine's units deliver, measured with stand-alone loops (no part of
 * the method): set beside the datasheet roofs when a kernel's share of its
 * roofline is reported.  `sink` is a device float that no launch ever writes
 * (it keeps the loops alive).  All three launch on `stream` and return at once.
 *   sbn_roof_mfma: four waves per SIMD issue `iters` x 16 independent
 *     v_mfma_f32_4x4x1 (the instruction of the sparse kernels, broadcast operand);
 *     *flops_out = floating-point operations of the launch.
 *   sbn_roof_lds:  the same waves read 16 bytes per lane from LDS, `iters` x 16
 *     times, in the 1x1 kernel's row layout; *bytes_out = bytes read.
 *   sbn_roof_read: reads `bytes` (a multiple of 16) of device memory once.
 */
int sbn_roof_mfma(int iters, float* sink, void* stream, double* flops_out);
int sbn_roof_lds(int iters, float* sink, void* stream, double* bytes_out);
int sbn_roof_read(const void* src, size_t bytes, float* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SBN_H */
