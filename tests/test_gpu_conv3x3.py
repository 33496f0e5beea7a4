"""Parity of the HIP kernel-level group-sparse 3x3 convolution with the CPU oracle (gpu)."""
import numpy as np
import pytest
import torch

import paper_2310_19509_amd as S
from oracle import reference as R
import workloads as W
from helpers import assert_within_bound

pytestmark = pytest.mark.gpu


def run_layer(x, w, go, gi, stride=1, mask=None, bias=None, perm_out=None, perm_in=None, act=S.SBN_ACT_NONE,
              pct=None):
    wp = R.permute_weights(w, perm_out, perm_in)
    if pct is not None:
        mask = S.sbn_prune_magnitude(wp, S.SBN_CONV3X3, go, gi, pct)
        assert np.array_equal(mask, R.prune_mask(wp, go, gi, pct))
    p = S.sbn_pack(S.SBN_CONV3X3, w, go, gi, mask=mask, bias=bias, perm_out=perm_out, perm_in=perm_in,
                   stride=stride, act=act)
    n, h, ww, _ = x.shape
    oh, ow = (h - 1) // stride + 1, (ww - 1) // stride + 1
    xd = torch.from_numpy(x).cuda()
    yd = torch.full((n, oh, ow, w.shape[0]), float("nan"), device="cuda", dtype=torch.float32)
    S.sbn_conv3x3_sparse(p, xd, yd, n, h, ww)
    torch.cuda.synchronize()
    y_ref, bound = R.sparse_conv_reference(x, w, mask, go, gi, bias=bias, perm_out=perm_out, perm_in=perm_in,
                                           stride=stride, pad=1, act=act)
    return yd.cpu().numpy(), y_ref, bound


CASES = [
    # n, h, w, K, N, go, gi, stride, pct, bias, relu, perms
    (1, 1, 1, 8, 8, 4, 4, 1, 50, True, False, False),        # a single pixel: only the centre tap sees data
    (2, 4, 4, 8, 8, 4, 4, 1, 0, True, False, False),         # all kept, borders everywhere
    (2, 4, 4, 8, 8, 4, 4, 2, 0, True, True, False),          # stride 2
    (1, 7, 7, 64, 64, 4, 4, 1, 70, True, True, True),        # 7x7: one ragged tile
    (1, 14, 14, 32, 48, 4, 4, 1, 70, True, False, False),    # 2x2 tiles, ragged
    (1, 9, 17, 40, 24, 4, 4, 1, 50, True, True, True),       # odd sizes, K=40 (ragged sub-chunk), N=24
    (1, 9, 17, 40, 24, 8, 4, 2, 50, True, True, False),      # stride 2, go=8
    (2, 16, 16, 96, 64, 4, 4, 1, 70, False, False, False),   # three sub-chunks
    (1, 10, 10, 64, 32, 4, 1, 1, 50, True, False, False),    # gi=1
    (1, 10, 10, 64, 32, 4, 8, 1, 30, True, False, True),     # gi=8
    (1, 12, 12, 128, 128, 4, 4, 2, 70, True, True, False),   # stride 2, several chunks
    (1, 5, 5, 16, 16, 4, 4, 1, 100, True, True, False),      # everything pruned
    (1, 8, 8, 32, 16, 4, 4, 1, 90, True, False, False),      # empty rows
    (3, 19, 33, 72, 80, 4, 4, 1, 60, True, True, True),      # three 16-wide tiles with a ragged one, odd height
    (2, 8, 16, 36, 20, 4, 4, 1, 40, True, False, False),     # exactly one 16-wide tile; K, N not multiples of 16
]


@pytest.fixture
def kernel_variant():
    """Forces one form of the stride-1 kernel for the launches of the test:
    1 = one pixel per lane, row-ahead; 2 = two pixels per lane; 3 = one pixel per lane, entry-ahead;
    32 = entry-ahead with the input channels split over two slices of four waves."""
    yield lambda v: S.sbn_force_kernel_form(S.SBN_CONV3X3, v)
    S.sbn_force_kernel_form(S.SBN_CONV3X3, 0)


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 32])
@pytest.mark.parametrize("n,h,w,K,N,go,gi,stride,pct,use_bias,relu,perms", CASES)
def test_shapes(n, h, w, K, N, go, gi, stride, pct, use_bias, relu, perms, variant, kernel_variant):
    if variant and stride != 1:
        pytest.skip("stride 2 has one form")
    kernel_variant(variant)
    seed = 8000 + 3 * K + N + go + gi + pct + stride
    wt = W.he_weights(seed, N, 3, 3, K)
    b = W.small_bias(seed + 1, N) * 20 if use_bias else None
    x = W.uniform_activation(seed + 2, (n, h, w, K))
    po = W.random_permutation(seed + 3, N) if perms else None
    pi = W.random_permutation(seed + 4, K) if perms else None
    y, ref, bound = run_layer(x, wt, go, gi, stride=stride, bias=b, perm_out=po, perm_in=pi,
                              act=S.SBN_ACT_RELU if relu else S.SBN_ACT_NONE, pct=pct)
    assert_within_bound(y, ref, bound, f"3x3 case {n,h,w,K,N,go,gi,stride,pct}")


def test_taps_are_not_transposed():
    """A kernel that is 1 at (ky=0, kx=2) only: y(oy, ox) = x(oy-1, ox+1)."""
    K = N = 8
    w = np.zeros((N, 3, 3, K), dtype=np.float32)
    for o in range(N):
        w[o, 0, 2, o] = 1.0
    x = W.uniform_activation(8101, (1, 6, 9, K))
    y, ref, bound = run_layer(x, w, 4, 4)
    expect = np.zeros_like(x)
    expect[0, 1:, :-1, :] = x[0, :-1, 1:, :]
    assert np.array_equal(ref, expect)
    assert np.array_equal(y, expect)


@pytest.mark.parametrize("share,stride", [(4, 1), (2, 1), (1, 2)])
def test_pattern_pruned_kernels(share, stride):
    """Section 3.2, Conv3x3: 4 of 9 weights kept inside every kernel (pattern shared by `share`
    adjacent filters of the order the layer runs in), then whole kernels removed by block magnitude."""
    K, N = 72, 48
    w = W.normal_weights(8200 + share, (N, 3, 3, K), (2.0 / (9 * K)) ** 0.5)
    bias = W.normal_weights(8210 + share, (N,), 0.01)
    x = W.uniform_activation(8220 + share, (2, 13, 18, K))
    perm_out = np.random.default_rng(8230 + share).permutation(N).astype(np.int32)
    wp = R.permute_weights(w, perm_out, None)
    ids = S.sbn_conv3x3_pattern_select(wp, share)
    assert ids.tolist() == R.conv3x3_pattern_select(wp, share).tolist()
    wm_p = S.sbn_conv3x3_pattern_apply(wp, ids, share)
    assert np.array_equal(wm_p.view(np.uint32), R.conv3x3_pattern_apply(wp, ids, share).view(np.uint32))
    wm = np.empty_like(wm_p)
    wm[perm_out] = wm_p                                           # back to the original filter order
    y, ref, bound = run_layer(x, wm, 4, 4, stride=stride, bias=bias, perm_out=perm_out, act=S.SBN_ACT_RELU, pct=60)
    assert_within_bound(y, ref, bound, f"pattern share {share}")
    # the oracle's layer on weights masked by hand: kept kernels carry exactly four weights
    per_kernel = np.count_nonzero(wm.transpose(0, 3, 1, 2).reshape(N * K, 9), axis=1)
    assert per_kernel.max() <= 4 and (per_kernel == 4).mean() > 0.99


@pytest.mark.parametrize("ordered", [False, True])
@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_resnet50_shapes_batch32_sampled(idx, ordered):
    """Config 5: ResNet-50-shaped 3x3 layers at batch 32, 70 % kernel-group sparsity; sampled images.
    ordered: as the benchmark packs them, the original grouping with whole filter groups reordered
    for the kernel (the output then comes in that order, and so does the oracle's)."""
    t = W.conv3x3_layer_tensors(5000, idx, 32, with_x=False)
    c, hw = t["c"], t["hw"]
    po = None
    if ordered:
        po = S.sbn_order_groups([dict(kind=S.SBN_CONV3X3, w=t["w"], go=4, gi=4)], [-1], 70, [np.arange(c, dtype=np.int32)])[0]
        assert np.array_equal(R.canonicalize(po, 4), np.arange(c))           # the grouping is the original one
    g = torch.Generator(device="cuda").manual_seed(5000 + idx)
    xd = torch.rand((32, hw, hw, c), device="cuda", generator=g) * 2 - 1
    mask = S.sbn_prune_magnitude(R.permute_weights(t["w"], po, None), S.SBN_CONV3X3, 4, 4, 70)
    p = S.sbn_pack(S.SBN_CONV3X3, t["w"], 4, 4, mask=mask, bias=t["bias"], perm_out=po, act=S.SBN_ACT_RELU)
    yd = torch.full((32, hw, hw, c), float("nan"), device="cuda")
    S.sbn_conv3x3_sparse(p, xd, yd, 32, hw, hw)
    torch.cuda.synchronize()
    assert torch.isfinite(yd).all()
    imgs = [0, 31] if hw >= 28 else [0, 13, 31]
    xs = xd[imgs].cpu().numpy()
    ys = yd[imgs].cpu().numpy()
    if hw == 56:          # keep the oracle's work to seconds: the top and the bottom band of 16 rows
        # (each needs one extra input row on its inner side; the outer side is the image border)
        ref, bound = R.sparse_conv_reference(xs[:, :17], t["w"], mask, 4, 4, bias=t["bias"], perm_out=po, stride=1, pad=1,
                                             act=S.SBN_ACT_RELU)
        assert_within_bound(ys[:, :16], ref[:, :16], bound[:, :16], f"resnet shape {idx} top rows")
        ref, bound = R.sparse_conv_reference(np.ascontiguousarray(xs[:, hw - 17:]), t["w"], mask, 4, 4, bias=t["bias"],
                                             perm_out=po, stride=1, pad=1, act=S.SBN_ACT_RELU)
        assert_within_bound(ys[:, hw - 16:], ref[:, 1:], bound[:, 1:], f"resnet shape {idx} bottom rows")
    else:
        ref, bound = R.sparse_conv_reference(xs, t["w"], mask, 4, 4, bias=t["bias"], perm_out=po, stride=1, pad=1,
                                             act=S.SBN_ACT_RELU)
        assert_within_bound(ys, ref, bound, f"resnet shape {idx}")


def test_activations_beyond_4_gib():
    """5400 images of 56x56x64: input and output are 4.3 GB each, so image byte offsets pass 2^32;
    whole images at the start, around the crossing and at the end are checked against the oracle."""
    c, hw, n = 64, 56, 5400
    free, _ = torch.cuda.mem_get_info()
    if free < 10 * (1 << 30):
        pytest.skip("needs 10 GiB of device memory")
    wt = W.he_weights(8900, c, 3, 3, c)
    b = W.small_bias(8901, c)
    mask = S.sbn_prune_magnitude(wt, S.SBN_CONV3X3, 4, 4, 70)
    p = S.sbn_pack(S.SBN_CONV3X3, wt, 4, 4, mask=mask, bias=b, act=S.SBN_ACT_RELU)
    g = torch.Generator(device="cuda").manual_seed(8902)
    xd = torch.rand((n, hw, hw, c), device="cuda", generator=g) * 2 - 1
    yd = torch.full((n, hw, hw, c), float("nan"), device="cuda")
    S.sbn_conv3x3_sparse(p, xd, yd, n, hw, hw)
    torch.cuda.synchronize()
    cross = (1 << 32) // (4 * hw * hw * c)             # the image that straddles 4 GiB
    imgs = [0, cross - 1, cross, cross + 1, n - 1]
    idx = torch.tensor(imgs, device="cuda")
    ref, bound = R.sparse_conv_reference(xd[idx].cpu().numpy(), wt, mask, 4, 4, bias=b, stride=1, pad=1, act=R.ACT_RELU)
    assert_within_bound(yd[idx].cpu().numpy(), ref, bound, "images around 4 GiB")
    assert not torch.isnan(yd[::97, ::11, ::13]).any()
