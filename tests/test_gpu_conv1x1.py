"""Parity of the HIP group-sparse 1x1 convolution with the CPU oracle (gpu)."""
import numpy as np
import pytest
import torch

import paper_2310_19509_amd as S
from oracle import reference as R
import workloads as W
from helpers import assert_within_bound

pytestmark = pytest.mark.gpu


def run_layer(x, w, go, gi, mask=None, bias=None, perm_out=None, perm_in=None, act=S.SBN_ACT_NONE, pct=None):
    """x: NHWC numpy in PERMUTED channel order.  Returns (y_gpu, y_ref, bound)."""
    if pct is not None:
        mask = S.sbn_prune_magnitude(R.permute_weights(w, perm_out, perm_in), S.SBN_CONV1X1, go, gi, pct)
        assert np.array_equal(mask, R.prune_mask(R.permute_weights(w, perm_out, perm_in), go, gi, pct))
    p = S.sbn_pack(S.SBN_CONV1X1, w, go, gi, mask=mask, bias=bias, perm_out=perm_out, perm_in=perm_in, act=act)
    n, h, ww, _ = x.shape
    xd = torch.from_numpy(x).cuda()
    yd = torch.full((n, h, ww, w.shape[0]), float("nan"), device="cuda", dtype=torch.float32)
    S.sbn_conv1x1_sparse(p, xd, yd, n, h, ww)
    torch.cuda.synchronize()
    y_ref, bound = R.sparse_conv_reference(x, w, mask, go, gi, bias=bias, perm_out=perm_out, perm_in=perm_in, act=act)
    return yd.cpu().numpy(), y_ref, bound


def test_config1():
    c = W.config1()
    y, ref, bound = run_layer(c["x"], c["w"], 4, 4, mask=c["mask"])
    assert_within_bound(y, ref, bound, "config1")


CASES = [
    # n, h, w, K, N, go, gi, pct, bias, relu, perms
    (1, 1, 1, 8, 8, 4, 4, 50, True, False, False),          # one pixel
    (1, 7, 7, 32, 64, 4, 4, 90, True, True, False),         # M=49, empty rows
    (1, 14, 14, 64, 128, 4, 4, 0, False, False, False),     # M=196, all kept
    (1, 14, 14, 64, 128, 8, 4, 50, True, True, True),       # go=8
    (2, 5, 5, 64, 32, 4, 1, 50, True, False, True),         # gi=1
    (2, 5, 5, 64, 32, 4, 2, 70, True, False, False),        # gi=2
    (2, 5, 5, 64, 32, 8, 8, 30, False, True, True),         # gi=8
    (1, 3, 3, 24, 24, 4, 4, 30, True, False, True),         # K, N not multiples of 32 / 16
    (1, 3, 3, 40, 72, 8, 4, 50, True, True, False),         # K=40, N=72
    (1, 3, 3, 6, 12, 4, 2, 30, True, False, False),         # K not a multiple of 4 (scalar staging)
    (1, 3, 3, 70, 12, 4, 1, 50, True, False, True),         # K=70, two chunks, scalar staging
    (1, 7, 7, 1024, 1024, 4, 4, 30, True, True, False),     # widest layer
    (1, 7, 7, 512, 1024, 8, 4, 70, True, False, False),
    (3, 9, 11, 128, 256, 4, 4, 30, True, True, True),       # M=297: several tiles + ragged tail
    (1, 2, 2, 32, 16, 4, 4, 100, True, True, False),        # everything pruned
]


@pytest.mark.parametrize("n,h,w,K,N,go,gi,pct,use_bias,relu,perms", CASES)
def test_shapes(n, h, w, K, N, go, gi, pct, use_bias, relu, perms):
    seed = 7000 + K + N + go + gi + pct
    wt = W.he_weights(seed, N, 1, 1, K)
    b = W.small_bias(seed + 1, N) * 20 if use_bias else None
    x = W.uniform_activation(seed + 2, (n, h, w, K))
    po = W.random_permutation(seed + 3, N) if perms else None
    pi = W.random_permutation(seed + 4, K) if perms else None
    y, ref, bound = run_layer(x, wt, go, gi, bias=b, perm_out=po, perm_in=pi,
                              act=S.SBN_ACT_RELU if relu else S.SBN_ACT_NONE, pct=pct)
    assert_within_bound(y, ref, bound, f"case {n,h,w,K,N,go,gi,pct}")
    if pct == 100:
        expect = np.zeros(N, np.float32) if b is None else (b if po is None else b[po])
        if relu:
            expect = np.maximum(expect, 0)
        assert np.array_equal(y, np.broadcast_to(expect, y.shape))


@pytest.mark.parametrize("variant", [11, 12, 14, 21, 22, 112, 121, 504, 508, 516, 1012, 1021, 1112, 1121])
@pytest.mark.parametrize("n,h,w,K,N,pct", [(3, 9, 11, 128, 256, 30), (1, 7, 7, 512, 1024, 70), (2, 13, 5, 72, 40, 50),
                                             (1, 20, 20, 320, 64, 0), (1, 26, 50, 128, 96, 50)])
def test_every_multi_chunk_kernel_form(variant, n, h, w, K, N, pct):
    """Layers with more than 64 input channels have several kernel forms (pixel sets per wave,
    partial sums per group, 64- or 32-channel chunks, input channels split over waves, and the
    mixed forms 112 / 121 whose last pixel tiles run as few-pixel workgroups inside the same
    launch) chosen by launch size; each is forced in turn and must match the oracle on the same
    input.  The 1300-pixel case gives the mixed forms 16 (8) whole tiles and a ragged remainder.
    Forms above 1000 walk the every-piece tables, which layers that keep at least 60 % of their
    pieces have (a layer without them runs the plain form); 72 and 320 channels end in a ragged chunk."""
    seed = 7500 + K + N + pct
    wt = W.he_weights(seed, N, 1, 1, K)
    b = W.small_bias(seed + 1, N) * 20
    x = W.uniform_activation(seed + 2, (n, h, w, K))
    S.sbn_force_kernel_form(S.SBN_CONV1X1, variant)
    try:
        y, ref, bound = run_layer(x, wt, 4, 4, bias=b, act=S.SBN_ACT_RELU, pct=pct)
    finally:
        S.sbn_force_kernel_form(S.SBN_CONV1X1, 0)
    assert_within_bound(y, ref, bound, f"variant {variant} case {n,h,w,K,N,pct}")


def test_uneven_rows_from_hand_mask():
    """One row keeps every block, one keeps none, others one block each."""
    K, N = 64, 32
    w = W.he_weights(7101, N, 1, 1, K)
    mask = np.zeros((N // 4, K // 4), dtype=np.uint8)
    mask[0, :] = 1
    for i in range(2, 8):
        mask[i, (5 * i) % 16] = 1
    x = W.uniform_activation(7102, (1, 9, 9, K))
    y, ref, bound = run_layer(x, w, 4, 4, mask=mask, bias=W.small_bias(7103, N))
    assert_within_bound(y, ref, bound, "hand mask")


def test_large_m_uses_two_pixel_sets_per_wave():
    """Enough pixels for the 128-pixel-per-workgroup variant, with a ragged tail."""
    K, N = 32, 64
    m = 1024 * 128 + 77
    w = W.he_weights(7201, N, 1, 1, K)
    x = W.uniform_activation(7202, (1, 1, m, K))
    y, ref, bound = run_layer(x, w, 4, 4, bias=W.small_bias(7203, N), act=S.SBN_ACT_RELU, pct=50)
    assert_within_bound(y, ref, bound, "large M")


def test_zero_pixels_and_argument_errors():
    c = W.config1()
    p = S.sbn_pack(S.SBN_CONV1X1, c["w"], 4, 4, mask=c["mask"])
    x = torch.zeros(8, 64, device="cuda")
    y = torch.zeros(4, 128, device="cuda")
    S.sbn_conv1x1_sparse(p, x, y, 0, 14, 14)          # nothing to do
    with pytest.raises(S.SbnError):
        S.sbn_conv1x1_sparse(p, x, x, 1, 2, 2)        # aliasing
    with pytest.raises(S.SbnError):
        S.sbn_conv3x3_sparse(p, x, y, 1, 2, 2)        # wrong kind
    with pytest.raises(S.SbnError):
        S.sbn_conv1x1_sparse(p, x, y, -1, 2, 2)
    with pytest.raises(S.SbnError) as ei:                 # 4-byte offset: not 16-byte aligned
        S.sbn_conv1x1_sparse(p, torch.zeros(8 * 64 + 1, device="cuda")[1:], y, 1, 2, 2)
    assert ei.value.code == -1 and "aligned" in str(ei.value)
    with pytest.raises(ValueError):                       # the binding compares sizes with the extents
        S.sbn_conv1x1_sparse(p, x, y, 1, 3, 3)


def test_nonblocking_stream():
    c = W.config1()
    p = S.sbn_pack(S.SBN_CONV1X1, c["w"], 4, 4, mask=c["mask"])
    st = torch.cuda.Stream()
    xd = torch.from_numpy(c["x"]).cuda()
    yd = torch.empty(1, 14, 14, 128, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        S.sbn_conv1x1_sparse(p, xd, yd, 1, 14, 14)
    st.synchronize()
    ref, bound = R.sparse_conv_reference(c["x"], c["w"], c["mask"], 4, 4)
    assert_within_bound(yd.cpu().numpy(), ref, bound, "side stream")


@pytest.mark.parametrize("layer_idx", list(range(1, 14)))
def test_full_size_batch64_sampled(layer_idx):
    """Config 3 at full size: every MobileNet-v1 pointwise layer at batch 64, at 30/50/70/90 %
    sparsity and with 4 and 8 filters per block, in the launch configuration the benchmark times;
    every output channel of about 600 sampled pixels (the first and the last tile among them)
    is compared with the oracle."""
    L = W.MOBILENET_V1_PW[layer_idx - 1]
    t = W.pw_layer_tensors(3000, L, 64, with_x=False)
    m = 64 * L.hw * L.hw
    g = torch.Generator(device="cuda").manual_seed(3000 + layer_idx)
    xd = torch.rand((m, L.c_in), device="cuda", generator=g) * 2 - 1
    rng = np.random.default_rng(layer_idx)
    idx = np.unique(np.concatenate([rng.integers(0, m, 480), np.arange(0, 64), np.arange(m - 64, m)]))
    idx_d = torch.from_numpy(idx).cuda()
    xs = xd[idx_d].cpu().numpy()
    yd = torch.empty((m, L.c_out), device="cuda")
    for go in (4, 8):
        for pct in (30, 50, 70, 90):
            mask = S.sbn_prune_magnitude(t["w"], S.SBN_CONV1X1, go, 4, pct)
            p = S.sbn_pack(S.SBN_CONV1X1, t["w"], go, 4, mask=mask, bias=t["bias"], act=S.SBN_ACT_RELU)
            yd.fill_(float("nan"))
            S.sbn_conv1x1_sparse(p, xd, yd, 64, L.hw, L.hw)
            torch.cuda.synchronize()
            assert torch.isfinite(yd).all()
            ys = yd[idx_d].cpu().numpy()
            ref, bound = R.sparse_conv_reference(xs[None, None], t["w"], mask, go, 4, bias=t["bias"],
                                                 act=S.SBN_ACT_RELU)
            assert_within_bound(ys[None, None], ref, bound, f"pw{layer_idx} rho={pct} go={go}")
            S.sbn_free(p)


def test_the_benchmarks_own_layers_at_full_size_sampled():
    """The default benchmark's step itself: the 13 layers as bench.py builds them (filters rearranged
    as a chain, groups ordered for the kernels, 30 % by block magnitude, batch 64), launched as the
    benchmark launches them; every output channel of about 300 sampled pixels per layer against
    the oracle on the same permuted, masked weights."""
    import bench
    tens, perms, packed, _ = bench.build_layers(S, W, 64, 30, 4, True)
    pin = None
    for L, t, po, p in zip(W.MOBILENET_V1_PW, tens, perms, packed):
        m = 64 * L.hw * L.hw
        g = torch.Generator(device="cuda").manual_seed(3100 + L.index)
        xd = torch.rand((m, L.c_in), device="cuda", generator=g) * 2 - 1      # channels in perm_in order
        rng = np.random.default_rng(100 + L.index)
        idx = np.unique(np.concatenate([rng.integers(0, m, 200), np.arange(0, 32), np.arange(m - 64, m)]))
        idx_d = torch.from_numpy(idx).cuda()
        yd = torch.full((m, L.c_out), float("nan"), device="cuda")
        S.sbn_conv1x1_sparse(p, xd, yd, 64, L.hw, L.hw)
        torch.cuda.synchronize()
        assert torch.isfinite(yd).all()
        wp = R.permute_weights(t["w"], po, pin)
        mask = R.prune_mask(wp, 4, 4, 30)
        assert S.sbn_packed_work(p)["nnz_blocks"] == int(mask.sum())
        # the oracle on the permuted layer: its input order is the order xd is in, its output order yd's
        ref, bound = R.sparse_conv_reference(xd[idx_d].cpu().numpy()[None, None], wp, mask, 4, 4, bias=t["bias"][po],
                                             act=S.SBN_ACT_RELU)
        assert_within_bound(yd[idx_d].cpu().numpy()[None, None], ref, bound, f"bench layer pw{L.index}")
        pin = po


def test_config2_all_13_layers_batch1_rearranged_chained_perms():
    """Config 2: the 13 pointwise layers at batch 1, each on its own input, 30 % by block magnitude
    after rearrangement, permutations chained across the stack; every output is compared."""
    layers = [W.pw_layer_tensors(2000, L, 1) for L in W.MOBILENET_V1_PW]
    descs = [dict(kind=S.SBN_CONV1X1, w=t["w"], go=4, gi=4) for t in layers]
    perms = S.sbn_rearrange(descs, [-1] + list(range(12)), 30, seed=2000, max_iters=300,
                            keep_output_order=[0] * 12 + [1])
    pin = None
    for L, t, po in zip(W.MOBILENET_V1_PW, layers, perms):
        wp = R.permute_weights(t["w"], po, pin)
        mask = S.sbn_prune_magnitude(wp, S.SBN_CONV1X1, 4, 4, 30)
        assert np.array_equal(mask, R.prune_mask(wp, 4, 4, 30))
        assert R.retained_l1(wp, 4, 4, 30) >= R.retained_l1(R.permute_weights(t["w"], None, pin), 4, 4, 30) * (1 - 1e-12)
        x = t["x"] if pin is None else np.ascontiguousarray(t["x"][..., pin])
        y, ref, bound = run_layer(x, t["w"], 4, 4, mask=mask, bias=t["bias"], perm_out=po, perm_in=pin,
                                  act=S.SBN_ACT_RELU)
        assert_within_bound(y, ref, bound, f"config2 pw{L.index}")
        pin = po


def test_config1_with_per_input_channel_masks():
    """Secondary reading of 'group of 4 output channels sharing the input-channel mask': gi = 1."""
    c = W.config1()
    mask = W.uniform_block_mask(1004, 128 // 4, 64, (128 // 4) * 64 // 2)
    y, ref, bound = run_layer(c["x"], c["w"], 4, 1, mask=mask)
    assert_within_bound(y, ref, bound, "config1 gi=1")


def test_very_wide_input():
    """Many chunks, few outputs: c_in = 2048, c_out = 16, odd pixel count."""
    w = W.he_weights(7301, 16, 1, 1, 2048)
    x = W.uniform_activation(7302, (1, 1, 71, 2048))
    y, ref, bound = run_layer(x, w, 4, 4, bias=W.small_bias(7303, 16), pct=60)
    assert_within_bound(y, ref, bound, "wide K")


def test_same_layer_on_two_streams_and_repeated_launches():
    """Launches of one packed layer on different streams and buffers do not interfere."""
    L = W.MOBILENET_V1_PW[4]
    t = W.pw_layer_tensors(7400, L, 2)
    mask = S.sbn_prune_magnitude(t["w"], S.SBN_CONV1X1, 4, 4, 50)
    p = S.sbn_pack(S.SBN_CONV1X1, t["w"], 4, 4, mask=mask, bias=t["bias"])
    xs = [torch.from_numpy(t["x"]).cuda(), torch.from_numpy(t["x"][::-1].copy()).cuda()]
    ys = [torch.empty(2, L.hw, L.hw, L.c_out, device="cuda") for _ in range(2)]
    sts = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(3):
        for i in range(2):
            S.sbn_conv1x1_sparse(p, xs[i], ys[i], 2, L.hw, L.hw, stream=sts[i])
    torch.cuda.synchronize()
    ref, bound = R.sparse_conv_reference(t["x"], t["w"], mask, 4, 4, bias=t["bias"])
    assert_within_bound(ys[0].cpu().numpy(), ref, bound, "stream 0")
    assert_within_bound(ys[1].cpu().numpy(), ref[::-1], bound[::-1], "stream 1")


def test_activations_beyond_4_gib():
    """17 million pixels x 64 channels: input and output are 4.35 GB each, so byte offsets pass
    2^32 and pixel*channel indices pass 2^30; sampled pixels from the start, the 4 GiB crossing and
    the ragged end are checked against the oracle."""
    K = N = 64
    m = 17_000_011                                     # not a multiple of the 64-pixel tile
    free, _ = torch.cuda.mem_get_info()
    if free < 10 * (1 << 30):
        pytest.skip("needs 10 GiB of device memory")
    wt = W.he_weights(7900, N, 1, 1, K)
    b = W.small_bias(7901, N)
    mask = S.sbn_prune_magnitude(wt, S.SBN_CONV1X1, 4, 4, 50)
    p = S.sbn_pack(S.SBN_CONV1X1, wt, 4, 4, mask=mask, bias=b, act=S.SBN_ACT_RELU)
    g = torch.Generator(device="cuda").manual_seed(7902)
    xd = torch.rand((m, K), device="cuda", generator=g) * 2 - 1
    yd = torch.full((m, N), float("nan"), device="cuda")
    S.sbn_conv1x1_sparse(p, xd, yd, 1, 1, m)
    torch.cuda.synchronize()
    cross = (1 << 32) // (4 * K)                       # first pixel whose bytes start beyond 4 GiB
    rows = np.concatenate([np.arange(0, 200), np.arange(cross - 100, cross + 100), np.arange(m - 300, m)])
    idx = torch.from_numpy(rows).cuda()
    xs = xd[idx].cpu().numpy().reshape(1, 1, len(rows), K)
    ref, bound = R.sparse_conv_reference(xs, wt, mask, 4, 4, bias=b, act=R.ACT_RELU)
    assert_within_bound(yd[idx].cpu().numpy().reshape(ref.shape), ref, bound, "rows around 4 GiB")
    assert not torch.isnan(yd[::100003]).any()
