"""Pins for the CPU oracle's convolutions (not gpu).

The oracle is checked against things other than itself: a pure-Python
brute-force loop nest on tiny layers, library routines (numpy matmul,
scipy.signal.correlate2d, torch conv2d in fp64), closed forms and invariants.
Each planted-mistake class (dropped tap, transposed operand, wrong stride/pad
index, missing bias, wrong activation) fails at least one of these.
"""
import numpy as np
import pytest
import scipy.signal
import torch

from oracle import reference as R
import workloads as W


def brute_conv(x, w, bias, stride, pad, act):
    """Definition (Section 3.1 notation) in pure Python loops, fp64."""
    n, ih, iw, ic = x.shape
    oc, kh, kw, _ = w.shape
    oh = (ih + 2 * pad - kh) // stride + 1
    ow = (iw + 2 * pad - kw) // stride + 1
    y = np.zeros((n, oh, ow, oc), dtype=np.float64)
    for b in range(n):
        for oy in range(oh):
            for ox in range(ow):
                for o in range(oc):
                    acc = float(bias[o]) if bias is not None else 0.0
                    for ky in range(kh):
                        for kx in range(kw):
                            iy, ix = oy * stride + ky - pad, ox * stride + kx - pad
                            if 0 <= iy < ih and 0 <= ix < iw:
                                for c in range(ic):
                                    acc += float(x[b, iy, ix, c]) * float(w[o, ky, kx, c])
                    if act == R.ACT_RELU:
                        acc = max(acc, 0.0)
                    y[b, oy, ox, o] = acc
    return y


@pytest.mark.parametrize("kh,stride,pad,ih,iw", [(1, 1, 0, 1, 3), (3, 1, 1, 4, 4), (3, 2, 1, 4, 4),
                                                 (3, 2, 1, 5, 7), (3, 1, 0, 5, 4)])
@pytest.mark.parametrize("act", [R.ACT_NONE, R.ACT_RELU])
def test_brute_force_tiny(kh, stride, pad, ih, iw, act):
    x = W.uniform_activation(11, (2, ih, iw, 8))
    w = W.normal_weights(12, (8, kh, kh, 8), 0.3)
    b = W.small_bias(13, 8) * 30
    y, bound = R.conv_nhwc(x, w, b, stride=stride, pad=pad, act=act)
    ref = brute_conv(x, w, b, stride, pad, act)
    assert y.shape == ref.shape
    np.testing.assert_allclose(y, ref.astype(np.float32), rtol=0, atol=1e-6)
    assert np.all(bound >= np.abs(ref - (b if act == R.ACT_NONE else 0)) - 1e-9) or act == R.ACT_RELU


def test_1x1_all_kept_is_a_gemm():
    """All blocks kept: a 1x1 layer is the matrix product [M,K] x [K,N] (Section 3.2, Conv1x1)."""
    x = W.uniform_activation(21, (3, 5, 7, 24))
    w = W.normal_weights(22, (16, 1, 1, 24), 0.2)
    y, _ = R.conv_nhwc(x, w)
    ref = x.reshape(-1, 24).astype(np.float64) @ w.reshape(16, 24).astype(np.float64).T
    np.testing.assert_allclose(y.reshape(-1, 16), ref.astype(np.float32), rtol=0, atol=2e-6)


def test_3x3_matches_scipy_correlate():
    x = W.uniform_activation(31, (1, 9, 6, 3))
    w = W.normal_weights(32, (2, 3, 3, 3), 0.4)
    y, _ = R.conv_nhwc(x, w, stride=1, pad=1)
    for o in range(2):
        acc = np.zeros((9, 6))
        for c in range(3):
            acc += scipy.signal.correlate2d(x[0, :, :, c].astype(np.float64),
                                            w[o, :, :, c].astype(np.float64), mode="same")
        np.testing.assert_allclose(y[0, :, :, o], acc.astype(np.float32), rtol=0, atol=2e-6)


@pytest.mark.parametrize("stride", [1, 2])
def test_matches_torch_conv2d_fp64(stride):
    x = W.uniform_activation(41, (2, 11, 10, 12))
    w = W.normal_weights(42, (8, 3, 3, 12), 0.2)
    b = W.small_bias(43, 8)
    y, _ = R.conv_nhwc(x, w, b, stride=stride, pad=1, act=R.ACT_RELU)
    t = torch.nn.functional.conv2d(torch.from_numpy(x).double().permute(0, 3, 1, 2),
                                   torch.from_numpy(w).double().permute(0, 3, 1, 2),
                                   torch.from_numpy(b).double(), stride=stride, padding=1).relu()
    np.testing.assert_allclose(y, t.permute(0, 2, 3, 1).numpy().astype(np.float32), rtol=0, atol=2e-6)


@pytest.mark.parametrize("stride", [1, 2])
def test_depthwise_matches_torch_grouped_conv(stride):
    x = W.uniform_activation(51, (2, 9, 8, 16))
    w = W.normal_weights(52, (16, 3, 3), 0.5)
    b = W.small_bias(53, 16)
    y, bound = R.dwconv3x3_nhwc(x, w, b, stride=stride, act=R.ACT_RELU)
    t = torch.nn.functional.conv2d(torch.from_numpy(x).double().permute(0, 3, 1, 2),
                                   torch.from_numpy(w).double()[:, None], torch.from_numpy(b).double(),
                                   stride=stride, padding=1, groups=16).relu()
    np.testing.assert_allclose(y, t.permute(0, 2, 3, 1).numpy().astype(np.float32), rtol=0, atol=2e-6)
    assert bound.shape == y.shape and np.all(bound >= 0)


@pytest.mark.parametrize("stride", [1, 2])
def test_depthwise_bound_is_sum_of_magnitudes(stride):
    """The depthwise bound is the tolerance scale of every depthwise and fused-pair parity test.
    Pinned three ways: pure-Python brute force of sum |x||w| over the taps inside the image, the
    identity bound(x, w) = dwconv(|x|, |w|) without bias, and torch's grouped convolution on the
    magnitudes.  A ones-kernel on a ones-image counts the taps inside the image (9 / 6 / 4)."""
    x = W.uniform_activation(54, (2, 5, 4, 8))
    w = W.normal_weights(55, (8, 3, 3), 0.5)
    b = W.small_bias(56, 8) * 50            # the bias must not enter the bound
    _, bound = R.dwconv3x3_nhwc(x, w, b, stride=stride, act=R.ACT_RELU)
    n, ih, iw, c = x.shape
    oh, ow = (ih - 1) // stride + 1, (iw - 1) // stride + 1
    brute = np.zeros((n, oh, ow, c))
    for bi in range(n):
        for oy in range(oh):
            for ox in range(ow):
                for ch in range(c):
                    s = 0.0
                    for ky in range(3):
                        for kx in range(3):
                            iy, ix = oy * stride + ky - 1, ox * stride + kx - 1
                            if 0 <= iy < ih and 0 <= ix < iw:
                                s += abs(float(x[bi, iy, ix, ch])) * abs(float(w[ch, ky, kx]))
                    brute[bi, oy, ox, ch] = s
    np.testing.assert_allclose(bound, brute, rtol=1e-14, atol=0)
    y_abs, _ = R.dwconv3x3_nhwc(np.abs(x), np.abs(w), None, stride=stride)
    np.testing.assert_allclose(bound, y_abs, rtol=1e-6)
    t = torch.nn.functional.conv2d(torch.from_numpy(np.abs(x)).double().permute(0, 3, 1, 2),
                                   torch.from_numpy(np.abs(w)).double()[:, None], None,
                                   stride=stride, padding=1, groups=c)
    np.testing.assert_allclose(bound, t.permute(0, 2, 3, 1).numpy(), rtol=1e-13)


def test_depthwise_bound_counts_taps_inside_the_image():
    ones = np.ones((1, 3, 3, 4), np.float32)
    _, bound = R.dwconv3x3_nhwc(ones, np.ones((4, 3, 3), np.float32))
    assert np.array_equal(bound[0, :, :, 0], np.array([[4, 6, 4], [6, 9, 6], [4, 6, 4]], float))
    _, bound2 = R.dwconv3x3_nhwc(ones, np.ones((4, 3, 3), np.float32), stride=2)
    assert np.array_equal(bound2[0, :, :, 0], np.array([[4, 4], [4, 4]], float))


def test_avgpool_is_mean():
    x = W.uniform_activation(61, (3, 7, 7, 10))
    np.testing.assert_allclose(R.avgpool_nhwc(x), x.astype(np.float64).mean(axis=(1, 2)).astype(np.float32),
                               rtol=0, atol=1e-7)


def test_all_pruned_gives_act_of_bias():
    x = W.uniform_activation(71, (1, 3, 3, 8))
    w = np.zeros((8, 1, 1, 8), dtype=np.float32)
    b = np.array([-1, 2, -3, 4, -5, 6, -7, 8], dtype=np.float32)
    y, bound = R.conv_nhwc(x, w, b, act=R.ACT_RELU)
    assert np.array_equal(y, np.broadcast_to(np.maximum(b, 0), y.shape))
    assert np.all(bound == 0)


def test_one_kept_block_closed_form():
    """Only block (row 1, col 0) of a 8x8 layer kept, go=gi=4: y[:,4:8] = x[:,0:4] @ Wblk^T."""
    x = W.uniform_activation(81, (1, 2, 2, 8))
    w = W.normal_weights(82, (8, 1, 1, 8), 0.3)
    mask = np.zeros((2, 2), dtype=np.uint8)
    mask[1, 0] = 1
    wt = R.apply_mask(w, mask, 4, 4)
    y, _ = R.conv_nhwc(x, wt)
    assert np.all(y[..., 0:4] == 0)
    ref = x.reshape(4, 8)[:, 0:4].astype(np.float64) @ w.reshape(8, 8)[4:8, 0:4].astype(np.float64).T
    np.testing.assert_allclose(y.reshape(4, 8)[:, 4:8], ref.astype(np.float32), rtol=0, atol=1e-6)


def test_bound_is_sum_of_magnitudes():
    x = W.uniform_activation(91, (1, 4, 4, 8))
    w = W.normal_weights(92, (4, 3, 3, 8), 0.3)
    _, bound = R.conv_nhwc(x, w, stride=1, pad=1)
    y_abs, _ = R.conv_nhwc(np.abs(x), np.abs(w), stride=1, pad=1)
    np.testing.assert_allclose(bound, y_abs, rtol=1e-6)


def test_sparse_equals_dense_on_zeroed_weights_and_linearity():
    """W = W~ + (W - W~): conv(x, W) = conv(x, W~) + conv(x, W - W~) (Section 3.1, W~ = W (.) M)."""
    c = W.config1()
    wt = R.apply_mask(c["w"], c["mask"], 4, 4)
    y_s, _ = R.conv_nhwc(c["x"], wt)
    y_d, _ = R.conv_nhwc(c["x"], c["w"])
    y_r, _ = R.conv_nhwc(c["x"], c["w"] - wt)
    np.testing.assert_allclose(y_s.astype(np.float64) + y_r, y_d, rtol=0, atol=1e-6)
    # the masked tensor has exactly the removed blocks at +0.0
    assert int((wt == 0).sum()) >= 256 * 16
    assert not np.signbit(wt[wt == 0]).any()


def test_output_permutation_is_exact():
    """Filter rearrangement only reorders outputs (Section 3.4)."""
    x = W.uniform_activation(101, (1, 3, 3, 8))
    w = W.normal_weights(102, (16, 1, 1, 8), 0.3)
    b = W.small_bias(103, 16)
    po = W.random_permutation(104, 16)
    y0, _ = R.conv_nhwc(x, w, b)
    y1, _ = R.sparse_conv_reference(x, w, np.ones((4, 2), np.uint8), 4, 4, bias=b, perm_out=po)
    assert np.array_equal(y1, y0[..., po])


def test_input_permutation_within_rounding():
    x = W.uniform_activation(111, (1, 3, 3, 8))
    w = W.normal_weights(112, (8, 1, 1, 8), 0.3)
    pi = W.random_permutation(113, 8)
    y0, bound = R.conv_nhwc(x, w)
    y1, _ = R.sparse_conv_reference(x[..., pi], w, np.ones((2, 2), np.uint8), 4, 4, perm_in=pi)
    assert np.all(np.abs(y1.astype(np.float64) - y0) <= 1e-6 * bound + 1e-12)
