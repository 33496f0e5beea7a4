"""Pins of the oracle's 3:9 depthwise pattern pruning (Section 3.2, DwConv3x3) against what the
paper and the mathematics fix: the pattern family, the 33 % sparsity, the grouping rule, and a
closed form of the selection that does not enumerate patterns."""
import numpy as np
import pytest

from oracle import reference as R
import workloads as W


def test_pattern_family_is_what_the_paper_describes():
    masks = [R.dw_pattern_mask(p) for p in range(8)]
    assert len({m.tobytes() for m in masks}) == 8                 # 2^3 distinct patterns
    for m in masks:
        assert m.sum() == 6                                       # 3 of 9 removed: "33 % sparsity"
        assert (m[:, 1] == 1).all()                               # the middle column is never touched
        assert ((m[:, 0] + m[:, 2]) == 1).all()                   # one of first / third column per row
    assert abs(3 / 9 - 0.33) < 0.01
    assert R.dw_pattern_mask(R.DW_PATTERN_DENSE).sum() == 9      # the dense ("full-1") pattern
    # ids decode bit by bit: bit r set -> row r loses the third column
    assert R.dw_pattern_mask(0b101).tolist() == [[1, 1, 0], [0, 1, 1], [1, 1, 0]]


@pytest.mark.parametrize("c,go,expect", [
    (32, 16, [(0, 16), (16, 16)]),
    (24, 16, [(0, 16), (16, 8)]),
    (28, 16, [(0, 16), (16, 8), (24, 4)]),
    (12, 16, [(0, 8), (8, 4)]),
    (24, 8, [(0, 8), (8, 8), (16, 8)]),
    (4, 16, [(0, 4)]),
])
def test_groups_of_16_then_8_and_4(c, go, expect):
    assert R.dw_pattern_groups(c, go) == expect


def test_selection_equals_the_row_wise_closed_form():
    """Rows are independent: the best pattern keeps, in every row, whichever of the first and the
    third column carries the larger group-summed magnitude.  The oracle enumerates the 8 patterns."""
    rng = np.random.default_rng(77)
    for trial in range(20):
        c = int(rng.choice([16, 32, 24, 28, 48]))
        w = rng.standard_normal((c, 3, 3)).astype(np.float32)
        ids = R.dw_pattern_select(w, 16)
        for (c0, n), pid in zip(R.dw_pattern_groups(c, 16), ids):
            a = np.abs(w[c0:c0 + n].astype(np.float64))
            first, third = a[:, :, 0].sum(axis=0), a[:, :, 2].sum(axis=0)
            expect = sum(1 << r for r in range(3) if first[r] > third[r])   # keep the first -> remove the third
            assert pid == expect
            kept = a.sum() - np.minimum(first, third).sum()
            assert np.isclose((a * R.dw_pattern_mask(int(pid))).sum(), kept, rtol=1e-12)


def test_selection_on_a_hand_made_group():
    w = np.zeros((4, 3, 3), dtype=np.float32)
    w[:, :, 1] = 1.0
    w[:, 0, 0], w[:, 0, 2] = 5.0, 1.0      # row 0: first column heavier -> drop the third (bit 0 set)
    w[:, 1, 0], w[:, 1, 2] = 1.0, 5.0      # row 1: third heavier -> drop the first (bit 1 clear)
    w[:, 2, 0], w[:, 2, 2] = 2.0, 2.0      # row 2: tie -> lowest id -> bit 2 clear
    assert R.dw_pattern_select(w, 4).tolist() == [0b001]
    wm = R.dw_pattern_apply(w, [0b001], 4)
    assert (wm[:, 0, 2] == 0).all() and (wm[:, 1, 0] == 0).all() and (wm[:, 2, 0] == 0).all()
    assert (wm != 0).sum() == 4 * 6


def test_apply_is_a_select_and_dense_groups_stay_dense():
    w = W.normal_weights(4321, (40, 3, 3), 0.5)
    w[3, 0, 0] = -0.0
    ids = R.dw_pattern_select(w, 16, dense_groups=(1,))
    assert ids[1] == R.DW_PATTERN_DENSE and (ids[[0, 2]] < 8).all()
    wm = R.dw_pattern_apply(w, ids, 16)
    assert np.array_equal(wm[16:32], w[16:32])
    kept = wm != 0
    assert np.array_equal(wm[kept].view(np.uint32), w[kept].view(np.uint32))      # kept weights bit for bit
    assert not np.signbit(wm[~kept]).any()                                          # removed ones are +0.0
    assert (kept[:16].sum(), kept[32:].sum()) == (16 * 6, 8 * 6) or (w[:16] == 0).any()


def test_pattern_pruned_layer_equals_dense_layer_on_masked_weights():
    """The pruned depthwise layer is the plain depthwise convolution of W (.) M, which for a
    one-hot input reads the surviving taps back."""
    w = W.normal_weights(99, (16, 3, 3), 1.0)
    ids = R.dw_pattern_select(w, 16)
    wm = R.dw_pattern_apply(w, ids, 16)
    x = np.zeros((1, 5, 5, 16), dtype=np.float32)
    x[0, 2, 2, :] = 1.0
    y, _ = R.dwconv3x3_nhwc(x, wm, None, stride=1)
    # y[oy, ox] = w[2 + 1 - oy, 2 + 1 - ox] for the 3x3 window around the centre
    for oy in range(1, 4):
        for ox in range(1, 4):
            assert np.allclose(y[0, oy, ox], wm[:, 3 - oy, 3 - ox])
    assert (y[0, 0] == 0).all() and (y[0, 4] == 0).all()
