"""Pins of the oracle's 4-of-9 pattern pruning of 3x3 kernels (Section 3.2, Conv3x3) against
what the paper and the mathematics fix: the size and shape of the pattern family, and a closed
form of the selection that sorts instead of enumerating."""
import math

import numpy as np
import pytest

from oracle import reference as R


def test_pattern_family_is_what_the_paper_describes():
    masks = [R.conv3x3_pattern_mask(p) for p in range(R.K3_PATTERNS)]
    assert R.K3_PATTERNS == 56 == math.comb(8, 3)                 # the paper's count
    assert len({m.tobytes() for m in masks}) == 56                # all different
    for m in masks:
        assert m.sum() == 4                                       # 4 of 9 kept ("5:9" removed)
        assert m[1, 1] == 1                                       # the centre always stays
    assert R.conv3x3_pattern_mask(R.K3_PATTERN_DENSE).sum() == 9
    # numbering: lexicographic 3-subsets of taps 0,1,2,3,5,6,7,8
    assert R.conv3x3_pattern_mask(0).reshape(9).tolist() == [1, 1, 1, 0, 1, 0, 0, 0, 0]
    assert R.conv3x3_pattern_mask(1).reshape(9).tolist() == [1, 1, 0, 1, 1, 0, 0, 0, 0]
    assert R.conv3x3_pattern_mask(55).reshape(9).tolist() == [0, 0, 0, 0, 1, 0, 1, 1, 1]
    # every non-centre tap is in C(7,2) = 21 of the patterns
    counts = np.sum([m.reshape(9) for m in masks], axis=0)
    assert counts.tolist() == [21, 21, 21, 21, 56, 21, 21, 21, 21]


@pytest.mark.parametrize("share", [1, 2, 4])
def test_selection_equals_top_three_by_summed_magnitude(share):
    """The score is additive over taps, so the best pattern keeps the centre and the three other
    taps with the largest magnitude summed over the filters sharing it.  The oracle enumerates."""
    rng = np.random.default_rng(90 + share)
    w = rng.standard_normal((8, 3, 3, 6)).astype(np.float32)
    ids = R.conv3x3_pattern_select(w, share)
    assert ids.shape == (8 // share, 6)
    for f in range(8 // share):
        for c in range(6):
            a = np.abs(w[f * share:(f + 1) * share, :, :, c].astype(np.float64)).sum(axis=0).reshape(9)
            a[4] = -1.0
            top = set(np.argsort(-a)[:3].tolist())
            kept = set(np.nonzero(R.conv3x3_pattern_mask(int(ids[f, c])).reshape(9))[0].tolist())
            assert kept == top | {4}


def test_ties_take_the_lowest_id_and_apply_is_a_select():
    w = np.ones((4, 3, 3, 2), dtype=np.float32)                   # every pattern scores the same
    assert R.conv3x3_pattern_select(w, 4).tolist() == [[0, 0]]
    w[:, 2, 2, 1] = 3.0                                           # channel 1: tap 8 must be kept;
    ids = R.conv3x3_pattern_select(w, 4)                          # lowest such subset is {0, 1, 8}
    assert R.conv3x3_pattern_mask(int(ids[0, 1])).reshape(9).tolist() == [1, 1, 0, 0, 1, 0, 0, 0, 1]
    w = -np.abs(np.random.default_rng(5).standard_normal((4, 3, 3, 3)).astype(np.float32))
    ids = R.conv3x3_pattern_select(w, 2)
    wm = R.conv3x3_pattern_apply(w, ids, 2)
    assert not np.signbit(wm[wm == 0]).any()                      # removed weights are +0.0
    assert np.count_nonzero(wm) == 4 * 4 * 3                      # four weights per kernel stay
    assert np.array_equal(wm[wm != 0], w[wm != 0])
    dense = np.full_like(ids, R.K3_PATTERN_DENSE)
    assert np.array_equal(R.conv3x3_pattern_apply(w, dense, 2), w)


def test_pattern_pruned_layer_equals_a_convolution_with_hand_masked_weights():
    """One kernel, one pattern: the layer's output is the sum over exactly the four kept taps."""
    rng = np.random.default_rng(17)
    w = rng.standard_normal((1, 3, 3, 1)).astype(np.float32)
    x = rng.uniform(-1, 1, (1, 5, 5, 1)).astype(np.float32)
    ids = R.conv3x3_pattern_select(w, 1)
    wm = R.conv3x3_pattern_apply(w, ids, 1)
    y, _ = R.conv_nhwc(x, wm, None, stride=1, pad=1, act=0)
    keep = np.nonzero(R.conv3x3_pattern_mask(int(ids[0, 0])).reshape(9))[0]
    xp = np.pad(x[0, :, :, 0].astype(np.float64), 1)
    want = np.zeros((5, 5))
    for t in keep:
        want += xp[t // 3:t // 3 + 5, t % 3:t % 3 + 5] * float(w[0, t // 3, t % 3, 0])
    assert np.allclose(y[0, :, :, 0], want, rtol=0, atol=1e-6)
