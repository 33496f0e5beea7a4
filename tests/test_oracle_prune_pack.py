"""Pins for the oracle's host-side pieces: block importance, pruning,
canonical packing, rearrangement objective and enumerator, FLOP accounting."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import reference as R
import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_kv(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            out[k] = float(v)
    return out


# ---------------------------------------------------------------- FLOP accounting

def test_mobilenet_macs_match_paper_table3():
    g = read_kv("paper_table3_flops.txt")
    m = W.mobilenet_v1_macs()
    assert abs(m["total"] / 1e6 - g["baseline_total_M"]) < 1.0
    for pct in (10, 20, 30, 40, 50):
        ours = (m["total"] - m["pw"] * pct / 100.0) / 1e6
        assert abs(ours - g[f"fkgp_M_at_{pct}pct"]) < 1.0, (pct, ours)
    assert abs(100.0 * m["stem"] / m["total"] - g["stem_conv3x3_share_percent"]) < 0.01


def test_pw_and_dw_tables_chain():
    for a, b in zip(W.MOBILENET_V1_PW[:-1], W.MOBILENET_V1_PW[1:]):
        assert a.c_out == b.c_in
    for d, p in zip(W.MOBILENET_V1_DW, W.MOBILENET_V1_PW):
        assert d.c == p.c_in and d.hw_out == p.hw


# ---------------------------------------------------------------- block norms / pruning

def brute_block_norm(w, go, gi, i, j):
    s = 0.0
    for o in range(go):
        for ky in range(w.shape[1]):
            for kx in range(w.shape[2]):
                for c in range(gi):
                    s += abs(float(w[i * go + o, ky, kx, j * gi + c]))
    return s


@pytest.mark.parametrize("kh,go,gi", [(1, 4, 4), (3, 4, 4), (1, 8, 4), (1, 4, 1), (3, 2, 2)])
def test_block_norms_brute_force(kh, go, gi):
    w = W.normal_weights(201, (16, kh, kh, 8), 0.5)
    s = R.block_norms(w, go, gi)
    assert s.shape == (16 // go, 8 // gi)
    for i in range(s.shape[0]):
        for j in range(s.shape[1]):
            assert s[i, j] == brute_block_norm(w, go, gi, i, j)


def test_block_norm_not_transposed():
    """A weight placed at (filter 5, channel 2) must land in block (1, 0) for go=gi=4."""
    w = np.zeros((8, 1, 1, 8), dtype=np.float32)
    w[5, 0, 0, 2] = -3.0
    s = R.block_norms(w, 4, 4)
    assert s[1, 0] == 3.0 and s.sum() == 3.0


@pytest.mark.parametrize("pct", [0, 10, 30, 33, 50, 70, 90, 100])
def test_prune_count_and_threshold(pct):
    w = W.he_weights(211, 32, 1, 1, 24)
    m = R.prune_mask(w, 4, 4, pct)
    nb = 8 * 6
    assert int(m.sum()) == nb - (nb * pct) // 100
    s = R.block_norms(w, 4, 4)
    if 0 < m.sum() < nb:
        assert s[m == 1].min() >= s[m == 0].max()


def test_prune_brute_force_and_ties():
    """Exhaustive: the kept set maximises the retained norm (Eq. 2); ties drop the lower index first."""
    w = W.normal_weights(221, (8, 1, 1, 12), 1.0)
    s = R.block_norms(w, 4, 4)          # 2 x 3 blocks
    m = R.prune_mask(w, 4, 4, 50)       # removes 3 of 6
    best = max(itertools.combinations(range(6), 3), key=lambda keep: sum(s.ravel()[list(keep)]))
    assert sorted(np.flatnonzero(m.ravel())) == sorted(best)
    wt = np.ones((8, 1, 1, 8), dtype=np.float32)    # all four blocks tie
    mt = R.prune_mask(wt, 4, 4, 50)
    assert mt.ravel().tolist() == [0, 0, 1, 1]


def test_retained_l1_is_norm_of_masked_weights():
    w = W.he_weights(231, 16, 3, 3, 16)
    for pct in (30, 70):
        m = R.prune_mask(w, 4, 4, pct)
        assert math.isclose(R.retained_l1(w, 4, 4, pct),
                            float(np.abs(R.apply_mask(w, m, 4, 4).astype(np.float64)).sum()), rel_tol=1e-12)


# ---------------------------------------------------------------- packing

@pytest.mark.parametrize("kh,go,gi,pct", [(1, 4, 4, 50), (3, 4, 4, 70), (1, 8, 4, 30), (1, 4, 1, 50), (1, 4, 4, 100),
                                          (1, 4, 4, 0)])
def test_pack_invariants_and_round_trip(kh, go, gi, pct):
    w = W.he_weights(241, 32, kh, kh, 16)
    w[3, 0, 0, 5] = np.float32(-0.0)                 # sign of zero inside a block must survive
    w[9, 0, 0, 1] = np.float32(1e-42)                # denormal too
    m = R.prune_mask(w, go, gi, pct)
    row_ptr, kidx, vals = R.canonical_pack(w, m, go, gi)
    assert row_ptr[0] == 0 and row_ptr[-1] == kidx.size == vals.shape[0] == int(m.sum())
    assert np.all(np.diff(row_ptr.astype(np.int64)) >= 0)
    for i in range(32 // go):
        seg = kidx[row_ptr[i]:row_ptr[i + 1]].astype(np.int64)
        assert np.all(np.diff(seg) > 0) and np.all(seg % gi == 0)
    w2, m2 = R.canonical_unpack(row_ptr, kidx, vals, 32, 16, go, gi)
    assert np.array_equal(m2, m)
    assert np.array_equal(w2.view(np.uint32), R.apply_mask(w, m, go, gi).view(np.uint32))


def test_pack_vals_layout_is_ci_major_co_minor():
    w = np.arange(8 * 8, dtype=np.float32).reshape(8, 1, 1, 8)     # w[o, c] = 8*o + c
    m = np.array([[0, 1], [1, 0]], dtype=np.uint8)
    row_ptr, kidx, vals = R.canonical_pack(w, m, 4, 4)
    assert row_ptr.tolist() == [0, 1, 2] and kidx.tolist() == [4, 0]
    # block (row 0, col 1): element [ci][co] = w[co, 4 + ci]
    assert vals[0, 0, 0, 1, 2] == w[2, 0, 0, 5]
    assert vals[1, 0, 0, 3, 0] == w[4, 0, 0, 3]


def test_nonzero_block_mask():
    w = np.zeros((8, 1, 1, 8), dtype=np.float32)
    w[0, 0, 0, 0] = np.float32(-0.0)      # magnitude zero: does not keep the block
    w[4, 0, 0, 7] = np.float32(1e-45)     # smallest denormal keeps it
    assert R.nonzero_block_mask(w, 4, 4).tolist() == [[0, 0], [0, 1]]


# ---------------------------------------------------------------- permutations

def test_permute_round_trip():
    w = W.he_weights(251, 12, 3, 3, 8)
    po, pi = W.random_permutation(252, 12), W.random_permutation(253, 8)
    wp = R.permute_weights(w, po, pi)
    assert wp[3, 1, 2, 5] == w[po[3], 1, 2, pi[5]]
    assert np.array_equal(R.unpermute_weights(wp, po, pi), w)
    inv = R.inverse_permutation(po)
    assert np.array_equal(po[inv], np.arange(12)) and np.array_equal(inv[po], np.arange(12))
    assert R.is_permutation(po, 12) and not R.is_permutation(np.zeros(12, np.int32), 12)


def test_canonical_grouping_counts_match_section_3_4():
    with open(os.path.join(GOLD, "paper_sec34_canonical.txt")) as f:
        rows = [tuple(map(int, l.split())) for l in f if l.strip() and not l.startswith("#")]
    for n, go, count in rows:
        gs = list(R.canonical_groupings(n, go))
        assert len(gs) == count == math.factorial(n) // (math.factorial(go) ** (n // go) * math.factorial(n // go))
        assert len(set(gs)) == count
        for g in gs:
            assert sorted(g) == list(range(n))
            assert np.array_equal(R.canonicalize(g, go), np.asarray(g))


def test_canonicalize_preserves_objective():
    w = W.he_weights(261, 8, 1, 1, 8)
    p = W.random_permutation(262, 8)
    c = R.canonicalize(p, 4)
    assert R.is_permutation(c, 8)
    assert math.isclose(R.retained_l1(w[p], 4, 4, 50), R.retained_l1(w[c], 4, 4, 50), rel_tol=1e-12)


def test_exhaustive_grouping_beats_identity_and_finds_planted_structure():
    """Two 'strong' and two 'weak' filters interleaved: grouping like with like retains more (Section 3.4)."""
    w = np.zeros((4, 1, 1, 4), dtype=np.float32)
    w[0] = 5.0
    w[2] = 4.0
    w[1] = 0.1
    w[3] = 0.2
    ident = R.retained_l1(w, 2, 2, 50)
    perm, obj = R.best_row_grouping(w, 2, 2, 50)
    assert perm.tolist() == [0, 2, 1, 3]
    assert obj > ident
    # identity: blocks 10.2, 10.2, 8.4, 8.4 -> top two kept; regrouped: 18, 18, 0.6, 0.6
    assert math.isclose(obj, 36.0, rel_tol=1e-6) and math.isclose(ident, 20.4, rel_tol=1e-6)


def test_network_function_invariant_under_edge_permutations():
    """Parent's filter order = child's channel order leaves the network output unchanged (Section 3.4)."""
    x = W.uniform_activation(271, (1, 4, 4, 8))
    w1, b1 = W.he_weights(272, 16, 1, 1, 8), W.small_bias(273, 16)
    w2, b2 = W.he_weights(274, 8, 1, 1, 16), W.small_bias(275, 8)
    h, _ = R.conv_nhwc(x, w1, b1, act=R.ACT_RELU)
    y, bound = R.conv_nhwc(h, w2, b2)
    p = W.random_permutation(276, 16)
    ones1, ones2 = np.ones((4, 2), np.uint8), np.ones((2, 4), np.uint8)
    hp, _ = R.sparse_conv_reference(x, w1, ones1, 4, 4, bias=b1, perm_out=p, act=R.ACT_RELU)
    yp, _ = R.sparse_conv_reference(hp, w2, ones2, 4, 4, bias=b2, perm_in=p)
    assert np.array_equal(hp, h[..., p])
    assert np.all(np.abs(yp.astype(np.float64) - y) <= 1e-6 * bound + 1e-12)
