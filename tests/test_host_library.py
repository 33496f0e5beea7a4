"""Host-side library code (prune, pack, unpack, export, rearrange, argument
checks) against the numpy oracle, bit-exact.  Runs without a GPU: layers are
packed with device = -1."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

import paper_2310_19509_amd as S
from paper_2310_19509_amd import _lib
from oracle import reference as R
import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "sbn.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(sbn_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(_lib.SYMBOLS), declared ^ set(_lib.SYMBOLS)
    lib = C.CDLL(_lib.LIB_PATH)
    for name in declared:
        getattr(lib, name)
    _lib.lib()


@pytest.mark.parametrize("kind,go,gi,pct", [(S.SBN_CONV1X1, 4, 4, 30), (S.SBN_CONV1X1, 8, 4, 50),
                                           (S.SBN_CONV1X1, 4, 1, 70), (S.SBN_CONV3X3, 4, 4, 70),
                                           (S.SBN_CONV1X1, 4, 8, 90), (S.SBN_CONV1X1, 4, 2, 0),
                                           (S.SBN_CONV3X3, 8, 2, 100)])
def test_prune_matches_oracle_bit_exact(kind, go, gi, pct):
    k = 3 if kind == S.SBN_CONV3X3 else 1
    w = W.he_weights(301, 64, k, k, 48)
    m = S.sbn_prune_magnitude(w, kind, go, gi, pct)
    assert np.array_equal(m, R.prune_mask(w, go, gi, pct))
    assert math.isclose(S.sbn_retained_l1(w, kind, go, gi, pct), R.retained_l1(w, go, gi, pct), rel_tol=1e-12)


def test_prune_ties_lower_index_first():
    w = np.ones((8, 1, 1, 8), dtype=np.float32)
    assert S.sbn_prune_magnitude(w, S.SBN_CONV1X1, 4, 4, 50).ravel().tolist() == [0, 0, 1, 1]


@pytest.mark.parametrize("kind,go,gi,pct", [(S.SBN_CONV1X1, 4, 4, 50), (S.SBN_CONV1X1, 8, 4, 30),
                                           (S.SBN_CONV1X1, 4, 1, 50), (S.SBN_CONV1X1, 8, 8, 70),
                                           (S.SBN_CONV1X1, 4, 2, 50), (S.SBN_CONV3X3, 4, 4, 70),
                                           (S.SBN_CONV3X3, 8, 1, 50), (S.SBN_CONV1X1, 4, 4, 100)])
def test_pack_export_unpack_bit_exact(kind, go, gi, pct):
    k = 3 if kind == S.SBN_CONV3X3 else 1
    w = W.he_weights(311, 48, k, k, 40)
    w[5, 0, 0, 7] = np.float32(-0.0)
    w[6, 0, 0, 3] = np.float32(1e-42)
    b = W.small_bias(312, 48)
    po, pi = W.random_permutation(313, 48), W.random_permutation(314, 40)
    wp = R.permute_weights(w, po, pi)
    mask = R.prune_mask(wp, go, gi, pct)
    p = S.sbn_pack(kind, w, go, gi, mask=mask, bias=b, perm_out=po, perm_in=pi, device=-1)
    ex = S.sbn_export(p)
    row_ptr, kidx, vals = R.canonical_pack(wp, mask, go, gi)
    assert np.array_equal(ex["row_ptr"], row_ptr) and np.array_equal(ex["kidx"], kidx)
    assert np.array_equal(ex["vals"].view(np.uint32), vals.view(np.uint32))
    assert np.array_equal(ex["perm_out"], po) and np.array_equal(ex["perm_in"], pi)
    assert np.array_equal(ex["bias"], b[po])
    assert ex["nnz"] == int(mask.sum())
    wu, mu = S.sbn_unpack(p)
    assert np.array_equal(mu, mask)
    expect = R.unpermute_weights(R.apply_mask(wp, mask, go, gi), po, pi)
    assert np.array_equal(wu.view(np.uint32), expect.view(np.uint32))
    work = S.sbn_packed_work(p)
    assert work["nnz_blocks"] == ex["nnz"] and work["macs_per_pixel"] == ex["nnz"] * go * gi * k * k
    S.sbn_free(p)
    S.sbn_free(p)      # idempotent through the binding


def test_pack_with_implied_mask():
    w = W.he_weights(321, 16, 1, 1, 16)
    m = R.prune_mask(w, 4, 4, 50)
    wt = R.apply_mask(w, m, 4, 4)
    wt[0, 0, 0, 0] = np.float32(-0.0) if m[0, 0] == 0 else wt[0, 0, 0, 0]
    p = S.sbn_pack(S.SBN_CONV1X1, wt, 4, 4, device=-1)
    _, mu = S.sbn_unpack(p)
    assert np.array_equal(mu, R.nonzero_block_mask(wt, 4, 4))


def test_config1_pack_counts():
    c = W.config1()
    p = S.sbn_pack(S.SBN_CONV1X1, c["w"], 4, 4, mask=c["mask"], device=-1)
    assert S.sbn_export(p)["nnz"] == 256


def _err(fn, code):
    with pytest.raises(S.SbnError) as ei:
        fn()
    assert ei.value.code == code, str(ei.value)
    assert S.sbn_last_error() != ""


def test_argument_errors():
    w = W.he_weights(331, 16, 1, 1, 16)
    _err(lambda: S.sbn_pack(S.SBN_CONV1X1, w, 3, 4, device=-1), -1)
    _err(lambda: S.sbn_pack(S.SBN_CONV1X1, w[:, :, :, :14], 4, 4, device=-1), -2)
    _err(lambda: S.sbn_pack(S.SBN_CONV1X1, w[:14], 4, 4, device=-1), -2)
    _err(lambda: S.sbn_pack(S.SBN_CONV1X1, w, 4, 4, perm_out=np.zeros(16, np.int32), device=-1), -3)
    _err(lambda: S.sbn_pack(S.SBN_CONV1X1, w, 4, 4, perm_in=np.arange(16, dtype=np.int32) + 1, device=-1), -3)
    _err(lambda: S.sbn_pack(S.SBN_CONV1X1, w, 4, 4, stride=2, device=-1), -1)
    _err(lambda: S.sbn_pack(S.SBN_CONV1X1, w, 4, 4, act=7, device=-1), -1)
    _err(lambda: S.sbn_prune_magnitude(w, S.SBN_CONV1X1, 4, 4, 101), -1)
    _err(lambda: S.sbn_prune_magnitude(w, 2, 4, 4, 10), -1)
    p = S.sbn_pack(S.SBN_CONV1X1, w, 4, 4, device=-1)
    assert S.sbn_packed_info(p) == dict(kind=1, c_in=16, c_out=16, go=4, gi=4, stride=1, act=0, device=-1)
    # run call on a host-only layer: refused before anything touches a GPU
    rc = _lib.lib().sbn_conv1x1_sparse(p.handle, 16, 32, 1, 1, 1, None)
    assert rc == -6 and "device" in S.sbn_last_error()
    rc = _lib.lib().sbn_conv3x3_sparse(p.handle, 16, 32, 1, 1, 1, None)
    assert rc == -1
    assert _lib.lib().sbn_conv1x1_sparse(None, 16, 32, 1, 1, 1, None) == -1


def test_nonfinite_weights_and_device_3x3_channel_rule_are_refused():
    """Importance has no order with NaN in it; a 3x3 layer packed for a device needs c_in % 4 == 0
    (refused at pack time, before any GPU call, so this runs without a GPU)."""
    w = W.he_weights(341, 16, 1, 1, 16)
    w[3, 0, 0, 5] = np.nan
    _err(lambda: S.sbn_prune_magnitude(w, S.SBN_CONV1X1, 4, 4, 30), -1)
    _err(lambda: S.sbn_retained_l1(w, S.SBN_CONV1X1, 4, 4, 30), -1)
    w[3, 0, 0, 5] = np.inf
    _err(lambda: S.sbn_prune_magnitude(w, S.SBN_CONV1X1, 4, 4, 30), -1)
    w3 = W.he_weights(342, 8, 3, 3, 6)
    _err(lambda: S.sbn_pack(S.SBN_CONV3X3, w3, 4, 2, device=0), -2)
    assert "multiple of 4" in S.sbn_last_error()
    p = S.sbn_pack(S.SBN_CONV3X3, w3, 4, 2, device=-1)          # host-only packing has no such limit
    wt, _ = S.sbn_unpack(p)
    assert np.array_equal(wt.view(np.uint32), w3.view(np.uint32))


def test_packed_layout_reports_entries_and_every_piece_tables():
    """Entries = (bundle of 16 filters, 4-channel piece) pairs with a kept block, counted here from
    the oracle's mask; the every-piece tables exist for 1x1 layers of more than 64 input channels
    that keep at least 60 % of those pairs."""
    w = W.he_weights(331, 64, 1, 1, 128)
    for pct, expect in ((0, True), (50, True), (70, True), (90, False)):
        mask = S.sbn_prune_magnitude(w, S.SBN_CONV1X1, 4, 4, pct)
        lay = S.sbn_packed_layout(S.sbn_pack(S.SBN_CONV1X1, w, 4, 4, mask=mask, device=-1))
        m = R.prune_mask(w, 4, 4, pct).astype(bool)
        entries = sum(int(m[b:b + 4].any(axis=0).sum()) for b in range(0, m.shape[0], 4))
        assert lay["entries"] == entries
        assert lay["every_piece"] == expect, (pct, entries, 4 * 32)
        assert lay["table_bytes"] > 0
    small = S.sbn_pack(S.SBN_CONV1X1, W.he_weights(332, 32, 1, 1, 64), 4, 4, device=-1)      # one chunk: no such tables
    assert not S.sbn_packed_layout(small)["every_piece"]
    k3 = S.sbn_pack(S.SBN_CONV3X3, W.he_weights(333, 16, 3, 3, 128), 4, 4, device=-1)
    assert not S.sbn_packed_layout(k3)["every_piece"]


# ---------------------------------------------------------------- rearrangement

def _layers(seed, chans, go=4, gi=4):
    return [dict(kind=S.SBN_CONV1X1, w=W.he_weights(seed + i, chans[i + 1], 1, 1, chans[i]), go=go, gi=gi)
            for i in range(len(chans) - 1)]


def test_rearrange_valid_canonical_monotone_deterministic():
    layers = _layers(341, [16, 32, 64, 32])
    parent = [-1, 0, 1]
    perms = S.sbn_rearrange(layers, parent, 50, seed=7, max_iters=400, keep_output_order=[0, 0, 1])
    again = S.sbn_rearrange(layers, parent, 50, seed=7, max_iters=400, keep_output_order=[0, 0, 1])
    for p, q in zip(perms, again):
        assert np.array_equal(p, q)
    assert np.array_equal(perms[2], np.arange(32))
    pin = None
    improved = 0
    for l, p in zip(layers, perms):
        n = l["w"].shape[0]
        assert R.is_permutation(p, n)
        assert np.array_equal(R.canonicalize(p, 4), p)
        base = R.retained_l1(R.permute_weights(l["w"], None, pin), 4, 4, 50)
        got = R.retained_l1(R.permute_weights(l["w"], p, pin), 4, 4, 50)
        assert got >= base * (1 - 1e-12)
        improved += got > base * (1 + 1e-9)
        pin = p
    assert improved >= 2


def test_rearrange_exhaustive_equals_brute_force_optimum():
    """c_out <= 8: every canonical grouping is tried (Section 3.4's canonical form)."""
    for seed, go, gi in ((351, 4, 4), (352, 4, 2)):
        w = W.he_weights(seed, 8, 1, 1, 8)
        perm = S.sbn_rearrange([dict(kind=S.SBN_CONV1X1, w=w, go=go, gi=gi)], [-1], 50)[0]
        best, obj = R.best_row_grouping(w, go, gi, 50)
        assert np.array_equal(perm, best)
        assert math.isclose(R.retained_l1(w[perm], go, gi, 50), obj, rel_tol=1e-12)


def test_rearrange_exhaustive_reaches_to_twelve_filters():
    """12 filters in groups of 4 (5 775 canonical groupings) and 16 in groups of 8 (6 435) are
    still enumerated: the result is the oracle's brute-force optimum."""
    for seed, n, go, pct in ((353, 12, 4, 30), (354, 12, 4, 70), (355, 16, 8, 50)):
        w = W.he_weights(seed, n, 1, 1, 16)
        perm = S.sbn_rearrange([dict(kind=S.SBN_CONV1X1, w=w, go=go, gi=4)], [-1], pct)[0]
        best, obj = R.best_row_grouping(w, go, 4, pct)
        assert np.array_equal(perm, best)
        assert math.isclose(R.retained_l1(w[perm], go, 4, pct), obj, rel_tol=1e-12)


def _tiny_residual_graph(seed):
    """x (8 ch) -> conv_a -> u (8 ch) -> conv_b -> y (8 ch), out = y + x: the skip connection makes
    tensor y carry the order of tensor x, i.e. conv_b writes the tensor conv_a reads."""
    wa, wb = W.he_weights(seed, 8, 1, 1, 8), W.he_weights(seed + 1, 8, 1, 1, 8)
    layers = [dict(kind=S.SBN_CONV1X1, w=wa, go=4, gi=4), dict(kind=S.SBN_CONV1X1, w=wb, go=4, gi=4)]
    return layers, [0, 1], [1, 0]             # tensor 0 = x = y's order class, tensor 1 = u


def test_rearrange_graph_residual_block_keeps_the_function_and_finds_the_joint_optimum():
    layers, tin, tout = _tiny_residual_graph(371)
    perms = S.sbn_rearrange_graph(layers, tin, tout, 2, 50, seed=3, max_iters=200)
    p0, p1 = perms
    assert R.is_permutation(p0, 8) and R.is_permutation(p1, 8)
    # tensor 0 is decided first: its only writer conv_b still has its channels in original order
    # then; 8 filters are enumerated, so the result is the brute-force optimum of that problem
    best0, _ = R.best_row_grouping(layers[1]["w"], 4, 4, 50)
    assert np.array_equal(p0, best0)
    # tensor 1: its writer conv_a reads tensor 0, already decided
    wa_cols = R.permute_weights(layers[0]["w"], None, p0)
    best1, _ = R.best_row_grouping(wa_cols, 4, 4, 50)
    assert np.array_equal(p1, best1)
    # the block's function: out = conv_b(conv_a(x)) + x, evaluated in permuted channel space
    x = W.uniform_activation(372, (1, 3, 3, 8))
    u, _ = R.conv_nhwc(x, layers[0]["w"])
    y, _ = R.conv_nhwc(u, layers[1]["w"])
    ref = y.astype(np.float64) + x
    xp = x[..., p0]
    up, _ = R.conv_nhwc(xp, R.permute_weights(layers[0]["w"], p1, p0))
    yp, _ = R.conv_nhwc(up, R.permute_weights(layers[1]["w"], p0, p1))
    got = yp.astype(np.float64) + xp
    np.testing.assert_allclose(got, ref[..., p0], rtol=0, atol=1e-5)


def test_rearrange_graph_two_writers_share_one_order_maximising_the_sum():
    """Two branches summed into one tensor: one filter order for both, the one with the largest
    sum of retained importances (brute force over the 35 canonical groupings of 8 filters)."""
    w1, w2 = W.he_weights(381, 8, 1, 1, 8), W.he_weights(382, 8, 1, 1, 16)
    layers = [dict(kind=S.SBN_CONV1X1, w=w1, go=4, gi=4), dict(kind=S.SBN_CONV1X1, w=w2, go=4, gi=4)]
    perms = S.sbn_rearrange_graph(layers, [0, 1], [2, 2], 3, 50)
    assert np.array_equal(perms[0], np.arange(8)) and np.array_equal(perms[1], np.arange(16))   # network inputs
    best, best_obj = None, -1.0
    for g in R.canonical_groupings(8, 4):
        obj = R.retained_l1(w1[list(g)], 4, 4, 50) + R.retained_l1(w2[list(g)], 4, 4, 50)
        if obj > best_obj:
            best, best_obj = g, obj
    assert np.array_equal(perms[2], np.asarray(best, dtype=np.int32))
    with pytest.raises(S.SbnError):            # writers that disagree on the channel count
        S.sbn_rearrange_graph([layers[0], dict(kind=S.SBN_CONV1X1, w=W.he_weights(383, 16, 1, 1, 16), go=4, gi=4)],
                              [0, 1], [2, 2], 3, 50)


def test_rearrange_finds_planted_grouping():
    """Strong and weak filters interleaved: like must be grouped with like."""
    rng = np.random.default_rng(361)
    w = np.zeros((16, 1, 1, 8), dtype=np.float32)
    strong = [0, 3, 5, 6, 9, 10, 12, 15]
    for f in range(16):
        w[f] = (5.0 if f in strong else 0.05) * (1 + 0.01 * rng.standard_normal((1, 1, 8)))
    perm = S.sbn_rearrange([dict(kind=S.SBN_CONV1X1, w=w, go=4, gi=4)], [-1], 50, seed=1, max_iters=3000)[0]
    groups = perm.reshape(4, 4)
    kinds = sorted(sum(int(f in strong) for f in g) for g in groups)
    assert kinds == [0, 0, 4, 4]


def _bundle_unions(w_run, go, gi, pct):
    """Number of (bundle of 16 filters, 4-channel input piece) pairs with a kept block: what the
    device kernels walk.  From the oracle's mask."""
    m = R.prune_mask(w_run, go, gi, pct).astype(bool)
    c_in = w_run.shape[3]
    piece = np.zeros((m.shape[0], (c_in + 3) // 4), dtype=bool)
    for j in range(m.shape[1]):
        for ch in range(j * gi, (j + 1) * gi):
            piece[:, ch // 4] |= m[:, j]
    per = 16 // go
    return sum(int(piece[b:b + per].any(axis=0).sum()) for b in range(0, piece.shape[0], per))


def test_order_groups_keeps_the_grouping_and_shrinks_the_unions():
    layers = _layers(391, [32, 64, 128, 64])
    parent, keep = [-1, 0, 1], [0, 0, 1]
    perms = S.sbn_rearrange(layers, parent, 70, seed=5, max_iters=300, keep_output_order=keep)
    ordered = S.sbn_order_groups(layers, parent, 70, perms, keep_output_order=keep)
    again = S.sbn_order_groups(layers, parent, 70, perms, keep_output_order=keep)
    assert np.array_equal(ordered[2], np.arange(64))
    before = after = 0
    pin_a = pin_b = None
    for l, p, q, q2 in zip(layers, perms, ordered, again):
        assert np.array_equal(q, q2)
        assert R.is_permutation(q, l["w"].shape[0])
        # same groups (as sets), only their order differs
        assert np.array_equal(R.canonicalize(q, 4), R.canonicalize(p, 4))
        wa, wb = R.permute_weights(l["w"], p, pin_a), R.permute_weights(l["w"], q, pin_b)
        assert math.isclose(R.retained_l1(wa, 4, 4, 70), R.retained_l1(wb, 4, 4, 70), rel_tol=1e-12)
        before += _bundle_unions(wa, 4, 4, 70)
        after += _bundle_unions(wb, 4, 4, 70)
        pin_a, pin_b = p, q
    assert after < before


def test_order_groups_finds_planted_bundles():
    """Eight groups, alternately keeping the first and the second half of the input pieces: the
    groups of a kind belong in one bundle, which halves what a bundle walks."""
    rng = np.random.default_rng(392)
    w = (0.01 * rng.standard_normal((32, 1, 1, 64))).astype(np.float32)
    for g in range(8):
        half = slice(0, 32) if g % 2 == 0 else slice(32, 64)
        w[g * 4:(g + 1) * 4, :, :, half] += rng.choice([-1.0, 1.0], (4, 1, 1, 32)).astype(np.float32)
    layer = [dict(kind=S.SBN_CONV1X1, w=w, go=4, gi=4)]
    ident = [np.arange(32, dtype=np.int32)]
    assert _bundle_unions(w, 4, 4, 50) == 32
    q = S.sbn_order_groups(layer, [-1], 50, ident)[0]
    assert _bundle_unions(w[q], 4, 4, 50) == 16
    kinds = [sorted((int(f) // 4) % 2 for f in q[b:b + 16]) for b in (0, 16)]
    assert kinds[0][0] == kinds[0][-1] and kinds[1][0] == kinds[1][-1]


def test_order_groups_moves_whole_blocks_of_the_readers():
    """A reader with 8-channel blocks: filters move in runs of 8, so its blocks (hence its mask and
    retained importance) stay what they were."""
    w0, w1 = W.he_weights(393, 64, 1, 1, 32), W.he_weights(394, 32, 1, 1, 64)
    layers = [dict(kind=S.SBN_CONV1X1, w=w0, go=4, gi=4), dict(kind=S.SBN_CONV1X1, w=w1, go=4, gi=8)]
    ident = [np.arange(64, dtype=np.int32), np.arange(32, dtype=np.int32)]
    q = S.sbn_order_groups(layers, [-1, 0], 60, ident, keep_output_order=[0, 1])
    runs = q[0].reshape(8, 8)
    assert np.array_equal(runs, runs[:, :1] + np.arange(8)) and np.all(runs[:, 0] % 8 == 0)
    assert not np.array_equal(q[0], ident[0])
    assert math.isclose(R.retained_l1(R.permute_weights(w1, None, q[0]), 4, 8, 60), R.retained_l1(w1, 4, 8, 60), rel_tol=1e-12)
    # graph form, two writers of one tensor: same result as the chain form for a single writer
    g = S.sbn_order_groups_graph(layers, [2, 0], [0, 1], 3, 60, [ident[0], ident[1], np.arange(32, dtype=np.int32)],
                                 tensor_fixed=[0, 1, 1])
    assert np.array_equal(g[0], q[0]) and np.array_equal(g[1], ident[1])
    bad = [np.zeros(64, dtype=np.int32), ident[1]]
    _err(lambda: S.sbn_order_groups(layers, [-1, 0], 60, bad), -3)


def test_rearrange_errors():
    layers = _layers(371, [16, 32, 16])
    _err(lambda: S.sbn_rearrange(layers, [-1, 1], 50), -2)
    _err(lambda: S.sbn_rearrange(layers, [-1, 0], 150), -1)
    bad = [layers[0], dict(kind=S.SBN_CONV1X1, w=W.he_weights(372, 16, 1, 1, 24), go=4, gi=4)]
    _err(lambda: S.sbn_rearrange(bad, [-1, 0], 50), -2)


# ---- 3:9 pattern group pruning of depthwise kernels (Section 3.2, DwConv3x3)

@pytest.mark.parametrize("c,go", [(32, 16), (24, 16), (28, 16), (12, 16), (24, 8), (4, 16), (40, 4)])
def test_dw_pattern_groups_match_the_oracle(c, go):
    want = R.dw_pattern_groups(c, go)
    got = S.sbn_dw_pattern_groups(c, go)
    assert got.tolist() == [g[0] for g in want] + [c]


@pytest.mark.parametrize("c,go,seed", [(64, 16, 1), (40, 16, 2), (28, 16, 3), (32, 8, 4), (16, 4, 5)])
def test_dw_pattern_select_and_apply_bit_exact(c, go, seed):
    w = W.normal_weights(7700 + seed, (c, 3, 3), 0.4)
    w[1, 2, 0] = -0.0
    n_groups = len(R.dw_pattern_groups(c, go))
    dense = (1,) if n_groups > 1 else ()
    kd = np.zeros(n_groups, np.uint8)
    kd[list(dense)] = 1
    want = R.dw_pattern_select(w, go, dense_groups=dense)
    got = S.sbn_dw_pattern_select(w, go, keep_dense=kd)
    assert got.tolist() == want.tolist()
    wm = S.sbn_dw_pattern_apply(w, got, go)
    assert np.array_equal(wm.view(np.uint32), R.dw_pattern_apply(w, want, go).view(np.uint32))


def test_dw_pattern_ties_take_the_lowest_id():
    w = np.ones((16, 3, 3), dtype=np.float32)
    assert S.sbn_dw_pattern_select(w, 16).tolist() == [0] == R.dw_pattern_select(w, 16).tolist()


def test_dw_pattern_errors():
    w = np.zeros((6, 3, 3), np.float32)
    with pytest.raises(S.SbnError):
        S.sbn_dw_pattern_select(w, 16)                       # 6 channels: not a multiple of 4
    with pytest.raises(S.SbnError):
        S.sbn_dw_pattern_groups(16, 5)                       # group size
    with pytest.raises(S.SbnError):
        S.sbn_dw_pattern_apply(np.zeros((16, 3, 3), np.float32), np.array([9], np.uint8), 16)


# ---- 4-of-9 pattern pruning inside kept 3x3 kernels (Section 3.2, Conv3x3)

def test_conv3x3_pattern_taps_match_the_oracle():
    for pid in list(range(S.SBN_K3_PATTERNS)) + [S.SBN_K3_PATTERN_DENSE]:
        want = sum(1 << t for t in range(9) if R.conv3x3_pattern_mask(pid).reshape(9)[t])
        assert S.sbn_conv3x3_pattern_taps(pid) == want
    assert S.SBN_K3_PATTERNS == R.K3_PATTERNS and S.SBN_K3_PATTERN_DENSE == R.K3_PATTERN_DENSE


@pytest.mark.parametrize("c_out,c_in,share,seed", [(8, 8, 4, 1), (8, 12, 2, 2), (12, 5, 1, 3), (16, 7, 4, 4)])
def test_conv3x3_pattern_select_and_apply_bit_exact(c_out, c_in, share, seed):
    w = W.normal_weights(7800 + seed, (c_out, 3, 3, c_in), 0.3)
    w[0, 1, 1, 0] = -0.0
    w[1, 0, 0, 1] = -0.0
    want = R.conv3x3_pattern_select(w, share)
    got = S.sbn_conv3x3_pattern_select(w, share)
    assert got.shape == want.shape and got.tolist() == want.tolist()
    got[0, 0] = S.SBN_K3_PATTERN_DENSE                   # a group left dense
    wm = S.sbn_conv3x3_pattern_apply(w, got, share)
    assert np.array_equal(wm.view(np.uint32), R.conv3x3_pattern_apply(w, got, share).view(np.uint32))
    kept = np.count_nonzero(wm.view(np.uint32) & 0x7FFFFFFF)
    assert kept <= 4 * c_out * c_in + 5 * share


def test_conv3x3_pattern_ties_and_errors():
    w = np.ones((4, 3, 3, 3), dtype=np.float32)
    assert S.sbn_conv3x3_pattern_select(w, 4).tolist() == [[0, 0, 0]] == R.conv3x3_pattern_select(w, 4).tolist()
    with pytest.raises(S.SbnError):
        S.sbn_conv3x3_pattern_select(w, 3)                   # share must be 4, 2 or 1
    with pytest.raises(S.SbnError):
        S.sbn_conv3x3_pattern_select(np.ones((6, 3, 3, 3), np.float32), 4)   # 6 filters, groups of 4
    with pytest.raises(S.SbnError):
        S.sbn_conv3x3_pattern_apply(w, np.full((1, 3), 57, np.uint8), 4)
    with pytest.raises(S.SbnError):
        S.sbn_conv3x3_pattern_taps(57)


def test_force_kernel_form_validates_its_arguments():
    S.sbn_force_kernel_form(S.SBN_CONV1X1, 21)
    S.sbn_force_kernel_form(S.SBN_CONV1X1, 0)
    S.sbn_force_kernel_form(S.SBN_CONV3X3, 2)
    S.sbn_force_kernel_form(S.SBN_CONV3X3, 0)
    for kind, form in [(S.SBN_CONV1X1, 13), (S.SBN_CONV3X3, 4), (S.SBN_CONV3X3, -1), (99, 0)]:
        with pytest.raises(S.SbnError):
            S.sbn_force_kernel_form(kind, form)
