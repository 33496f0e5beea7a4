"""Property tests of the offline host calls over random layer geometries (hypothesis): the
library's mask, canonical arrays and round trip must equal the numpy oracle's bit for bit, and the
canonical arrays must keep their structural invariants (Algorithm 1's per-row start-channel lists)."""
import numpy as np
from hypothesis import HealthCheck, given, settings, strategies as st

import paper_2310_19509_amd as S
from oracle import reference as R


@st.composite
def layers(draw):
    kind = draw(st.sampled_from([S.SBN_CONV1X1, S.SBN_CONV3X3]))
    go = draw(st.sampled_from([4, 8]))
    gi = draw(st.sampled_from([1, 2, 4, 8]))
    c_out = go * draw(st.integers(1, 6))
    c_in = gi * draw(st.integers(1, 12))
    pct = draw(st.integers(0, 100))
    seed = draw(st.integers(0, 2 ** 31 - 1))
    perms = draw(st.booleans())
    return kind, go, gi, c_out, c_in, pct, seed, perms


@settings(max_examples=60, deadline=None, derandomize=True, database=None, suppress_health_check=[HealthCheck.too_slow])
@given(layers())
def test_prune_pack_export_unpack_agree_with_the_oracle(layer):
    kind, go, gi, c_out, c_in, pct, seed, perms = layer
    k = 3 if kind == S.SBN_CONV3X3 else 1
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((c_out, k, k, c_in)).astype(np.float32)
    w[rng.random(w.shape) < 0.05] = 0.0                        # some exact zeros and ties
    b = rng.standard_normal(c_out).astype(np.float32)
    po = rng.permutation(c_out).astype(np.int32) if perms else None
    pi = rng.permutation(c_in).astype(np.int32) if perms else None
    wp = R.permute_weights(w, po, pi)

    mask = S.sbn_prune_magnitude(wp, kind, go, gi, pct)
    assert np.array_equal(mask, R.prune_mask(wp, go, gi, pct))
    n_blocks = (c_out // go) * (c_in // gi)
    assert int(mask.sum()) == n_blocks - n_blocks * pct // 100

    p = S.sbn_pack(kind, w, go, gi, mask=mask, bias=b, perm_out=po, perm_in=pi, device=-1)
    ex = S.sbn_export(p)
    row_ptr, kidx, vals = R.canonical_pack(wp, mask, go, gi)
    assert np.array_equal(ex["row_ptr"], row_ptr) and np.array_equal(ex["kidx"], kidx)
    assert np.array_equal(ex["vals"].view(np.uint32), vals.view(np.uint32))
    # structure: rows monotone, last = nnz, start channels ascending inside a row and multiples of gi
    assert ex["row_ptr"][0] == 0 and ex["row_ptr"][-1] == ex["nnz"] == int(mask.sum())
    assert np.all(np.diff(ex["row_ptr"].astype(np.int64)) >= 0)
    for r in range(c_out // go):
        ks = ex["kidx"][ex["row_ptr"][r]:ex["row_ptr"][r + 1]].astype(np.int64)
        assert np.all(np.diff(ks) > 0) and np.all(ks % gi == 0) and np.all(ks < c_in)
    wu, mu = S.sbn_unpack(p)
    assert np.array_equal(mu, mask)
    expect = R.unpermute_weights(R.apply_mask(wp, mask, go, gi), po, pi)
    assert np.array_equal(wu.view(np.uint32), expect.view(np.uint32))
    S.sbn_free(p)
