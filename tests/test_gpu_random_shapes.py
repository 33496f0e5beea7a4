"""Randomised parity run (gpu): seeded random layer shapes, group sizes, sparsities, strides and
permutations inside the documented limits, every kernel form forced in turn, each output compared
with the CPU oracle element by element."""
import numpy as np
import pytest
import torch

import paper_2310_19509_amd as S
from oracle import reference as R
from helpers import assert_within_bound

pytestmark = pytest.mark.gpu

FORMS = {S.SBN_CONV1X1: [0, 11, 12, 14, 21, 22, 112, 121, 504, 508, 516, 1012, 1021, 1112, 1121], S.SBN_CONV3X3: [0, 1, 2, 3, 32]}


def random_case(rng):
    kind = int(rng.choice([S.SBN_CONV1X1, S.SBN_CONV3X3]))
    go, gi = int(rng.choice([4, 8])), int(rng.choice([1, 2, 4, 8]))
    K = int(rng.integers(1, 40)) * 8                       # 8 .. 312: one to ten 32-channel sub-chunks
    if kind == S.SBN_CONV1X1 and rng.random() < 0.2:
        K = int(rng.integers(1, 20)) * gi                  # 1x1 also takes channel counts that are not multiples of 4
    N = int(rng.integers(1, 30)) * 8
    n, h, w = int(rng.integers(1, 4)), int(rng.integers(1, 24)), int(rng.integers(1, 40))
    stride = int(rng.choice([1, 1, 2])) if kind == S.SBN_CONV3X3 else 1
    pct = int(rng.choice([0, 30, 50, 70, 90, 97, 100]))
    return dict(kind=kind, go=go, gi=gi, K=K, N=N, n=n, h=h, w=w, stride=stride, pct=pct,
                bias=rng.random() < 0.7, relu=rng.random() < 0.5, perms=rng.random() < 0.5)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_layers_every_form(seed):
    rng = np.random.default_rng(seed)
    try:
        for _ in range(60):
            c = random_case(rng)
            kind, K, N, k = c["kind"], c["K"], c["N"], 1 if c["kind"] == S.SBN_CONV1X1 else 3
            wt = (rng.standard_normal((N, k, k, K)) * (2.0 / (K * k * k)) ** 0.5).astype(np.float32)
            b = (rng.standard_normal(N) * 0.2).astype(np.float32) if c["bias"] else None
            x = rng.uniform(-1, 1, (c["n"], c["h"], c["w"], K)).astype(np.float32)
            po = rng.permutation(N).astype(np.int32) if c["perms"] else None
            pi = rng.permutation(K).astype(np.int32) if c["perms"] else None
            wp = R.permute_weights(wt, po, pi)
            mask = S.sbn_prune_magnitude(wp, kind, c["go"], c["gi"], c["pct"])
            assert np.array_equal(mask, R.prune_mask(wp, c["go"], c["gi"], c["pct"])), c
            act = S.SBN_ACT_RELU if c["relu"] else S.SBN_ACT_NONE
            p = S.sbn_pack(kind, wt, c["go"], c["gi"], mask=mask, bias=b, perm_out=po, perm_in=pi,
                           stride=c["stride"], act=act)
            ref, bound = R.sparse_conv_reference(x, wt, mask, c["go"], c["gi"], bias=b, perm_out=po, perm_in=pi,
                                                 stride=c["stride"], pad=k // 2, act=act)
            xd = torch.from_numpy(x).cuda()
            run = S.sbn_conv1x1_sparse if kind == S.SBN_CONV1X1 else S.sbn_conv3x3_sparse
            for form in FORMS[kind]:
                S.sbn_force_kernel_form(kind, form)
                yd = torch.full(ref.shape, float("nan"), device="cuda")
                run(p, xd, yd, c["n"], c["h"], c["w"])
                torch.cuda.synchronize()
                assert_within_bound(yd.cpu().numpy(), ref, bound, f"form {form} of {c}")
            S.sbn_force_kernel_form(kind, 0)
    finally:
        S.sbn_force_kernel_form(S.SBN_CONV1X1, 0)
        S.sbn_force_kernel_form(S.SBN_CONV3X3, 0)


@pytest.mark.parametrize("seed", [21, 22])
def test_random_depthwise_plus_pointwise_pairs(seed):
    """Random (depthwise 3x3, small 1x1) pairs through the chain: the fused launch and the two separate
    launches both within the two-layer tolerance of the oracle (|err| <= 1e-4 (bound_pw + |W| bound_dw))."""
    rng = np.random.default_rng(seed)
    for _ in range(25):
        K, N = int(rng.choice([32, 64, 96, 128])), int(rng.integers(1, 17)) * 8
        n, h, w = int(rng.integers(1, 4)), int(rng.integers(1, 30)), int(rng.integers(1, 30))
        stride, pct = int(rng.choice([1, 2])), int(rng.choice([0, 30, 50, 70, 90, 100]))
        act_dw = S.SBN_ACT_RELU if rng.random() < 0.8 else S.SBN_ACT_NONE
        act_pw = S.SBN_ACT_RELU if rng.random() < 0.5 else S.SBN_ACT_NONE
        dw_w = (rng.standard_normal((K, 3, 3)) * 0.4).astype(np.float32)
        dw_b = (rng.standard_normal(K) * 0.1).astype(np.float32) if rng.random() < 0.8 else None
        wt = (rng.standard_normal((N, 1, 1, K)) * (2.0 / K) ** 0.5).astype(np.float32)
        b = (rng.standard_normal(N) * 0.1).astype(np.float32)
        po = rng.permutation(N).astype(np.int32) if rng.random() < 0.5 else None
        mask = S.sbn_prune_magnitude(R.permute_weights(wt, po, None), S.SBN_CONV1X1, 4, 4, pct)
        p = S.sbn_pack(S.SBN_CONV1X1, wt, 4, 4, mask=mask, bias=b, perm_out=po, act=act_pw)
        chain = S.sbn_chain_create([S.dw_item(dw_w, dw_b, stride=stride, act=act_dw), S.sparse_item(p)])
        oh, ow, oc = S.sbn_chain_output_shape(chain, n, h, w)
        ws = torch.empty(S.sbn_chain_workspace(chain, n, h, w) // 4, device="cuda")
        x = rng.uniform(-1, 1, (n, h, w, K)).astype(np.float32)
        xd = torch.from_numpy(x).cuda()
        mid, bound_dw = R.dwconv3x3_nhwc(x, dw_w, dw_b, stride=stride, act=act_dw)
        ref, bound_pw = R.sparse_conv_reference(mid, wt, mask, 4, 4, bias=b, perm_out=po, act=act_pw)
        wm = np.abs(R.apply_mask(R.permute_weights(wt, po, None), mask, 4, 4).reshape(N, K).astype(np.float64))
        bound = bound_pw + (bound_dw.reshape(-1, K) @ wm.T).reshape(bound_pw.shape)
        for fused in (True, False):
            S.sbn_chain_set_fusion(chain, fused)
            yd = torch.full((n, oh, ow, oc), float("nan"), device="cuda")
            S.sbn_pointwise_chain(chain, xd, yd, n, h, w, ws)
            torch.cuda.synchronize()
            assert_within_bound(yd.cpu().numpy(), ref, bound,
                                f"fused={fused} n,h,w={n,h,w} K={K} N={N} stride={stride} pct={pct}")
