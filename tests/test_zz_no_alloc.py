"""sbn_pointwise_chain_static (the chain run for callers that cannot allocate: its intermediate
activations live in a fixed array inside the library) against sbn_pointwise_chain with a
caller-provided workspace, through the C ABI: same kernels, same launch order, so the outputs
must be identical bit for bit; both are also held to the oracle's bound.  Two calls in a row, the
second on a smaller input (what the first call left in the array must not matter), then the size
limit."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2310_19509_amd as S
from paper_2310_19509_amd import _lib
from oracle import reference as R
import workloads as W
from helpers import assert_within_bound

pytestmark = pytest.mark.gpu


def _chain():
    chans, strides = [16, 32, 64, 24], [1, 2, 1]
    pws = [W.he_weights(9700 + i, chans[i + 1], 1, 1, chans[i]) for i in range(3)]
    items, meta = [], []
    for i in range(3):
        dw_w, dw_b = W.normal_weights(9710 + i, (chans[i], 3, 3), 0.4), W.small_bias(9720 + i, chans[i])
        items.append(S.dw_item(dw_w, dw_b, stride=strides[i], act=S.SBN_ACT_RELU))
        meta.append(("dw", dw_w, dw_b, strides[i]))
        b = W.small_bias(9730 + i, chans[i + 1])
        mask = S.sbn_prune_magnitude(pws[i], S.SBN_CONV1X1, 4, 4, 50)
        items.append(S.sparse_item(S.sbn_pack(S.SBN_CONV1X1, pws[i], 4, 4, mask=mask, bias=b, act=S.SBN_ACT_RELU)))
        meta.append(("pw", pws[i], b, mask))
    return S.sbn_chain_create(items), meta, chans


def _oracle_last_item(meta, x_in):
    """The last item (a pointwise layer) on the GPU's own input to it."""
    _, w, b, mask = meta[-1]
    return R.sparse_conv_reference(x_in, w, mask, 4, 4, bias=b, act=R.ACT_RELU)


def test_static_workspace_chain_matches_the_workspace_call_twice_in_a_row():
    chain, meta, chans = _chain()
    lib = _lib.lib()
    st = torch.cuda.current_stream().cuda_stream
    for call, (n, hw) in enumerate([(3, 20), (1, 9)]):          # the second call is the smaller one
        x = torch.from_numpy(W.uniform_activation(9750 + call, (n, hw, hw, chans[0]))).cuda()
        oh, ow, oc = S.sbn_chain_output_shape(chain, n, hw, hw)
        ws = torch.empty(S.sbn_chain_workspace(chain, n, hw, hw) // 4, device="cuda")
        y_ws = torch.full((n, oh, ow, oc), float("nan"), device="cuda")
        y_st = torch.full((n, oh, ow, oc), float("nan"), device="cuda")
        # the input of the last item, copied out by both calls
        tap_shape = (n, oh, ow, chans[-2])
        tap_ws = torch.full(tap_shape, float("nan"), device="cuda")
        tap_st = torch.full(tap_shape, float("nan"), device="cuda")
        n_items = len(meta)
        lo_ws = (C.c_void_p * n_items)(*([None] * (n_items - 2) + [tap_ws.data_ptr(), None]))
        lo_st = (C.c_void_p * n_items)(*([None] * (n_items - 2) + [tap_st.data_ptr(), None]))
        print(f"call {call}: n={n} hw={hw}", flush=True)
        rc = lib.sbn_pointwise_chain(chain.handle, x.data_ptr(), y_ws.data_ptr(), n, hw, hw, ws.data_ptr(),
                                     ws.numel() * 4, lo_ws, st)
        assert rc == 0, S.sbn_last_error()
        rc = lib.sbn_pointwise_chain_static(chain.handle, x.data_ptr(), y_st.data_ptr(), n, hw, hw, lo_st, st)
        assert rc == 0, S.sbn_last_error()
        torch.cuda.synchronize()
        assert torch.equal(y_st, y_ws), "static-workspace call differs from the workspace call"
        assert torch.equal(tap_st, tap_ws)
        ref, bound = _oracle_last_item(meta, tap_st.cpu().numpy())
        assert_within_bound(y_st.cpu().numpy(), ref, bound, f"static chain, call {call}")


def test_static_workspace_chain_refuses_inputs_beyond_its_limit():
    chain, _, chans = _chain()
    n, hw = 64, 112                                   # 64 x 112 x 112 x 32 floats per intermediate: far too large
    assert S.sbn_chain_workspace(chain, n, hw, hw) > S.SBN_STATIC_WORKSPACE_BYTES
    x = torch.zeros(16, device="cuda")                # never read: the call is refused before any launch
    rc = _lib.lib().sbn_pointwise_chain_static(chain.handle, x.data_ptr(), x.data_ptr(), n, hw, hw, None, None)
    assert rc == -1 and "built-in workspace" in S.sbn_last_error()
