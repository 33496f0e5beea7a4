"""Argument marshalling for the C ABI (include/sbn.h).  No arithmetic here."""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence

import numpy as np

from . import _lib
from ._lib import ChainItem, LayerDesc

__all__ = [
    "SBN_CONV1X1", "SBN_CONV3X3", "SBN_ACT_NONE", "SBN_ACT_RELU",
    "SBN_ITEM_SPARSE", "SBN_ITEM_DW3X3", "SBN_ITEM_AVGPOOL", "SbnError", "Packed", "Chain",
    "sbn_last_error", "sbn_prune_magnitude", "sbn_retained_l1", "sbn_rearrange", "sbn_rearrange_graph", "sbn_order_groups", "sbn_order_groups_graph", "sbn_packed_layout", "sbn_pack", "sbn_unpack",
    "sbn_export", "sbn_packed_info", "sbn_packed_work", "sbn_free", "sbn_conv1x1_sparse", "sbn_conv3x3_sparse",
    "sbn_chain_create", "sbn_chain_workspace", "sbn_chain_output_shape", "sbn_pointwise_chain", "sbn_pointwise_chain_static",
    "SBN_STATIC_WORKSPACE_BYTES", "sbn_chain_free",
    "sbn_copy_bytes", "sbn_roof_mfma", "sbn_roof_lds", "sbn_roof_read", "dw_item", "sparse_item", "avgpool_item", "stem_item", "SBN_ITEM_STEM3X3",
    "SBN_DW_PATTERN_DENSE", "sbn_dw_pattern_groups", "sbn_dw_pattern_select", "sbn_dw_pattern_apply",
    "sbn_force_kernel_form", "sbn_chain_set_fusion", "sbn_chain_set_multi_layer", "sbn_chain_check", "SBN_K3_PATTERNS", "SBN_K3_PATTERN_DENSE", "sbn_conv3x3_pattern_taps", "sbn_conv3x3_pattern_select",
    "sbn_conv3x3_pattern_apply",
]

SBN_CONV1X1, SBN_CONV3X3 = 1, 3
SBN_ACT_NONE, SBN_ACT_RELU = 0, 1
SBN_ITEM_SPARSE, SBN_ITEM_DW3X3, SBN_ITEM_AVGPOOL, SBN_ITEM_STEM3X3 = 1, 2, 3, 4
SBN_DW_PATTERN_DENSE = 8
SBN_K3_PATTERNS = 56
SBN_K3_PATTERN_DENSE = 56


class SbnError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"sbn error {code}: {text}")
        self.code = code


def sbn_last_error() -> str:
    return _lib.lib().sbn_last_error().decode()


def _check(rc: int) -> None:
    if rc != 0:
        raise SbnError(rc, sbn_last_error())


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _dev_ptr(t) -> Optional[int]:
    """Device address of a torch tensor (or a raw int address / None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_cuda and t.is_contiguous() and t.dtype.is_floating_point and t.element_size() == 4
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _taps(kind: int) -> int:
    return 9 if kind == SBN_CONV3X3 else 1


class Packed:
    """Owner of an sbn_packed_t*; freed on garbage collection or by sbn_free."""

    def __init__(self, handle: int):
        self.handle = handle

    def __del__(self):
        try:
            sbn_free(self)
        except Exception:
            pass


class Chain:
    def __init__(self, handle: int, keep, n_items: int = 0, c_in: int = 0):
        self.handle = handle
        self._keep = keep
        self.n_items = n_items
        self.c_in = c_in

    def __del__(self):
        try:
            sbn_chain_free(self)
        except Exception:
            pass


def _desc(kind, w, go, gi, mask=None, bias=None, perm_out=None, perm_in=None, stride=1, pad=None,
          act=SBN_ACT_NONE):
    w = _f32(w)
    c_out, kh, kw, c_in = w.shape
    assert kh == kw == (3 if kind == SBN_CONV3X3 else 1)
    keep = [w]
    d = LayerDesc()
    d.kind, d.c_in, d.c_out, d.go, d.gi = kind, c_in, c_out, go, gi
    d.stride = stride
    d.pad = (1 if kind == SBN_CONV3X3 else 0) if pad is None else pad
    d.act = act
    d.w = w.ctypes.data
    for name, arr, dt in (("mask", mask, np.uint8), ("bias", bias, np.float32),
                          ("perm_out", perm_out, np.int32), ("perm_in", perm_in, np.int32)):
        if arr is not None:
            a = np.ascontiguousarray(arr, dtype=dt)
            keep.append(a)
            setattr(d, name, a.ctypes.data)
    return d, keep


def sbn_prune_magnitude(w_permuted, kind: int, go: int, gi: int, sparsity_percent: int) -> np.ndarray:
    w = _f32(w_permuted)
    c_out, _, _, c_in = w.shape
    mask = np.empty((max(c_out // go, 0), max(c_in // gi, 0)), dtype=np.uint8)
    _check(_lib.lib().sbn_prune_magnitude(w.ctypes.data, kind, c_in, c_out, go, gi, sparsity_percent,
                                          mask.ctypes.data))
    return mask


def sbn_retained_l1(w_permuted, kind: int, go: int, gi: int, sparsity_percent: int) -> float:
    w = _f32(w_permuted)
    c_out, _, _, c_in = w.shape
    out = C.c_double()
    _check(_lib.lib().sbn_retained_l1(w.ctypes.data, kind, c_in, c_out, go, gi, sparsity_percent, C.byref(out)))
    return out.value


def sbn_dw_pattern_groups(c: int, go: int = 16) -> np.ndarray:
    """First channel of every 3:9 pattern group of a depthwise layer, plus c at the end."""
    n = C.c_int()
    start = np.zeros(c // 4 + 2, dtype=np.int32)
    _check(_lib.lib().sbn_dw_pattern_groups(c, go, C.byref(n), start.ctypes.data))
    return start[:n.value + 1].copy()


def sbn_dw_pattern_select(w, go: int = 16, keep_dense=None) -> np.ndarray:
    """w [c][3][3] in the order the layer runs in -> uint8 pattern id per group."""
    w = _f32(w)
    c = w.shape[0]
    n = len(sbn_dw_pattern_groups(c, go)) - 1
    kd = None if keep_dense is None else np.ascontiguousarray(keep_dense, dtype=np.uint8)
    if kd is not None and kd.shape != (n,):
        raise ValueError(f"keep_dense must have one entry per group ({n})")
    out = np.zeros(n, dtype=np.uint8)
    _check(_lib.lib().sbn_dw_pattern_select(w.ctypes.data, c, go, _ptr(kd), out.ctypes.data))
    return out


def sbn_dw_pattern_apply(w, pattern, go: int = 16) -> np.ndarray:
    w = _f32(w)
    c = w.shape[0]
    pat = np.ascontiguousarray(pattern, dtype=np.uint8)
    if pat.shape != (len(sbn_dw_pattern_groups(c, go)) - 1,):
        raise ValueError("pattern must have one id per group")
    out = np.empty_like(w)
    _check(_lib.lib().sbn_dw_pattern_apply(w.ctypes.data, c, go, pat.ctypes.data, out.ctypes.data))
    return out


def sbn_force_kernel_form(kind: int, form: int) -> None:
    """Force one form of the 1x1 or 3x3 kernel for all later launches (0 = automatic); for tests."""
    _check(_lib.lib().sbn_force_kernel_form(int(kind), int(form)))


def sbn_conv3x3_pattern_taps(pattern: int) -> int:
    """9-bit mask of the taps (ky*3 + kx) that 4-of-9 pattern `pattern` keeps."""
    out = C.c_uint32()
    _check(_lib.lib().sbn_conv3x3_pattern_taps(int(pattern), C.byref(out)))
    return out.value


def sbn_conv3x3_pattern_select(w, share: int = 4) -> np.ndarray:
    """w OHWI [c_out][3][3][c_in] in the order the layer runs in -> uint8 [c_out/share][c_in] pattern ids."""
    w = _f32(w)
    if w.ndim != 4 or w.shape[1:3] != (3, 3):
        raise ValueError("w must be [c_out][3][3][c_in]")
    c_out, c_in = w.shape[0], w.shape[3]
    out = np.zeros((max(c_out // max(share, 1), 0), c_in), dtype=np.uint8)
    _check(_lib.lib().sbn_conv3x3_pattern_select(w.ctypes.data, c_out, c_in, share, out.ctypes.data))
    return out


def sbn_conv3x3_pattern_apply(w, pattern, share: int = 4) -> np.ndarray:
    w = _f32(w)
    if w.ndim != 4 or w.shape[1:3] != (3, 3):
        raise ValueError("w must be [c_out][3][3][c_in]")
    c_out, c_in = w.shape[0], w.shape[3]
    pat = np.ascontiguousarray(pattern, dtype=np.uint8)
    if share in (1, 2, 4) and c_out % share == 0 and pat.shape != (c_out // share, c_in):
        raise ValueError("pattern must be [c_out/share][c_in]")
    out = np.empty_like(w)
    _check(_lib.lib().sbn_conv3x3_pattern_apply(w.ctypes.data, c_out, c_in, share, pat.ctypes.data, out.ctypes.data))
    return out


def sbn_rearrange(layers: Sequence[dict], parent: Sequence[int], sparsity_percent: int, seed: int = 0,
                  max_iters: int = 2000, keep_output_order: Optional[Sequence[int]] = None) -> List[np.ndarray]:
    """layers: dicts with kind, w, go, gi.  Returns one filter permutation per layer."""
    n = len(layers)
    descs = (LayerDesc * n)()
    keep = []
    for i, l in enumerate(layers):
        d, k = _desc(l["kind"], l["w"], l["go"], l["gi"])
        descs[i] = d
        keep.append(k)
    par = (C.c_int * n)(*parent)
    koo = None if keep_output_order is None else (C.c_int * n)(*keep_output_order)
    perms = [np.empty(descs[i].c_out, dtype=np.int32) for i in range(n)]
    pp = (C.c_void_p * n)(*[p.ctypes.data for p in perms])
    _check(_lib.lib().sbn_rearrange(descs, n, par, koo, sparsity_percent, seed, max_iters, pp))
    return perms


def sbn_rearrange_graph(layers: Sequence[dict], in_tensor: Sequence[int], out_tensor: Sequence[int], n_tensors: int,
                        sparsity_percent: int, seed: int = 0, max_iters: int = 2000,
                        tensor_fixed: Optional[Sequence[int]] = None) -> List[np.ndarray]:
    """layers: dicts with kind, w, go, gi; layer l reads tensor in_tensor[l] and writes out_tensor[l].
    Returns one channel permutation per tensor."""
    n = len(layers)
    descs = (LayerDesc * n)()
    keep = []
    chans = [0] * n_tensors
    for i, l in enumerate(layers):
        d, k = _desc(l["kind"], l["w"], l["go"], l["gi"])
        descs[i] = d
        keep.append(k)
        if 0 <= in_tensor[i] < n_tensors:
            chans[in_tensor[i]] = d.c_in
        if 0 <= out_tensor[i] < n_tensors:
            chans[out_tensor[i]] = d.c_out
    perms = [np.empty(max(c, 1), dtype=np.int32) for c in chans]
    pp = (C.c_void_p * n_tensors)(*[p.ctypes.data for p in perms])
    fixed = None if tensor_fixed is None else (C.c_int * n_tensors)(*tensor_fixed)
    _check(_lib.lib().sbn_rearrange_graph(descs, n, (C.c_int * n)(*in_tensor), (C.c_int * n)(*out_tensor), n_tensors,
                                          fixed, sparsity_percent, seed, max_iters, pp))
    return perms


def _perm_copies(perms, sizes):
    out = [np.ascontiguousarray(p, dtype=np.int32).copy() for p in perms]
    for p, c in zip(out, sizes):
        if p.shape != (c,):
            raise ValueError(f"an order of length {c} is expected, got shape {p.shape}")
    return out


def sbn_order_groups(layers: Sequence[dict], parent: Sequence[int], sparsity_percent: int, perms: Sequence[np.ndarray],
                     keep_output_order: Optional[Sequence[int]] = None) -> List[np.ndarray]:
    """Reorders whole filter groups of the given per-layer orders (copies are returned)."""
    n = len(layers)
    descs = (LayerDesc * n)()
    keep = []
    for i, l in enumerate(layers):
        d, k = _desc(l["kind"], l["w"], l["go"], l["gi"])
        descs[i] = d
        keep.append(k)
    if len(perms) != n:
        raise ValueError("one order per layer is expected")
    out = _perm_copies(perms, [descs[i].c_out for i in range(n)])
    koo = None if keep_output_order is None else (C.c_int * n)(*keep_output_order)
    pp = (C.c_void_p * n)(*[p.ctypes.data for p in out])
    _check(_lib.lib().sbn_order_groups(descs, n, (C.c_int * n)(*parent), koo, sparsity_percent, pp))
    return out


def sbn_order_groups_graph(layers: Sequence[dict], in_tensor: Sequence[int], out_tensor: Sequence[int], n_tensors: int,
                           sparsity_percent: int, perms: Sequence[np.ndarray],
                           tensor_fixed: Optional[Sequence[int]] = None) -> List[np.ndarray]:
    """Reorders whole filter groups of the given per-tensor orders (copies are returned)."""
    n = len(layers)
    descs = (LayerDesc * n)()
    keep = []
    chans = [0] * n_tensors
    for i, l in enumerate(layers):
        d, k = _desc(l["kind"], l["w"], l["go"], l["gi"])
        descs[i] = d
        keep.append(k)
        if 0 <= in_tensor[i] < n_tensors:
            chans[in_tensor[i]] = d.c_in
        if 0 <= out_tensor[i] < n_tensors:
            chans[out_tensor[i]] = d.c_out
    if len(perms) != n_tensors:
        raise ValueError("one order per tensor is expected")
    out = _perm_copies(perms, [max(c, 1) for c in chans])
    pp = (C.c_void_p * n_tensors)(*[p.ctypes.data for p in out])
    fixed = None if tensor_fixed is None else (C.c_int * n_tensors)(*tensor_fixed)
    _check(_lib.lib().sbn_order_groups_graph(descs, n, (C.c_int * n)(*in_tensor), (C.c_int * n)(*out_tensor), n_tensors,
                                             fixed, sparsity_percent, pp))
    return out


def sbn_pack(kind: int, w, go: int, gi: int, mask=None, bias=None, perm_out=None, perm_in=None, stride: int = 1,
             pad: Optional[int] = None, act: int = SBN_ACT_NONE, device: int = 0) -> Packed:
    d, keep = _desc(kind, w, go, gi, mask, bias, perm_out, perm_in, stride, pad, act)
    out = C.c_void_p()
    _check(_lib.lib().sbn_pack(C.byref(d), device, C.byref(out)))
    del keep
    return Packed(out.value)


def sbn_packed_info(p: Packed) -> dict:
    v = [C.c_int() for _ in range(8)]
    _check(_lib.lib().sbn_packed_info(p.handle, *[C.byref(x) for x in v]))
    names = ("kind", "c_in", "c_out", "go", "gi", "stride", "act", "device")
    return {k: x.value for k, x in zip(names, v)}


def sbn_packed_work(p: Packed) -> dict:
    nnz, macs = C.c_size_t(), C.c_size_t()
    _check(_lib.lib().sbn_packed_work(p.handle, C.byref(nnz), C.byref(macs)))
    return dict(nnz_blocks=nnz.value, macs_per_pixel=macs.value)


def sbn_packed_layout(p: Packed) -> dict:
    entries, nbytes, every = C.c_size_t(), C.c_size_t(), C.c_int()
    _check(_lib.lib().sbn_packed_layout(p.handle, C.byref(entries), C.byref(nbytes), C.byref(every)))
    return dict(entries=entries.value, table_bytes=nbytes.value, every_piece=bool(every.value))


def sbn_unpack(p: Packed):
    """Returns (masked weights OHWI in original order, mask in permuted block coordinates)."""
    i = sbn_packed_info(p)
    k = 3 if i["kind"] == SBN_CONV3X3 else 1
    w = np.empty((i["c_out"], k, k, i["c_in"]), dtype=np.float32)
    m = np.empty((i["c_out"] // i["go"], i["c_in"] // i["gi"]), dtype=np.uint8)
    _check(_lib.lib().sbn_unpack(p.handle, w.ctypes.data, m.ctypes.data))
    return w, m


def sbn_export(p: Packed) -> dict:
    i = sbn_packed_info(p)
    nnz = C.c_size_t()
    _check(_lib.lib().sbn_export(p.handle, None, None, None, None, None, None, C.byref(nnz)))
    k = 3 if i["kind"] == SBN_CONV3X3 else 1
    row_ptr = np.empty(i["c_out"] // i["go"] + 1, dtype=np.uint32)
    kidx = np.empty(nnz.value, dtype=np.uint16)
    vals = np.empty((nnz.value, k, k, i["gi"], i["go"]), dtype=np.float32)
    perm_out = np.empty(i["c_out"], dtype=np.int32)
    perm_in = np.empty(i["c_in"], dtype=np.int32)
    bias = np.empty(i["c_out"], dtype=np.float32)
    _check(_lib.lib().sbn_export(p.handle, row_ptr.ctypes.data, kidx.ctypes.data, vals.ctypes.data,
                                 perm_out.ctypes.data, perm_in.ctypes.data, bias.ctypes.data, C.byref(nnz)))
    return dict(row_ptr=row_ptr, kidx=kidx, vals=vals, perm_out=perm_out, perm_in=perm_in, bias=bias,
                nnz=nnz.value)


def sbn_free(p: Packed) -> None:
    if p is not None and p.handle:
        _lib.lib().sbn_free(p.handle)
        p.handle = None


def _shape_of(p: Packed) -> dict:
    """Channel counts and stride of a packed layer (asked once, kept with the handle)."""
    info = getattr(p, "_info", None)
    if info is None:
        info = p._info = sbn_packed_info(p)
    return info


def _check_extent(t, elements: int, what: str) -> None:
    """The C side sees raw addresses: a tensor smaller than the extents given would be read or
    written out of bounds, so sizes are compared here (raw int addresses are the caller's business)."""
    if t is not None and not isinstance(t, int) and t.numel() < elements:
        raise ValueError(f"{what} holds {t.numel()} elements, the extents given need {elements}")


def sbn_conv1x1_sparse(p: Packed, x, y, n: int, h: int, w: int, stream=None) -> None:
    if n > 0 and h > 0 and w > 0:
        info = _shape_of(p)
        _check_extent(x, n * h * w * info["c_in"], "x")
        _check_extent(y, n * h * w * info["c_out"], "y")
    _check(_lib.lib().sbn_conv1x1_sparse(p.handle, _dev_ptr(x), _dev_ptr(y), n, h, w, _stream(stream)))


def sbn_conv3x3_sparse(p: Packed, x, y, n: int, h: int, w: int, stream=None) -> None:
    if n > 0 and h > 0 and w > 0:
        info = _shape_of(p)
        s = max(1, info["stride"])
        _check_extent(x, n * h * w * info["c_in"], "x")
        _check_extent(y, n * ((h - 1) // s + 1) * ((w - 1) // s + 1) * info["c_out"], "y")
    _check(_lib.lib().sbn_conv3x3_sparse(p.handle, _dev_ptr(x), _dev_ptr(y), n, h, w, _stream(stream)))


def sparse_item(p: Packed) -> dict:
    return dict(item=SBN_ITEM_SPARSE, packed=p)


def dw_item(w, bias=None, stride: int = 1, act: int = SBN_ACT_RELU, pattern=None, go: int = 16) -> dict:
    """Depthwise 3x3 item; pattern: one 3:9 pattern id per group of the channels in the order the
    layer runs in (None = dense)."""
    pat = None if pattern is None else np.ascontiguousarray(pattern, dtype=np.uint8)
    return dict(item=SBN_ITEM_DW3X3, w=_f32(w), bias=None if bias is None else _f32(bias), stride=stride, act=act,
                pattern=pat, go=go)


def stem_item(w_ohwi, bias=None, stride: int = 2, act: int = SBN_ACT_RELU) -> dict:
    w = _f32(w_ohwi)
    return dict(item=SBN_ITEM_STEM3X3, w=w, bias=None if bias is None else _f32(bias), stride=stride, act=act)


def avgpool_item() -> dict:
    return dict(item=SBN_ITEM_AVGPOOL)


def sbn_chain_create(items: Sequence[dict], device: int = 0) -> Chain:
    n = len(items)
    arr = (ChainItem * n)()
    keep = []
    for i, it in enumerate(items):
        arr[i].item = it["item"]
        if it["item"] == SBN_ITEM_SPARSE:
            arr[i].packed = it["packed"].handle
            keep.append(it["packed"])
        elif it["item"] == SBN_ITEM_STEM3X3:
            arr[i].channels = it["w"].shape[3]
            arr[i].c_out = it["w"].shape[0]
            arr[i].stride = it["stride"]
            arr[i].act = it["act"]
            arr[i].dw_w = it["w"].ctypes.data
            arr[i].dw_bias = _ptr(it["bias"])
            keep.append(it)
        elif it["item"] == SBN_ITEM_DW3X3:
            arr[i].channels = it["w"].shape[0]
            arr[i].stride = it["stride"]
            arr[i].act = it["act"]
            arr[i].dw_w = it["w"].ctypes.data
            arr[i].dw_bias = _ptr(it["bias"])
            if it.get("pattern") is not None:
                n_groups = len(sbn_dw_pattern_groups(it["w"].shape[0], it["go"])) - 1
                if it["pattern"].shape != (n_groups,):
                    raise ValueError(f"chain item {i}: pattern must have one id per group ({n_groups})")
                arr[i].dw_pattern = it["pattern"].ctypes.data
                arr[i].dw_go = it["go"]
            keep.append(it)
    out = C.c_void_p()
    _check(_lib.lib().sbn_chain_create(arr, n, device, C.byref(out)))
    first = items[0]
    c_in = (_shape_of(first["packed"])["c_in"] if first["item"] == SBN_ITEM_SPARSE else
            first["w"].shape[3] if first["item"] == SBN_ITEM_STEM3X3 else first["w"].shape[0])
    return Chain(out.value, keep, n, c_in)


def sbn_chain_workspace(c: Chain, n: int, h: int, w: int) -> int:
    b = C.c_size_t()
    _check(_lib.lib().sbn_chain_workspace(c.handle, n, h, w, C.byref(b)))
    return b.value


def sbn_chain_output_shape(c: Chain, n: int, h: int, w: int):
    oh, ow, oc = C.c_int(), C.c_int(), C.c_int()
    _check(_lib.lib().sbn_chain_output_shape(c.handle, n, h, w, C.byref(oh), C.byref(ow), C.byref(oc)))
    return oh.value, ow.value, oc.value


def sbn_chain_set_fusion(c: Chain, enable: bool) -> None:
    """Switch the fused depthwise + small 1x1 launches of a chain on (default) or off."""
    _check(_lib.lib().sbn_chain_set_fusion(c.handle, 1 if enable else 0))


def sbn_pointwise_chain(c: Chain, x, y, n: int, h: int, w: int, workspace, layer_outputs=None, stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    if n > 0 and h > 0 and w > 0:
        oh, ow, oc = sbn_chain_output_shape(c, n, h, w)
        _check_extent(x, n * h * w * c.c_in, "x")
        _check_extent(y, n * oh * ow * oc, "y")
    lo = None
    if layer_outputs is not None:
        if len(layer_outputs) != c.n_items:       # the C side reads one pointer per item
            raise ValueError(f"layer_outputs has {len(layer_outputs)} entries, the chain has {c.n_items} items")
        lo = (C.c_void_p * len(layer_outputs))(*[_dev_ptr(t) for t in layer_outputs])
    _check(_lib.lib().sbn_pointwise_chain(c.handle, _dev_ptr(x), _dev_ptr(y), n, h, w,
                                          None if workspace is None else workspace.data_ptr(), ws_bytes, lo,
                                          _stream(stream)))


SBN_STATIC_WORKSPACE_BYTES = 32 << 20


def sbn_pointwise_chain_static(c: Chain, x, y, n: int, h: int, w: int, layer_outputs=None, stream=None) -> None:
    """sbn_pointwise_chain with the library's built-in workspace: allocates nothing."""
    if n > 0 and h > 0 and w > 0:
        oh, ow, oc = sbn_chain_output_shape(c, n, h, w)
        _check_extent(x, n * h * w * c.c_in, "x")
        _check_extent(y, n * oh * ow * oc, "y")
    lo = None
    if layer_outputs is not None:
        if len(layer_outputs) != c.n_items:
            raise ValueError(f"layer_outputs has {len(layer_outputs)} entries, the chain has {c.n_items} items")
        lo = (C.c_void_p * len(layer_outputs))(*[_dev_ptr(t) for t in layer_outputs])
    _check(_lib.lib().sbn_pointwise_chain_static(c.handle, _dev_ptr(x), _dev_ptr(y), n, h, w, lo, _stream(stream)))


def sbn_chain_set_multi_layer(c: Chain, enable: bool) -> None:
    """Switch the one-launch path for runs of small items on (default) or off."""
    _check(_lib.lib().sbn_chain_set_multi_layer(c.handle, 1 if enable else 0))


def sbn_chain_check(c: Chain) -> None:
    """Raises if a multi-layer launch of the chain gave up at a grid barrier (synchronous)."""
    _check(_lib.lib().sbn_chain_check(c.handle))


def sbn_chain_free(c: Chain) -> None:
    if c is not None and c.handle:
        _lib.lib().sbn_chain_free(c.handle)
        c.handle = None


def sbn_copy_bytes(src, dst, nbytes: int, stream=None) -> None:
    _check(_lib.lib().sbn_copy_bytes(src.data_ptr(), dst.data_ptr(), nbytes, _stream(stream)))


def sbn_roof_mfma(iters: int, sink, stream=None) -> float:
    """Launches the matrix-pipe loop; returns the floating-point operations of the launch."""
    out = C.c_double()
    _check(_lib.lib().sbn_roof_mfma(iters, sink.data_ptr(), _stream(stream), C.byref(out)))
    return out.value


def sbn_roof_lds(iters: int, sink, stream=None) -> float:
    """Launches the LDS read loop; returns the bytes the launch reads."""
    out = C.c_double()
    _check(_lib.lib().sbn_roof_lds(iters, sink.data_ptr(), _stream(stream), C.byref(out)))
    return out.value


def sbn_roof_read(src, nbytes: int, sink, stream=None) -> None:
    _check(_lib.lib().sbn_roof_read(src.data_ptr(), nbytes, sink.data_ptr(), _stream(stream)))
