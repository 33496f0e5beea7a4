"""ctypes loader for libsbn.so (the C ABI declared in include/sbn.h).

There is no fallback: if the shared library is missing and cannot be built,
importing the binding raises.  Nothing here computes anything."""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import sys

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
LIB_PATH = os.path.join(_PKG, "libsbn.so")
CSRC = os.path.join(_PKG, "csrc")

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
               # packed fp32 VALU ops are kept off on purpose
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".cpp")))


def build(verbose: bool = False) -> str:
    """Compile every source under csrc/ into libsbn.so with hipcc (gfx950)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-shared", "-I" + os.path.join(_ROOT, "include"), "-I" + CSRC,
           *sources(), "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("building libsbn.so failed:\n" + r.stdout)
    return LIB_PATH


class LayerDesc(C.Structure):
    _fields_ = [("kind", C.c_int), ("c_in", C.c_int), ("c_out", C.c_int), ("go", C.c_int), ("gi", C.c_int),
                ("stride", C.c_int), ("pad", C.c_int),
                ("w", C.c_void_p), ("mask", C.c_void_p), ("bias", C.c_void_p),
                ("perm_out", C.c_void_p), ("perm_in", C.c_void_p), ("act", C.c_int)]


class ChainItem(C.Structure):
    _fields_ = [("item", C.c_int), ("packed", C.c_void_p), ("channels", C.c_int), ("stride", C.c_int),
                ("act", C.c_int), ("dw_w", C.c_void_p), ("dw_bias", C.c_void_p), ("c_out", C.c_int),
                ("dw_pattern", C.c_void_p), ("dw_go", C.c_int)]


# name -> (restype, argtypes): every symbol include/sbn.h declares
SYMBOLS = {
    "sbn_last_error": (C.c_char_p, []),
    "sbn_prune_magnitude": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "sbn_retained_l1": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                  C.POINTER(C.c_double)]),
    "sbn_chain_set_fusion": (C.c_int, [C.c_void_p, C.c_int]),
    "sbn_force_kernel_form": (C.c_int, [C.c_int, C.c_int]),
    "sbn_dw_pattern_groups": (C.c_int, [C.c_int, C.c_int, C.POINTER(C.c_int), C.c_void_p]),
    "sbn_dw_pattern_select": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]),
    "sbn_dw_pattern_apply": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]),
    "sbn_conv3x3_pattern_taps": (C.c_int, [C.c_int, C.POINTER(C.c_uint32)]),
    "sbn_conv3x3_pattern_select": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "sbn_conv3x3_pattern_apply": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]),
    "sbn_rearrange": (C.c_int, [C.POINTER(LayerDesc), C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int), C.c_int,
                                C.c_uint64, C.c_int, C.POINTER(C.c_void_p)]),
    "sbn_rearrange_graph": (C.c_int, [C.POINTER(LayerDesc), C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int), C.c_int,
                                      C.POINTER(C.c_int), C.c_int, C.c_uint64, C.c_int, C.POINTER(C.c_void_p)]),
    "sbn_order_groups": (C.c_int, [C.POINTER(LayerDesc), C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int), C.c_int,
                                   C.POINTER(C.c_void_p)]),
    "sbn_order_groups_graph": (C.c_int, [C.POINTER(LayerDesc), C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int), C.c_int,
                                         C.POINTER(C.c_int), C.c_int, C.POINTER(C.c_void_p)]),
    "sbn_pack": (C.c_int, [C.POINTER(LayerDesc), C.c_int, C.POINTER(C.c_void_p)]),
    "sbn_unpack": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "sbn_export": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                             C.POINTER(C.c_size_t)]),
    "sbn_packed_info": (C.c_int, [C.c_void_p] + [C.POINTER(C.c_int)] * 8),
    "sbn_free": (None, [C.c_void_p]),
    "sbn_conv1x1_sparse": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "sbn_conv3x3_sparse": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "sbn_chain_create": (C.c_int, [C.POINTER(ChainItem), C.c_int, C.c_int, C.POINTER(C.c_void_p)]),
    "sbn_chain_workspace": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_size_t)]),
    "sbn_chain_output_shape": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int] + [C.POINTER(C.c_int)] * 3),
    "sbn_pointwise_chain": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                      C.c_size_t, C.POINTER(C.c_void_p), C.c_void_p]),
    "sbn_pointwise_chain_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                             C.POINTER(C.c_void_p), C.c_void_p]),
    "sbn_chain_set_multi_layer": (C.c_int, [C.c_void_p, C.c_int]),
    "sbn_chain_check": (C.c_int, [C.c_void_p]),
    "sbn_chain_free": (None, [C.c_void_p]),
    "sbn_packed_work": (C.c_int, [C.c_void_p, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]),
    "sbn_packed_layout": (C.c_int, [C.c_void_p, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t), C.POINTER(C.c_int)]),
    "sbn_copy_bytes": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "sbn_roof_mfma": (C.c_int, [C.c_int, C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]),
    "sbn_roof_lds": (C.c_int, [C.c_int, C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]),
    "sbn_roof_read": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]),
}

_lib = None


def lib() -> C.CDLL:
    """The loaded library; built first if no libsbn.so exists yet."""
    global _lib
    if _lib is None:
        # torch ships its own HIP runtime; import it first so that libsbn.so binds to the
        # runtime that also owns the device memory and streams it is handed
        import torch  # noqa: F401
        if not os.path.exists(LIB_PATH):
            build()
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(l, name)          # AttributeError if the symbol is missing: fail loudly
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib
