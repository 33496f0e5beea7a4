"""CPU ORACLE -- TEST INFRASTRUCTURE ONLY.

Plain numpy / ctypes code that states what the hot path must compute.  Only
tests, the smoke check and the benchmark's cpu_baseline leg may import it;
the product (the HIP library and its Python binding) never does, and this
module imports nothing from the product.

Contents, each following the passage it cites:
  * select-masking of weights                      (Section 3.1, W~ = W (.) M)
  * block l1 importance and magnitude pruning      (Section 3.2, Conv1x1 / Conv3x3; Eq. 2)
  * canonical group-sparse packing ("sparse info") (Algorithm 1, SD / kStartIndex)
  * filter / channel rearrangement and its objective (Section 3.4)
  * the layer itself: dense direct convolution on masked weights, via the C
    oracle in sbn_oracle.c                         (Section 3.1; Algorithm 1 result)
  * 3:9 pattern group pruning of depthwise 3x3 kernels (Section 3.2, DwConv3x3;
    Algorithm 2's PatternInfo)
  * 4-of-9 pattern pruning inside kept 3x3 kernels (Section 3.2, Conv3x3)

Pinned by tests/test_oracle_*.py against brute force, library routines,
closed forms and the paper's printed FLOP totals.  Parity unpinned: quality of
a permutation *search* (the paper's worked example, retained l1 57 -> 70, is
inside a figure whose numbers are not available); the oracle therefore only
defines the objective and an exhaustive optimum for tiny layers.
"""
from __future__ import annotations

import ctypes
import itertools
import os
import subprocess
from typing import Iterator, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libsbn_oracle.so")
_SRC = os.path.join(_HERE, "sbn_oracle.c")

ACT_NONE = 0
ACT_RELU = 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2 + OpenMP); returns the .so path."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"])
    return _SO


_lib = None


def _c():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.oracle_conv_nhwc.argtypes = [fp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                         fp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                         fp, ctypes.c_int, ctypes.c_int, ctypes.c_int, fp, dp]
        lib.oracle_conv_nhwc.restype = ctypes.c_int
        lib.oracle_dwconv3x3_nhwc.argtypes = [fp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                              fp, fp, ctypes.c_int, ctypes.c_int, fp, dp]
        lib.oracle_dwconv3x3_nhwc.restype = ctypes.c_int
        lib.oracle_avgpool_nhwc.argtypes = [fp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, fp]
        lib.oracle_avgpool_nhwc.restype = ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_c().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _c().oracle_set_num_threads(int(n))


def _fptr(a: Optional[np.ndarray]):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


# ----------------------------------------------------------------------------
# The layer (Section 3.1): dense direct convolution on already-masked weights.
# ----------------------------------------------------------------------------

def conv_nhwc(x: np.ndarray, w: np.ndarray, bias: Optional[np.ndarray] = None,
              stride: int = 1, pad: int = 0, act: int = ACT_NONE,
              want_bound: bool = True) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """y = act(bias + conv(x, w)); x NHWC fp32, w OHWI fp32 (masked by the caller).

    Returns (y fp32 [n][oh][ow][oc], bound fp64 = sum |x||w| per output or None)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    n, ih, iw, ic = x.shape
    oc, kh, kw, ic2 = w.shape
    assert ic == ic2
    oh = (ih + 2 * pad - kh) // stride + 1
    ow = (iw + 2 * pad - kw) // stride + 1
    y = np.empty((n, oh, ow, oc), dtype=np.float32)
    bound = np.empty((n, oh, ow, oc), dtype=np.float64) if want_bound else None
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    rc = _c().oracle_conv_nhwc(_fptr(x), n, ih, iw, ic, _fptr(w), oc, kh, kw, _fptr(b),
                               stride, pad, act, _fptr(y),
                               None if bound is None else bound.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    assert rc == 0
    return y, bound


def dwconv3x3_nhwc(x: np.ndarray, w: np.ndarray, bias: Optional[np.ndarray] = None,
                   stride: int = 1, act: int = ACT_NONE,
                   want_bound: bool = True) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """Dense depthwise 3x3, pad 1; x NHWC, w [c][3][3]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    n, ih, iw, c = x.shape
    assert w.shape == (c, 3, 3)
    oh = (ih - 1) // stride + 1
    ow = (iw - 1) // stride + 1
    y = np.empty((n, oh, ow, c), dtype=np.float32)
    bound = np.empty((n, oh, ow, c), dtype=np.float64) if want_bound else None
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    rc = _c().oracle_dwconv3x3_nhwc(_fptr(x), n, ih, iw, c, _fptr(w), _fptr(b), stride, act, _fptr(y),
                                    None if bound is None else bound.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    assert rc == 0
    return y, bound


def avgpool_nhwc(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    n, h, w, c = x.shape
    y = np.empty((n, c), dtype=np.float32)
    assert _c().oracle_avgpool_nhwc(_fptr(x), n, h, w, c, _fptr(y)) == 0
    return y


# ----------------------------------------------------------------------------
# Rearrangement (Section 3.4): packed filter r is original filter perm_out[r],
# packed channel c is original channel perm_in[c].
# ----------------------------------------------------------------------------

def permute_weights(w: np.ndarray, perm_out: Optional[Sequence[int]],
                    perm_in: Optional[Sequence[int]]) -> np.ndarray:
    """Wp[r, :, :, c] = W[perm_out[r], :, :, perm_in[c]]."""
    wp = w
    if perm_out is not None:
        wp = wp[np.asarray(perm_out, dtype=np.int64)]
    if perm_in is not None:
        wp = wp[..., np.asarray(perm_in, dtype=np.int64)]
    return np.ascontiguousarray(wp)


def inverse_permutation(p: Sequence[int]) -> np.ndarray:
    p = np.asarray(p, dtype=np.int64)
    inv = np.empty_like(p)
    inv[p] = np.arange(p.size)
    return inv


def is_permutation(p: Sequence[int], n: int) -> bool:
    p = np.asarray(p)
    return p.shape == (n,) and np.array_equal(np.sort(p), np.arange(n))


# ----------------------------------------------------------------------------
# Block importance and magnitude pruning (Section 3.2; Eq. 2).
# A block is go output channels x gi input channels, all kh*kw taps included.
# ----------------------------------------------------------------------------

def block_norms(wp: np.ndarray, go: int, gi: int) -> np.ndarray:
    """fp64 l1 norm of every block of an OHWI tensor, summed in (o, ky, kx, c) order."""
    n, kh, kw, c = wp.shape
    assert n % go == 0 and c % gi == 0
    v = np.abs(wp.astype(np.float64)).reshape(n // go, go, kh, kw, c // gi, gi)
    s = np.zeros((n // go, c // gi), dtype=np.float64)
    for o in range(go):
        for ky in range(kh):
            for kx in range(kw):
                for ci in range(gi):
                    s = s + v[:, o, ky, kx, :, ci]
    return s


def n_removed(n_blocks: int, sparsity_percent: int) -> int:
    """Number of blocks removed at an integer-percent sparsity (rounded down)."""
    return (n_blocks * int(sparsity_percent)) // 100


def prune_mask(wp: np.ndarray, go: int, gi: int, sparsity_percent: int) -> np.ndarray:
    """uint8 [n/go][c/gi]; the lowest-importance blocks of the layer get 0.

    Ties are broken by block position: the lower linear index goes first."""
    s = block_norms(wp, go, gi)
    r = n_removed(s.size, sparsity_percent)
    flat = s.ravel()
    order = np.lexsort((np.arange(flat.size), flat))   # by norm, then by index
    m = np.ones(flat.size, dtype=np.uint8)
    m[order[:r]] = 0
    return m.reshape(s.shape)


def apply_mask(wp: np.ndarray, mask: np.ndarray, go: int, gi: int) -> np.ndarray:
    """W~: weights of removed blocks become +0.0 (a select, so no -0.0 appears)."""
    n, kh, kw, c = wp.shape
    full = np.repeat(np.repeat(mask.astype(bool), go, axis=0), gi, axis=1)   # [n][c]
    out = np.where(full[:, None, None, :], wp, np.float32(0.0)).astype(np.float32)
    return np.ascontiguousarray(out)


def nonzero_block_mask(wp: np.ndarray, go: int, gi: int) -> np.ndarray:
    """Mask implied by the weights: a block is kept iff any element has nonzero magnitude."""
    n, kh, kw, c = wp.shape
    bits = wp.view(np.uint32) & np.uint32(0x7FFFFFFF)
    nz = (bits != 0).reshape(n // go, go, kh, kw, c // gi, gi)
    return nz.any(axis=(1, 2, 3, 5)).astype(np.uint8)


def retained_l1(wp: np.ndarray, go: int, gi: int, sparsity_percent: int) -> float:
    """The rearrangement objective: total importance of the blocks that survive pruning."""
    s = np.sort(block_norms(wp, go, gi).ravel())
    return float(np.sum(s[n_removed(s.size, sparsity_percent):]))


# ----------------------------------------------------------------------------
# Canonical packed format (Algorithm 1's "sparse info"): one row per output
# group; a row lists its kept blocks by ascending first input channel.
# ----------------------------------------------------------------------------

def canonical_pack(wp: np.ndarray, mask: np.ndarray, go: int, gi: int):
    """Returns (row_ptr uint32 [n/go+1], kidx uint16 [nnz], vals fp32 [nnz][kh][kw][gi][go])."""
    n, kh, kw, c = wp.shape
    rows, cols = n // go, c // gi
    assert mask.shape == (rows, cols)
    row_ptr = np.zeros(rows + 1, dtype=np.uint32)
    kidx: List[int] = []
    vals: List[np.ndarray] = []
    for i in range(rows):
        for j in range(cols):
            if mask[i, j]:
                kidx.append(j * gi)
                blk = wp[i * go:(i + 1) * go, :, :, j * gi:(j + 1) * gi]     # [go][kh][kw][gi]
                vals.append(np.transpose(blk, (1, 2, 3, 0)))                 # [kh][kw][gi][go]
        row_ptr[i + 1] = len(kidx)
    v = (np.stack(vals).astype(np.float32) if vals
         else np.zeros((0, kh, kw, gi, go), dtype=np.float32))
    return row_ptr, np.asarray(kidx, dtype=np.uint16), np.ascontiguousarray(v)


def canonical_unpack(row_ptr, kidx, vals, n: int, c: int, go: int, gi: int) -> Tuple[np.ndarray, np.ndarray]:
    """Inverse of canonical_pack: (masked weights in permuted order, mask)."""
    nnz, kh, kw, gi2, go2 = vals.shape
    assert gi2 == gi and go2 == go
    wp = np.zeros((n, kh, kw, c), dtype=np.float32)
    mask = np.zeros((n // go, c // gi), dtype=np.uint8)
    for i in range(n // go):
        for e in range(int(row_ptr[i]), int(row_ptr[i + 1])):
            k0 = int(kidx[e])
            wp[i * go:(i + 1) * go, :, :, k0:k0 + gi] = np.transpose(vals[e], (3, 0, 1, 2))
            mask[i, k0 // gi] = 1
    return wp, mask


def unpermute_weights(wp: np.ndarray, perm_out, perm_in) -> np.ndarray:
    """Inverse of permute_weights: W[perm_out[r], :, :, perm_in[c]] = Wp[r, :, :, c]."""
    n, kh, kw, c = wp.shape
    po = np.arange(n) if perm_out is None else np.asarray(perm_out, dtype=np.int64)
    pi = np.arange(c) if perm_in is None else np.asarray(perm_in, dtype=np.int64)
    w = np.empty_like(wp)
    w[np.ix_(po, np.arange(kh), np.arange(kw), pi)] = wp
    return w


# ----------------------------------------------------------------------------
# Canonical groupings (Section 3.4): filters sorted inside every group, groups
# sorted by their first filter.  Exhaustive optimum for tiny layers.
# ----------------------------------------------------------------------------

def canonical_groupings(n: int, go: int) -> Iterator[Tuple[int, ...]]:
    """All canonical permutations of n filters into groups of go, as flat tuples."""
    assert n % go == 0

    def rec(remaining: Tuple[int, ...]):
        if not remaining:
            yield ()
            return
        first, rest = remaining[0], remaining[1:]
        for others in itertools.combinations(rest, go - 1):
            group = (first,) + others
            left = tuple(v for v in rest if v not in others)
            for tail in rec(left):
                yield group + tail

    yield from rec(tuple(range(n)))


def canonicalize(perm: Sequence[int], go: int) -> np.ndarray:
    """Sort filters inside each group, then groups by first filter."""
    g = np.sort(np.asarray(perm, dtype=np.int64).reshape(-1, go), axis=1)
    g = g[np.argsort(g[:, 0], kind="stable")]
    return g.reshape(-1).astype(np.int32)


def best_row_grouping(w_cols_permuted: np.ndarray, go: int, gi: int, sparsity_percent: int):
    """Exhaustive search over canonical filter groupings; returns (perm, objective).

    The first grouping reaching the maximum (in enumeration order) is returned."""
    n = w_cols_permuted.shape[0]
    best, best_obj = None, -1.0
    for g in canonical_groupings(n, go):
        obj = retained_l1(w_cols_permuted[list(g)], go, gi, sparsity_percent)
        if obj > best_obj:
            best, best_obj = g, obj
    return np.asarray(best, dtype=np.int32), best_obj


# ----------------------------------------------------------------------------
# One sparse layer end to end, as the definition states it.
# ----------------------------------------------------------------------------

def sparse_conv_reference(x_perm: np.ndarray, w: np.ndarray, mask: Optional[np.ndarray], go: int, gi: int,
                          bias: Optional[np.ndarray] = None, perm_out=None, perm_in=None,
                          stride: int = 1, pad: int = 0, act: int = ACT_NONE):
    """Result of a packed layer in PERMUTED channel space.

    x_perm has channels in perm_in order; y comes out in perm_out order.
    w and bias are in original order; mask is in permuted block coordinates
    (None: a block is kept iff it holds a nonzero)."""
    wp = permute_weights(w, perm_out, perm_in)
    if mask is None:
        mask = nonzero_block_mask(wp, go, gi)
    wt = apply_mask(wp, mask, go, gi)
    bp = None
    if bias is not None:
        bp = np.asarray(bias, dtype=np.float32)
        if perm_out is not None:
            bp = bp[np.asarray(perm_out, dtype=np.int64)]
    return conv_nhwc(x_perm, wt, bp, stride=stride, pad=pad, act=act)


# ----------------------------------------------------------------------------
# Section 3.2, DwConv3x3: 3:9 pattern group pruning.  Every kernel loses three
# weights, one per row, each taken from the first or the third column: 2^3
# patterns.  go consecutive channels (16; a remainder forms groups of 8 or 4)
# share one pattern, the one that keeps the largest l1-norm.  A group may be
# left dense (Section 3.3's "full-1" pattern); which groups is the caller's
# choice.
# ----------------------------------------------------------------------------

DW_PATTERN_DENSE = 8


def dw_pattern_mask(pid: int) -> np.ndarray:
    """uint8 [3][3] keep-mask of pattern pid: bit r of pid set -> row r loses its THIRD column,
    clear -> its FIRST column; DW_PATTERN_DENSE keeps everything."""
    m = np.ones((3, 3), dtype=np.uint8)
    if pid == DW_PATTERN_DENSE:
        return m
    assert 0 <= pid < 8
    for r in range(3):
        m[r, 2 if (pid >> r) & 1 else 0] = 0
    return m


def dw_pattern_groups(c: int, go: int = 16) -> List[Tuple[int, int]]:
    """(first channel, size) of every pattern group: as many groups of go as fit, then the
    remainder in groups of 8 and 4 (Section 3.3); c must be a multiple of 4."""
    assert c % 4 == 0 and go in (4, 8, 16)
    out, pos = [], 0
    while c - pos >= go:
        out.append((pos, go))
        pos += go
    for g in (8, 4):
        while g < go and c - pos >= g:
            out.append((pos, g))
            pos += g
    assert pos == c
    return out


def dw_pattern_select(w: np.ndarray, go: int = 16, dense_groups: Sequence[int] = ()) -> np.ndarray:
    """Pattern id per group of w[C][3][3]: the pattern with the largest kept l1-norm over the
    group's kernels (fp64 sums in channel, row, column order; ties -> the lowest id)."""
    ids = []
    for gidx, (c0, n) in enumerate(dw_pattern_groups(w.shape[0], go)):
        if gidx in dense_groups:
            ids.append(DW_PATTERN_DENSE)
            continue
        best, best_id = -1.0, 0
        for pid in range(8):
            m = dw_pattern_mask(pid)
            tot = 0.0
            for ch in range(c0, c0 + n):
                for r in range(3):
                    for col in range(3):
                        if m[r, col]:
                            tot += abs(float(w[ch, r, col]))
            if tot > best:
                best, best_id = tot, pid
        ids.append(best_id)
    return np.array(ids, dtype=np.uint8)


def dw_pattern_apply(w: np.ndarray, ids: Sequence[int], go: int = 16) -> np.ndarray:
    """W (.) M for the depthwise layer: a select, removed weights become +0.0."""
    out = w.copy()
    for (c0, n), pid in zip(dw_pattern_groups(w.shape[0], go), ids):
        m = dw_pattern_mask(int(pid)).astype(bool)
        out[c0:c0 + n][:, ~m] = 0.0
    return out


# ----------------------------------------------------------------------------
# Section 3.2, Conv3x3: pattern pruning inside the kept kernels.  Every 3x3
# kernel keeps 4 of its 9 weights, the centre always among them: C(8,3) = 56
# patterns.  Adjacent filters (4, 2 or 1) use the same pattern for a given
# input channel (Section 3.3, closing remarks); the pattern kept is the one
# with the largest l1-norm.  Numbering (a reading; the paper shows the
# patterns in a figure only): taps are ky*3 + kx, id p is the p-th 3-subset of
# the eight non-centre taps in lexicographic order.
# ----------------------------------------------------------------------------

K3_PATTERNS = 56
K3_PATTERN_DENSE = 56


def conv3x3_pattern_mask(pid: int) -> np.ndarray:
    """uint8 [3][3] keep-mask of 4-of-9 pattern pid; K3_PATTERN_DENSE keeps everything."""
    if pid == K3_PATTERN_DENSE:
        return np.ones((3, 3), dtype=np.uint8)
    assert 0 <= pid < K3_PATTERNS
    others = [t for t in range(9) if t != 4]
    subsets = list(itertools.combinations(others, 3))       # lexicographic in (a, b, c)
    m = np.zeros(9, dtype=np.uint8)
    m[4] = 1
    m[list(subsets[pid])] = 1
    return m.reshape(3, 3)


def conv3x3_pattern_select(w: np.ndarray, share: int = 4) -> np.ndarray:
    """uint8 [c_out/share][c_in] pattern ids for w OHWI [c_out][3][3][c_in]: per group of `share`
    adjacent filters and per input channel, the pattern keeping the largest summed magnitude
    (fp64: per tap over the group's filters in order, then over the pattern's three non-centre
    taps in ascending order; ties -> the lowest id)."""
    c_out, _, _, c_in = w.shape
    assert share in (1, 2, 4) and c_out % share == 0
    masks = [conv3x3_pattern_mask(p).reshape(9) for p in range(K3_PATTERNS)]
    ids = np.zeros((c_out // share, c_in), dtype=np.uint8)
    for f in range(c_out // share):
        for c in range(c_in):
            s = [0.0] * 9
            for t in range(9):
                for i in range(share):
                    s[t] += abs(float(w[f * share + i, t // 3, t % 3, c]))
            best, best_id = -1.0, 0
            for p in range(K3_PATTERNS):
                tot = 0.0
                for t in range(9):
                    if t != 4 and masks[p][t]:
                        tot += s[t]
                if tot > best:
                    best, best_id = tot, p
            ids[f, c] = best_id
    return ids


def conv3x3_pattern_apply(w: np.ndarray, ids: np.ndarray, share: int = 4) -> np.ndarray:
    """W (.) M for a 3x3 layer: a select, removed weights become +0.0."""
    c_out, _, _, c_in = w.shape
    out = w.copy()
    for n in range(c_out):
        for c in range(c_in):
            m = conv3x3_pattern_mask(int(ids[n // share, c])).astype(bool)
            out[n, :, :, c][~m] = 0.0
    return out
