"""ctypes binding of liboracle.so plus a thin pipeline helper (test infrastructure)."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build(force=False))
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def _chk(rc, what):
    if rc != 0:
        raise RuntimeError("%s failed with %d" % (what, rc))


def saliency(W: Optional[np.ndarray], G_or_T: Optional[np.ndarray], kind: int, S: int, K: int) -> np.ndarray:
    T = np.empty((S, K), dtype=np.float32)
    _chk(lib().oracle_saliency(S, K, kind, _p(W), _p(G_or_T), _p(T)), "oracle_saliency")
    return T


def nm_select(T: np.ndarray, n: int, m: int) -> np.ndarray:
    S, K = T.shape
    keep = np.empty((S, K), dtype=np.uint8)
    _chk(lib().oracle_nm_select(S, K, n, m, _p(np.ascontiguousarray(T, dtype=np.float32)), _p(keep)), "oracle_nm_select")
    return keep


def keep_to_bits(keep: np.ndarray) -> np.ndarray:
    S, K = keep.shape
    bits = np.empty((S, (K + 31) // 32), dtype=np.uint32)
    _chk(lib().oracle_keep_to_bits(S, K, _p(keep), _p(bits)), "oracle_keep_to_bits")
    return bits


def block_score(T: np.ndarray, keep: np.ndarray, B: int) -> np.ndarray:
    S, K = T.shape
    sc = np.empty(((S + B - 1) // B, (K + B - 1) // B), dtype=np.float64)
    _chk(lib().oracle_block_score(S, K, B, _p(np.ascontiguousarray(T, dtype=np.float32)), _p(keep), _p(sc)), "oracle_block_score")
    return sc


def k_row(density: float, Kb: int) -> int:
    f = lib().oracle_k_row
    f.argtypes = [C.c_double, C.c_int]
    r = f(density, Kb)
    if r < 1:
        raise RuntimeError("oracle_k_row: bad arguments")
    return r


def block_select(score: np.ndarray, k_row_: int, mode: int):
    Sb, Kb = score.shape
    row_ptr = np.empty(Sb + 1, dtype=np.int32)
    col_idx = np.full(Sb * Kb, -1, dtype=np.int32)
    _chk(lib().oracle_block_select(Sb, Kb, k_row_, mode, _p(np.ascontiguousarray(score)), _p(row_ptr), _p(col_idx)), "oracle_block_select")
    return row_ptr, col_idx[: row_ptr[-1]].copy()


def dense_mask(keep: np.ndarray, B: int, row_ptr: np.ndarray, col_idx: np.ndarray) -> np.ndarray:
    S, K = keep.shape
    mask = np.empty((S, K), dtype=np.uint8)
    ci = col_idx if col_idx.size else np.zeros(1, dtype=np.int32)
    _chk(lib().oracle_dense_mask(S, K, B, _p(keep), _p(row_ptr), _p(ci), _p(mask)), "oracle_dense_mask")
    return mask


def pack_geometry(n: int, m: int, B: int):
    w = {4: 2, 8: 3}[m]
    slots = B // m * n
    wpr = (slots * w + 31) // 32
    return w, slots, wpr


def pack(W: np.ndarray, keep: np.ndarray, n: int, m: int, B: int, row_ptr: np.ndarray, col_idx: np.ndarray):
    S, K = W.shape
    _, slots, wpr = pack_geometry(n, m, B)
    nk = int(row_ptr[-1])
    vals = np.zeros((max(nk, 1), B, slots), dtype=np.uint16)
    idxw = np.zeros((max(nk, 1), B, wpr), dtype=np.uint32)
    flags = np.zeros(4, dtype=np.int32)
    ci = col_idx if col_idx.size else np.zeros(1, dtype=np.int32)
    _chk(lib().oracle_pack(S, K, n, m, B, _p(W), _p(keep), _p(row_ptr), _p(ci), _p(vals), _p(idxw), _p(flags)), "oracle_pack")
    return vals[:nk], idxw[:nk], flags


def unpack(S: int, K: int, n: int, m: int, B: int, row_ptr, col_idx, vals, idxw) -> np.ndarray:
    Wd = np.empty((S, K), dtype=np.uint16)
    ci = col_idx if col_idx.size else np.zeros(1, dtype=np.int32)
    v = vals if vals.size else np.zeros(1, dtype=np.uint16)
    i = idxw if idxw.size else np.zeros(1, dtype=np.uint32)
    _chk(lib().oracle_unpack(S, K, n, m, B, _p(row_ptr), _p(ci), _p(np.ascontiguousarray(v)), _p(np.ascontiguousarray(i)), _p(Wd)), "oracle_unpack")
    return Wd


def gemm_masked(W: np.ndarray, mask: np.ndarray, X: np.ndarray, c0: int = 0, nc: Optional[int] = None, want_abs: bool = True):
    """Y* = (W.mask) X and A* = |W.mask||X| for columns [c0, c0+nc) of X (bf16 bits, K x ldx)."""
    S, K = W.shape
    assert X.shape[0] == K and X.dtype == np.uint16
    ldx = X.shape[1]
    if nc is None:
        nc = ldx - c0
    Y = np.empty((S, nc), dtype=np.float64)
    A = np.empty((S, nc), dtype=np.float64) if want_abs else None
    f = lib().oracle_gemm_masked
    f.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_long, C.c_long, C.c_long, C.c_void_p, C.c_void_p]
    _chk(f(S, K, _p(W), _p(mask), _p(X), ldx, c0, nc, _p(Y), _p(A)), "oracle_gemm_masked")
    return Y, A


def spmm_packed(S, K, n, m, B, row_ptr, col_idx, vals, idxw, X: np.ndarray, c0: int = 0, nc: Optional[int] = None):
    ldx = X.shape[1]
    if nc is None:
        nc = ldx - c0
    Y = np.empty((S, nc), dtype=np.float64)
    f = lib().oracle_spmm_packed
    f.argtypes = [C.c_int] * 5 + [C.c_void_p] * 5 + [C.c_long, C.c_long, C.c_long, C.c_void_p]
    ci = col_idx if col_idx.size else np.zeros(1, dtype=np.int32)
    v = vals if vals.size else np.zeros(1, dtype=np.uint16)
    i = idxw if idxw.size else np.zeros(1, dtype=np.uint32)
    _chk(f(S, K, n, m, B, _p(row_ptr), _p(ci), _p(np.ascontiguousarray(v)), _p(np.ascontiguousarray(i)), _p(X), ldx, c0, nc, _p(Y)), "oracle_spmm_packed")
    return Y


def im2col(act: np.ndarray, kh: int, kw: int, stride: int, pad: int) -> np.ndarray:
    Cc, batch, H, Wd = act.shape
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (Wd + 2 * pad - kw) // stride + 1
    X = np.empty((kh * kw * Cc, batch * Ho * Wo), dtype=np.uint16)
    f = lib().oracle_im2col
    f.argtypes = [C.c_int] * 8 + [C.c_void_p, C.c_void_p, C.c_long]
    _chk(f(Cc, H, Wd, batch, kh, kw, stride, pad, _p(np.ascontiguousarray(act)), _p(X), X.shape[1]), "oracle_im2col")
    return X


def metadata_bits(S, K, Kp, n, m, B):
    out = np.zeros(3, dtype=np.float64)
    _chk(lib().oracle_metadata_bits(S, K, Kp, n, m, B, _p(out)), "oracle_metadata_bits")
    return out


@dataclass
class Selection:
    T: np.ndarray
    keep: np.ndarray       # N:M keep map, uint8 S x K
    nm_bits: np.ndarray    # same, bit-packed
    score: np.ndarray      # fp64 Sb x Kb
    k_row: int
    row_ptr: np.ndarray
    col_idx: np.ndarray
    mask: np.ndarray       # final hybrid mask, uint8 S x K


def select(W: np.ndarray, G_or_T: Optional[np.ndarray], n: int, m: int, B: int, density: float,
           sal_kind: int, select_mode: int = 0) -> Selection:
    """Saliency -> N:M -> block scores -> per-row block choice -> dense mask."""
    S, K = W.shape
    T = saliency(W, G_or_T, sal_kind, S, K)
    keep = nm_select(T, n, m)
    sc = block_score(T, keep, B)
    kr = k_row(density, sc.shape[1])
    row_ptr, col_idx = block_select(sc, kr, select_mode)
    mask = dense_mask(keep, B, row_ptr, col_idx)
    return Selection(T, keep, keep_to_bits(keep), sc, kr, row_ptr, col_idx, mask)


def epilogue(Y: np.ndarray, A: Optional[np.ndarray], scale=None, bias=None, residual=None, relu=False):
    """Tail of a layer on the exact product Y (fp64): y*scale[s] + bias[s] + residual[s][j], then
    ReLU; absent parts are skipped.  A, the bound |W|.|X| that the element-wise tolerance uses, is
    scaled by |scale| (bias and residual are exact inputs and add no error of their own).
    Plain definition; not part of the paper's method (folded batch normalisation, ReLU, shortcut)."""
    Y = np.array(Y, dtype=np.float64, copy=True)
    A = None if A is None else np.array(A, dtype=np.float64, copy=True)
    if scale is not None:
        sc = np.asarray(scale, dtype=np.float64)[:, None]
        Y *= sc
        if A is not None:
            A *= np.abs(sc)
    if bias is not None:
        Y += np.asarray(bias, dtype=np.float64)[:, None]
    if residual is not None:
        Y += np.asarray(residual, dtype=np.float64)
    if relu:
        Y = np.maximum(Y, 0.0)
    return Y, A


def maxpool(act: np.ndarray, kh: int, kw: int, stride: int, pad: int) -> np.ndarray:
    """Max over kh x kw windows of act [C][batch][H][W] (bf16 bits), positions outside the image
    excluded; returns bf16 bits [C][batch][Ho][Wo].  Plain loops over the window."""
    a = (np.ascontiguousarray(act, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    C_, b, H, W = a.shape
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    out = np.full((C_, b, Ho, Wo), -np.inf, dtype=np.float32)
    for oh in range(Ho):
        for ow in range(Wo):
            for da in range(kh):
                ih = oh * stride + da - pad
                if ih < 0 or ih >= H:
                    continue
                for db in range(kw):
                    iw = ow * stride + db - pad
                    if iw < 0 or iw >= W:
                        continue
                    out[:, :, oh, ow] = np.maximum(out[:, :, oh, ow], a[:, :, ih, iw])
    return (out.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def global_budget(layers, scores, target: float):
    """layers: list of (S, K, n, m, B); scores: list of fp64 Sb x Kb arrays.  Returns (k_row list, achieved sparsity)."""
    L = len(layers)
    arr = lambda i: (C.c_int * L)(*[int(x[i]) for x in layers])
    sc = [np.ascontiguousarray(s, dtype=np.float64) for s in scores]
    ptrs = (C.c_void_p * L)(*[s.ctypes.data for s in sc])
    k_row = (C.c_int * L)()
    ach = (C.c_double * 1)()
    f = lib().oracle_global_budget
    f.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_double, C.c_void_p,
                  C.c_void_p]
    _chk(f(L, arr(0), arr(1), arr(2), arr(3), arr(4), ptrs, float(target), k_row, ach), "oracle_global_budget")
    return list(k_row), float(ach[0])
