"""fp64 CPU oracle for Attention Pruning's masked attention -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import this
package.  It shares no code with the GPU library and never imports it.

The arithmetic lives in ``ap_oracle.c`` (plain loops, double precision, OpenMP over query
rows); this module compiles it with gcc on first use and marshals numpy arrays.

Functions
---------
masked_attention   Section 3.2, masked-attention equation: softmax((QK^T + M_p)/sqrt(d_k)) V
build_layout       block-sparse layout (block rows, block columns, per-block element bitmaps)
                   of an element mask; Section 9.2 uses block-structured sparseness patterns
macs_fraction      Appendix A's multiply-accumulate count, the model behind Eq. (3)
kept_entry_flops   4*D flops per kept (query, key) connection: both N^2-sized products

The backward pass (gradients of the masked-attention equation) is in ``backward.py`` (numpy):
masked_attention_backward.

Masked attention with the 1.5-entmax normaliser of Section 6 is in ``entmax.py`` (numpy): entmax15,
masked_entmax15_attention and their gradients (entmax15_backward, masked_entmax15_attention_backward).

Mask construction (Section 3.2, Eq. (1) and Eq. (2)) is in ``mask_construction.py`` (numpy):
attention_maps, mean_attention_map, percentile_threshold, prune_mask.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from .backward import masked_attention_backward  # noqa: F401
from .entmax import (entmax15, entmax15_backward, masked_entmax15_attention,  # noqa: F401
                     masked_entmax15_attention_backward)
from .mask_construction import (attention_maps, mean_attention_map,  # noqa: F401
                                percentile_threshold, prune_mask)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ap_oracle.c")
_LIB = os.path.join(_HERE, "libap_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ap_oracle.c into libap_oracle.so (gcc -O2 -fopenmp, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        lib.ap_oracle_masked_attention.restype = ctypes.c_int
        lib.ap_oracle_masked_attention.argtypes = [
            dp, dp, dp, u8p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_double, dp, dp]
        lib.ap_oracle_build_layout.restype = ctypes.c_longlong
        lib.ap_oracle_build_layout.argtypes = [
            u8p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32),
            ctypes.POINTER(ctypes.c_uint64), ctypes.c_longlong]
        lib.ap_oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the OpenMP loops use (OMP_NUM_THREADS or all cores)."""
    return int(_load().ap_oracle_num_threads())


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def masked_attention(Q, K, V, mask, causal: bool = False, scale: float = 0.0):
    """Masked softmax attention in fp64 (Section 3.2, equation after Eq. (2)).

    Q [B,H,Lq,D], K [B,H,Lk,D], V [B,H,Lk,Dv]; mask [H,Lq,Lk], nonzero = kept.
    Returns (O [B,H,Lq,Dv], lse [B,H,Lq]).  A query without any visible kept key
    gets O = 0 and lse = -inf.  ``scale <= 0`` means 1/sqrt(D).
    """
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    mask = np.ascontiguousarray(np.asarray(mask) != 0).astype(np.uint8)
    if Q.ndim != 4 or K.ndim != 4 or V.ndim != 4 or mask.ndim != 3:
        raise ValueError("expected Q,K,V [B,H,L,D] and mask [H,Lq,Lk]")
    B, H, Lq, D = Q.shape
    Lk = K.shape[2]
    Dv = V.shape[3]
    if K.shape != (B, H, Lk, D) or V.shape != (B, H, Lk, Dv) or mask.shape != (H, Lq, Lk):
        raise ValueError("shape mismatch")
    O = np.empty((B, H, Lq, Dv), dtype=np.float64)
    lse = np.empty((B, H, Lq), dtype=np.float64)
    rc = _load().ap_oracle_masked_attention(
        _ptr(Q, ctypes.c_double), _ptr(K, ctypes.c_double), _ptr(V, ctypes.c_double),
        _ptr(mask, ctypes.c_uint8), B, H, Lq, Lk, D, Dv, int(bool(causal)), float(scale),
        _ptr(O, ctypes.c_double), _ptr(lse, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("ap_oracle_masked_attention failed (%d)" % rc)
    return O, lse


def build_layout(mask, block_m: int, block_n: int):
    """Block-sparse layout of an element mask [H,Lq,Lk] (nonzero = kept).

    Returns (row_ptr int32 [H*nQB+1], col_idx int32 [nnz], bitmaps uint64 [nnz, BM, ceil(BN/64)]).
    Tiles of a block row are in ascending block-column order; bit c%64 of word c//64 of
    local row r is mask[h, qb*BM + r, kb*BN + c] != 0 and 0 outside the mask.
    """
    mask = np.ascontiguousarray(np.asarray(mask) != 0).astype(np.uint8)
    H, Lq, Lk = mask.shape
    nQB = -(-Lq // block_m)
    W = -(-block_n // 64)
    lib = _load()
    row_ptr = np.zeros(H * nQB + 1, dtype=np.int32)
    nnz = lib.ap_oracle_build_layout(_ptr(mask, ctypes.c_uint8), H, Lq, Lk, block_m, block_n,
                                     _ptr(row_ptr, ctypes.c_int32), None, None, 0)
    if nnz < 0:
        raise RuntimeError("ap_oracle_build_layout failed")
    col_idx = np.zeros(max(nnz, 1), dtype=np.int32)
    bitmaps = np.zeros((max(nnz, 1), block_m, W), dtype=np.uint64)
    nnz2 = lib.ap_oracle_build_layout(_ptr(mask, ctypes.c_uint8), H, Lq, Lk, block_m, block_n,
                                      _ptr(row_ptr, ctypes.c_int32), _ptr(col_idx, ctypes.c_int32),
                                      _ptr(bitmaps, ctypes.c_uint64), nnz)
    assert nnz2 == nnz
    return row_ptr, col_idx[:nnz], bitmaps[:nnz]


def macs_fraction(N: int, d: int, p: float, B: int = 1, h: int = 1) -> float:
    """Fraction of attention-layer multiply-accumulates left after pruning a fraction p.

    Follows Appendix A step by step: (i) Q,K,V projections 3*B*N*d^2; (ii) scores
    B*h*N^2*d_k; (iii) probabilities times values B*h*N^2*d_k, the only step the paper
    credits with the saving (a fraction 1-p of it remains); (iv) output projection
    B*N*d^2; with d_k = d / h.  Eq. (3) is the closed form of this ratio.
    """
    d_k = d / h
    proj_in = 3.0 * B * N * d * d
    scores = B * h * float(N) * N * d_k
    pv = B * h * float(N) * N * d_k
    proj_out = 1.0 * B * N * d * d
    dense = proj_in + scores + pv + proj_out
    pruned = proj_in + scores + (1.0 - p) * pv + proj_out
    return pruned / dense


def kept_entry_flops(mask, B: int, D: int, causal: bool = False) -> int:
    """Flops of the two N^2-sized products restricted to kept connections.

    Each kept (query, key) pair costs D multiply-adds in Q K^T and D in P V (Appendix A,
    steps (ii) and (iii)), i.e. 4*D flops, for every batch element.
    """
    mask = np.asarray(mask) != 0
    H, Lq, Lk = mask.shape
    if causal:
        i = np.arange(Lq)[:, None]
        j = np.arange(Lk)[None, :]
        mask = mask & (j <= i + (Lk - Lq))[None]
    return int(4 * D * int(mask.sum()) * B)
