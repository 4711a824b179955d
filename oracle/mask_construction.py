"""fp64 CPU oracle for Attention Pruning's mask construction -- TEST INFRASTRUCTURE ONLY.

Plain numpy, double precision, no blocking: every function is the definition written out.
It shares no code with the GPU library and never imports it.

Functions
---------
attention_maps        Section 3.2: A_i = softmax(Q_i K_i^T / sqrt(d_k)), the attention matrix of
                      example i for every head (the masked-attention equation with M_p = 0)
mean_attention_map    Section 3.2, Eq. (1): the element-wise mean of the A_i over the examples
percentile_threshold  Section 3.2, paragraph before Eq. (2): the layer's threshold tau, the
                      p-th percentile of the entries of all heads of the layer
prune_mask            Section 3.2, Eq. (2): an entry is pruned iff its mean is strictly below tau

Readings (the paper does not fix them):
* percentile without interpolation: with the N participating entries sorted ascending as
  v[0] <= ... <= v[N-1], tau = v[floor(p * N)] (p in [0, 1); p = 1 gives tau = +inf).  With
  distinct values exactly floor(p * N) entries are pruned, "the percentage of entries we want
  to prune"; entries equal to tau are kept because Eq. (2) compares with a strict "<".
* a causal (auto-regressive) attention never uses the entries j > i + Lk - Lq; they do not
  take part in the percentile and are never kept.
"""
from __future__ import annotations

import math

import numpy as np


def _visible(Lq: int, Lk: int, causal: bool) -> np.ndarray:
    """[Lq, Lk] bool: the entries an (optionally causal, bottom-right aligned) attention uses."""
    if not causal:
        return np.ones((Lq, Lk), dtype=bool)
    i = np.arange(Lq)[:, None]
    j = np.arange(Lk)[None, :]
    return j <= i + (Lk - Lq)


def attention_maps(Q, K, causal: bool = False, scale: float = 0.0) -> np.ndarray:
    """A[b,h] = softmax_j(scale * Q[b,h] K[b,h]^T), fp64, [B,H,Lq,Lk].

    ``scale <= 0`` means 1/sqrt(D).  With ``causal`` the hidden entries are exactly 0 and each
    row is normalised over its visible entries.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    B, H, Lq, D = Q.shape
    Lk = K.shape[2]
    if K.shape != (B, H, Lk, D):
        raise ValueError("shape mismatch")
    if scale <= 0:
        scale = 1.0 / math.sqrt(D)
    vis = _visible(Lq, Lk, causal)
    A = np.empty((B, H, Lq, Lk), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            S = (Q[b, h] @ K[b, h].T) * scale
            S = np.where(vis, S, -np.inf)
            S = S - S.max(axis=1, keepdims=True)
            E = np.exp(S)
            A[b, h] = E / E.sum(axis=1, keepdims=True)
    return A


def mean_attention_map(Q, K, causal: bool = False, scale: float = 0.0) -> np.ndarray:
    """Eq. (1): (1/n) sum_i A_i over the n = B examples, element-wise; [H,Lq,Lk] fp64."""
    A = attention_maps(Q, K, causal, scale)
    return A.sum(axis=0) / A.shape[0]


def percentile_threshold(abar, p: float, causal: bool = False):
    """tau of one layer: abar [H,Lq,Lk] holds the mean maps of all its heads.

    Returns (tau, rank, n): rank = floor(p * n) is the 0-based position of tau in the ascending
    order of the n participating entries.  abar's dtype is kept (a float32 input gives the
    float32 order statistic, no arithmetic is done on the values).
    """
    abar = np.asarray(abar)
    H, Lq, Lk = abar.shape
    if not (0.0 <= p <= 1.0):
        raise ValueError("p must lie in [0, 1]")
    vis = _visible(Lq, Lk, causal)
    vals = abar[:, vis].ravel()
    n = int(vals.size)
    rank = int(math.floor(p * n))
    if rank >= n:
        return abar.dtype.type(np.inf), rank, n
    return np.sort(vals, kind="stable")[rank], rank, n


def prune_mask(abar, p: float, causal: bool = False):
    """Eq. (2) as a keep mask: uint8 [H,Lq,Lk], 1 = kept (mean >= tau and visible), 0 = pruned.

    Returns (mask, tau).
    """
    abar = np.asarray(abar)
    tau, _, _ = percentile_threshold(abar, p, causal)
    vis = _visible(abar.shape[1], abar.shape[2], causal)
    pruned = abar < tau                      # Eq. (2): Iverson bracket of the strict comparison
    return (~pruned & vis[None]).astype(np.uint8), tau
