"""fp64 CPU oracle for masked attention with the 1.5-entmax normaliser -- TEST INFRASTRUCTURE ONLY.

Section 6 repeats the experiments with 1.5-entmax in place of softmax as the attention's
normalising activation, together with the pruning mask.  The paper takes the activation from the
literature it cites there; its definition is

    entmax_a(z) = argmax over the probability simplex of  <p, z> + H_a(p),
    H_a(p) = (1 / (a (a - 1))) sum_j (p_j - p_j^a)                          (Tsallis entropy)

whose optimality conditions give, for a = 1.5,

    p_j = [z_j / 2 - tau]_+^2     with tau such that sum_j p_j = 1.

Here the condition is solved exactly: with x = z / 2 sorted in descending order, a support of the
k largest entries fixes tau as the smaller root of  k tau^2 - 2 tau sum x + sum x^2 - 1 = 0,  and
the support is right iff  x_(k) > tau >= x_(k+1); the largest k with x_(k) > tau_k is that
support.  Plain numpy, one row at a time.

masked_entmax15_attention   O = entmax_1.5(scale * Q K^T restricted to kept, visible keys) V
"""
from __future__ import annotations

import math

import numpy as np


def entmax15(z: np.ndarray):
    """1.5-entmax of a 1-D score vector (fp64).  Returns (p, tau) with p = [z/2 - tau]_+^2."""
    z = np.asarray(z, dtype=np.float64)
    x = np.sort(z / 2.0)[::-1]
    k = np.arange(1, x.size + 1, dtype=np.float64)
    s1 = np.cumsum(x)
    s2 = np.cumsum(x * x)
    disc = s1 * s1 - k * (s2 - 1.0)
    tau_k = (s1 - np.sqrt(np.maximum(disc, 0.0))) / k
    # the consistent supports are a prefix of k = 1, 2, ...; the largest one is the solution
    # (at an exact tie x_(k+1) = tau both neighbours describe the same p)
    ok = (disc >= 0.0) & (x > tau_k)
    idx = np.flatnonzero(ok)
    tau = tau_k[idx[-1]]
    p = np.maximum(z / 2.0 - tau, 0.0) ** 2
    return p, tau


def masked_entmax15_attention(Q, K, V, mask, causal: bool = False, scale: float = 0.0):
    """Q [B,H,Lq,D], K [B,H,Lk,D], V [B,H,Lk,Dv]; mask [H,Lq,Lk], nonzero = kept.

    Returns (O [B,H,Lq,Dv], tau [B,H,Lq]) in fp64; a query without any visible kept key gets
    O = 0 and tau = +inf.  ``scale <= 0`` means 1/sqrt(D).
    """
    Q, K, V = (np.asarray(x, dtype=np.float64) for x in (Q, K, V))
    keep = np.asarray(mask) != 0
    B, H, Lq, D = Q.shape
    Lk = K.shape[2]
    if scale <= 0:
        scale = 1.0 / math.sqrt(D)
    if causal:
        keep = keep & (np.arange(Lk)[None, :] <= np.arange(Lq)[:, None] + (Lk - Lq))[None]
    O = np.zeros((B, H, Lq, V.shape[3]), dtype=np.float64)
    tau = np.full((B, H, Lq), np.inf, dtype=np.float64)
    for b in range(B):
        for h in range(H):
            S = (Q[b, h] @ K[b, h].T) * scale
            for i in range(Lq):
                cols = np.flatnonzero(keep[h, i])
                if cols.size == 0:
                    continue
                p, t = entmax15(S[i, cols])
                O[b, h, i] = p @ V[b, h, cols]
                tau[b, h, i] = t
    return O, tau
