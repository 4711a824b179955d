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

Backward (the models of Section 6 are trained with this activation).  The paper prints no
gradient; from the conditions above, with u_j = [z_j/2 - tau]_+ (so p_j = u_j^2) and sum_j p_j = 1
held fixed:  dp_j = 2 u_j (dz_j / 2 - dtau)  and  sum_j u_j (dz_j / 2 - dtau) = 0,  hence

    dtau = sum_j u_j dz_j / (2 sum_j u_j),
    dL/dz_j = u_j (g_j - gbar),   g_j = dL/dp_j,   gbar = sum_k u_k g_k / sum_k u_k

on the support and 0 outside it.

entmax15_backward                   dL/dz for one score vector
masked_entmax15_attention_backward  dQ, dK, dV of masked_entmax15_attention's O
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


def entmax15_backward(z: np.ndarray, g: np.ndarray) -> np.ndarray:
    """dL/dz of p = entmax15(z) for an upstream gradient g = dL/dp (1-D, fp64)."""
    z = np.asarray(z, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    _, tau = entmax15(z)
    u = np.maximum(z / 2.0 - tau, 0.0)
    gbar = float(u @ g) / float(u.sum())
    return u * (g - gbar)


def masked_entmax15_attention_backward(Q, K, V, mask, dO, causal: bool = False, scale: float = 0.0):
    """Gradients (dQ, dK, dV) of masked_entmax15_attention's O for an upstream gradient dO, fp64.

    With s_ij = scale <Q_i, K_j> on kept, visible entries, P_i = entmax15(s_i) and O_i = sum_j P_ij V_j:
    dV_j = sum_i P_ij dO_i,  g_ij = <dO_i, V_j>,  dS_i = entmax15_backward(s_i, g_i),
    dQ_i = scale sum_j dS_ij K_j,  dK_j = scale sum_i dS_ij Q_i.  Queries without a kept key
    contribute nothing.
    """
    Q, K, V, dO = (np.asarray(x, dtype=np.float64) for x in (Q, K, V, dO))
    keep = np.asarray(mask) != 0
    B, H, Lq, D = Q.shape
    Lk = K.shape[2]
    if scale <= 0:
        scale = 1.0 / math.sqrt(D)
    if causal:
        keep = keep & (np.arange(Lk)[None, :] <= np.arange(Lq)[:, None] + (Lk - Lq))[None]
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    for b in range(B):
        for h in range(H):
            S = (Q[b, h] @ K[b, h].T) * scale
            G = dO[b, h] @ V[b, h].T
            for i in range(Lq):
                cols = np.flatnonzero(keep[h, i])
                if cols.size == 0:
                    continue
                p, _ = entmax15(S[i, cols])
                ds = entmax15_backward(S[i, cols], G[i, cols])
                dV[b, h, cols] += np.outer(p, dO[b, h, i])
                dQ[b, h, i] = scale * (ds @ K[b, h, cols])
                dK[b, h, cols] += scale * np.outer(ds, Q[b, h, i])
    return dQ, dK, dV
