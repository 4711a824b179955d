"""fp64 CPU oracle for the backward pass of masked attention -- TEST INFRASTRUCTURE ONLY.

Plain numpy, double precision, one (example, head) at a time, no blocking.  It shares no code
with the GPU library and never imports it.

masked_attention_backward   gradients of the masked-attention equation of Section 3.2,
                            A~ = softmax((Q K^T + M_p) / sqrt(d_k)) V, with respect to Q, K and V
                            (step 4 of the algorithm of Section 3.2 trains the pruned model, which
                            needs them).  The paper gives no formulas; these follow from the
                            definition by the chain rule:

    P_ij  = exp(s_ij) / sum_{j' in S_i} exp(s_ij')        for j in S_i, else 0      (s = scale * Q K^T)
    dV_j  = sum_i P_ij dO_i
    dP_ij = <dO_i, V_j>
    dS_ij = P_ij (dP_ij - sum_j' P_ij' dP_ij')                                       (softmax Jacobian)
    dQ_i  = scale * sum_j dS_ij K_j ,   dK_j = scale * sum_i dS_ij Q_i

A query with no visible kept key has O = 0 whatever the inputs are: its row contributes nothing.
"""
from __future__ import annotations

import math

import numpy as np


def masked_attention_backward(Q, K, V, mask, dO, causal: bool = False, scale: float = 0.0):
    """Q [B,H,Lq,D], K [B,H,Lk,D], V [B,H,Lk,Dv], mask [H,Lq,Lk] (nonzero = kept), dO [B,H,Lq,Dv].

    Returns (dQ, dK, dV) in fp64.  ``scale <= 0`` means 1/sqrt(D).
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
            S = np.where(keep[h], (Q[b, h] @ K[b, h].T) * scale, -np.inf)
            m = S.max(axis=1, keepdims=True)
            m = np.where(np.isfinite(m), m, 0.0)             # rows without a kept key: all-zero P
            E = np.exp(S - m)
            Z = E.sum(axis=1, keepdims=True)
            P = np.divide(E, Z, out=np.zeros_like(E), where=Z > 0)
            dV[b, h] = P.T @ dO[b, h]
            dP = dO[b, h] @ V[b, h].T
            dS = P * (dP - (P * dP).sum(axis=1, keepdims=True))
            dQ[b, h] = scale * (dS @ K[b, h])
            dK[b, h] = scale * (dS.T @ Q[b, h])
    return dQ, dK, dV
