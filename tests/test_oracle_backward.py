"""Pins for the backward oracle: central finite differences of the separately pinned forward
oracle, a library autograd in fp64 with the additive large-negative mask of Eq. (2)'s footnote,
and the identities the softmax Jacobian forces."""
import math

import numpy as np
import pytest
import torch

import oracle


def case(seed, B, H, Lq, Lk, D, Dv, density):
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((B, H, Lq, D))
    K = rng.standard_normal((B, H, Lk, D))
    V = rng.standard_normal((B, H, Lk, Dv))
    dO = rng.standard_normal((B, H, Lq, Dv))
    mask = (rng.random((H, Lq, Lk)) < density).astype(np.uint8)
    return Q, K, V, dO, mask


@pytest.mark.parametrize("causal", [False, True])
def test_backward_matches_finite_differences_of_forward_oracle(causal):
    Q, K, V, dO, mask = case(1, 1, 2, 5, 7, 3, 4, 0.6)
    mask[0, 2, :] = 0                                       # a query without any kept key
    dQ, dK, dV = oracle.masked_attention_backward(Q, K, V, mask, dO, causal=causal)

    def loss(q, k, v):
        O, _ = oracle.masked_attention(q, k, v, mask, causal=causal)
        return float((O * dO).sum())

    eps = 1e-6
    for X, G, which in ((Q, dQ, 0), (K, dK, 1), (V, dV, 2)):
        num = np.zeros_like(X)
        it = np.nditer(X, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            args = [Q.copy(), K.copy(), V.copy()]
            args[which][idx] += eps
            up = loss(*args)
            args[which][idx] -= 2 * eps
            dn = loss(*args)
            num[idx] = (up - dn) / (2 * eps)
        np.testing.assert_allclose(G, num, rtol=0, atol=1e-8)


@pytest.mark.parametrize("shape,causal", [((2, 2, 9, 9, 4, 4), True), ((1, 3, 6, 11, 5, 2), False),
                                          ((2, 1, 7, 12, 3, 3), True)])
def test_backward_matches_library_autograd(shape, causal):
    B, H, Lq, Lk, D, Dv = shape
    Q, K, V, dO, mask = case(2, B, H, Lq, Lk, D, Dv, 0.5)
    mask[:, np.arange(Lq), np.arange(Lq) % Lk] = 1          # keep every row non-empty
    if causal:
        mask[:, :, 0] = 1
    q, k, v = (torch.tensor(x, requires_grad=True) for x in (Q, K, V))
    keep = torch.from_numpy(mask != 0)
    if causal:
        keep = keep & (torch.arange(Lk)[None, :] <= torch.arange(Lq)[:, None] + (Lk - Lq))[None]
    s = torch.matmul(q, k.transpose(-1, -2)) / math.sqrt(D)
    s = s + torch.where(keep, 0.0, -1e30)[None]             # additive large negative value
    o = torch.matmul(torch.softmax(s, dim=-1), v)
    o.backward(torch.from_numpy(dO))
    dQ, dK, dV = oracle.masked_attention_backward(Q, K, V, mask, dO, causal=causal)
    np.testing.assert_allclose(dQ, q.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dK, k.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dV, v.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_pruned_keys_get_no_gradient_and_empty_rows_give_none():
    Q, K, V, dO, mask = case(3, 1, 1, 6, 8, 4, 4, 0.5)
    mask[0, :, 5] = 0                                       # key 5 pruned everywhere
    mask[0, 3, :] = 0                                       # query 3 sees nothing
    dQ, dK, dV = oracle.masked_attention_backward(Q, K, V, mask, dO)
    assert np.all(dK[0, 0, 5] == 0) and np.all(dV[0, 0, 5] == 0)
    assert np.all(dQ[0, 0, 3] == 0)


def test_single_kept_key_rows():
    """One kept key per query: P = 1, so dV collects dO and the scores get no gradient."""
    rng = np.random.default_rng(4)
    Q, K, V, dO, _ = case(4, 1, 1, 5, 5, 3, 3, 1.0)
    mask = np.zeros((1, 5, 5), np.uint8)
    cols = rng.permutation(5)
    mask[0, np.arange(5), cols] = 1
    dQ, dK, dV = oracle.masked_attention_backward(Q, K, V, mask, dO)
    np.testing.assert_allclose(dV[0, 0, cols], dO[0, 0], rtol=0, atol=0)
    assert np.all(dQ == 0) and np.all(dK == 0)


def test_gradient_is_orthogonal_to_a_common_shift_of_the_scores():
    """softmax is invariant to adding a constant to a row of scores; with K -> K + c (same c for
    every key) each row of scores shifts by <q_i, c>, so sum_j dK_j must vanish when the mask
    keeps whole rows, and does in general once weighted by kept entries: check the dense case."""
    Q, K, V, dO, _ = case(5, 1, 2, 6, 6, 4, 4, 1.0)
    mask = np.ones((2, 6, 6), np.uint8)
    dQ, dK, dV = oracle.masked_attention_backward(Q, K, V, mask, dO)
    np.testing.assert_allclose(dK.sum(axis=2), 0.0, atol=1e-13)
    np.testing.assert_allclose(dV.sum(axis=2), dO.sum(axis=2), atol=1e-13)   # rows of P sum to 1


def test_scale_argument():
    Q, K, V, dO, mask = case(6, 1, 1, 4, 6, 16, 4, 0.7)
    mask[0, :, 0] = 1
    a = oracle.masked_attention_backward(Q, K, V, mask, dO)
    b = oracle.masked_attention_backward(Q, K, V, mask, dO, scale=0.25)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
