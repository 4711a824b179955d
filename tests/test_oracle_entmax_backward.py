"""Pins for the gradient of the 1.5-entmax oracle (Section 6's normaliser under the pruning mask):
central finite differences of the separately pinned forward oracle, fp64 autograd through a
forward written with differentiable tensor ops, and the properties the Jacobian must have."""
import math

import numpy as np
import pytest
import torch

import oracle


def finite_difference(f, x, eps=1e-6):
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[i] += eps
        xm[i] -= eps
        g[i] = (f(xp) - f(xm)) / (2 * eps)
    return g


@pytest.mark.parametrize("seed", range(5))
def test_vector_jacobian_against_finite_differences(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 10))
    z = rng.standard_normal(n) * rng.choice([0.5, 1.5])
    g = rng.standard_normal(n)
    want = finite_difference(lambda zz: float(oracle.entmax15(zz)[0] @ g), z)
    np.testing.assert_allclose(oracle.entmax15_backward(z, g), want, atol=2e-8)


def entmax15_torch(z):
    """The same conditions with differentiable tensor ops (sort, cumsum, sqrt): autograd then
    derives the Jacobian on its own."""
    x, _ = torch.sort(z / 2, descending=True)
    k = torch.arange(1, x.numel() + 1, dtype=z.dtype)
    s1, s2 = torch.cumsum(x, 0), torch.cumsum(x * x, 0)
    disc = s1 * s1 - k * (s2 - 1)
    tau_k = (s1 - torch.sqrt(torch.clamp(disc, min=0))) / k
    ksup = int(torch.nonzero((disc >= 0) & (x > tau_k)).max())
    return torch.clamp(z / 2 - tau_k[ksup], min=0) ** 2


@pytest.mark.parametrize("seed", range(4))
def test_vector_jacobian_against_autograd(seed):
    rng = np.random.default_rng(50 + seed)
    z = rng.standard_normal(9) * 1.2
    g = rng.standard_normal(9)
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    (entmax15_torch(zt) @ torch.tensor(g)).backward()
    np.testing.assert_allclose(oracle.entmax15_backward(z, g), zt.grad.numpy(), atol=1e-12)


def test_jacobian_properties():
    rng = np.random.default_rng(7)
    z = rng.standard_normal(11) * 2.0
    g = rng.standard_normal(11)
    p, _ = oracle.entmax15(z)
    dz = oracle.entmax15_backward(z, g)
    assert abs(dz.sum()) < 1e-13                       # a common shift of the scores changes nothing
    assert np.all(dz[p == 0] == 0)                     # no gradient outside the support
    np.testing.assert_allclose(oracle.entmax15_backward(z, g + 4.2), dz, atol=1e-13)   # sum p = 1
    # one-hot output (gap >= 2 to the runner-up): the output does not move with the scores
    assert np.all(oracle.entmax15_backward(np.array([0.0, 5.0, 2.5]), np.array([1.0, -2.0, 0.3])) == 0)
    # two entries, closed form: p1 = ((d + r) / 2)^2, r = sqrt(2 - d^2), d = (z1 - z2) / 2
    d = 0.3
    r = math.sqrt(2 - d * d)
    dp1_dz1 = 2 * ((d + r) / 2) * (0.5 - d / (2 * r)) / 2          # d p1 / d z1 = (d p1 / d d) / 2
    got = oracle.entmax15_backward(np.array([0.4 + 2 * d, 0.4]), np.array([1.0, 0.0]))
    np.testing.assert_allclose(got, [dp1_dz1, -dp1_dz1], rtol=1e-12)


def loss(Q, K, V, mask, W, causal, scale):
    O, _ = oracle.masked_entmax15_attention(Q, K, V, mask, causal=causal, scale=scale)
    return float((O * W).sum())


@pytest.mark.parametrize("causal", [False, True])
def test_attention_gradients_against_finite_differences(causal):
    rng = np.random.default_rng(11 + causal)
    B, H, Lq, Lk, D = 1, 2, 5, 7, 4
    Q, K, V, W = (rng.standard_normal(s) for s in ((B, H, Lq, D), (B, H, Lk, D), (B, H, Lk, D), (B, H, Lq, D)))
    mask = (rng.random((H, Lq, Lk)) < 0.6).astype(np.uint8)
    mask[0, 2] = 0                                       # a query without kept keys
    mask[:, :, 0] = 1
    if not causal:
        mask[0, 2] = 0
    dQ, dK, dV = oracle.masked_entmax15_attention_backward(Q, K, V, mask, W, causal=causal, scale=0.7)
    np.testing.assert_allclose(dQ, finite_difference(lambda x: loss(x, K, V, mask, W, causal, 0.7), Q), atol=5e-8)
    np.testing.assert_allclose(dK, finite_difference(lambda x: loss(Q, x, V, mask, W, causal, 0.7), K), atol=5e-8)
    np.testing.assert_allclose(dV, finite_difference(lambda x: loss(Q, K, x, mask, W, causal, 0.7), V), atol=5e-8)
    assert np.all(dQ[0, 0, 2] == 0) or causal            # the empty query gets no gradient


def test_single_kept_key_and_default_scale():
    rng = np.random.default_rng(3)
    B, H, L, D = 1, 1, 6, 8
    Q, K, V, W = (rng.standard_normal((B, H, L, D)) for _ in range(4))
    mask = np.eye(L, dtype=np.uint8)[None]               # every query keeps exactly its own key
    dQ, dK, dV = oracle.masked_entmax15_attention_backward(Q, K, V, mask, W)
    assert np.all(dQ == 0) and np.all(dK == 0)           # p = 1 whatever the score
    np.testing.assert_allclose(dV, W, atol=1e-15)        # dV_j collects dO_j
    full = np.ones((1, L, L), np.uint8)
    a = oracle.masked_entmax15_attention_backward(Q, K, V, full, W)
    b = oracle.masked_entmax15_attention_backward(Q, K, V, full, W, scale=1 / math.sqrt(D))
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
    # unpruned: sum_j dK_j = 0 would need sum_j dS_ij = 0 per query, which the Jacobian gives
    np.testing.assert_allclose(a[1].sum(axis=2), 0.0, atol=1e-12)
