"""Pins for the mask-construction oracle (Section 3.2, Eq. (1) and Eq. (2)): hand-computed
fixtures, closed forms, a library softmax, the already pinned masked-attention oracle, numpy's
order statistics, and the counting properties the percentile must have."""
import json
import math
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_qk(seed, B, H, Lq, Lk, D):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((B, H, Lq, D)), rng.standard_normal((B, H, Lk, D))


# --- attention maps: A_i = softmax(Q K^T / sqrt(d_k)) ---------------------------------------------

def test_maps_hand_example_and_mean():
    g = json.load(open(os.path.join(GOLDEN, "mean_map_two_examples.json")))
    Q, K = np.array(g["Q"]), np.array(g["K"])
    A = oracle.attention_maps(Q, K, scale=g["scale"])
    np.testing.assert_allclose(A, np.array(g["A"]), rtol=0, atol=1e-15)
    abar = oracle.mean_attention_map(Q, K, scale=g["scale"])
    np.testing.assert_allclose(abar, np.array(g["abar"]), rtol=0, atol=1e-15)


@pytest.mark.parametrize("shape,causal", [((2, 3, 7, 7, 5), False), ((2, 2, 5, 11, 4), True),
                                          ((1, 2, 9, 9, 8), True), ((3, 1, 6, 4, 3), False)])
def test_maps_match_library_softmax(shape, causal):
    B, H, Lq, Lk, D = shape
    Q, K = rand_qk(3, *shape)
    A = oracle.attention_maps(Q, K, causal=causal)
    S = torch.matmul(torch.from_numpy(Q), torch.from_numpy(K).transpose(-1, -2)) / math.sqrt(D)
    if causal:
        i = torch.arange(Lq)[:, None]
        j = torch.arange(Lk)[None, :]
        S = S.masked_fill(j > i + (Lk - Lq), float("-inf"))
    ref = torch.softmax(S, dim=-1).numpy()
    np.testing.assert_allclose(A, ref, rtol=1e-13, atol=1e-15)


def test_maps_are_row_stochastic_and_causal_zeros_exact():
    Q, K = rand_qk(5, 2, 2, 6, 9, 4)
    A = oracle.attention_maps(Q, K, causal=True)
    np.testing.assert_allclose(A.sum(-1), 1.0, rtol=0, atol=1e-14)
    for i in range(6):
        assert np.all(A[..., i, i + 4:] == 0.0)          # j > i + (Lk - Lq) = i + 3
        assert np.all(A[..., i, :i + 4] > 0.0)
    abar = oracle.mean_attention_map(Q, K, causal=True)
    np.testing.assert_allclose(abar.sum(-1), 1.0, rtol=0, atol=1e-14)   # a mean of stochastic rows


def test_zero_queries_give_uniform_rows():
    Q, K = rand_qk(7, 2, 1, 5, 5, 3)
    A = oracle.attention_maps(np.zeros_like(Q), K, causal=True)
    for i in range(5):
        np.testing.assert_allclose(A[:, :, i, :i + 1], 1.0 / (i + 1), rtol=0, atol=1e-15)


def test_two_keys_closed_form_is_a_sigmoid():
    q, k1, k2, scale = 1.7, 0.4, -1.1, 0.6
    A = oracle.attention_maps(np.array([[[[q]]]]), np.array([[[[k1], [k2]]]]), scale=scale)
    sig = 1.0 / (1.0 + math.exp(-scale * q * (k1 - k2)))
    np.testing.assert_allclose(A[0, 0, 0], [sig, 1.0 - sig], rtol=1e-14)


def test_default_scale_is_inverse_sqrt_dk():
    Q, K = rand_qk(8, 1, 1, 4, 6, 16)
    np.testing.assert_array_equal(oracle.attention_maps(Q, K), oracle.attention_maps(Q, K, scale=0.25))
    assert not np.allclose(oracle.attention_maps(Q, K), oracle.attention_maps(Q, K, scale=1.0))


@pytest.mark.parametrize("causal", [False, True])
def test_maps_times_values_is_the_pinned_attention(causal):
    """A V must be the unmasked output of the masked-attention oracle (pinned on its own):
    a transposed operand or a wrong causal alignment in the maps shows here."""
    Q, K = rand_qk(11, 2, 2, 6, 8, 5)
    V = np.random.default_rng(12).standard_normal((2, 2, 8, 3))
    A = oracle.attention_maps(Q, K, causal=causal)
    O, _ = oracle.masked_attention(Q, K, V, np.ones((2, 6, 8), np.uint8), causal=causal)
    np.testing.assert_allclose(A @ V, O, rtol=1e-12, atol=1e-14)


def test_mean_is_over_examples_not_heads():
    Q, K = rand_qk(13, 3, 2, 4, 4, 2)
    A = oracle.attention_maps(Q, K)
    abar = oracle.mean_attention_map(Q, K)
    assert abar.shape == (2, 4, 4)
    np.testing.assert_allclose(abar, (A[0] + A[1] + A[2]) / 3.0, rtol=1e-15)


# --- threshold and mask: Eq. (2) --------------------------------------------------------------------

def test_percentile_hand_example():
    g = json.load(open(os.path.join(GOLDEN, "percentile_two_heads.json")))
    abar = np.array(g["abar"])
    tau, rank, n = oracle.percentile_threshold(abar, g["p"])
    assert (tau, rank, n) == (g["tau"], g["rank"], 12)
    mask, tau2 = oracle.prune_mask(abar, g["p"])
    assert tau2 == g["tau"]
    np.testing.assert_array_equal(mask, np.array(g["keep"], dtype=np.uint8))


def test_threshold_is_layer_wise_not_per_head():
    rng = np.random.default_rng(17)
    small = rng.random((1, 4, 6)) * 0.1                   # every entry of head 0 below every entry of head 1
    large = 0.5 + rng.random((1, 4, 6)) * 0.1
    mask, tau = oracle.prune_mask(np.concatenate([small, large]), 0.5)
    assert mask[0].sum() == 0 and mask[1].sum() == 24
    assert tau == large.min()


def test_ties_with_the_threshold_are_kept():
    abar = np.array([[[0.2, 0.2, 0.5, 0.2]]])
    mask, tau = oracle.prune_mask(abar, 0.5)               # rank 2 -> tau = 0.2, nothing is below it
    assert tau == 0.2 and mask.tolist() == [[[1, 1, 1, 1]]]
    mask, tau = oracle.prune_mask(abar, 0.75)              # rank 3 -> tau = 0.5
    assert tau == 0.5 and mask.tolist() == [[[0, 0, 1, 0]]]


@pytest.mark.parametrize("p", [0.0, 0.1, 0.3, 0.5, 0.9, 0.99])
@pytest.mark.parametrize("causal", [False, True])
def test_pruned_count_and_numpy_order_statistics(p, causal):
    rng = np.random.default_rng(19)
    H, Lq, Lk = 3, 10, 13
    abar = rng.random((H, Lq, Lk))                         # distinct with probability 1
    vis = np.arange(Lk)[None, :] <= np.arange(Lq)[:, None] + (Lk - Lq) if causal else np.ones((Lq, Lk), bool)
    vals = abar[:, vis].ravel()
    tau, rank, n = oracle.percentile_threshold(abar, p, causal)
    assert n == vals.size and rank == math.floor(p * n)
    assert tau == np.partition(vals, rank)[rank]
    # numpy's interpolating percentile brackets it
    assert np.percentile(vals, 100 * p, method="lower") <= tau <= np.percentile(vals, 100 * p, method="higher")
    mask, _ = oracle.prune_mask(abar, p, causal)
    assert int(vis.sum()) * H - int(mask.sum()) == rank    # exactly floor(p n) visible entries pruned
    assert np.all(mask[:, ~vis] == 0)                      # hidden entries are never kept
    kept_min = abar[mask == 1].min()
    pruned = abar[(mask == 0) & vis[None]]
    assert pruned.size == 0 or pruned.max() < tau <= kept_min


def test_p_zero_keeps_everything_and_p_one_nothing():
    abar = np.random.default_rng(23).random((2, 5, 5))
    mask, _ = oracle.prune_mask(abar, 0.0, causal=True)
    assert mask.sum() == 2 * 15
    mask, tau = oracle.prune_mask(abar, 1.0)
    assert mask.sum() == 0 and np.isinf(tau)


def test_float32_input_gives_a_float32_element():
    abar = np.random.default_rng(29).random((2, 7, 9)).astype(np.float32)
    tau, rank, _ = oracle.percentile_threshold(abar, 0.9)
    assert tau.dtype == np.float32 and tau in abar
    assert (abar < tau).sum() == rank
