"""Pins for the fp64 CPU oracle: it is checked here against things other than itself --
a library softmax/matmul, the additive large-negative formulation of the paper's footnote,
closed forms, invariances, brute-force enumeration and hand-computed fixtures."""
import itertools
import json
import math
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_qkv(seed, B, H, Lq, Lk, D, Dv=None):
    rng = np.random.default_rng(seed)
    Dv = D if Dv is None else Dv
    return (rng.standard_normal((B, H, Lq, D)), rng.standard_normal((B, H, Lk, D)),
            rng.standard_normal((B, H, Lk, Dv)))


def rand_mask(seed, H, Lq, Lk, density, nonempty=True):
    rng = np.random.default_rng(seed)
    m = rng.random((H, Lq, Lk)) < density
    if nonempty:
        cols = rng.integers(0, Lk, size=(H, Lq))
        hh, ii = np.meshgrid(np.arange(H), np.arange(Lq), indexing="ij")
        m[hh, ii, cols] = True
    return m.astype(np.uint8)


# --- Section 3.1 / sentence after the masked equation: M_p = 0 gives ordinary attention ---------

@pytest.mark.parametrize("shape", [(2, 3, 7, 7, 5, 5), (1, 2, 5, 11, 4, 6), (1, 1, 13, 3, 8, 2)])
def test_all_ones_mask_is_dense_attention_library(shape):
    B, H, Lq, Lk, D, Dv = shape
    Q, K, V = rand_qkv(1, B, H, Lq, Lk, D, Dv)
    O, lse = oracle.masked_attention(Q, K, V, np.ones((H, Lq, Lk), np.uint8))
    tq, tk, tv = (torch.from_numpy(x) for x in (Q, K, V))
    s = tq @ tk.transpose(-1, -2) / math.sqrt(D)
    ref = torch.softmax(s, dim=-1) @ tv
    np.testing.assert_allclose(O, ref.numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, torch.logsumexp(s, dim=-1).numpy(), rtol=0, atol=1e-13)


def test_dense_matches_torch_sdpa_kernel():
    B, H, Lq, Lk, D = 2, 2, 9, 12, 8
    Q, K, V = rand_qkv(2, B, H, Lq, Lk, D)
    O, _ = oracle.masked_attention(Q, K, V, np.ones((H, Lq, Lk), np.uint8))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V))
    np.testing.assert_allclose(O, ref.numpy(), rtol=0, atol=1e-12)


def test_explicit_scale_is_used():
    B, H, Lq, Lk, D = 1, 1, 4, 6, 3
    Q, K, V = rand_qkv(3, B, H, Lq, Lk, D)
    O, lse = oracle.masked_attention(Q, K, V, np.ones((H, Lq, Lk), np.uint8), scale=0.37)
    s = torch.from_numpy(Q) @ torch.from_numpy(K).transpose(-1, -2) * 0.37
    np.testing.assert_allclose(O, (torch.softmax(s, -1) @ torch.from_numpy(V)).numpy(), atol=1e-13)
    np.testing.assert_allclose(lse, torch.logsumexp(s, -1).numpy(), atol=1e-13)


# --- Eq. (2) footnote: the mask is a large negative number added before the softmax -----------

@pytest.mark.parametrize("density", [0.05, 0.3, 0.8])
def test_additive_large_negative_formulation(density):
    B, H, Lq, Lk, D = 2, 3, 17, 23, 6
    Q, K, V = rand_qkv(4, B, H, Lq, Lk, D)
    mask = rand_mask(5, H, Lq, Lk, density)
    O, lse = oracle.masked_attention(Q, K, V, mask)
    # (Q K^T + M)/sqrt(d_k) with M = -1e9 on pruned entries; exp(-1e9/sqrt(d)) underflows to 0
    M = np.where(mask != 0, 0.0, -1e9)[None]
    s = (np.einsum("bhid,bhjd->bhij", Q, K) + M) / math.sqrt(D)
    ref = torch.softmax(torch.from_numpy(s), dim=-1).numpy() @ V
    np.testing.assert_allclose(O, ref, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, torch.logsumexp(torch.from_numpy(s), -1).numpy(), atol=1e-12)


# --- closed forms ---------------------------------------------------------------------------

def test_single_kept_entry_returns_that_value_row_exactly():
    B, H, Lq, Lk, D = 2, 2, 6, 9, 4
    Q, K, V = rand_qkv(6, B, H, Lq, Lk, D)
    rng = np.random.default_rng(7)
    cols = rng.integers(0, Lk, size=(H, Lq))
    mask = np.zeros((H, Lq, Lk), np.uint8)
    for h in range(H):
        mask[h, np.arange(Lq), cols[h]] = 1
    O, lse = oracle.masked_attention(Q, K, V, mask)
    for b in range(B):
        for h in range(H):
            for i in range(Lq):
                j = cols[h, i]
                assert np.array_equal(O[b, h, i], V[b, h, j])          # bitwise
                s = float(np.dot(Q[b, h, i], K[b, h, j])) / math.sqrt(D)
                assert abs(lse[b, h, i] - s) < 1e-14


def test_zero_queries_give_mean_of_kept_values():
    B, H, Lq, Lk, D = 1, 2, 8, 10, 5
    _, K, V = rand_qkv(8, B, H, Lq, Lk, D)
    Q = np.zeros((B, H, Lq, D))
    mask = rand_mask(9, H, Lq, Lk, 0.4)
    O, lse = oracle.masked_attention(Q, K, V, mask)
    for h in range(H):
        for i in range(Lq):
            kept = np.nonzero(mask[h, i])[0]
            np.testing.assert_allclose(O[0, h, i], V[0, h, kept].mean(axis=0), atol=1e-14)
            assert abs(lse[0, h, i] - math.log(len(kept))) < 1e-14


def test_constant_values_pass_through():
    B, H, Lq, Lk, D = 1, 2, 8, 10, 5
    Q, K, _ = rand_qkv(10, B, H, Lq, Lk, D)
    V = np.ones((B, H, Lk, 3))
    O, _ = oracle.masked_attention(Q, K, V, rand_mask(11, H, Lq, Lk, 0.3))
    np.testing.assert_allclose(O, 1.0, atol=1e-14)


def test_two_key_worked_example_fixture():
    # tests/golden/two_key_example.json: hand-computed softmax over scores (0, ln 3)
    with open(os.path.join(GOLDEN, "two_key_example.json")) as f:
        g = json.load(f)
    Q = np.array(g["Q"], float)[None, None]
    K = np.array(g["K"], float)[None, None]
    V = np.array(g["V"], float)[None, None]
    mask = np.array(g["mask"], np.uint8)[None]
    O, lse = oracle.masked_attention(Q, K, V, mask, scale=g["scale"])
    np.testing.assert_allclose(O[0, 0], np.array(g["O"], float), atol=1e-14)
    np.testing.assert_allclose(lse[0, 0], np.array(g["lse"], float), atol=1e-14)


# --- invariances ------------------------------------------------------------------------------

def test_key_permutation_invariance():
    B, H, Lq, Lk, D = 2, 2, 7, 12, 4
    Q, K, V = rand_qkv(12, B, H, Lq, Lk, D)
    mask = rand_mask(13, H, Lq, Lk, 0.4)
    perm = np.random.default_rng(14).permutation(Lk)
    O1, l1 = oracle.masked_attention(Q, K, V, mask)
    O2, l2 = oracle.masked_attention(Q, K[:, :, perm], V[:, :, perm], mask[:, :, perm])
    np.testing.assert_allclose(O1, O2, atol=1e-13)
    np.testing.assert_allclose(l1, l2, atol=1e-13)


def test_key_shift_invariance():
    B, H, Lq, Lk, D = 1, 2, 7, 12, 4
    Q, K, V = rand_qkv(15, B, H, Lq, Lk, D)
    mask = rand_mask(16, H, Lq, Lk, 0.4)
    c = np.random.default_rng(17).standard_normal(D)
    O1, l1 = oracle.masked_attention(Q, K, V, mask)
    O2, l2 = oracle.masked_attention(Q, K + c, V, mask)
    np.testing.assert_allclose(O1, O2, atol=1e-12)
    np.testing.assert_allclose(l2 - l1, (Q @ c) / math.sqrt(D), atol=1e-12)


def test_mask_has_no_batch_index():
    # the same global mask applies to every example of the batch (Section 3.2)
    B, H, Lq, Lk, D = 3, 2, 5, 6, 4
    Q, K, V = rand_qkv(18, B, H, Lq, Lk, D)
    mask = rand_mask(19, H, Lq, Lk, 0.5)
    O, lse = oracle.masked_attention(Q, K, V, mask)
    for b in range(B):
        Ob, lb = oracle.masked_attention(Q[b:b + 1], K[b:b + 1], V[b:b + 1], mask)
        assert np.array_equal(O[b], Ob[0]) and np.array_equal(lse[b], lb[0])


# --- causal composition (Transformer-XL figure caption) --------------------------------------------

@pytest.mark.parametrize("Lq,Lk", [(9, 9), (5, 12)])
def test_causal_flag_equals_intersection_with_bottom_right_triangle(Lq, Lk):
    B, H, D = 2, 2, 4
    Q, K, V = rand_qkv(20, B, H, Lq, Lk, D)
    mask = rand_mask(21, H, Lq, Lk, 0.6)
    tri = (np.arange(Lk)[None, :] <= np.arange(Lq)[:, None] + (Lk - Lq)).astype(np.uint8)
    O1, l1 = oracle.masked_attention(Q, K, V, mask, causal=True)
    O2, l2 = oracle.masked_attention(Q, K, V, mask * tri[None], causal=False)
    assert np.array_equal(O1, O2) and np.array_equal(l1, l2)
    # first query of a square causal problem sees only key 0
    if Lq == Lk:
        m1 = np.ones((H, Lq, Lk), np.uint8)
        O3, _ = oracle.masked_attention(Q, K, V, m1, causal=True)
        np.testing.assert_array_equal(O3[:, :, 0], V[:, :, 0])


def test_empty_rows_give_zero_and_minus_inf():
    B, H, Lq, Lk, D = 1, 1, 4, 5, 3
    Q, K, V = rand_qkv(22, B, H, Lq, Lk, D)
    mask = np.ones((H, Lq, Lk), np.uint8)
    mask[0, 2] = 0
    O, lse = oracle.masked_attention(Q, K, V, mask)
    assert np.all(O[0, 0, 2] == 0.0) and lse[0, 0, 2] == -np.inf
    assert np.all(np.isfinite(lse[0, 0, [0, 1, 3]]))
    # kept keys that all lie in the causal future also leave the row empty
    mask2 = np.zeros((H, Lq, Lk), np.uint8)
    mask2[0, :, 4] = 1
    O, lse = oracle.masked_attention(Q, K, V, mask2, causal=True)   # Lk - Lq = 1: row 3 sees key 4
    assert np.all(O[0, 0, :3] == 0.0) and np.all(lse[0, 0, :3] == -np.inf)
    assert np.array_equal(O[0, 0, 3], V[0, 0, 4])


# --- brute force on tiny shapes ------------------------------------------------------------------

def test_brute_force_enumeration_of_all_masks():
    # every one of the 2^(Lq*Lk) masks of a 2x3 problem, sums written out with math.exp
    Lq, Lk, D, Dv = 2, 3, 2, 2
    Q, K, V = rand_qkv(23, 1, 1, Lq, Lk, D, Dv)
    for bits in itertools.product([0, 1], repeat=Lq * Lk):
        mask = np.array(bits, np.uint8).reshape(1, Lq, Lk)
        for causal in (False, True):
            O, lse = oracle.masked_attention(Q, K, V, mask, causal=causal)
            for i in range(Lq):
                num = [0.0] * Dv
                den = 0.0
                for j in range(Lk):
                    if not mask[0, i, j] or (causal and j > i + (Lk - Lq)):
                        continue
                    s = sum(Q[0, 0, i, t] * K[0, 0, j, t] for t in range(D)) / math.sqrt(D)
                    e = math.exp(s)
                    den += e
                    for t in range(Dv):
                        num[t] += e * V[0, 0, j, t]
                if den == 0.0:
                    assert np.all(O[0, 0, i] == 0.0) and lse[0, 0, i] == -np.inf
                else:
                    np.testing.assert_allclose(O[0, 0, i], [x / den for x in num], rtol=1e-13, atol=1e-15)
                    assert abs(lse[0, 0, i] - math.log(den)) < 1e-13


def test_large_scores_do_not_overflow():
    # max-subtraction: scores around 800 would overflow a naive exp
    Q = np.full((1, 1, 1, 1), 40.0)
    K = np.array([20.0, 19.0, -5.0]).reshape(1, 1, 3, 1)
    V = np.array([1.0, 2.0, 3.0]).reshape(1, 1, 3, 1)
    O, lse = oracle.masked_attention(Q, K, V, np.ones((1, 1, 3), np.uint8), scale=1.0)
    e = math.exp(-40.0)
    np.testing.assert_allclose(O[0, 0, 0, 0], (1.0 + 2.0 * e) / (1.0 + e), rtol=1e-13)
    assert abs(lse[0, 0, 0] - (800.0 + math.log1p(e))) < 1e-10


# --- Eq. (3): multiply-accumulate model --------------------------------------------------------

@pytest.mark.parametrize("N,d,h", [(128, 768, 12), (384, 768, 12), (4096, 4096, 32)])
def test_macs_fraction_matches_equation_3(N, d, h):
    for p in (0.0, 0.25, 0.5, 0.9, 1.0):
        closed = (4 * d + (2 - p) * N) / (4 * d + 2 * N)
        assert abs(oracle.macs_fraction(N, d, p, B=3, h=h) - closed) < 1e-12
    assert oracle.macs_fraction(N, d, 0.0) == 1.0
    assert abs(oracle.macs_fraction(N, d, 1.0) - (4 * d + N) / (4 * d + 2 * N)) < 1e-12


def test_kept_entry_flops_counts_both_products():
    mask = np.zeros((2, 4, 4), np.uint8)
    mask[0, 1, 0] = mask[0, 1, 3] = mask[1, 3, 3] = 1
    assert oracle.kept_entry_flops(mask, B=5, D=8) == 4 * 8 * 3 * 5
    assert oracle.kept_entry_flops(mask, B=5, D=8, causal=True) == 4 * 8 * 2 * 5
    ones = np.ones((1, 6, 6), np.uint8)
    assert oracle.kept_entry_flops(ones, B=1, D=2, causal=True) == 4 * 2 * 21
