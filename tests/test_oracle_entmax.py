"""Pins for the 1.5-entmax oracle (Section 6's normaliser): the defining optimisation problem
solved by a library optimiser, closed forms for two entries and for equal scores, the optimality
conditions, invariances, and a brute-force comparison of the objective on the simplex."""
import itertools
import math

import numpy as np
import pytest
from scipy.optimize import minimize

import oracle


def objective(p, z):
    """<p, z> + Tsallis entropy with a = 1.5: what entmax maximises over the simplex."""
    return float(p @ z + (4.0 / 3.0) * np.sum(p - p ** 1.5))


@pytest.mark.parametrize("seed", range(6))
def test_solves_the_defining_problem_library_optimiser(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 9))
    z = rng.standard_normal(n) * rng.choice([0.3, 1.0, 3.0])
    p, tau = oracle.entmax15(z)
    cons = ({"type": "eq", "fun": lambda q: q.sum() - 1.0},)
    res = minimize(lambda q: -objective(np.clip(q, 0, None), z), np.full(n, 1.0 / n), method="SLSQP",
                   bounds=[(0.0, 1.0)] * n, constraints=cons, options={"ftol": 1e-14, "maxiter": 500})
    assert objective(p, z) >= objective(np.clip(res.x, 0, None), z) - 1e-9
    np.testing.assert_allclose(p, res.x, atol=2e-5)


def test_two_entries_closed_form():
    for d in (0.0, 0.3, 0.9, 1.0, 1.7):                     # d = (z1 - z2) / 2
        z = np.array([0.4 + 2 * d, 0.4])
        p, _ = oracle.entmax15(z)
        if d >= 1.0:
            np.testing.assert_allclose(p, [1.0, 0.0], atol=1e-15)
        else:
            r = math.sqrt(2.0 - d * d)
            np.testing.assert_allclose(p, [((d + r) / 2) ** 2, ((r - d) / 2) ** 2], rtol=1e-13)


def test_equal_scores_give_uniform_and_large_gap_gives_one_hot():
    p, _ = oracle.entmax15(np.full(7, 1.3))
    np.testing.assert_allclose(p, 1.0 / 7, rtol=1e-14)
    p, _ = oracle.entmax15(np.array([0.1, 5.0, 2.9, -1.0]))     # gap to the runner-up >= 2
    assert p.tolist() == [0.0, 1.0, 0.0, 0.0]


@pytest.mark.parametrize("seed", range(4))
def test_optimality_conditions_and_invariances(seed):
    rng = np.random.default_rng(100 + seed)
    z = rng.standard_normal(12) * 2.0
    p, tau = oracle.entmax15(z)
    assert abs(p.sum() - 1.0) < 1e-13 and np.all(p >= 0)
    np.testing.assert_allclose(p, np.maximum(z / 2 - tau, 0.0) ** 2, rtol=0, atol=1e-16)
    assert np.all(z[p == 0] / 2 <= tau) and np.all(z[p > 0] / 2 > tau)
    p2, tau2 = oracle.entmax15(z + 3.7)                          # common shift: same p, tau moves by half of it
    np.testing.assert_allclose(p2, p, atol=1e-13)
    assert abs(tau2 - tau - 1.85) < 1e-13
    perm = rng.permutation(12)
    np.testing.assert_allclose(oracle.entmax15(z[perm])[0], p[perm], atol=1e-15)


def test_brute_force_on_a_grid_of_the_simplex():
    z = np.array([0.9, 0.2, -0.4])
    p, _ = oracle.entmax15(z)
    best = objective(p, z)
    n = 60
    for a, b in itertools.product(range(n + 1), repeat=2):
        if a + b <= n:
            q = np.array([a, b, n - a - b]) / n
            assert objective(q, z) <= best + 1e-12


def test_masked_attention_uses_only_kept_visible_keys():
    rng = np.random.default_rng(7)
    Q, K, V = rng.standard_normal((1, 2, 5, 4)), rng.standard_normal((1, 2, 7, 4)), rng.standard_normal((1, 2, 7, 3))
    mask = (rng.random((2, 5, 7)) < 0.6).astype(np.uint8)
    mask[0, 1, :] = 0                                            # a query without kept keys
    O, tau = oracle.masked_entmax15_attention(Q, K, V, mask, causal=True)
    assert np.all(O[0, 0, 1] == 0) and np.isinf(tau[0, 0, 1])
    vis = np.arange(7)[None, :] <= np.arange(5)[:, None] + 2
    for h in range(2):
        for i in range(5):
            cols = np.flatnonzero((mask[h, i] != 0) & vis[i])
            if cols.size == 0:
                continue
            z = (Q[0, h, i] @ K[0, h, cols].T) / 2.0             # 1/sqrt(4)
            p, _ = oracle.entmax15(z)
            np.testing.assert_allclose(O[0, h, i], p @ V[0, h, cols], rtol=1e-13, atol=1e-15)
    # single kept key: the output is that value row
    m1 = np.zeros((2, 5, 7), np.uint8)
    m1[:, np.arange(5), np.arange(5)] = 1
    O1, _ = oracle.masked_entmax15_attention(Q, K, V, m1)
    np.testing.assert_allclose(O1[0, :, :, :], V[0][:, :5, :], rtol=1e-15, atol=0)   # p = (x - (x - 1))^2
