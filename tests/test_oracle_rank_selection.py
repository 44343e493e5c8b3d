"""Pins of the rank-selection oracle (Sec. 3.3, Eq. 5-9, App. A.2) against what the mathematics fixes:
planted spectra, hand-worked thresholds, the HOSVD truncation bound, a worked selection table and a
dynamic-programming solution of the same budgeted choice (a different algorithm)."""
import itertools

import numpy as np
import pytest

from oracle import asi_oracle as O
from oracle import rank_selection as R


def _orth(rng, n, k):
    q, _ = np.linalg.qr(rng.standard_normal((n, k)))
    return q


def test_spectrum_of_a_matrix_with_planted_singular_values():
    # A_1 = Q diag(s) Z^T folded to (6, 4, 5): its mode-1 spectrum is s^2, by construction
    rng = np.random.default_rng(1)
    s = np.array([9.0, 4.0, 2.0, 1.0, 0.5, 0.25])
    A1 = _orth(rng, 6, 6) @ np.diag(s) @ _orth(rng, 20, 6).T
    A = A1.reshape(6, 4, 5)
    np.testing.assert_allclose(R.mode_spectrum(A, 0), s * s, rtol=1e-12)
    # every mode's spectrum sums to the squared Frobenius norm (trace of the Gram matrix)
    for m in range(3):
        lam = R.mode_spectrum(A, m)
        assert lam.shape == (A.shape[m],)
        assert np.all(np.diff(lam) <= 1e-12)
        np.testing.assert_allclose(lam.sum(), np.sum(A * A), rtol=1e-12)


def test_spectrum_is_padded_when_the_mode_is_longer_than_the_unfolding_is_wide():
    A = np.random.default_rng(2).standard_normal((7, 2, 2))           # A_1 is 7 x 4: at most 4 nonzero values
    lam = R.mode_spectrum(A, 0)
    assert lam.shape == (7,) and np.all(lam[4:] == 0.0) and np.all(lam[:4] > 0.0)
    G = O.unfold(A, 0) @ O.unfold(A, 0).T
    np.testing.assert_allclose(lam, np.sort(np.linalg.eigvalsh(G))[::-1].clip(min=0.0), atol=1e-12)


def test_explained_variance_rank_worked_by_hand():
    lam = np.array([4.0, 3.0, 2.0, 1.0])                              # cumulative 0.4, 0.7, 0.9, 1.0
    want = {0.1: 1, 0.4: 1, 0.5: 2, 0.6: 2, 0.7: 2, 0.8: 3, 0.9: 3, 0.95: 4, 1.0: 4}
    for eps, r in want.items():
        assert R.explained_variance_rank(lam, eps) == r, eps
    assert R.explained_variance_rank(np.array([5.0, 0.0, 0.0]), 0.9) == 1
    assert R.explained_variance_rank(np.array([1.0, 1.0, 1.0, 1.0]), 0.75) == 3


def test_ranks_of_a_tensor_with_one_planted_spectrum_per_mode():
    # core with a dominant corner: every mode sees a spectrum it can be asked about
    rng = np.random.default_rng(3)
    dims = (6, 5, 4, 7)
    S = np.zeros(dims)
    for k in range(4):
        S[k, k, k, k] = [8.0, 4.0, 2.0, 1.0][k]                       # superdiagonal core: every mode has spectrum 64, 16, 4, 1
    U = [_orth(rng, n, n) for n in dims]
    A = O.reconstruct(S, U)
    for m in range(4):
        np.testing.assert_allclose(R.mode_spectrum(A, m)[:4], [64.0, 16.0, 4.0, 1.0], rtol=1e-10)
    # cumulative fractions 64/85 = 0.753, 80/85 = 0.941, 84/85 = 0.988
    assert R.explained_variance_ranks(A, 0.7) == (1, 1, 1, 1)
    assert R.explained_variance_ranks(A, 0.8) == (2, 2, 2, 2)
    assert R.explained_variance_ranks(A, 0.95) == (3, 3, 3, 3)
    assert R.explained_variance_ranks(A, 0.999) == (4, 4, 4, 4)


def test_truncated_hosvd_is_exact_on_a_tucker_tensor_and_obeys_the_tail_bound():
    rng = np.random.default_rng(4)
    dims, ranks = (7, 6, 5, 4), (3, 2, 4, 2)
    A = O.reconstruct(rng.standard_normal(ranks), [_orth(rng, n, r) for n, r in zip(dims, ranks)])
    S, U = R.hosvd_truncate(A, ranks)
    for u, r in zip(U, ranks):
        np.testing.assert_allclose(u.T @ u, np.eye(r), atol=1e-12)
    np.testing.assert_allclose(O.reconstruct(S, U), A, atol=1e-10)
    # a full tensor: squared error at most the discarded tails of all modes, at least the largest single tail
    B = rng.standard_normal(dims)
    S, U = R.hosvd_truncate(B, ranks)
    err = np.sum((B - O.reconstruct(S, U)) ** 2)
    tails = [R.mode_spectrum(B, m)[r:].sum() for m, r in enumerate(ranks)]
    assert max(tails) * (1 - 1e-12) <= err <= sum(tails) * (1 + 1e-12)
    # full ranks: nothing is lost
    S, U = R.hosvd_truncate(B, dims)
    np.testing.assert_allclose(O.reconstruct(S, U), B, atol=1e-10)


def test_truncation_by_threshold_keeps_the_asked_variance_per_mode():
    rng = np.random.default_rng(5)
    A = O.reconstruct(rng.standard_normal((5, 6, 4)) * np.array([4.0, 2.0, 1.0, 0.5])[None, None, :],
                      [_orth(rng, n, r) for n, r in zip((9, 8, 10), (5, 6, 4))])
    for eps in (0.4, 0.6, 0.9):
        ranks = R.explained_variance_ranks(A, eps)
        for m, r in enumerate(ranks):
            lam = R.mode_spectrum(A, m)
            assert lam[:r].sum() >= eps * lam.sum()
            assert r == 1 or lam[: r - 1].sum() < eps * lam.sum()


def test_perplexity_and_memory_by_hand():
    assert R.perplexity(np.array([[3.0, 0.0], [0.0, 0.0]]), np.array([[0.0, 0.0], [0.0, 4.0]])) == 5.0
    assert R.perplexity(np.ones((2, 3)), np.ones((2, 3))) == 0.0
    assert R.activation_memory((2, 3, 4, 5), (1, 2, 3, 4)) == 24 + (2 + 6 + 12 + 20)      # Eq. 5
    assert R.activation_memory((8, 512, 768), (2, 20, 20)) == 800 + 16 + 10240 + 15360
    assert R.activation_memory((2, 3, 4, 5), (1, 2, 3, 4)) == O.storage_elements((2, 3, 4, 5), (1, 2, 3, 4))


def test_rank_select_worked_table():
    P = np.array([[1.0, 5.0], [2.0, 3.0]])
    M = np.array([[10, 4], [10, 5]])
    # (0,0): 20 elements, (0,1): 15, (1,0): 14 -> total 7, (1,1): 9 -> total 8
    assert R.rank_select(P, M, 14) == ((1, 0), 7.0)
    assert R.rank_select(P, M, 13) == ((1, 1), 8.0)
    assert R.rank_select(P, M, 15) == ((0, 1), 4.0)
    assert R.rank_select(P, M, 20) == ((0, 0), 3.0)
    assert R.rank_select(P, M, 8) is None
    # no constraint: every layer takes its own minimum; ties go to the first index
    assert R.rank_select(np.array([[2.0, 2.0, 1.0], [0.5, 0.5, 0.7]]), np.ones((2, 3), dtype=int), 10) == ((2, 0), 1.5)


def _knapsack(P, M, budget):
    """Multiple-choice knapsack by dynamic programming over the memory spent: best[b] = least total
    perplexity of the layers so far with exactly b elements."""
    INF = float("inf")
    best = np.full(budget + 1, INF)
    best[0] = 0.0
    for i in range(P.shape[0]):
        nxt = np.full(budget + 1, INF)
        for j in range(P.shape[1]):
            m = int(M[i, j])
            if m <= budget:
                cand = best[: budget + 1 - m] + P[i, j]
                nxt[m:] = np.minimum(nxt[m:], cand)
        best = nxt
    return None if not np.isfinite(best.min()) else float(best.min())


@pytest.mark.parametrize("seed", range(6))
def test_rank_select_agrees_with_dynamic_programming(seed):
    rng = np.random.default_rng(100 + seed)
    n, e = int(rng.integers(2, 6)), int(rng.integers(2, 5))
    # perplexity falls and memory rises with the threshold, as in the method; integers keep sums exact
    P = np.sort(rng.integers(1, 50, (n, e)), axis=1)[:, ::-1].astype(np.float64)
    M = np.sort(rng.integers(1, 40, (n, e)), axis=1)
    budget = int(M.min(axis=1).sum() + rng.integers(0, 30))
    got = R.rank_select(P, M, budget)
    want = _knapsack(P, M, budget)
    assert got is not None and want is not None
    J, tot = got
    assert tot == want
    assert sum(int(M[i, j]) for i, j in enumerate(J)) <= budget
    assert tot == sum(P[i, j] for i, j in enumerate(J))
    assert R.rank_select(P, M, int(M.min(axis=1).sum()) - 1) is None
