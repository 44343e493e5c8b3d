"""The host half of rank selection through the C ABI (no GPU needed): the budgeted backtracking search of
Eq. 8-9 against the oracle's exhaustive search, and Eq. 5."""
import itertools

import numpy as np
import pytest

from oracle import rank_selection as R
from paper_2505_05086_amd import binding as B


def _tables(rng, n, e, integer):
    P = np.sort(rng.random((n, e)) * 10, axis=1)[:, ::-1]
    if integer:
        P = np.round(P * 4)                      # many equal totals: the tie rule shows
    M = np.sort(rng.integers(5, 400, (n, e)), axis=1)
    return np.ascontiguousarray(P), M


@pytest.mark.parametrize("seed", range(8))
def test_backtracking_matches_the_exhaustive_search(seed):
    rng = np.random.default_rng(seed)
    n, e = int(rng.integers(1, 7)), int(rng.integers(1, 7))
    P, M = _tables(rng, n, e, integer=seed % 2 == 0)
    lo, hi = int(M.min(axis=1).sum()), int(M.max(axis=1).sum())
    for budget in sorted({lo, (lo + hi) // 2, (2 * lo + hi) // 3, hi, hi + 5}):
        want = R.rank_select(P, M, budget)
        choice, total = B.asi_rank_select(P.tolist(), M.tolist(), budget)
        assert want is not None
        assert tuple(choice) == want[0]                           # same tie rule: first in lexicographic order
        assert total == pytest.approx(want[1], rel=1e-13, abs=0)
        assert sum(int(M[i, j]) for i, j in enumerate(choice)) <= budget


def test_monotone_tables_of_fourteen_layers_reach_the_knapsack_optimum():
    # too many combinations for the exhaustive search (6^14): the optimum is checked against a dynamic
    # program over the memory spent, a different algorithm
    rng = np.random.default_rng(42)
    n, e = 14, 6
    P = np.sort(rng.integers(1, 60, (n, e)), axis=1)[:, ::-1].astype(np.float64)
    M = np.sort(rng.integers(1, 50, (n, e)), axis=1)
    budget = int(M.min(axis=1).sum()) + 120
    best = np.full(budget + 1, np.inf)
    best[0] = 0.0
    for i in range(n):
        nxt = np.full(budget + 1, np.inf)
        for j in range(e):
            m = int(M[i, j])
            nxt[m:] = np.minimum(nxt[m:], best[: budget + 1 - m] + P[i, j])
        best = nxt
    choice, total = B.asi_rank_select(P.tolist(), M.tolist(), budget)
    assert total == best.min()
    assert sum(int(M[i, j]) for i, j in enumerate(choice)) <= budget
    assert total == sum(P[i, j] for i, j in enumerate(choice))


def test_infeasible_budget_and_bad_arguments():
    P, M = [[1.0, 2.0], [3.0, 4.0]], [[10, 5], [10, 5]]
    with pytest.raises(B.AsiError) as e:
        B.asi_rank_select(P, M, 9)
    assert e.value.status == 6
    assert B.asi_rank_select(P, M, 10) == ([1, 1], 6.0)
    with pytest.raises(B.AsiError) as e:
        B.asi_rank_select([[float("nan"), 1.0]], [[1, 1]], 5)
    assert e.value.status == 1
    with pytest.raises(B.AsiError) as e:
        B.asi_rank_select([[1.0] * 17], [[1] * 17], 5)
    assert e.value.status == 1
    with pytest.raises(ValueError):
        B.asi_rank_select([[1.0, 2.0], [1.0]], [[1, 1], [1, 1]], 5)


def test_activation_memory_is_eq5():
    for dims, ranks in [((2, 3, 4, 5), (1, 2, 3, 4)), ((8, 512, 768), (2, 20, 20)), ((32, 128, 56, 56), (16, 32, 24, 24))]:
        assert B.asi_activation_memory(B.make_desc(dims, ranks)) == R.activation_memory(dims, ranks)
    with pytest.raises(B.AsiError):
        B.asi_activation_memory(B.make_desc((2, 3, 4), (3, 1, 1)))


def test_spectrum_argument_checks_need_no_gpu():
    assert B.asi_mode_spectrum_workspace_bytes(B.make_desc((4, 600, 8, 8), (1, 1, 1, 1)), 1) == 0      # longer than 512
    assert B.asi_mode_spectrum_workspace_bytes(B.make_desc((4, 60, 8, 8), (1, 1, 1, 1)), 4) == 0
    assert B.asi_mode_spectrum_workspace_bytes(B.make_desc((4, 60, 8, 8), (1, 1, 1, 1)), 1) > 60 * 60 * 8
