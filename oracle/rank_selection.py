"""Float64 CPU oracle for the rank-selection front end of ASI (Sec. 3.3, Eq. 5-9, App. A.2).

THIS IS TEST INFRASTRUCTURE, like asi_oracle.py: only the tests may call it; the GPU library never
does, and the two share no code.  Everything here is a definition written out (singular values of
an unfolding, a truncated HOSVD, a Frobenius norm, an exhaustive search), on library SVD and plain
loops.

Readings of the paper (each also listed in the design notes):
  * "Truncating with respect to eps" (Sec. 3.3, Step 1; HOSVD_eps of App. A.2): per mode, keep the
    smallest number r of principal components whose explained variance
    sum_{k <= r} sigma_k^2 / sum_k sigma_k^2 reaches eps, sigma the singular values of the mode's
    unfolding; at least one component is kept.
  * Eq. 9 prints a double sum over i and j in J; J holds ONE threshold index per fine-tuned layer,
    so the objective is sum_i P[i, j_i] and the constraint sum_i M_i(R[i, j_i]) <= B.
  * M_i is Eq. 5: prod_m r_m + sum_m D_m r_m elements.

Parity pins: every function here is pinned by tests/test_oracle_rank_selection.py.
"""
from __future__ import annotations

import itertools
from typing import List, Optional, Sequence, Tuple

import numpy as np

from .asi_oracle import core_project, unfold


def mode_spectrum(A: np.ndarray, m: int) -> np.ndarray:
    """Squared singular values of the mode-m unfolding, descending, padded with zeros to length
    D_m: the eigenvalues of A_m A_m^T (App. A.2)."""
    Am = unfold(np.asarray(A, dtype=np.float64), m)
    s = np.linalg.svd(Am, compute_uv=False)
    lam = np.zeros(Am.shape[0])
    lam[: s.size] = s * s
    return lam


def explained_variance_rank(lam: np.ndarray, eps: float) -> int:
    """Smallest r >= 1 with sum_{k <= r} lam_k >= eps * sum_k lam_k (Sec. 3.3, Step 1)."""
    lam = np.asarray(lam, dtype=np.float64)
    total = float(lam.sum())
    run = 0.0
    for r in range(1, lam.size + 1):
        run += float(lam[r - 1])
        if run >= eps * total:
            return r
    return int(lam.size)


def explained_variance_ranks(A: np.ndarray, eps: float) -> Tuple[int, ...]:
    """One rank per mode for one threshold: a row of the rank tensor R (Sec. 3.3)."""
    return tuple(explained_variance_rank(mode_spectrum(A, m), eps) for m in range(A.ndim))


def hosvd_truncate(A: np.ndarray, ranks: Sequence[int]) -> Tuple[np.ndarray, List[np.ndarray]]:
    """Truncated HOSVD (App. A.2): U_m = the first r_m left singular vectors of A_m, core
    S = A x_1 U_1^T ... x_d U_d^T."""
    A = np.asarray(A, dtype=np.float64)
    U = []
    for m, r in enumerate(ranks):
        Um, _, _ = np.linalg.svd(unfold(A, m), full_matrices=False)
        U.append(Um[:, :r].copy())
    return core_project(A, U), U


def perplexity(dW: np.ndarray, dW_lowrank: np.ndarray) -> float:
    """Eq. 7: Frobenius norm of the difference between the exact and the compressed weight gradient."""
    d = np.asarray(dW, dtype=np.float64) - np.asarray(dW_lowrank, dtype=np.float64)
    return float(np.sqrt(np.sum(d * d)))


def activation_memory(dims: Sequence[int], ranks: Sequence[int]) -> int:
    """Eq. 5: elements kept for one layer, prod_m r_m + sum_m D_m r_m."""
    prod = 1
    for r in ranks:
        prod *= int(r)
    return prod + sum(int(n) * int(r) for n, r in zip(dims, ranks))


def rank_select(P: np.ndarray, M: np.ndarray, budget: int) -> Optional[Tuple[Tuple[int, ...], float]]:
    """Eq. 8-9 by exhaustive search: one threshold index per layer, minimal sum of perplexities
    among the choices whose memories sum to at most `budget`.  P, M: (layers, thresholds).
    Returns (indices, total perplexity), or None if no choice fits.  Among equal totals the first
    in lexicographic order of the indices is returned."""
    P = np.asarray(P, dtype=np.float64)
    M = np.asarray(M)
    n, e = P.shape
    best = None
    for J in itertools.product(range(e), repeat=n):
        mem = sum(int(M[i, j]) for i, j in enumerate(J))
        if mem > budget:
            continue
        tot = 0.0
        for i, j in enumerate(J):
            tot += float(P[i, j])
        if best is None or tot < best[1]:
            best = (J, tot)
    return best
