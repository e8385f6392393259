"""Exact solvers for one MxM block of Eq. (2) / Eq. (3).  TEST INFRASTRUCTURE ONLY.

They pin the oracle from outside: the heuristic mask may never beat the true
optimum, and on the paper's worked example the optimum is the printed value.
  * ``feasible_masks`` / ``brute_force_optimum``: enumerate every 0/1 matrix
    with all row and column sums equal to N (90 of them for 2:4).
  * ``lp_optimum``: the relaxed problem of Eq. (3) solved with HiGHS; Sec. 3.1
    states that its vertices are integral, so its value is the optimum of Eq. (2).
"""
from __future__ import annotations

import itertools

import numpy as np


def feasible_masks(M: int, N: int) -> np.ndarray:
    """All M x M 0/1 matrices whose row sums and column sums are all N."""
    row_patterns = [np.array([1 if k in c else 0 for k in range(M)], dtype=np.int64)
                    for c in itertools.combinations(range(M), N)]
    found = []

    def extend(rows, col_counts):
        depth = len(rows)
        if depth == M:
            if np.all(col_counts == N):
                found.append(np.stack(rows))
            return
        remaining = M - depth - 1
        for pat in row_patterns:
            cc = col_counts + pat
            if np.any(cc > N) or np.any(cc + remaining < N):
                continue
            extend(rows + [pat], cc)

    extend([], np.zeros(M, dtype=np.int64))
    return np.stack(found).astype(np.uint8)


def brute_force_optimum(imp_block: np.ndarray, N: int, masks: np.ndarray | None = None) -> float:
    """max over all feasible masks of <S, imp> for one block (double accumulation)."""
    imp_block = np.asarray(imp_block, dtype=np.float64)
    M = imp_block.shape[0]
    if masks is None:
        masks = feasible_masks(M, N)
    return float(np.max(np.tensordot(masks.astype(np.float64), imp_block, axes=([1, 2], [0, 1]))))


def lp_optimum(imp_block: np.ndarray, N: int):
    """Optimum value and an optimal vertex of Eq. (3) for one block (HiGHS dual simplex)."""
    from scipy.optimize import linprog

    imp_block = np.asarray(imp_block, dtype=np.float64)
    M = imp_block.shape[0]
    A = np.zeros((2 * M, M * M))
    for i in range(M):
        A[i, i * M:(i + 1) * M] = 1.0          # row i sums to N
        A[M + i, i::M] = 1.0                   # column i sums to N
    res = linprog(-imp_block.ravel(), A_eq=A, b_eq=np.full(2 * M, float(N)), bounds=(0.0, 1.0),
                  method="highs-ds")
    if res.status != 0:
        raise RuntimeError(f"linprog failed: {res.message}")
    return float(-res.fun), res.x.reshape(M, M)


def blocks(a: np.ndarray, M: int) -> np.ndarray:
    """View a (rows, cols) array as (rows/M * cols/M, M, M) blocks, block-row major."""
    rows, cols = a.shape
    return a.reshape(rows // M, M, cols // M, M).transpose(0, 2, 1, 3).reshape(-1, M, M)


def is_transposable_nm(mask: np.ndarray, N: int, M: int) -> bool:
    """Every row and column of every MxM block holds exactly N ones and entries are 0/1."""
    b = blocks(np.asarray(mask), M).astype(np.int64)
    return bool(np.all((b == 0) | (b == 1)) and np.all(b.sum(axis=1) == N) and np.all(b.sum(axis=2) == N))
