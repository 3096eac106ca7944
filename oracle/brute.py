"""Brute-force definition of the linear-chain CRF.  TEST INFRASTRUCTURE ONLY.

The paper defines a structured distribution by normalising the product of the
part potentials over *all* structures (section "Structured Distributions", Eq. 1
and Eq. 2) and a part's marginal as the total probability of the structures that
contain it (section "Computing Marginals", Eq. 3).  For a chain of L positions
over T tags the structures are the T**L tag paths.  This file enumerates them:
nothing here is a dynamic program, so it can pin the dynamic-programming oracle.

Only usable while T**L stays around 10**6.  float64 throughout; bfloat16 inputs
must be widened by the caller.
"""
from __future__ import annotations

import numpy as np


def all_paths(T: int, L: int) -> np.ndarray:
    """int64 [T**L, L]: every tag path, in lexicographic order (y_0 slowest)."""
    if L == 0:
        return np.zeros((1, 0), dtype=np.int64)
    idx = np.arange(T ** L, dtype=np.int64)
    cols = []
    for i in range(L):
        cols.append((idx // (T ** (L - 1 - i))) % T)
    return np.stack(cols, axis=1)


def path_scores(phi: np.ndarray, L: int, paths: np.ndarray) -> np.ndarray:
    """Log-potential of each path: phi[0, 0, y_0] + sum_i phi[i, y_{i-1}, y_i] (log of Eq. 1)."""
    phi = np.asarray(phi, dtype=np.float64)
    if L == 0:
        return np.zeros((paths.shape[0],), dtype=np.float64)
    sc = phi[0, 0, paths[:, 0]].copy()
    for i in range(1, L):
        sc += phi[i, paths[:, i - 1], paths[:, i]]
    return sc


def enumerate_sequence(phi: np.ndarray, L: int):
    """Everything the definition gives for ONE sequence ``phi[N, T, T]`` of length ``L``.

    Returns a dict with
      logZ      log of the sum over all paths of exp(score)            (Eq. 2)
      mu        [N, T, T] edge marginals; position 0 uses row 0 only    (Eq. 3)
      path      int [N] best path (lexicographically first among exact ties), -1 past L
      score     its score
      gap       best score minus the best score among all *other* paths (inf if none)
      entropy   -sum_y p(y) log p(y)
    """
    phi = np.asarray(phi, dtype=np.float64)
    N, T, _ = phi.shape
    paths = all_paths(T, L)
    sc = path_scores(phi, L, paths)
    m = sc.max()
    if np.isneginf(m):
        logZ = -np.inf
        p = np.zeros_like(sc)
    else:
        logZ = m + np.log(np.exp(sc - m).sum())
        p = np.exp(sc - logZ)
    mu = np.zeros((N, T, T), dtype=np.float64)
    if L > 0:
        np.add.at(mu[0, 0], paths[:, 0], p)
        for i in range(1, L):
            np.add.at(mu[i], (paths[:, i - 1], paths[:, i]), p)
    best = int(np.argmax(sc))  # first maximum = lexicographically first path
    path = np.full((N,), -1, dtype=np.int64)
    path[:L] = paths[best]
    if sc.shape[0] > 1:
        rest = np.delete(sc, best)
        second = rest.max()
        gap = sc[best] - second if np.isfinite(sc[best]) else 0.0
    else:
        gap = np.inf
    with np.errstate(divide="ignore", invalid="ignore"):
        plogp = np.where(p > 0, p * (sc - logZ), 0.0)
    return {"logZ": float(logZ), "mu": mu, "path": path, "score": float(sc[best]),
            "gap": float(gap), "entropy": float(-plogp.sum())}
