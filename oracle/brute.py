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


def segmentations(L: int, K: int):
    """All splits of positions 0..L-1 into consecutive segments of 1..K positions, as tuples of
    segment lengths (compositions of L with parts <= K)."""
    if L == 0:
        return [()]
    out = []
    for first in range(1, min(K, L) + 1):
        out += [(first,) + rest for rest in segmentations(L - first, K)]
    return out


def semi_markov_log_partition(phi: np.ndarray, L: int) -> float:
    """log sum over every labelled segmentation of exp(score), by enumeration.  phi: [N, K, T, T]
    float64, phi[i][k][s][t] the score of a segment with tag t ending at i, covering k + 1
    positions, after a segment tagged s (row 0 for the first segment)."""
    import itertools
    _, K, T, _ = phi.shape
    scores = []
    for seg in segmentations(L, K):
        ends = np.cumsum(seg) - 1
        for tags in itertools.product(range(T), repeat=len(seg)):
            sc, prev = 0.0, 0
            for e, n, t in zip(ends, seg, tags):
                sc += phi[e, n - 1, prev, t]
                prev = t
            scores.append(sc)
    scores = np.array(scores)
    m = scores.max()
    return float(m + np.log(np.exp(scores - m).sum())) if np.isfinite(m) else float("-inf")
