"""CPU oracle for the adaptive peer selection of Alg. 3 (and Alg. 1 line 2).  TEST INFRASTRUCTURE ONLY.

Plain numpy/Python statements of the pieces whose outcome is unique: the filtered graph
B*, the recently-connected graph and its components, the candidate matrix E, the size of a
maximum matching (exact, by dynamic programming over vertex subsets, small n only) and the
rules a result must obey.  The matching itself is not unique (RandomlyMaxMatch), so callers
compare sizes and validity, not edges.  Imports nothing of the GPU package.
"""
from __future__ import annotations

from functools import lru_cache
from typing import List, Tuple

import numpy as np

NEVER = np.iinfo(np.int64).min


def symmetrise(B: np.ndarray) -> np.ndarray:
    """Sec. II-C: B_ij = B_ji = min(B_ij, B_ji); diagonal unused (set to 0)."""
    S = np.minimum(B, B.T).astype(np.float64)
    np.fill_diagonal(S, 0.0)
    return S


def filtered_graph(B: np.ndarray, B_thres: float) -> np.ndarray:
    """Alg. 1, GetNewConnectedGraph: B*_ij = 1 iff B_ij >= B_thres (i != j)."""
    E = (symmetrise(B) >= B_thres).astype(np.uint8)
    np.fill_diagonal(E, 0)
    return E


def recently_connected(R: np.ndarray, T_thres: int, t: int) -> np.ndarray:
    """Alg. 3, IfConnected / GetOverTimeMatrix: Q_ij = 1 iff R_ij > t - T_thres."""
    Q = np.zeros(R.shape, dtype=np.uint8)
    ok = R != NEVER
    Q[ok] = R[ok] > t - T_thres
    return Q


def component_labels(Q: np.ndarray) -> Tuple[int, np.ndarray]:
    """Connected components by repeated flooding (no library)."""
    n = Q.shape[0]
    lab = -np.ones(n, dtype=np.int64)
    c = 0
    for s in range(n):
        if lab[s] >= 0:
            continue
        front = [s]; lab[s] = c
        while front:
            v = front.pop()
            for u in range(n):
                if lab[u] < 0 and (Q[v, u] or Q[u, v]):
                    lab[u] = c; front.append(u)
        c += 1
    return c, lab


def candidate_matrix(Bstar: np.ndarray, R: np.ndarray, T_thres: int, t: int) -> Tuple[bool, int, np.ndarray]:
    """Alg. 3 lines 1-5: E = B* if the recently-connected graph is connected, else all pairs
    that join two different components of it."""
    Q = recently_connected(R, T_thres, t)
    ncomp, lab = component_labels(Q)
    if ncomp == 1:
        return True, 1, Bstar.copy()
    E = (lab[:, None] != lab[None, :]).astype(np.uint8)
    return False, ncomp, E


def max_matching_size(E: np.ndarray) -> int:
    """Exact maximum matching size by DP over subsets of vertices (n <= 20)."""
    n = E.shape[0]
    assert n <= 20
    nb = [sum(1 << j for j in range(n) if j != i and (E[i, j] or E[j, i])) for i in range(n)]

    @lru_cache(maxsize=None)
    def best(avail: int) -> int:
        if avail == 0:
            return 0
        i = (avail & -avail).bit_length() - 1          # lowest free vertex: leave it unmatched or match it
        rest = avail & ~(1 << i)
        r = best(rest)
        cand = nb[i] & rest
        while cand:
            j = (cand & -cand).bit_length() - 1
            cand &= cand - 1
            r = max(r, 1 + best(rest & ~(1 << j)))
        return r

    return best((1 << n) - 1)


def check_matching(peer: np.ndarray, E: np.ndarray) -> int:
    """peer must be an involution whose pairs are edges of E; returns the number of pairs."""
    n = len(peer)
    assert np.array_equal(peer[peer], np.arange(n)), "not an involution"
    pairs = 0
    for i in range(n):
        p = int(peer[i])
        if p > i:
            assert E[i, p] or E[p, i], f"pair ({i},{p}) is not an edge"
            pairs += 1
    return pairs
