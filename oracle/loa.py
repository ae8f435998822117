"""Layout reformatting oracle (Section V-B, Alg. 5, Eq. 5).  TEST INFRASTRUCTURE ONLY.

The basic greedy algorithm, written with Python sets and exact fractions so that it can be read
against the paper: every candidate's computing intensity is recomputed from scratch as
(#non-zero elements) / (#non-zero columns) of the window with the candidate added (Eq. 5).  The
library's implementation follows the optimised algorithm (Alg. 6, Eq. 6: incremental intersection
counts); the two must produce the same windows.

Readings where the paper leaves a choice open (each is also listed in the design notes):
  * N(v) is the set of distinct column indices of row v; |N(v)| is "the degree".
  * the sort by min(N(v)) is ascending and stable in the vertex id; a vertex with no neighbours
    sorts after every vertex that has one.
  * the vertices window of a row window seeded at sorted position p covers the sorted positions
    p .. p + VW inclusive; visited vertices inside it are skipped.
  * the best intensity is searched afresh in each of the 15 growth steps.
  * ties on the intensity go to the higher degree (Alg. 5), remaining ties to the earlier sorted
    position.  Intensities are compared as exact rationals; 0/0 (nothing in the window, candidate
    without neighbours) counts as 0.
  * when the vertices window holds no unvisited vertex, the growth step takes the first unvisited
    vertex of the sorted list, so that every row window except the last holds exactly 16 vertices.
"""
from __future__ import annotations

from fractions import Fraction
from typing import List

import numpy as np

H = 16


def neighbour_sets(rowptr, colind) -> List[frozenset]:
    return [frozenset(int(c) for c in colind[rowptr[v]:rowptr[v + 1]]) for v in range(len(rowptr) - 1)]


def sorted_vertex_list(nbrs: List[frozenset]) -> List[int]:
    """Vertices by their smallest neighbour index (Alg. 5, the sort before the loop)."""
    inf = float("inf")
    return sorted(range(len(nbrs)), key=lambda v: (min(nbrs[v]) if nbrs[v] else inf, v))


def intensity(n_elements: int, n_columns: int) -> Fraction:
    """Eq. 5."""
    return Fraction(n_elements, n_columns) if n_columns else Fraction(0)


def loa_order(rowptr, colind, vw: int, window_rows: int = H) -> np.ndarray:
    """Row windows after layout reformatting, concatenated: entry i is the old id of new vertex i."""
    nbrs = neighbour_sets(rowptr, colind)
    n = len(nbrs)
    so = sorted_vertex_list(nbrs)
    visited = [False] * n
    order: List[int] = []
    first = 0
    while len(order) < n:
        while visited[so[first]]:
            first += 1
        p0 = first
        v0 = so[p0]
        visited[v0] = True
        rw = [v0]
        cols = set(nbrs[v0])
        eles = len(nbrs[v0])
        for _ in range(window_rows - 1):
            if len(order) + len(rw) == n:
                break
            cands = [j for j in range(p0, min(p0 + vw, n - 1) + 1) if not visited[so[j]]]
            if not cands:
                j = p0
                while visited[so[j]]:
                    j += 1
                cands = [j]
            best_key, best_j = None, None
            for j in cands:
                v = so[j]
                p = intensity(eles + len(nbrs[v]), len(cols | nbrs[v]))
                key = (p, len(nbrs[v]), -j)
                if best_key is None or key > best_key:
                    best_key, best_j = key, j
            v = so[best_j]
            visited[v] = True
            rw.append(v)
            cols |= nbrs[v]
            eles += len(nbrs[v])
        order.extend(rw)
    return np.asarray(order, dtype=np.int64)


def permute_graph(rowptr, colind, vals, order):
    """Relabel the square matrix so that old vertex order[i] becomes vertex i (rows and columns);
    columns of each row ascending.  Returns (rowptr, colind, vals)."""
    order = np.asarray(order, dtype=np.int64)
    n = len(rowptr) - 1
    new_of_old = np.empty(n, dtype=np.int64)
    new_of_old[order] = np.arange(n)
    rp = [0]
    ci, va = [], []
    for i in range(n):
        old = int(order[i])
        s, e = int(rowptr[old]), int(rowptr[old + 1])
        c = new_of_old[np.asarray(colind[s:e], dtype=np.int64)]
        idx = np.argsort(c, kind="stable")
        ci.append(c[idx])
        va.append(np.asarray(vals[s:e])[idx])
        rp.append(rp[-1] + (e - s))
    cat = (lambda parts, dt: np.concatenate(parts).astype(dt) if parts else np.empty(0, dtype=dt))
    return np.asarray(rp, dtype=np.int32), cat(ci, np.int32), cat(va, np.float32)


def mean_intensity(rowptr, colind, window_rows: int = H) -> float:
    """Sum of non-zeros over sum of distinct columns per window (Eq. 5 aggregated over the matrix)."""
    n = len(rowptr) - 1
    nnz = cols = 0
    for w0 in range(0, n, window_rows):
        s, e = int(rowptr[w0]), int(rowptr[min(w0 + window_rows, n)])
        nnz += len(set(zip(np.repeat(np.arange(w0, min(w0 + window_rows, n)),
                                     np.diff(rowptr[w0:min(w0 + window_rows, n) + 1])).tolist(),
                           np.asarray(colind[s:e]).tolist())))
        cols += len(set(np.asarray(colind[s:e]).tolist()))
    return nnz / cols if cols else 0.0
