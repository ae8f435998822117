"""Seeded synthetic graph / feature generators for the five benchmark configs.

Everything here is input plumbing.  No datasets are read: the graphs are
synthetic stand-ins that share node count, edge count, degree law and feature
width with the workloads named by the benchmark configuration.

Recipes
-------
Chung-Lu power law (configs 1, 2, 4, 5)
    weights ``w_i = (i + i0) ** (-1/(gamma-1))`` for i = 1..N, ``i0 >= 0`` found by
    bisection so that the largest expected degree ``E * w_1 / sum(w)`` equals
    ``max_degree`` (default ``floor(sqrt(E))``).  Endpoint multiset: a
    multinomial draw of ``2*M`` endpoints with probabilities ``w / sum(w)``,
    expanded and shuffled; consecutive entries form undirected pairs.  Loops
    are dropped, duplicate pairs collapsed, and a seeded random subset of
    exactly ``E/2`` distinct pairs is kept (more pairs are drawn until enough
    exist).  The pairs are symmetrised, a self-loop is added to every node and
    every row's columns are ascending.  Node ids are as generated, i.e. in
    descending expected degree.
Stochastic block model (config 3)
    ``n_blocks`` blocks of ``block`` consecutive ids, every intra-block
    unordered pair present with probability ``p_in``; ``N * inter_deg / 2``
    distinct inter-block undirected pairs with endpoints uniform in different
    blocks; ids are then permuted at random inside each block.  No self-loops.
Mixed (config 6, not one of the benchmark's five)
    the block model (75 % fill) and the power law of config 2 as a disjoint union, block-model nodes first.
Values
    1.0f, or the GCN normalisation ``1/sqrt(d_i d_j)`` with ``d_i`` the row
    length (self-loop included), computed in fp64 and rounded once to fp32.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import numpy as np
import scipy.sparse as sp


@dataclasses.dataclass
class CSRGraph:
    n_rows: int
    n_cols: int
    rowptr: np.ndarray  # int32 [n_rows+1]
    colind: np.ndarray  # int32 [nnz]
    vals: np.ndarray    # float32 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])


# ----------------------------------------------------------------------------
# helpers
# ----------------------------------------------------------------------------

def _pairs_to_csr(n: int, u: np.ndarray, v: np.ndarray, self_loops: bool) -> CSRGraph:
    """u < v, pairs sorted by (u, v) and distinct -> symmetric CSR, ascending columns.

    Entries are fed to a counting sort by row in an order that is already
    ascending within each row: reverse edges (row v, col u < v) first, then the
    self-loop, then forward edges (row u, col v > u).
    """
    if self_loops:
        loop = np.arange(n, dtype=np.int32)
        rows = np.concatenate([v, loop, u]).astype(np.int32, copy=False)
        cols = np.concatenate([u, loop, v]).astype(np.int32, copy=False)
    else:
        rows = np.concatenate([v, u]).astype(np.int32, copy=False)
        cols = np.concatenate([u, v]).astype(np.int32, copy=False)
    counts = np.bincount(rows, minlength=n).astype(np.int64)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    order = np.argsort(rows, kind="stable")
    colind = cols[order]
    del order
    assert rowptr[-1] < 2 ** 31
    return CSRGraph(n, n, rowptr.astype(np.int32), np.ascontiguousarray(colind, dtype=np.int32),
                    np.ones(colind.shape[0], dtype=np.float32))


def _solve_i0(n: int, alpha: float, target_ratio: float) -> float:
    """Find i0 >= 0 with w_1 / sum(w) == target_ratio for w_i = (i+i0)^-alpha."""
    idx = np.arange(1, n + 1, dtype=np.float64)

    def ratio(i0: float) -> float:
        w = (idx + i0) ** (-alpha)
        return float(w[0] / w.sum())

    if ratio(0.0) <= target_ratio:
        return 0.0
    lo, hi = 0.0, 1.0
    while ratio(hi) > target_ratio:
        hi *= 2.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if ratio(mid) > target_ratio:
            lo = mid
        else:
            hi = mid
    return hi


def chung_lu_graph(n: int, n_directed_edges: int, gamma: float, seed: int,
                   max_degree: Optional[int] = None, self_loops: bool = True) -> CSRGraph:
    """Symmetrised Chung-Lu graph with exactly ``n_directed_edges`` off-diagonal entries."""
    assert n_directed_edges % 2 == 0
    target_pairs = n_directed_edges // 2
    rng = np.random.Generator(np.random.PCG64(seed))
    alpha = 1.0 / (gamma - 1.0)
    if max_degree is None:
        max_degree = int(math.isqrt(n_directed_edges))
    i0 = _solve_i0(n, alpha, max_degree / float(n_directed_edges))
    w = (np.arange(1, n + 1, dtype=np.float64) + i0) ** (-alpha)
    p = w / w.sum()
    keys = np.empty(0, dtype=np.int64)
    draw = int(target_pairs * 1.08) + 64
    for _ in range(64):
        counts = rng.multinomial(2 * draw, p)
        ends = np.repeat(np.arange(n, dtype=np.int32), counts)
        rng.shuffle(ends)
        a = ends[0::2].astype(np.int64)
        b = ends[1::2].astype(np.int64)
        del ends
        keep = a != b
        lo = np.minimum(a, b)[keep]
        hi = np.maximum(a, b)[keep]
        del a, b, keep
        new = lo * n + hi
        del lo, hi
        keys = np.unique(np.concatenate([keys, new]))
        del new
        if keys.shape[0] >= target_pairs:
            break
        draw = int((target_pairs - keys.shape[0]) * 1.5) + 64
    else:
        raise RuntimeError("could not draw enough distinct pairs")
    if keys.shape[0] > target_pairs:
        sel = rng.permutation(keys.shape[0])[:target_pairs]
        sel.sort()
        keys = keys[sel]
        del sel
    u = (keys // n).astype(np.int32)
    v = (keys % n).astype(np.int32)
    del keys
    return _pairs_to_csr(n, u, v, self_loops)


def sbm_graph(n_blocks: int, block: int, p_in: float, inter_deg: float, seed: int) -> CSRGraph:
    n = n_blocks * block
    rng = np.random.Generator(np.random.PCG64(seed))
    iu, iv = np.triu_indices(block, k=1)
    present = rng.random((n_blocks, iu.shape[0])) < p_in
    b_idx, p_idx = np.nonzero(present)
    u_in = (b_idx * block + iu[p_idx]).astype(np.int64)
    v_in = (b_idx * block + iv[p_idx]).astype(np.int64)
    del present
    target_inter = int(n * inter_deg / 2)
    keys = np.empty(0, dtype=np.int64)
    draw = target_inter + target_inter // 16 + 64
    for _ in range(64):
        a = rng.integers(0, n, size=draw, dtype=np.int64)
        b = rng.integers(0, n, size=draw, dtype=np.int64)
        keep = (a // block) != (b // block)
        lo = np.minimum(a, b)[keep]
        hi = np.maximum(a, b)[keep]
        keys = np.unique(np.concatenate([keys, lo * n + hi]))
        if keys.shape[0] >= target_inter:
            break
        draw = (target_inter - keys.shape[0]) * 2 + 64
    if keys.shape[0] > target_inter:
        sel = rng.permutation(keys.shape[0])[:target_inter]
        sel.sort()
        keys = keys[sel]
    u = np.concatenate([u_in, keys // n])
    v = np.concatenate([v_in, keys % n])
    # random relabel inside each block
    perm = rng.permuted(np.tile(np.arange(block, dtype=np.int64), (n_blocks, 1)), axis=1)
    perm = (perm + (np.arange(n_blocks, dtype=np.int64) * block)[:, None]).reshape(-1)
    u = perm[u]
    v = perm[v]
    lo = np.minimum(u, v)
    hi = np.maximum(u, v)
    keys = np.unique(lo * n + hi)
    return _pairs_to_csr(n, (keys // n).astype(np.int32), (keys % n).astype(np.int32), self_loops=False)


def disjoint_union(a: CSRGraph, b: CSRGraph) -> CSRGraph:
    """Block-diagonal union: the nodes of ``b`` follow those of ``a``; no edge joins the two parts."""
    rowptr = np.concatenate([a.rowptr.astype(np.int64), a.rowptr[-1].astype(np.int64) + b.rowptr[1:].astype(np.int64)])
    assert rowptr[-1] < 2 ** 31
    colind = np.concatenate([a.colind, (b.colind.astype(np.int64) + a.n_cols).astype(np.int32)])
    vals = np.concatenate([a.vals, b.vals])
    return CSRGraph(a.n_rows + b.n_rows, a.n_cols + b.n_cols, rowptr.astype(np.int32), colind, vals)


def gcn_normalise(g: CSRGraph) -> CSRGraph:
    """values <- 1/sqrt(d_i d_j), d_i = row length of i (self-loop already in the graph)."""
    deg = np.diff(g.rowptr.astype(np.int64)).astype(np.float64)
    rows = np.repeat(np.arange(g.n_rows, dtype=np.int64), np.diff(g.rowptr.astype(np.int64)))
    with np.errstate(divide="ignore"):
        vals = 1.0 / np.sqrt(deg[rows] * deg[g.colind])
    return CSRGraph(g.n_rows, g.n_cols, g.rowptr, g.colind, vals.astype(np.float32))


def random_relabel(g: CSRGraph, seed: int) -> CSRGraph:
    """Symmetric seeded random permutation of node ids (stress variant: removes window density)."""
    assert g.n_rows == g.n_cols
    rng = np.random.Generator(np.random.PCG64(seed))
    perm = rng.permutation(g.n_rows)
    m = sp.csr_matrix((g.vals, g.colind, g.rowptr), shape=(g.n_rows, g.n_cols))
    coo = m.tocoo()
    m2 = sp.csr_matrix((coo.data, (perm[coo.row], perm[coo.col])), shape=m.shape)
    m2.sort_indices()
    return CSRGraph(g.n_rows, g.n_cols, m2.indptr.astype(np.int32), m2.indices.astype(np.int32),
                    m2.data.astype(np.float32))


# ----------------------------------------------------------------------------
# dense inputs and 16-bit encodings
# ----------------------------------------------------------------------------

def dense_uniform(rows: int, cols: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.random((rows, cols), dtype=np.float32)
    x *= 2.0
    x -= 1.0
    return x


def dense_normal(rows: int, cols: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.standard_normal((rows, cols), dtype=np.float32)


def glorot_uniform(fan_in: int, fan_out: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    a = math.sqrt(6.0 / (fan_in + fan_out))
    return ((rng.random((fan_in, fan_out)) * 2.0 - 1.0) * a).astype(np.float32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even; finite inputs."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f16_bits(x: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


# ----------------------------------------------------------------------------
# the five configurations
# ----------------------------------------------------------------------------

BASE_SEED = 20241208

CONFIGS = {
    "C1": dict(kind="chung_lu", n=2708, edges=10556, gamma=2.1, max_degree=None, values="ones",
               d=32, x="uniform", index=0),
    "C2": dict(kind="chung_lu", n=169343, edges=2_300_000, gamma=2.0, max_degree=13000, values="gcn",
               d=128, x="normal", index=1),
    "C3": dict(kind="sbm", n_blocks=2048, block=64, p_in=0.25, inter_deg=4.0, values="ones",
               d=64, x="normal", index=2),
    "C4": dict(kind="chung_lu", n=2_449_029, edges=123_700_000, gamma=2.2, max_degree=None, values="gcn",
               d=32, x="uniform", index=3),
    "C5": dict(kind="chung_lu", n=232_965, edges=114_600_000, gamma=1.9, max_degree=None, values="gcn",
               d=128, d_in=602, x="normal", index=4),
    # Not one of the benchmark's five: a graph whose row windows are of both kinds -- dense communities (blocks of 64
    # at 75 % fill) followed by a sparse power-law part (the recipe of C2) -- for the claim that per-window routing
    # beats both single-path plans.
    "C6": dict(kind="mixed", n_blocks=2048, block=64, p_in=0.75, inter_deg=4.0,
               n=169343, edges=2_300_000, gamma=2.0, max_degree=13000, values="gcn", d=128, x="normal", index=5),
}


def make_config(name: str, scale: float = 1.0, with_dense: bool = True):
    """Return (graph, X, W-or-None) for config ``name``.

    ``scale`` < 1 shrinks node and edge counts proportionally (used by tests that
    want the same structure at a size a CPU finishes quickly); scale == 1 is the
    benchmark size.  For C5, X has ``d_in`` columns and W is d_in x d.
    """
    c = CONFIGS[name]
    seed = BASE_SEED + c["index"]
    if c["kind"] == "chung_lu":
        n = max(64, int(round(c["n"] * scale)))
        e = int(round(c["edges"] * scale)) // 2 * 2
        md = c["max_degree"]
        if md is not None and scale != 1.0:
            md = max(8, min(int(md * scale), n // 2))
        g = chung_lu_graph(n, e, c["gamma"], seed, max_degree=md)
    elif c["kind"] == "mixed":
        nb = max(2, int(round(c["n_blocks"] * scale)))
        n = max(64, int(round(c["n"] * scale)))
        md = c["max_degree"] if scale == 1.0 else max(8, min(int(c["max_degree"] * scale), n // 2))
        g = disjoint_union(sbm_graph(nb, c["block"], c["p_in"], c["inter_deg"], seed),
                           chung_lu_graph(n, int(round(c["edges"] * scale)) // 2 * 2, c["gamma"], seed + 1, max_degree=md))
    else:
        nb = max(2, int(round(c["n_blocks"] * scale)))
        g = sbm_graph(nb, c["block"], c["p_in"], c["inter_deg"], seed)
    if c["values"] == "gcn":
        g = gcn_normalise(g)
    if not with_dense:
        return g, None, None
    width = c.get("d_in", c["d"])
    gen = dense_uniform if c["x"] == "uniform" else dense_normal
    x = gen(g.n_rows, width, seed + 100)
    w = glorot_uniform(c["d_in"], c["d"], seed + 200) if "d_in" in c else None
    return g, x, w


def tiny_random_csr(n_rows: int, n_cols: int, density: float, seed: int, sorted_rows: bool = True,
                    duplicates: bool = False, integer_values: bool = False) -> CSRGraph:
    """Small unstructured CSR for property tests (may have empty rows, ragged last window)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    rows_l, cols_l = [], []
    for i in range(n_rows):
        k = rng.binomial(n_cols, density)
        c = rng.choice(n_cols, size=k, replace=False) if k else np.empty(0, dtype=np.int64)
        if duplicates and k:
            c = np.concatenate([c, rng.choice(c, size=max(1, k // 3))])
        if sorted_rows:
            c = np.sort(c)
        else:
            rng.shuffle(c)
        rows_l.append(np.full(c.shape[0], i, dtype=np.int64))
        cols_l.append(c.astype(np.int64))
    rows = np.concatenate(rows_l) if rows_l else np.empty(0, dtype=np.int64)
    cols = np.concatenate(cols_l) if cols_l else np.empty(0, dtype=np.int64)
    rowptr = np.zeros(n_rows + 1, dtype=np.int32)
    np.cumsum(np.bincount(rows, minlength=n_rows), out=rowptr[1:])
    if integer_values:
        vals = rng.integers(-3, 4, size=cols.shape[0]).astype(np.float32)
    else:
        vals = rng.standard_normal(cols.shape[0]).astype(np.float32)
    return CSRGraph(n_rows, n_cols, rowptr, cols.astype(np.int32), vals)
