"""Pins for the layout-reformatting oracle (Section V-B, Alg. 5 / Eq. 5): hand-worked examples,
closed-form cases and invariants -- none of them computed by the oracle itself."""
import os

import numpy as np
import pytest

from oracle import loa
from workloads import chung_lu_graph, sbm_graph, random_relabel, tiny_random_csr

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "loa_worked_examples.txt")


def read_examples():
    out, cur = [], None
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if tok[0] == "example":
            cur = dict(name=tok[1], window_rows=int(tok[3]), vw=int(tok[5]), rows=[], order=None)
            out.append(cur)
        elif tok[0] == "row":
            assert int(tok[1].rstrip(":")) == len(cur["rows"])
            cur["rows"].append([int(t) for t in tok[2:]])
        elif tok[0] == "order:":
            cur["order"] = [int(t) for t in tok[1:]]
    return out


def csr_of(rows):
    rowptr = np.zeros(len(rows) + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colind = np.asarray([c for r in rows for c in r], dtype=np.int32)
    return rowptr, colind


@pytest.mark.parametrize("ex", read_examples(), ids=lambda e: e["name"])
def test_worked_examples(ex):
    rowptr, colind = csr_of(ex["rows"])
    got = loa.loa_order(rowptr, colind, ex["vw"], window_rows=ex["window_rows"])
    assert got.tolist() == ex["order"]


def scrambled_cliques(n_cliques, size, seed):
    """Disjoint cliques with self loops under a random vertex labelling."""
    rng = np.random.Generator(np.random.PCG64(seed))
    label = rng.permutation(n_cliques * size)
    rows = [None] * (n_cliques * size)
    for c in range(n_cliques):
        members = sorted(int(x) for x in label[c * size:(c + 1) * size])
        for m in members:
            rows[m] = members
    return rows, label


def test_disjoint_cliques_are_recovered():
    """Closed form: with the whole graph in the vertices window, a member of the seed's clique
    keeps the column count (intensity (16k+16)/16) while any other vertex adds 16 columns, so every
    row window must come out as exactly one clique, and the layout's intensity is 16."""
    rows, label = scrambled_cliques(12, 16, seed=7)
    rowptr, colind = csr_of(rows)
    order = loa.loa_order(rowptr, colind, vw=len(rows))
    assert sorted(order.tolist()) == list(range(len(rows)))
    clique_of = np.empty(len(rows), dtype=np.int64)
    clique_of[label] = np.arange(len(rows)) // 16
    for w in range(12):
        assert len(set(clique_of[order[16 * w:16 * w + 16]].tolist())) == 1
    rp, ci, _ = loa.permute_graph(rowptr, colind, np.ones(len(colind), dtype=np.float32), order)
    assert loa.mean_intensity(rp, ci) == 16.0
    assert loa.mean_intensity(rowptr, colind) < 3.0          # scrambled: windows mix up to 16 cliques


def test_vw_zero_is_the_sorted_list():
    """With an empty vertices window every growth step falls through to the next unvisited vertex
    of the sorted list, so the result is the sort by smallest neighbour itself."""
    g = tiny_random_csr(75, 75, 0.06, seed=5)
    order = loa.loa_order(g.rowptr, g.colind, vw=0)
    keys = []
    for v in range(75):
        c = g.colind[g.rowptr[v]:g.rowptr[v + 1]]
        keys.append((int(c.min()) if len(c) else 10 ** 9, v))
    assert order.tolist() == [v for _, v in sorted(keys)]


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_invariants_on_random_graphs(seed):
    g = chung_lu_graph(150, 900, 2.1, seed=seed)
    order = loa.loa_order(g.rowptr, g.colind, vw=24)
    assert sorted(order.tolist()) == list(range(150))                      # a permutation
    # the seed of every window is the first not-yet-placed vertex of the sorted list
    nb = loa.neighbour_sets(g.rowptr, g.colind)
    so = loa.sorted_vertex_list(nb)
    placed = set()
    for w0 in range(0, 150, 16):
        first = next(v for v in so if v not in placed)
        assert order[w0] == first
        placed.update(order[w0:w0 + 16].tolist())
    # every growth step is a greedy argmax: re-check one step per window with dense boolean algebra
    B = np.zeros((150, 150), dtype=bool)
    for v in range(150):
        B[v, g.colind[g.rowptr[v]:g.rowptr[v + 1]]] = True
    pos = {v: j for j, v in enumerate(so)}
    done = set()
    for w0 in range(0, 150 - 16, 16):
        rw = order[w0:w0 + 16].tolist()
        k = 5                                            # the 5th growth step of this window
        cur, chosen = rw[:k], rw[k]
        p0 = pos[rw[0]]
        cands = [so[j] for j in range(p0, min(p0 + 24, 149) + 1) if so[j] not in done and so[j] not in cur]
        if cands:
            def score(v):
                sel = B[cur + [v]]
                return int(sel.sum()), int(sel.any(axis=0).sum())
            num_c, den_c = score(chosen)
            for v in cands:
                num, den = score(v)
                assert num * den_c <= num_c * den, "a candidate beats the chosen vertex"
        done.update(rw)


def test_permute_graph_is_a_relabelling():
    g = chung_lu_graph(90, 500, 2.1, seed=9)
    order = loa.loa_order(g.rowptr, g.colind, vw=16)
    rp, ci, va = loa.permute_graph(g.rowptr, g.colind, g.vals, order)
    A = np.zeros((90, 90))
    for v in range(90):
        A[v, g.colind[g.rowptr[v]:g.rowptr[v + 1]]] = g.vals[g.rowptr[v]:g.rowptr[v + 1]]
    A2 = np.zeros((90, 90))
    for v in range(90):
        A2[v, ci[rp[v]:rp[v + 1]]] = va[rp[v]:rp[v + 1]]
        assert np.all(np.diff(ci[rp[v]:rp[v + 1]]) > 0)
    np.testing.assert_array_equal(A2, A[np.ix_(order, order)])


def test_layout_gain_on_scrambled_communities():
    """Property the method is built for: on a community graph whose labels were scrambled, the
    reformatted layout has a higher computing intensity than the scrambled one."""
    g = random_relabel(sbm_graph(12, 32, 0.5, 1.0, seed=11), seed=12)
    order = loa.loa_order(g.rowptr, g.colind, vw=g.n_rows)
    rp, ci, _ = loa.permute_graph(g.rowptr, g.colind, g.vals, order)
    before, after = loa.mean_intensity(g.rowptr, g.colind), loa.mean_intensity(rp, ci)
    assert after > 1.5 * before
