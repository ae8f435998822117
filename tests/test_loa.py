"""Layout reformatting in the library (host code, Alg. 6 / Eq. 6) against the oracle (Alg. 5 / Eq. 5):
index work, so the vertex orders must be identical."""
import numpy as np
import pytest

from oracle import loa as oracle_loa
from workloads import chung_lu_graph, sbm_graph, random_relabel, tiny_random_csr
from test_oracle_loa import read_examples, csr_of


def lib_order(rowptr, colind, n_cols, vw, window_rows=16):
    import paper_2412_08902_amd.binding as hc
    return hc.hcspmm_loa_order(len(rowptr) - 1, n_cols, rowptr, colind, vw, window_rows)


@pytest.mark.parametrize("ex", read_examples(), ids=lambda e: e["name"])
def test_worked_examples(ex):
    rowptr, colind = csr_of(ex["rows"])
    got = lib_order(rowptr, colind, int(colind.max()) + 1, ex["vw"], ex["window_rows"])
    assert got.tolist() == ex["order"]


@pytest.mark.parametrize("seed,n,edges,vw,h", [(1, 200, 1500, 16, 16), (2, 333, 4000, 64, 16), (3, 100, 300, 5, 4),
                                               (4, 257, 2000, 0, 16), (5, 180, 2500, 1000, 16), (6, 64, 900, 7, 3)])
def test_power_law_graphs_match_oracle(seed, n, edges, vw, h):
    g = chung_lu_graph(n, edges, 2.1, seed=seed)
    want = oracle_loa.loa_order(g.rowptr, g.colind, vw, window_rows=h)
    got = lib_order(g.rowptr, g.colind, g.n_cols, vw, h)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("seed", [11, 12])
def test_scrambled_communities_match_oracle(seed):
    g = random_relabel(sbm_graph(10, 32, 0.4, 2.0, seed=seed), seed=seed + 1)
    for vw in (8, 48, g.n_rows):
        np.testing.assert_array_equal(lib_order(g.rowptr, g.colind, g.n_cols, vw),
                                      oracle_loa.loa_order(g.rowptr, g.colind, vw))


def test_unsorted_duplicate_empty_and_rectangular_rows():
    g = tiny_random_csr(90, 140, 0.05, seed=21, sorted_rows=False, duplicates=True)
    assert (np.diff(g.rowptr) == 0).any()
    np.testing.assert_array_equal(lib_order(g.rowptr, g.colind, g.n_cols, 20),
                                  oracle_loa.loa_order(g.rowptr, g.colind, 20))
    empty = tiny_random_csr(40, 40, 0.0, seed=1)
    assert lib_order(empty.rowptr, empty.colind, 40, 8).tolist() == list(range(40))
    assert lib_order(np.zeros(1, dtype=np.int32), np.empty(0, dtype=np.int32), 0, 4).tolist() == []


def test_permute_csr_matches_oracle_and_rejects_bad_orders():
    import paper_2412_08902_amd.binding as hc
    g = chung_lu_graph(120, 800, 2.1, seed=31)
    order = lib_order(g.rowptr, g.colind, g.n_cols, 32)
    rp, ci, va = hc.hcspmm_permute_csr(g.n_rows, g.rowptr, g.colind, g.vals, order)
    wrp, wci, wva = oracle_loa.permute_graph(g.rowptr, g.colind, g.vals, order)
    np.testing.assert_array_equal(rp, wrp)
    np.testing.assert_array_equal(ci, wci)
    np.testing.assert_array_equal(va, wva)
    bad = order.copy()
    bad[0] = bad[1]
    with pytest.raises(hc.HcspmmError):
        hc.hcspmm_permute_csr(g.n_rows, g.rowptr, g.colind, g.vals, bad)


def test_bad_arguments():
    import paper_2412_08902_amd.binding as hc
    g = chung_lu_graph(50, 200, 2.1, seed=41)
    with pytest.raises(hc.HcspmmError):
        lib_order(g.rowptr, g.colind, g.n_cols, -1)
    with pytest.raises(hc.HcspmmError):
        lib_order(g.rowptr, g.colind, 10, 4)                 # column indices beyond n_cols
    rp = g.rowptr.copy()
    rp[5] = rp[6] + 1
    with pytest.raises(hc.HcspmmError):
        lib_order(rp, g.colind, g.n_cols, 4)


def test_random_structures_match_oracle():
    """Many small random structures (unsorted rows, duplicates, empty rows, rectangular), several window sizes."""
    from hypothesis import given, settings, strategies as st
    from test_oracle_properties import csr_structures

    @settings(max_examples=80, deadline=None, derandomize=True)
    @given(csr_structures(), st.integers(0, 40), st.integers(1, 16))
    def check(csr, vw, window_rows):
        n_rows, n_cols, rowptr, colind = csr
        want = oracle_loa.loa_order(rowptr, colind, vw, window_rows=window_rows)
        got = lib_order(rowptr, colind, n_cols, vw, window_rows)
        np.testing.assert_array_equal(got, want)

    check()


@pytest.mark.parametrize("shape", [(37, 53), (64, 64), (1, 9), (9, 1), (0, 5)])
def test_transpose_csr_matches_scipy(shape):
    """Host transpose (for the backward aggregation of a directed graph): structure and values against scipy,
    ascending columns, duplicates kept in row order."""
    import scipy.sparse as sp
    import paper_2412_08902_amd.binding as hc
    from workloads import tiny_random_csr
    n, m = shape
    g = tiny_random_csr(n, m, 0.2, seed=n + m, sorted_rows=False, duplicates=True)
    rp, ci, va = hc.hcspmm_transpose_csr(n, m, g.rowptr, g.colind, g.vals)
    assert rp.shape == (m + 1,) and rp[0] == 0 and rp[-1] == g.nnz
    A = sp.csr_matrix((g.vals.astype(np.float64), g.colind, g.rowptr), shape=(n, m))
    At = sp.csr_matrix((va.astype(np.float64), ci, rp), shape=(m, n))
    assert abs(A.T - At).sum() == 0
    for r in range(m):
        assert np.all(np.diff(ci[rp[r]:rp[r + 1]]) >= 0)
    # the entries keep their identity: every (row, col, value) of the input appears exactly once, transposed
    rows = np.repeat(np.arange(n), np.diff(g.rowptr))
    want = sorted(zip(g.colind.tolist(), rows.tolist(), g.vals.tolist()))
    trows = np.repeat(np.arange(m), np.diff(rp))
    got = sorted(zip(trows.tolist(), ci.tolist(), va.tolist()))
    assert got == want


def test_transpose_csr_rejects_bad_input():
    import paper_2412_08902_amd.binding as hc
    with pytest.raises(hc.HcspmmError):
        hc.hcspmm_transpose_csr(2, 3, np.array([0, 1, 2], np.int32), np.array([0, 3], np.int32), np.ones(2, np.float32))
    with pytest.raises(hc.HcspmmError):
        hc.hcspmm_transpose_csr(2, 3, np.array([0, 2, 1], np.int32), np.array([0, 1], np.int32), np.ones(2, np.float32))


def test_checked_order_reports_the_windows_distinct_columns_before_and_after():
    """total_ncols of the stored layout and of the returned order, against the plan oracle's own count; on a block
    graph whose blocks are contiguous the regrouping makes the layout worse, and the numbers say so."""
    import oracle
    import paper_2412_08902_amd.binding as hc
    g = sbm_graph(40, 64, 0.25, 4.0, seed=3)
    order, before, after = hc.hcspmm_loa_order_checked(g.n_rows, g.n_cols, g.rowptr, g.colind, 256)
    assert np.array_equal(order, hc.hcspmm_loa_order(g.n_rows, g.n_cols, g.rowptr, g.colind, 256))
    plan = oracle.derive_plan_vectorised(g.rowptr, g.colind, [0, 0, 1], n_cols=g.n_cols)
    assert before == int(plan["ncols"].sum())
    rp2, ci2, _ = hc.hcspmm_permute_csr(g.n_rows, g.rowptr, g.colind, g.vals, order)
    plan2 = oracle.derive_plan_vectorised(rp2, ci2, [0, 0, 1], n_cols=g.n_cols)
    assert after == int(plan2["ncols"].sum())
    assert after > before                               # contiguous blocks: leave this layout alone
    gs = random_relabel(g, seed=9)                      # no locality: here the regrouping helps
    _, before_s, after_s = hc.hcspmm_loa_order_checked(gs.n_rows, gs.n_cols, gs.rowptr, gs.colind, 256)
    assert after_s < before_s
