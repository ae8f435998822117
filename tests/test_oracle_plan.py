"""Pins for the plan oracle (windows, condensing, features, selector form)."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from workloads import tiny_random_csr, make_config, dense_normal


def _read_table(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([int(t) for t in line.split()])
    return rows


def test_sparsity_endpoints_from_paper(golden_dir):
    for ncols, nnzw, num, den in _read_table(os.path.join(golden_dir, "selector_training_features.txt")):
        assert oracle.sparsity(ncols, nnzw) == Fraction(num, den)


def test_intensity_from_paper(golden_dir):
    for nnzw, ncols, num, den in _read_table(os.path.join(golden_dir, "computing_intensity.txt")):
        assert oracle.computing_intensity(ncols, nnzw) == Fraction(num, den)


def test_disjoint_neighbours_give_128_columns():
    # 16 rows x 8 neighbours, no common neighbour (footnote 8 of Section IV-C)
    rowptr = np.arange(0, 16 * 8 + 1, 8, dtype=np.int32)
    colind = (np.arange(128, dtype=np.int32) * 7) % 1000 + 1000 * (np.arange(128) // 8 % 2)
    colind = np.concatenate([np.sort(colind[i * 8:(i + 1) * 8]) for i in range(16)]).astype(np.int32)
    assert len(set(colind.tolist())) == 128
    p = oracle.derive_plan(rowptr, colind, [0, 0, 1])
    assert p["ncols"].tolist() == [128] and p["nnzw"].tolist() == [128]


def test_identical_rows_give_ncols_equal_degree():
    deg = 11
    cols = np.sort(np.random.default_rng(1).choice(500, deg, replace=False)).astype(np.int32)
    rowptr = np.arange(0, 16 * deg + 1, deg, dtype=np.int32)
    p = oracle.derive_plan(rowptr, np.tile(cols, 16), [0, 0, 1])
    assert p["ncols"].tolist() == [deg] and p["nnzw"].tolist() == [16 * deg]
    assert oracle.sparsity(deg, 16 * deg) == 0
    assert np.array_equal(p["wcols"], cols)
    assert np.array_equal(p["ecol"], np.tile(np.arange(deg), 16))


def test_hand_built_window():
    # two windows with H = 4 for readability: rows 0-3 and rows 4-5 (ragged tail)
    rowptr = np.array([0, 2, 2, 5, 6, 8, 9], dtype=np.int32)
    colind = np.array([7, 3, 3, 9, 7, 0, 5, 5, 2], dtype=np.int32)   # row 0 unsorted on purpose
    p = oracle.derive_plan(rowptr, colind, [0, 0, 1], H=4)
    assert p["W"] == 2
    assert p["nnzw"].tolist() == [6, 3]
    assert p["ncols"].tolist() == [4, 2]
    assert p["wptr"].tolist() == [0, 4, 6]
    assert p["wcols"].tolist() == [0, 3, 7, 9, 2, 5]
    assert p["ecol"].tolist() == [2, 1, 1, 3, 2, 0, 1, 1, 0]


@pytest.mark.parametrize("seed,n,m,dens,sorted_rows,dups", [(1, 100, 80, 0.05, True, False),
                                                           (2, 37, 200, 0.1, False, True),
                                                           (3, 16, 16, 0.9, True, False),
                                                           (4, 15, 300, 0.0, True, False),
                                                           (5, 129, 40, 0.3, False, False)])
def test_condensed_structure_roundtrip_and_dense_tile(seed, n, m, dens, sorted_rows, dups):
    H = 16
    g = tiny_random_csr(n, m, dens, seed, sorted_rows=sorted_rows, duplicates=dups)
    p = oracle.derive_plan(g.rowptr, g.colind, [3, -5, 1])
    X = dense_normal(m, 6, seed + 9)
    Y = oracle.spmm(g.rowptr, g.colind, g.vals, X)
    assert p["wptr"][-1] == p["wcols"].shape[0] <= g.nnz
    for w in range(p["W"]):
        r0, r1 = H * w, min(H * w + H, n)
        s, e = g.rowptr[r0], g.rowptr[r1]
        wc = p["wcols"][p["wptr"][w]:p["wptr"][w + 1]]
        assert np.all(np.diff(wc) > 0)                                   # strictly ascending
        assert np.array_equal(wc[p["ecol"][s:e]], g.colind[s:e])          # round trip
        # scatter into the condensed dense tile and multiply by the gathered X rows
        tile = np.zeros((H, max(len(wc), 1)), dtype=np.float64)
        for i in range(r0, r1):
            for k in range(g.rowptr[i], g.rowptr[i + 1]):
                tile[i - r0, p["ecol"][k]] += float(g.vals[k])
        got = tile[:, :len(wc)] @ X[wc].astype(np.float64) if len(wc) else np.zeros((H, 6))
        np.testing.assert_allclose(got[:r1 - r0], Y[r0:r1], atol=1e-12)
    q = oracle.derive_plan_vectorised(g.rowptr, g.colind, [3, -5, 1], n_cols=m)
    for k in p:
        assert np.array_equal(np.asarray(p[k]), np.asarray(q[k])), k


def test_vectorised_equals_loop_on_config1():
    g, _, _ = make_config("C1", with_dense=False)
    coef = [37, 2500, -2600]
    p = oracle.derive_plan(g.rowptr, g.colind, coef)
    q = oracle.derive_plan_vectorised(g.rowptr, g.colind, coef, n_cols=g.n_cols)
    for k in p:
        assert np.array_equal(np.asarray(p[k]), np.asarray(q[k])), k
    assert p["W"] == 170 and int(p["nnzw"].sum()) == 13264


def test_selector_is_the_linear_form_and_polarity():
    # z = w1*ncols + w2*sparsity + b, route = matrix path iff z < 0 (label 1 = scalar cores faster)
    w1, w2, b = 3, 400, -330
    H = 16
    for ncols in [1, 2, 7, 32, 130, 1000]:
        for nnzw in sorted({ncols, 2 * ncols, 5 * ncols, 15 * ncols, 16 * ncols}):
            z = w1 * ncols + w2 * oracle.sparsity(ncols, nnzw, H) + b        # exact rational
            assert oracle.select_route(ncols, nnzw, [w1, w2, b], H) == (1 if z < 0 else 0)
    assert oracle.select_route(0, 0, [w1, w2, b]) == 0                       # empty window -> scalar path
    assert oracle.select_route(5, 5, [w1, w2, b], mode=oracle.plan.ROUTE_ALL_MFMA) == 1
    assert oracle.select_route(5, 80, [w1, w2, b], mode=oracle.plan.ROUTE_ALL_CSR) == 0


def test_selector_monotone_for_positive_weights():
    # with w1, w2 > 0: more non-zeros at fixed ncols never flips matrix -> scalar,
    # more columns at fixed sparsity never flips scalar -> matrix (Section IV-B)
    coef = [5, 900, -800]
    for ncols in range(1, 140, 7):
        routes = [oracle.select_route(ncols, nnzw, coef) for nnzw in range(ncols, 16 * ncols + 1)]
        assert routes == sorted(routes)
    for num in range(1, 16):                      # sparsity = 1 - num/16 exactly: nnzw = num*ncols
        routes = [oracle.select_route(c, num * c, coef) for c in range(1, 400)]
        assert routes == sorted(routes, reverse=True)


def test_eq6_equals_eq5_on_the_enlarged_window():
    # Eq. 6: (curEles + |N(v)|) / (curCols + |N(v)| - |N(v) ∩ allCols|) equals Eq. 5 on RW ∪ {v}
    rng = np.random.default_rng(3)
    rows = [set(rng.choice(60, size=rng.integers(1, 12), replace=False).tolist()) for _ in range(6)]
    rw, v = rows[:5], rows[5]
    all_cols = set().union(*rw)
    cur_eles = sum(len(r) for r in rw)
    eq6 = Fraction(cur_eles + len(v), len(all_cols) + len(v) - len(v & all_cols))
    cols = np.concatenate([np.array(sorted(r)) for r in rw + [v]])
    ncols, nnzw = oracle.window_features(cols)
    assert oracle.computing_intensity(ncols, nnzw) == eq6


def test_launch_guard_cases():
    """The launch guard of the hybrid mode on hand-set routes: the smaller side moves only when it is
    below 2^18 non-zeros AND below one eighth of the matrix; the matrix side is examined first."""
    ncols = np.array([10, 10, 10, 0, 10], dtype=np.int32)
    # matrix side 100 of 1000 non-zeros (< 1/8, < 2^18): joins the scalar path
    assert oracle.launch_guard([1, 0, 0, 0, 0], ncols, [100, 300, 300, 0, 300]).tolist() == [0, 0, 0, 0, 0]
    # matrix side 125 of 1000 = exactly 1/8: stays
    assert oracle.launch_guard([1, 0, 0, 0, 0], ncols, [125, 300, 300, 0, 275]).tolist() == [1, 0, 0, 0, 0]
    # scalar side small: joins the matrix path, the empty window keeps route 0
    assert oracle.launch_guard([1, 1, 0, 0, 1], ncols, [400, 400, 50, 0, 400]).tolist() == [1, 1, 1, 0, 1]
    # a side of 2^18 non-zeros or more is never moved, however small its share
    big = 1 << 18
    assert oracle.launch_guard([1, 0, 0, 0, 0], ncols, [big, 40 * big, 0, 0, 0]).tolist() == [1, 0, 0, 0, 0]
    assert oracle.launch_guard([1, 0, 0, 0, 0], ncols, [big - 1, 40 * big, 0, 0, 0]).tolist() == [0, 0, 0, 0, 0]
    # pure plans are left alone
    assert oracle.launch_guard([0, 0, 0, 0, 0], ncols, [5, 5, 5, 0, 5]).tolist() == [0, 0, 0, 0, 0]
    assert oracle.launch_guard([1, 1, 1, 0, 1], ncols, [5, 5, 5, 0, 5]).tolist() == [1, 1, 1, 0, 1]


def test_guard_applies_to_hybrid_mode_only():
    from workloads import sbm_graph
    g = sbm_graph(6, 64, 0.5, 1.0, seed=3)
    # a selector that sends exactly the windows with fewer than 70 columns to the matrix path
    coef = [1 << 20, 0, -70 * (1 << 20)]
    per_window = oracle.derive_plan(g.rowptr, g.colind, coef, mode=oracle.plan.ROUTE_PER_WINDOW)
    hybrid = oracle.derive_plan(g.rowptr, g.colind, coef, mode=oracle.plan.ROUTE_HYBRID)
    expect = np.array([oracle.select_route(c, z, coef) for c, z in zip(per_window["ncols"], per_window["nnzw"])])
    np.testing.assert_array_equal(per_window["route"], expect)
    np.testing.assert_array_equal(hybrid["route"], oracle.launch_guard(expect, per_window["ncols"], per_window["nnzw"]))
    vec = oracle.derive_plan_vectorised(g.rowptr, g.colind, coef, mode=oracle.plan.ROUTE_HYBRID, n_cols=g.n_cols)
    np.testing.assert_array_equal(vec["route"], hybrid["route"])


def test_runs_merge_the_column_lists_of_neighbouring_matrix_path_windows():
    # hand-worked: three matrix-path windows 0, 2, 5 whose column lists overlap; run length 2 -> runs (0, 2) and (5)
    wcols = np.array([1, 4, 9,   7,   4, 5, 9, 30,   0,   2, 30], np.int32)      # windows 0 | 1 | 2 | 3,4 (3 empty) | 5
    wptr = np.array([0, 3, 4, 8, 8, 9, 11], np.int64)
    runs = oracle.derive_runs([0, 2, 5], wptr, wcols, run_windows=2)
    assert len(runs) == 2
    assert runs[0]["windows"] == [0, 2] and runs[0]["union"].tolist() == [1, 4, 5, 9, 30]
    assert runs[0]["slots"][0].tolist() == [0, 1, 3] and runs[0]["slots"][1].tolist() == [1, 2, 3, 4]
    assert runs[1]["windows"] == [5] and runs[1]["union"].tolist() == [2, 30] and runs[1]["slots"][0].tolist() == [0, 1]
    # property on a random plan: the union is strictly ascending, a slot leads back to the column, and the union has
    # no column that none of the run's windows holds
    g = tiny_random_csr(200, 150, 0.1, seed=8)
    plan = oracle.derive_plan(g.rowptr, g.colind, [0, 0, -1])
    lst = np.nonzero(plan["ncols"] > 0)[0]
    for r in oracle.derive_runs(lst, plan["wptr"], plan["wcols"]):
        u = r["union"]
        assert np.all(np.diff(u) > 0)
        seen = np.zeros(u.shape[0], bool)
        for w, sl in zip(r["windows"], r["slots"]):
            cols = plan["wcols"][plan["wptr"][w]:plan["wptr"][w + 1]]
            assert np.array_equal(u[sl], cols)
            seen[sl] = True
        assert seen.all()
