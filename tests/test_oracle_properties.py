"""Randomised invariants of the CPU oracle (hypothesis): properties that hold for every CSR structure, checked
against definitions that do not go through the oracle's own code paths."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from oracle import loa as oracle_loa


@st.composite
def csr_structures(draw):
    n_rows = draw(st.integers(1, 70))
    n_cols = draw(st.integers(1, 90))
    rows = []
    for _ in range(n_rows):
        k = draw(st.integers(0, min(n_cols, 12)))
        cols = draw(st.lists(st.integers(0, n_cols - 1), min_size=k, max_size=k))
        rows.append(cols)                                  # unsorted, duplicates allowed
    rowptr = np.zeros(n_rows + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colind = np.asarray([c for r in rows for c in r], dtype=np.int32)
    return n_rows, n_cols, rowptr, colind


@settings(max_examples=60, deadline=None, derandomize=True)
@given(csr_structures(), st.integers(-50, 50), st.integers(0, 2 ** 21), st.integers(-2 ** 21, 0))
def test_plan_invariants(csr, c0, c1, c2):
    n_rows, n_cols, rowptr, colind = csr
    coef = [c0, c1, c2]
    plan = oracle.derive_plan(rowptr, colind, coef, mode=oracle.plan.ROUTE_PER_WINDOW)
    vec = oracle.derive_plan_vectorised(rowptr, colind, coef, mode=oracle.plan.ROUTE_PER_WINDOW, n_cols=n_cols)
    for key in ("ncols", "nnzw", "route", "wptr", "wcols", "ecol", "mfma_windows", "csr_windows"):
        np.testing.assert_array_equal(plan[key], vec[key], err_msg=key)
    W = plan["W"]
    assert W == (n_rows + 15) // 16 and int(plan["nnzw"].sum()) == len(colind)
    for w in range(W):
        s, e = int(rowptr[min(16 * w, n_rows)]), int(rowptr[min(16 * w + 16, n_rows)])
        wc = plan["wcols"][plan["wptr"][w]:plan["wptr"][w + 1]]
        assert np.all(np.diff(wc) > 0) and set(wc.tolist()) == set(colind[s:e].tolist())      # the distinct columns, ascending
        assert np.array_equal(wc[plan["ecol"][s:e]], colind[s:e])                               # round trip
        # the selector is the sign of the exact rational form w1*ncols + w2*sparsity + b
        nc, nz = int(plan["ncols"][w]), int(plan["nnzw"][w])
        if nc == 0:
            assert plan["route"][w] == 0
        else:
            z = c0 * nc + c1 * oracle.sparsity(nc, nz) + c2
            assert plan["route"][w] == (1 if z < 0 else 0)
    assert sorted(plan["mfma_windows"].tolist() + plan["csr_windows"].tolist()) == list(range(W))
    # the hybrid mode only ever merges one side into the other
    hyb = oracle.derive_plan(rowptr, colind, coef, mode=oracle.plan.ROUTE_HYBRID)["route"]
    per = plan["route"]
    assert np.array_equal(hyb, per) or hyb.sum() == 0 or np.array_equal(hyb, (plan["ncols"] > 0).astype(np.uint8))


@settings(max_examples=40, deadline=None, derandomize=True)
@given(csr_structures(), st.integers(0, 40), st.integers(1, 16))
def test_layout_order_invariants(csr, vw, window_rows):
    n_rows, n_cols, rowptr, colind = csr
    order = oracle_loa.loa_order(rowptr, colind, vw, window_rows=window_rows)
    assert sorted(order.tolist()) == list(range(n_rows))
    nb = oracle_loa.neighbour_sets(rowptr, colind)
    so = oracle_loa.sorted_vertex_list(nb)
    keys = [(min(nb[v]) if nb[v] else 10 ** 9, v) for v in so]
    assert keys == sorted(keys)
    placed = set()
    for w0 in range(0, n_rows, window_rows):
        first = next(v for v in so if v not in placed)
        assert order[w0] == first                            # every window is seeded by the first unplaced vertex
        placed.update(order[w0:w0 + window_rows].tolist())
