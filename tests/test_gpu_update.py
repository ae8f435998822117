"""hcspmm_plan_update: after edges are inserted or deleted, the plan re-prepared from the changed rows must equal,
array by array, the CPU re-derivation of the plan of the NEW matrix, and the product must match the oracle."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from workloads import CSRGraph, chung_lu_graph, gcn_normalise, dense_normal, tiny_random_csr
from gpu_util import device_graph, assert_close

pytestmark = pytest.mark.gpu
KEYS = ["ncols", "nnzw", "route", "wptr", "wcols", "ecol", "mfma_windows", "csr_windows"]


def edit(g, inserts=(), deletes=()):
    """New CSR (ascending columns) with the (row, col) pairs of `inserts` added and those of `deletes` removed;
    returns it with the sorted list of rows whose entries changed."""
    A = sp.csr_matrix((g.vals.astype(np.float64), g.colind, g.rowptr), shape=(g.n_rows, g.n_cols)).tolil()
    changed = set()
    for r, c in deletes:
        if A[r, c] != 0:
            A[r, c] = 0
            changed.add(int(r))
    for r, c in inserts:
        if A[r, c] == 0:
            A[r, c] = 0.5 + 0.001 * ((r + c) % 100)
            changed.add(int(r))
    A = A.tocsr()
    A.eliminate_zeros()
    A.sort_indices()
    g2 = CSRGraph(g.n_rows, g.n_cols, A.indptr.astype(np.int32), A.indices.astype(np.int32), A.data.astype(np.float32))
    return g2, np.array(sorted(changed), dtype=np.int32)


def update_and_check(plan, g2, changed, mode, d=32, X=None):
    """Runs the update, compares the exported plan with the CPU re-derivation on g2 and the product with the oracle."""
    import torch
    import paper_2412_08902_amd.binding as hc
    rp, ci, va = device_graph(g2)
    hc.hcspmm_plan_update(plan, rp, ci, va, changed)
    info = hc.hcspmm_plan_info(plan)
    assert info["nnz"] == g2.nnz
    got = hc.hcspmm_plan_export(plan)
    want = oracle.derive_plan_vectorised(g2.rowptr, g2.colind, info["sel_coef"], mode=mode, n_cols=g2.n_cols)
    for k in KEYS:
        assert np.array_equal(got[k], want[k]), k
    X = dense_normal(g2.n_cols, d, seed=5) if X is None else X
    Y = torch.full((g2.n_rows, d), float("nan"), device="cuda")
    hc.hcspmm_spmm(plan, torch.from_numpy(X).cuda(), Y)
    torch.cuda.synchronize()
    ref = oracle.spmm(g2.rowptr, g2.colind, g2.vals, X)
    bound = oracle.spmm(g2.rowptr, g2.colind, g2.vals, X, use_abs=True)
    assert_close(Y.cpu().numpy().astype(np.float64), ref, bound, 1e-5, "after update")
    return info, got


def prepare(g, mode, sel_coef=None, d=32):
    import paper_2412_08902_amd.binding as hc
    rp, ci, va = device_graph(g)
    return hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, sel_coef=sel_coef, d_hint=d)


@pytest.mark.parametrize("mode,coef", [(3, [1, 0, -120]), (0, [1, 0, -120]), (0, None), (2, None), (1, None)])
def test_random_insertions_and_deletions(mode, coef):
    g = gcn_normalise(chung_lu_graph(3000, 60000, 2.1, seed=61, max_degree=1500))
    rng = np.random.default_rng(62)
    plan = prepare(g, mode, coef)
    cur = g
    for n_edits in (1, 40, 400):                                   # a chain of updates on one plan
        rows = rng.integers(0, g.n_rows, n_edits)
        ins = [(int(r), int(rng.integers(0, g.n_cols))) for r in rows]
        dels = []
        for r in rng.integers(0, g.n_rows, n_edits):
            s, e = cur.rowptr[r], cur.rowptr[r + 1]
            if e > s:
                dels.append((int(r), int(cur.colind[rng.integers(s, e)])))
        cur, changed = edit(cur, ins, dels)
        assert changed.size > 0
        update_and_check(plan, cur, changed, mode)
    plan.destroy()


def test_window_crossing_the_selector_boundary_and_rows_crossing_the_tier_boundaries():
    # windows of 16 identical-length rows; selector: matrix path iff ncols < 120
    n, m = 160, 5000
    rng = np.random.default_rng(63)
    lens = np.full(n, 7)
    lens[16:32] = 7                    # window 1: 16 x 7 distinct columns = 112 < 120 -> matrix path, will grow beyond 120
    lens[40] = 128                     # row at the short tier's upper bound, will grow by one (mid tier)
    lens[70] = 1024                    # row at the mid tier's upper bound, will grow by one (long tier)
    lens[100] = 2048                   # one segment, will grow to two segments (partial rows)
    cols = [np.sort(rng.choice(m, size=int(l), replace=False)) for l in lens]
    base = np.arange(16 * 7).reshape(16, 7) + 1000
    for i in range(16):
        cols[16 + i] = base[i]         # window 1: all columns distinct
    rp = np.zeros(n + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    g = CSRGraph(n, m, rp, np.concatenate(cols).astype(np.int32), rng.standard_normal(int(lens.sum())).astype(np.float32))
    plan = prepare(g, 3, [1, 0, -120])
    import paper_2412_08902_amd.binding as hc
    before = hc.hcspmm_plan_export(plan, with_ecol=False)
    info0 = hc.hcspmm_plan_info(plan)
    assert before["route"][1] == 1 and before["ncols"][1] == 112
    ins = [(16, 2000 + j) for j in range(9)]                      # window 1: 121 distinct columns -> scalar path
    for r in (40, 70, 100):
        free = np.setdiff1d(np.arange(m), cols[r])
        ins.append((r, int(free[0])))
    g2, changed = edit(g, ins)
    assert changed.tolist() == [16, 40, 70, 100]
    info, after = update_and_check(plan, g2, changed, 3)
    assert after["route"][1] == 0 and after["ncols"][1] == 121
    assert info["n_segments"] == info0["n_segments"] + 2          # row 70 became a long row, row 100 got a second segment
    # and back: delete what was inserted
    g3, changed = edit(g2, deletes=ins)
    info, after = update_and_check(plan, g3, changed, 3)
    assert after["route"][1] == 1 and info["n_segments"] == info0["n_segments"]
    plan.destroy()


def test_rows_emptied_and_filled_and_most_windows_touched():
    g = tiny_random_csr(200, 150, 0.1, seed=64)
    plan = prepare(g, 3, [3, 500, -420])
    # empty three rows entirely, fill an empty window's row
    dels = [(r, int(c)) for r in (0, 17, 199) for c in g.colind[g.rowptr[r]:g.rowptr[r + 1]]]
    g2, changed = edit(g, inserts=[(5, 3), (5, 149)], deletes=dels)
    update_and_check(plan, g2, changed, 3)
    # most windows touched: the call prepares from scratch, same result
    rng = np.random.default_rng(65)
    ins = [(int(r), int(rng.integers(0, 150))) for r in range(0, 200, 3)]
    g3, changed = edit(g2, ins)
    update_and_check(plan, g3, changed, 3)
    # nothing changed: pointers move, plan stays
    update_and_check(plan, g3, np.zeros(0, np.int32), 3)
    plan.destroy()


def test_bad_arguments_leave_the_plan_usable():
    import torch
    import paper_2412_08902_amd.binding as hc
    g = tiny_random_csr(100, 80, 0.1, seed=66)
    plan = prepare(g, 0)
    rp, ci, va = device_graph(g)
    with pytest.raises(hc.HcspmmError) as e:
        hc.hcspmm_plan_update(plan, rp, ci, va, np.array([100], np.int32))      # row outside the matrix
    assert e.value.status == hc.HCSPMM_EINVAL
    bad_ci = ci.clone()
    bad_ci[g.rowptr[20]] = 80                                                      # column out of range in a listed row
    with pytest.raises(hc.HcspmmError) as e:
        hc.hcspmm_plan_update(plan, rp, bad_ci, va, np.array([20], np.int32))
    assert e.value.status == hc.HCSPMM_EBADCSR
    X = dense_normal(80, 16, seed=7)
    Y = torch.empty((100, 16), device="cuda")
    hc.hcspmm_spmm(plan, torch.from_numpy(X).cuda(), Y)                            # still the plan of the old arrays
    torch.cuda.synchronize()
    ref = oracle.spmm(g.rowptr, g.colind, g.vals, X)
    assert_close(Y.cpu().numpy().astype(np.float64), ref, oracle.spmm(g.rowptr, g.colind, g.vals, X, use_abs=True), 1e-5)
    plan.destroy()


def test_many_updates_reuse_their_blocks_and_release_them_with_the_plan():
    """A plan that is updated keeps the device blocks of its last update; a chain of updates must neither grow the
    process's device memory step by step nor leave anything behind once the plan is destroyed."""
    import torch
    g = gcn_normalise(chung_lu_graph(20000, 600000, 2.1, seed=71, max_degree=4000))
    rng = np.random.default_rng(72)
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    plan = prepare(g, 2)                      # every window on the matrix path: the largest plan arrays
    cur = g
    graphs = []
    for step in range(4):                     # the edited matrices first (host work), their device copies stay alive below
        ins = [(int(r), int(rng.integers(0, g.n_cols))) for r in rng.integers(0, g.n_rows, 30)]
        cur, changed = edit(cur, ins)
        graphs.append((cur, changed))
    used = []
    for rep in range(3):
        for cur, changed in graphs:
            # (going back to an earlier matrix of the list changes the rows of every edit in between: list them all)
            rows = np.unique(np.concatenate([c for _, c in graphs]))
            update_and_check(plan, cur, rows, 2) if rep == 0 else None
            import paper_2412_08902_amd.binding as hc
            rp, ci, va = device_graph(cur)
            hc.hcspmm_plan_update(plan, rp, ci, va, rows)
            torch.cuda.synchronize()
            used.append(free0 - torch.cuda.mem_get_info()[0])
    # after the first rounds the footprint no longer grows (blocks are reused, unused ones released)
    assert max(used[-4:]) <= max(used[:8]) + (8 << 20), used
    plan.destroy()
    del rp, ci, va
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    # (the library's per-GPU cache of small blocks may hold up to 64 MiB of what the plan released)
    assert free0 - torch.cuda.mem_get_info()[0] < (64 << 20) + (32 << 20)


def test_update_of_a_plan_with_run_tables_and_after_an_export():
    """The optional run tables (matrix_kernels = RUNS) are rebuilt by an update; an update after an export (which had
    completed the condensed structure of scalar-path windows) still equals the re-derivation."""
    import torch
    import paper_2412_08902_amd.binding as hc
    g = gcn_normalise(chung_lu_graph(5000, 150000, 2.1, seed=81, max_degree=2000))
    rng = np.random.default_rng(82)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=2, d_hint=32, matrix_kernels=hc.HCSPMM_MATRIX_RUNS)
    ins = [(int(r), int(rng.integers(0, g.n_cols))) for r in rng.integers(0, g.n_rows, 25)]
    g2, changed = edit(g, ins)
    update_and_check(plan, g2, changed, 2)                      # exports: the plan now holds every window's lists
    runs = hc.hcspmm_plan_export_runs(plan)
    got = hc.hcspmm_plan_export(plan)
    want = oracle.derive_runs(got["mfma_windows"], got["wptr"], got["wcols"])
    assert runs["run_nu"].tolist() == [r["union"].shape[0] for r in want]
    assert np.array_equal(runs["ucols"], np.concatenate([r["union"] for r in want]))
    for r in want:
        for w, slots in zip(r["windows"], r["slots"]):
            assert np.array_equal(runs["wslot"][got["wptr"][w]:got["wptr"][w + 1]], slots)
    dels = [(int(r), int(g2.colind[g2.rowptr[r]])) for r in rng.integers(0, g.n_rows, 25) if g2.rowptr[r + 1] > g2.rowptr[r]]
    g3, changed = edit(g2, deletes=dels)
    update_and_check(plan, g3, changed, 2)
    plan.destroy()


def test_random_update_chains_equal_a_preparation_from_scratch():
    """Random graphs, routings, selector coefficients and chains of edits (with an export thrown in, which completes
    the condensed structure the next update carries over): after every update the plan's arrays and its product are
    bit-identical to those of a plan prepared from scratch for the same matrix.  (The comparison with the CPU
    re-derivation is in the tests above; this one hunts for state that an update could leave behind.)
    HCSPMM_TEST_EXAMPLES=N runs N cases with a fresh seed."""
    import os
    import torch
    import paper_2412_08902_amd.binding as hc
    n_cases = int(os.environ.get("HCSPMM_TEST_EXAMPLES", "12"))
    rng = np.random.default_rng(None if "HCSPMM_TEST_EXAMPLES" in os.environ else 20250101)
    for case in range(n_cases):
        n = int(rng.integers(400, 4000))
        e = int(rng.integers(n, 20 * n)) // 2 * 2
        avg = max(1, e // n)
        g = gcn_normalise(chung_lu_graph(n, e, 2.1 + 0.4 * rng.random(), seed=int(rng.integers(1 << 30)),
                                         max_degree=int(rng.integers(8 * avg, max(8 * avg + 1, n // 2)))))
        mode = int(rng.integers(0, 4))
        coef = None
        if mode in (0, 3) and rng.random() < 0.7:
            coef = [int(rng.integers(0, 50)), int(rng.integers(0, 2000)), -int(rng.integers(100, 3000))]
        d = int(rng.choice([16, 32, 64, 128]))
        plan = prepare(g, mode, coef, d)
        cur = g
        for step in range(int(rng.integers(1, 4))):
            ins = [(int(r), int(rng.integers(0, g.n_cols))) for r in rng.integers(0, g.n_rows, int(rng.integers(0, 50)))]
            dels = []
            for r in rng.integers(0, g.n_rows, int(rng.integers(0, 50))):
                if cur.rowptr[r + 1] > cur.rowptr[r]:
                    dels.append((int(r), int(cur.colind[rng.integers(cur.rowptr[r], cur.rowptr[r + 1])])))
            cur, changed = edit(cur, ins, dels)
            if rng.random() < 0.3:
                hc.hcspmm_plan_export(plan)
            rp, ci, va = device_graph(cur)
            hc.hcspmm_plan_update(plan, rp, ci, va, changed)
            fresh = prepare(cur, mode, coef, d)
            a, b = hc.hcspmm_plan_export(plan), hc.hcspmm_plan_export(fresh)
            for k in KEYS:
                assert np.array_equal(a[k], b[k]), (case, step, k, n, e, mode, coef)
            X = torch.from_numpy(dense_normal(cur.n_cols, d, seed=case)).cuda()
            Y1 = torch.empty((cur.n_rows, d), device="cuda")
            Y2 = torch.empty_like(Y1)
            hc.hcspmm_spmm(plan, X, Y1)
            hc.hcspmm_spmm(fresh, X, Y2)
            torch.cuda.synchronize()
            assert torch.equal(Y1, Y2), (case, step, n, e, mode, coef)
            fresh.destroy()
        plan.destroy()
