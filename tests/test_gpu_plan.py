"""GPU parity of the preprocessing plan: every exported index array bit-exact against the CPU re-derivation."""
import numpy as np
import pytest

import oracle
from workloads import tiny_random_csr, make_config, CSRGraph, sbm_graph, chung_lu_graph, gcn_normalise, dense_normal
from gpu_util import device_graph

pytestmark = pytest.mark.gpu

KEYS = ["ncols", "nnzw", "route", "wptr", "wcols", "ecol", "mfma_windows", "csr_windows"]


def gpu_plan(g, mode=0, sel_coef=None, d_hint=64, mfma_dtype=0):
    import paper_2412_08902_amd.binding as hc
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, sel_coef=sel_coef, d_hint=d_hint,
                             mfma_dtype=mfma_dtype)
    info = hc.hcspmm_plan_info(plan)
    out = hc.hcspmm_plan_export(plan)
    plan.destroy()
    return out, info


def check_plan(g, mode=0, sel_coef=None, d_hint=64):
    got, info = gpu_plan(g, mode, sel_coef, d_hint)
    coef = info["sel_coef"]
    if sel_coef is not None:
        assert coef == list(sel_coef)
    want = oracle.derive_plan_vectorised(g.rowptr, g.colind, coef, mode=mode, n_cols=g.n_cols)
    assert got["H"] == want["H"] == 16 and got["W"] == want["W"]
    for k in KEYS:
        assert got[k].dtype == want[k].dtype, k
        assert np.array_equal(got[k], want[k]), k
    assert info["total_ncols"] == want["wptr"][-1]
    assert info["nnz_mfma"] == int(want["nnzw"][want["route"] == 1].sum())
    return got, info


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
@pytest.mark.parametrize("case", [(83, 70, 0.12, True, False), (200, 5000, 0.01, False, True),
                                  (16, 16, 1.0, True, False), (15, 90, 0.0, True, False),
                                  (1000, 300, 0.3, True, False)])
def test_small_plans(case, mode):
    n, m, dens, srt, dup = case
    g = tiny_random_csr(n, m, dens, seed=n + m, sorted_rows=srt, duplicates=dup)
    check_plan(g, mode, sel_coef=[3, 500, -420])


@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_config_plans_default_selector(name):
    g, _, _ = make_config(name, with_dense=False)
    check_plan(g)


def test_plan_with_windows_beyond_lds_sort_and_many_columns():
    # windows with more non-zeros than the LDS sort handles, over more columns than one bitmap pass
    n, m = 64, 3_000_000
    rng = np.random.default_rng(3)
    lens = np.full(n, 5)
    lens[0:16] = 700                      # window 0: 11,200 non-zeros
    lens[40] = 30000                      # window 2: one huge row
    cols = [np.sort(rng.choice(m, size=l, replace=False)) for l in lens]
    cols[3] = cols[2].copy()              # shared columns inside window 0
    rp = np.zeros(n + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    g = CSRGraph(n, m, rp, np.concatenate(cols).astype(np.int32), np.ones(int(lens.sum()), np.float32))
    got, _ = check_plan(g, sel_coef=[1, 100, -50])
    assert 700 * 14 < got["ncols"][0] <= 700 * 15 and got["nnzw"][0] == 11200
    assert got["ncols"][2] > 30000 and got["wcols"].max() > (1 << 21)


def test_selector_routes_change_with_coefficients():
    g = sbm_graph(32, 64, 0.25, 4.0, seed=8)
    a, _ = check_plan(g, sel_coef=[0, 0, 1])        # z = 1 > 0 everywhere: scalar path
    b, _ = check_plan(g, sel_coef=[0, 0, -1])       # z < 0 everywhere: matrix path
    c, _ = check_plan(g, mode=3, sel_coef=[1, 0, -125])     # ncols < 125, decision per window as it stands
    assert a["route"].sum() == 0 and b["route"].all() and 0 < c["route"].sum() < c["W"]
    check_plan(g, mode=0, sel_coef=[1, 0, -125])            # with the launch guard on top


def test_launch_guard_merges_a_small_side():
    """Hybrid mode: a handful of dense windows in a sparse matrix do not get a launch of their own,
    and a handful of sparse windows in a dense matrix do not either; per-window mode keeps them."""
    dense = sbm_graph(2, 64, 1.0, 0.0, seed=5)              # 8 windows of 64 shared columns
    sparse = tiny_random_csr(128 * 400, 128, 0.02, seed=6)
    rows = np.concatenate([np.diff(dense.rowptr), np.diff(sparse.rowptr)])
    rp = np.zeros(rows.shape[0] + 1, np.int32)
    np.cumsum(rows, out=rp[1:])
    g = CSRGraph(rows.shape[0], 128, rp, np.concatenate([dense.colind, sparse.colind]).astype(np.int32),
                 np.concatenate([dense.vals, sparse.vals]).astype(np.float32))
    coef = [0, 1 << 20, -(1 << 19)]                         # matrix path iff sparsity < 1/2
    per, _ = check_plan(g, mode=3, sel_coef=coef)
    hyb, _ = check_plan(g, mode=0, sel_coef=coef)
    assert per["route"][:8].all() and per["route"].sum() == 8 and hyb["route"].sum() == 0
    coef = [0, -(1 << 20), 1 << 19]                         # matrix path iff sparsity > 1/2
    per, _ = check_plan(g, mode=3, sel_coef=coef)
    hyb, _ = check_plan(g, mode=0, sel_coef=coef)
    assert not per["route"][:8].any() and per["route"][8:].all() and hyb["route"].all()


def test_errors_are_status_codes():
    import torch
    import paper_2412_08902_amd.binding as hc
    g = tiny_random_csr(40, 30, 0.2, seed=1)
    rp, ci, va = device_graph(g)
    bad_rp = rp.clone()
    bad_rp[5] = bad_rp[6] + 1                                    # not monotone
    with pytest.raises(hc.HcspmmError) as e:
        hc.hcspmm_prepare(g.n_rows, g.n_cols, bad_rp, ci, va)
    assert e.value.status == hc.HCSPMM_EBADCSR
    bad_ci = ci.clone()
    bad_ci[3] = g.n_cols
    with pytest.raises(hc.HcspmmError) as e:
        hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, bad_ci, va)
    assert e.value.status == hc.HCSPMM_EBADCSR
    with pytest.raises(hc.HcspmmError) as e:
        hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, nnz=g.nnz - 1)
    assert e.value.status == hc.HCSPMM_EBADCSR
    with pytest.raises(hc.HcspmmError) as e:
        hc.hcspmm_prepare(-1, g.n_cols, rp, ci, va)
    assert e.value.status == hc.HCSPMM_EINVAL
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va)
    X = torch.zeros((g.n_cols, 8), device="cuda")
    Y = torch.zeros((g.n_rows, 8), device="cuda")
    with pytest.raises(hc.HcspmmError) as e:                     # ldx < d
        hc.hcspmm_spmm(plan, X, Y, d=16)
    assert e.value.status == hc.HCSPMM_EINVAL
    hc.hcspmm_spmm(plan, X, Y)                                    # still usable after an error
    torch.cuda.synchronize()
    plan.destroy()


def test_random_structures_plan_and_product():
    """Randomised small structures (hypothesis): unsorted rows, duplicates, empty rows and windows, ragged last
    window, random selector coefficients and widths -- plan arrays bit-exact, product within the fp32 gate."""
    import torch
    import paper_2412_08902_amd.binding as hc
    from hypothesis import given, settings, strategies as st
    from test_oracle_properties import csr_structures
    from gpu_util import assert_close

    import os
    n_examples = int(os.environ.get("HCSPMM_TEST_EXAMPLES", "40"))      # a larger, non-derandomised hunt on request

    @settings(max_examples=n_examples, deadline=None, derandomize=(n_examples == 40))
    @given(csr_structures(), st.integers(0, 40), st.integers(0, 2 ** 21), st.integers(-2 ** 21, -1), st.sampled_from([0, 3]),
           st.sampled_from([1, 3, 8, 16, 33, 64, 130]), st.integers(0, 2 ** 31 - 1))
    def check(csr, c0, c1, c2, mode, d, seed):
        n_rows, n_cols, rowptr, colind = csr
        rng = np.random.default_rng(seed)
        vals = rng.standard_normal(len(colind)).astype(np.float32)
        g = CSRGraph(n_rows, n_cols, rowptr, colind, vals)
        got, info = check_plan(g, mode=mode, sel_coef=[c0, c1, c2], d_hint=d)
        X = rng.standard_normal((n_cols, d)).astype(np.float32)
        rp, ci, va = device_graph(g)
        plan = hc.hcspmm_prepare(n_rows, n_cols, rp, ci, va, route_mode=mode, sel_coef=[c0, c1, c2], d_hint=d)
        Y = torch.full((n_rows, d), float("nan"), device="cuda")
        hc.hcspmm_spmm(plan, torch.from_numpy(X).cuda(), Y)
        torch.cuda.synchronize()
        plan.destroy()
        ref = oracle.spmm(rowptr, colind, vals, X)
        bound = oracle.spmm(rowptr, colind, vals, X, use_abs=True)
        assert_close(Y.cpu().numpy().astype(np.float64), ref, bound, 1e-5)

    check()


def test_random_skewed_structures_plan_product_and_layer():
    """Seeded random structures with heavy-tailed row lengths (rows of every tier, windows of every width class,
    unsorted rows, duplicates): plan bit-exact; SpMM, the fused aggregate-then-update layer and the backward pass
    (fused update forced on) within the gates."""
    import os
    import torch
    import paper_2412_08902_amd.binding as hc
    from hypothesis import given, settings, strategies as st
    from gpu_util import assert_close
    from workloads import glorot_uniform
    n_examples = int(os.environ.get("HCSPMM_TEST_EXAMPLES", "25"))

    @settings(max_examples=n_examples, deadline=None, derandomize=(n_examples == 25))
    @given(st.integers(0, 2 ** 31 - 1), st.integers(1, 260), st.integers(1, 6000), st.sampled_from([0, 1, 2, 3]),
           st.sampled_from([16, 32, 48, 64, 128, 256, 20, 7]), st.sampled_from([1, 16, 40, 64]), st.booleans())
    def check(seed, n_rows, n_cols, mode, d, d_out, sort_rows):
        rng = np.random.default_rng(seed)
        lens = np.minimum((rng.pareto(0.9, n_rows) * 3).astype(np.int64), 3500)
        lens[rng.random(n_rows) < 0.1] = 0
        cols = []
        for l in lens:
            c = rng.integers(0, n_cols, size=int(l))
            cols.append(np.sort(c) if sort_rows else c)
        rowptr = np.zeros(n_rows + 1, dtype=np.int32)
        np.cumsum(lens, out=rowptr[1:])
        colind = (np.concatenate(cols) if lens.sum() else np.empty(0)).astype(np.int32)
        vals = rng.standard_normal(len(colind)).astype(np.float32)
        g = CSRGraph(n_rows, n_cols, rowptr, colind, vals)
        coef = [int(rng.integers(0, 64)), int(rng.integers(0, 2 ** 21)), -int(rng.integers(1, 2 ** 21))]
        check_plan(g, mode=mode, sel_coef=coef, d_hint=d)
        X = rng.standard_normal((n_cols, d)).astype(np.float32)
        rp, ci, va = device_graph(g)
        plan = hc.hcspmm_prepare(n_rows, n_cols, rp, ci, va, route_mode=mode, sel_coef=coef, d_hint=d)
        Xd = torch.from_numpy(X).cuda()
        Y = torch.full((n_rows, d), float("nan"), device="cuda")
        hc.hcspmm_spmm(plan, Xd, Y)
        torch.cuda.synchronize()
        ref = oracle.spmm(rowptr, colind, vals, X)
        bound = oracle.spmm(rowptr, colind, vals, X, use_abs=True)
        assert_close(Y.cpu().numpy().astype(np.float64), ref, bound, 1e-5, "spmm")
        W = glorot_uniform(d, d_out, seed=seed % 1000)
        ws = torch.empty(hc.hcspmm_aggregate_update_workspace_bytes(plan, d, d_out), dtype=torch.uint8, device="cuda")
        Y2 = torch.full((n_rows, d_out), float("nan"), device="cuda")
        hc.hcspmm_plan_set_update_fusion(plan, hc.HCSPMM_UPDATE_FUSED)
        if True:
            hc.hcspmm_aggregate_update(plan, Xd, torch.from_numpy(W).cuda(), Y2, ws, apply_relu=False)
            torch.cuda.synchronize()
            # backward pass of a layer with a d_out x d weight matrix: G = X (n_cols x d), layer input n_rows x d_out
            Xin = rng.standard_normal((n_rows, d_out)).astype(np.float32)
            Wb = glorot_uniform(d_out, d, seed=seed % 999)
            Yf = rng.standard_normal((n_cols, d)).astype(np.float32)
            ws3 = torch.empty(max(256, hc.hcspmm_layer_backward_workspace_bytes(plan, d_out, d)), dtype=torch.uint8, device="cuda")
            dX = torch.full((n_rows, d_out), float("nan"), device="cuda")
            dW = torch.full((d_out, d), float("nan"), device="cuda")
            hc.hcspmm_layer_backward(plan, Xd, torch.from_numpy(Xin).cuda(), torch.from_numpy(Wb).cuda(), dX, dW, ws3,
                                     Y_fwd=torch.from_numpy(Yf).cuda())
            torch.cuda.synchronize()
        plan.destroy()
        ref2 = oracle.aggregate_update(rowptr, colind, vals, X, W, relu=False)
        bound2 = oracle.aggregate_update(rowptr, colind, vals, X, W, use_abs=True)
        assert_close(Y2.cpu().numpy().astype(np.float64), ref2, bound2, 1e-5, "aggregate-update")
        ref_dx, ref_dw = oracle.layer_backward(rowptr, colind, vals, X, Xin, Wb, Y_fwd=Yf)
        b_dx, b_dw = oracle.layer_backward(rowptr, colind, vals, X, Xin, Wb, Y_fwd=Yf, use_abs=True)
        assert_close(dX.cpu().numpy().astype(np.float64), ref_dx, b_dx, 1e-5, "backward dX")
        assert_close(dW.cpu().numpy().astype(np.float64), ref_dw, b_dw, 1e-5, "backward dW")

    check()


def test_scalar_only_plan_defers_the_window_features():
    """A scalar-only plan skips the condensing step: SpMM works at once, and the features arrive on the first
    export (asked for here through the C function directly, before any info call) or info call, bit-exact."""
    import ctypes
    import torch
    import paper_2412_08902_amd.binding as hc
    from workloads import chung_lu_graph, dense_normal
    from gpu_util import assert_close, oracle_pair
    g = chung_lu_graph(5000, 90000, 2.0, seed=11, max_degree=3000)
    rp, ci, va = device_graph(g)
    want = oracle.derive_plan_vectorised(g.rowptr, g.colind, [1, 1, 1], mode=1, n_cols=g.n_cols)
    for first in ("export", "info"):
        plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=hc.HCSPMM_ROUTE_ALL_CSR, d_hint=32)
        X = dense_normal(g.n_cols, 32, seed=12)
        Y = torch.empty((g.n_rows, 32), device="cuda")
        hc.hcspmm_spmm(plan, torch.from_numpy(X).cuda(), Y)
        torch.cuda.synchronize()
        ref, bound = oracle_pair(g, X)
        assert_close(Y.cpu().numpy().astype(np.float64), ref, bound, 1e-5)
        if first == "export":
            ncols = np.full(want["W"], -1, np.int32)
            wptr = np.full(want["W"] + 1, -1, np.int64)
            st = hc.load_library().hcspmm_plan_export(plan.handle, ncols.ctypes.data_as(ctypes.c_void_p), None, None,
                                                      wptr.ctypes.data_as(ctypes.c_void_p), None, None, None, None)
            assert st == 0
            assert np.array_equal(ncols, want["ncols"]) and np.array_equal(wptr, want["wptr"])
        info = hc.hcspmm_plan_info(plan)
        assert info["total_ncols"] == want["wptr"][-1] and info["n_mfma_windows"] == 0
        got = hc.hcspmm_plan_export(plan)
        for k in KEYS:
            assert np.array_equal(got[k], want[k]), k
        hc.hcspmm_spmm(plan, torch.from_numpy(X).cuda(), Y)       # still usable after the completion
        torch.cuda.synchronize()
        assert_close(Y.cpu().numpy().astype(np.float64), ref, bound, 1e-5)
        plan.destroy()


@pytest.mark.parametrize("m", [200_000, 3_000_000, 6_000_000])
@pytest.mark.parametrize("srt", [True, False])
def test_large_matrix_path_windows_lists_and_positions(m, srt):
    """Windows beyond the LDS sort (11,200 and 30,000+ non-zeros) forced onto the matrix path: their sorted column
    lists and every non-zero's position come from bitmap ranks (narrower matrices) or from the bitmap list plus a
    search (matrices too wide for that), with sorted and with shuffled rows; plan bit-exact, product within the gate."""
    import torch
    import paper_2412_08902_amd.binding as hc
    from workloads import dense_normal
    from gpu_util import assert_close, oracle_pair
    n = 64
    rng = np.random.default_rng(5)
    lens = np.full(n, 5)
    lens[0:16] = 700
    lens[40] = 30000
    lens[50] = 4100
    cols = [rng.choice(m, size=l, replace=False) for l in lens]
    cols[3] = cols[2].copy()
    cols = [np.sort(c) if srt else c for c in cols]
    rp = np.zeros(n + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    vals = rng.standard_normal(int(lens.sum())).astype(np.float32)
    g = CSRGraph(n, m, rp, np.concatenate(cols).astype(np.int32), vals)
    got, info = check_plan(g, mode=2)
    assert info["n_mfma_windows"] == 4 and got["ncols"][2] > 30000
    X = dense_normal(m, 16, seed=6)
    rpd, cid, vad = device_graph(g)
    plan = hc.hcspmm_prepare(n, m, rpd, cid, vad, route_mode=2, d_hint=16)
    Y = torch.empty((n, 16), device="cuda")
    hc.hcspmm_spmm(plan, torch.from_numpy(X).cuda(), Y)
    torch.cuda.synchronize()
    plan.destroy()
    ref, bound = oracle_pair(g, X)
    assert_close(Y.cpu().numpy().astype(np.float64), ref, bound, 1e-5)


def test_concurrent_preparations_share_the_library_state():
    """Four host threads prepare, use and destroy plans at the same time, each on its own stream (the binding releases
    the GIL during a call): the pinned read-back pages and the per-GPU cache of device blocks are shared by all of
    them.  Every thread's plans and products must equal those computed alone."""
    import threading
    import torch
    import paper_2412_08902_amd.binding as hc
    graphs = [gcn_normalise(chung_lu_graph(1500 + 300 * i, 30000 + 9000 * i, 2.2, seed=90 + i, max_degree=600)) for i in range(4)]
    Xs = [dense_normal(g.n_cols, 32, seed=95 + i) for i, g in enumerate(graphs)]
    ref = []
    for g, X in zip(graphs, Xs):
        rp, ci, va = device_graph(g)
        plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=3, sel_coef=[1, 0, -150], d_hint=32)
        Y = torch.empty((g.n_rows, 32), device="cuda")
        hc.hcspmm_spmm(plan, torch.from_numpy(X).cuda(), Y)
        torch.cuda.synchronize()
        ref.append((hc.hcspmm_plan_export(plan), Y.clone()))
        plan.destroy()
    errors = []

    def worker(i):
        try:
            g, X = graphs[i], Xs[i]
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                rp, ci, va = device_graph(g)
                Xd = torch.from_numpy(X).cuda()
                Y = torch.empty((g.n_rows, 32), device="cuda")
            stream.synchronize()
            for it in range(25):
                plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=3, sel_coef=[1, 0, -150], d_hint=32,
                                         stream=stream)
                hc.hcspmm_spmm(plan, Xd, Y, stream=stream)
                stream.synchronize()
                if it % 8 == 0:
                    got = hc.hcspmm_plan_export(plan)
                    for k in ("ncols", "route", "wptr", "wcols", "ecol"):
                        assert np.array_equal(got[k], ref[i][0][k]), (i, it, k)
                assert torch.equal(Y, ref[i][1]), (i, it)
                plan.destroy()
        except Exception as ex:      # noqa: BLE001 - reported below, in the main thread
            errors.append((i, repr(ex)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
