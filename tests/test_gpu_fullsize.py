"""GPU parity at the benchmark's full sizes (C4, C5), in the launch configuration bench.py times:
sampled output rows against the oracle, sampled windows of the plan against the CPU re-derivation,
and properties that hold at any size."""
import numpy as np
import pytest

import oracle
from workloads import make_config, CONFIGS, dense_normal
from gpu_util import device_graph, assert_close

pytestmark = pytest.mark.gpu
TOL_F32 = 1e-5


def sample_rows(g, n, seed):
    rng = np.random.default_rng(seed)
    deg = np.diff(g.rowptr)
    rows = set(rng.choice(g.n_rows, n, replace=False).tolist())
    rows.update([0, 1, 15, 16, g.n_rows - 1, int(np.argmax(deg)), int(np.argmin(deg))])
    # some rows of every length tier: longest, around the tier boundaries, shortest
    order = np.argsort(deg)
    for frac in (0.0, 0.5, 0.9, 0.99, 0.999, 0.9999):
        rows.add(int(order[min(g.n_rows - 1, int(frac * g.n_rows))]))
    for bound in (128, 129, 256, 257, 1024, 1025, 2048, 2049):
        idx = np.nonzero(deg == bound)[0]
        if idx.size:
            rows.add(int(idx[0]))
    return np.array(sorted(rows), dtype=np.int64)


def check_plan_windows(g, plan_arrays, info, windows):
    coef = info["sel_coef"]
    for w in windows:
        wc, ec, cnt = oracle.derive_window(int(w), g.rowptr, g.colind)
        lo, hi = plan_arrays["wptr"][w], plan_arrays["wptr"][w + 1]
        s = g.rowptr[min(16 * w, g.n_rows)]
        assert plan_arrays["nnzw"][w] == cnt and plan_arrays["ncols"][w] == wc.shape[0]
        assert np.array_equal(plan_arrays["wcols"][lo:hi], wc)
        assert np.array_equal(plan_arrays["ecol"][s:s + cnt], ec)
        assert plan_arrays["route"][w] == oracle.select_route(wc.shape[0], cnt, coef)


_CONFIG_CACHE = {}


def cached_config(name, with_w=False):
    """Graph and dense matrix (and W) of a benchmark configuration, generated once per test process."""
    if name not in _CONFIG_CACHE:
        print("generating %s ..." % name, flush=True)
        _CONFIG_CACHE[name] = make_config(name)
    g, X, Wm = _CONFIG_CACHE[name]
    return (g, X, Wm) if with_w else (g, X)


def spmm_sampled(g, X, rows, what, **prepare_args):
    """prepare + SpMM through the C ABI, every output row written, the sampled rows against the oracle."""
    import torch
    import paper_2412_08902_amd.binding as hc
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, d_hint=X.shape[1], **prepare_args)
    info = hc.hcspmm_plan_info(plan)
    Xd = torch.from_numpy(X).cuda()
    Y = torch.full((g.n_rows, X.shape[1]), float("nan"), device="cuda")
    hc.hcspmm_spmm(plan, Xd, Y)
    torch.cuda.synchronize()
    assert not torch.isnan(Y).any().item(), what + ": a row was not written"
    got = Y[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    plan.destroy()
    ref = oracle.spmm_rows(rows, g.rowptr, g.colind, g.vals, X)
    bound = oracle.spmm_rows(rows, g.rowptr, g.colind, g.vals, X, use_abs=True)
    assert_close(got, ref, bound, TOL_F32, what)
    return info


@pytest.fixture(scope="module")
def c4():
    return cached_config("C4")


def test_c4_spmm_and_plan(c4):
    import torch
    import paper_2412_08902_amd.binding as hc
    g, X = c4
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, d_hint=X.shape[1])
    info = hc.hcspmm_plan_info(plan)
    Xd = torch.from_numpy(X).cuda()
    Y = torch.full((g.n_rows, X.shape[1]), float("nan"), device="cuda")
    hc.hcspmm_spmm(plan, Xd, Y)
    torch.cuda.synchronize()
    assert not torch.isnan(Y).any().item()                       # every row was written
    rows = sample_rows(g, 4096, seed=1)
    got = Y[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    ref = oracle.spmm_rows(rows, g.rowptr, g.colind, g.vals, X)
    bound = oracle.spmm_rows(rows, g.rowptr, g.colind, g.vals, X, use_abs=True)
    assert_close(got, ref, bound, TOL_F32, "C4 sampled rows")
    # property at any size: A applied to the all-ones matrix gives the row sums of the stored values
    ones = torch.ones((g.n_cols, 8), device="cuda")
    Y1 = torch.empty((g.n_rows, 8), device="cuda")
    hc.hcspmm_spmm(plan, ones, Y1)
    rs = np.add.reduceat(g.vals.astype(np.float64), g.rowptr[:-1].astype(np.int64))
    np.testing.assert_allclose(Y1[:, 0].cpu().numpy(), rs, rtol=1e-5)
    # plan: aggregate invariants everywhere, exact arrays on sampled windows
    arrays = hc.hcspmm_plan_export(plan)
    W = info["n_windows"]
    assert W == (g.n_rows + 15) // 16 and int(arrays["nnzw"].sum()) == g.nnz
    assert arrays["wptr"][-1] == info["total_ncols"] == int(arrays["ncols"].sum())
    assert np.all(arrays["ncols"] <= arrays["nnzw"]) and np.all((arrays["ncols"] > 0) == (arrays["nnzw"] > 0))
    assert np.array_equal(np.sort(np.concatenate([arrays["mfma_windows"], arrays["csr_windows"]])), np.arange(W))
    wins = np.unique(np.concatenate([[0, 1, 2, 100, W - 1, W - 2], np.random.default_rng(2).choice(W, 300)]))
    check_plan_windows(g, arrays, info, wins)
    plan.destroy()


@pytest.mark.parametrize("mode", ["all_mfma", "per_window"])
def test_c4_matrix_path_at_full_size(c4, mode):
    """The matrix-path kernels at C4's size (the shipped selector keeps C4 on the scalar path): every window
    on the matrix path, and a per-window selector with hand-set coefficients that splits the matrix."""
    g, X = c4
    rows = sample_rows(g, 4096, seed=11)
    if mode == "all_mfma":
        info = spmm_sampled(g, X, rows, "C4 all-matrix", route_mode=2)
        assert info["n_csr_windows"] == 0 or info["nnz_mfma"] == g.nnz
    else:
        # z' = H ncols (ncols - 700): windows with fewer than 700 distinct columns take the matrix path
        info = spmm_sampled(g, X, rows, "C4 per-window", route_mode=3, sel_coef=[1, 0, -700])
        share = info["n_mfma_windows"] / info["n_windows"]
        assert 0.1 < share < 0.9, share
        assert info["n_mfma_small"] > 0 and info["n_mfma_big"] > 0


@pytest.mark.parametrize("mode", ["hybrid", "all_csr", "all_mfma", "per_window"])
def test_c5_spmm_at_full_size(mode):
    """C5's aggregation stage (d = 128) on every routing, 4,096 sampled rows against the oracle."""
    g, _ = cached_config("C5")
    T = dense_normal(g.n_cols, CONFIGS["C5"]["d"], seed=1)
    rows = sample_rows(g, 4096, seed=12)
    args = {"hybrid": dict(route_mode=0), "all_csr": dict(route_mode=1), "all_mfma": dict(route_mode=2),
            # windows with fewer than 6,000 distinct columns take the matrix path
            "per_window": dict(route_mode=3, sel_coef=[1, 0, -6000])}[mode]
    info = spmm_sampled(g, T, rows, "C5 " + mode, **args)
    if mode == "per_window":
        share = info["n_mfma_windows"] / info["n_windows"]
        assert 0.1 < share < 0.9, share


def test_mixed_graph_routes_both_ways():
    """The mixed graph (dense communities followed by a power-law part, d = 128): the shipped selector sends the
    community windows to the matrix path and the power-law windows to the scalar path; sampled rows of both parts
    against the oracle."""
    g, X = cached_config("C6")
    rows = sample_rows(g, 4096, seed=13)
    info = spmm_sampled(g, X, rows, "C6 hybrid", route_mode=0)
    n_comm = CONFIGS["C6"]["n_blocks"] * CONFIGS["C6"]["block"] // 16
    assert info["n_mfma_windows"] == n_comm, (info["n_mfma_windows"], n_comm)
    assert info["n_windows"] > n_comm


def test_c5_hybrid_call_replays_from_a_hip_graph():
    """A call that forks onto the plan's side streams (large matrix, work on both paths) captured in a HIP graph:
    every replay, with eager work between the replays, reproduces the eager result bit for bit."""
    import torch
    import paper_2412_08902_amd.binding as hc
    g, _ = cached_config("C5")
    T = dense_normal(g.n_cols, CONFIGS["C5"]["d"], seed=1)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, d_hint=T.shape[1])
    info = hc.hcspmm_plan_info(plan)
    assert 0 < info["n_mfma_windows"] < info["n_windows"] and g.nnz >= 16000000       # the side-stream route
    Xd = torch.from_numpy(T).cuda()
    Y_eager = torch.empty((g.n_rows, T.shape[1]), device="cuda")
    hc.hcspmm_spmm(plan, Xd, Y_eager)                       # also sizes the plan's scratch before the capture
    torch.cuda.synchronize()
    Y = torch.zeros_like(Y_eager)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        hc.hcspmm_spmm(plan, Xd, Y)
    for rep in range(3):
        Y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, Y_eager), "replay %d differs from the eager call" % rep
        Y2 = torch.empty_like(Y_eager)                      # the program's own eager work between replays
        hc.hcspmm_spmm(plan, Xd, Y2)
        torch.cuda.synchronize()
        assert torch.equal(Y2, Y_eager)
    del graph
    plan.destroy()


def test_c5_layer_and_plan():
    import torch
    import paper_2412_08902_amd.binding as hc
    g, X, Wm = cached_config("C5", with_w=True)
    rp, ci, va = device_graph(g)
    d_out = Wm.shape[1]
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, d_hint=d_out)
    info = hc.hcspmm_plan_info(plan)
    assert info["n_mfma_windows"] > 0 and info["n_csr_windows"] > 0          # both paths are exercised
    ws = torch.empty(hc.hcspmm_gcn_workspace_bytes(plan, X.shape[1], d_out), dtype=torch.uint8, device="cuda")
    Y = torch.full((g.n_rows, d_out), float("nan"), device="cuda")
    hc.hcspmm_gcn_layer(plan, torch.from_numpy(X).cuda(), torch.from_numpy(Wm).cuda(), Y, ws)
    torch.cuda.synchronize()
    assert not torch.isnan(Y).any().item() and Y.min().item() >= 0.0
    rows = sample_rows(g, 256, seed=3)
    got = Y[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    ref = oracle.gcn_layer_rows(rows, g.rowptr, g.colind, g.vals, X, Wm)
    bound = oracle.gcn_layer_rows(rows, g.rowptr, g.colind, g.vals, X, Wm, use_abs=True)
    assert_close(got, ref, bound, TOL_F32, "C5 layer sampled rows")
    arrays = hc.hcspmm_plan_export(plan)
    W = info["n_windows"]
    wins = np.unique(np.concatenate([[0, 1, W - 1], np.random.default_rng(4).choice(W, 40)]))
    check_plan_windows(g, arrays, info, wins)
    plan.destroy()


@pytest.mark.parametrize("name,d_out", [("C3", 64), ("C2", 128), ("C4", 32)])
def test_aggregate_update_fused_at_full_size(name, d_out):
    """The fused aggregate-then-update launch at sizes where its workgroups are handed out in XCD-local runs:
    sampled rows of Y = ReLU((A X) W) against the oracle, and the whole Y against the SpMM + GEMM route."""
    import torch
    import paper_2412_08902_amd.binding as hc
    from workloads import glorot_uniform
    g, X = cached_config(name)
    Wm = glorot_uniform(X.shape[1], d_out, seed=77)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, d_hint=X.shape[1])
    Xd, Wd = torch.from_numpy(X).cuda(), torch.from_numpy(Wm).cuda()
    ws = torch.empty(hc.hcspmm_aggregate_update_workspace_bytes(plan, X.shape[1], d_out), dtype=torch.uint8, device="cuda")
    Y = torch.full((g.n_rows, d_out), float("nan"), device="cuda")
    hc.hcspmm_plan_set_update_fusion(plan, hc.HCSPMM_UPDATE_FUSED)   # the fused kernels, also where the library would pick the other route
    hc.hcspmm_aggregate_update(plan, Xd, Wd, Y, ws)
    torch.cuda.synchronize()
    rows = sample_rows(g, 300, seed=5)
    ref = oracle.aggregate_update_rows(rows, g.rowptr, g.colind, g.vals, X, Wm)
    bound = oracle.aggregate_update_rows(rows, g.rowptr, g.colind, g.vals, X, Wm, use_abs=True)
    got = Y[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    assert_close(got, ref, bound, TOL_F32, name)
    assert torch.isfinite(Y).all()
    hc.hcspmm_plan_set_update_fusion(plan, hc.HCSPMM_UPDATE_SPLIT)
    Y2 = torch.empty_like(Y)
    hc.hcspmm_aggregate_update(plan, Xd, Wd, Y2, ws)
    torch.cuda.synchronize()
    # same mathematics, different summation order in the update: agree to fp32 rounding of the row sums
    assert float((Y - Y2).abs().max()) <= 1e-4 * max(1.0, float(Y2.abs().max()))
    plan.destroy()


@pytest.mark.parametrize("name,d_in", [("C3", 64), ("C2", 128), ("C4", 32)])
def test_layer_backward_at_full_size(name, d_in):
    """Backward pass at the benchmark sizes: the whole dW (a reduction over every row) and sampled rows of dX against
    the oracle, with the workload's dense matrix as the incoming gradient."""
    import torch
    import paper_2412_08902_amd.binding as hc
    from workloads import glorot_uniform
    g, G = cached_config(name)
    d_out = G.shape[1]
    Wm = glorot_uniform(d_in, d_out, seed=78)
    X = dense_normal(g.n_rows, d_in, seed=79)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, d_hint=d_out)
    ws = torch.empty(hc.hcspmm_layer_backward_workspace_bytes(plan, d_in, d_out), dtype=torch.uint8, device="cuda")
    dX = torch.full((g.n_rows, d_in), float("nan"), device="cuda")
    dW = torch.full((d_in, d_out), float("nan"), device="cuda")
    hc.hcspmm_layer_backward(plan, torch.from_numpy(G).cuda(), torch.from_numpy(X).cuda(), torch.from_numpy(Wm).cuda(),
                             dX, dW, ws)
    torch.cuda.synchronize()
    plan.destroy()
    assert torch.isfinite(dX).all()
    ref_dx, ref_dw = oracle.layer_backward(g.rowptr, g.colind, g.vals, G, X, Wm)
    b_dx, b_dw = oracle.layer_backward(g.rowptr, g.colind, g.vals, G, X, Wm, use_abs=True)
    assert_close(dW.cpu().numpy().astype(np.float64), ref_dw, b_dw, TOL_F32, name + " dW")
    rows = sample_rows(g, 300, seed=6)
    got = dX[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    assert_close(got, ref_dx[rows], b_dx[rows], TOL_F32, name + " dX")
