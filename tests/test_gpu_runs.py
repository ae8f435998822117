"""GPU parity of the optional run kernel (matrix_kernels = RUNS): runs of four neighbouring matrix-path windows
share their gathered X rows through LDS.  The run table is compared bit for bit with its CPU re-derivation, the
product with the oracle, on shapes that reach every part of the kernel (ragged runs, slices of wide runs, both
element kinds, several column spans)."""
import numpy as np
import pytest

import oracle
from workloads import tiny_random_csr, make_config, dense_normal, CSRGraph, chung_lu_graph, gcn_normalise, sbm_graph, to_bf16_bits, to_f16_bits
from gpu_util import assert_close, device_graph

pytestmark = pytest.mark.gpu
ALL_MFMA, PER_WINDOW = 2, 3
RUNS = 2


def run_spmm(g, X, mode=ALL_MFMA, sel_coef=None, kind="f32", check_table=True):
    import torch
    import paper_2412_08902_amd.binding as hc
    rp, ci, va = device_graph(g)
    d = X.shape[1]
    code = {"f32": 0, "bf16": 1, "f16": 2}[kind]
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=d, sel_coef=sel_coef, mfma_dtype=code,
                             matrix_kernels=hc.HCSPMM_MATRIX_RUNS)
    info = hc.hcspmm_plan_info(plan)
    if kind == "f32":
        Xd, x_or, x_code = torch.from_numpy(X).cuda(), X, None
    else:
        bits = to_bf16_bits(X) if kind == "bf16" else to_f16_bits(X)
        Xd = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16 if kind == "bf16" else torch.float16)
        x_or, x_code = bits, (oracle.DT_BF16 if kind == "bf16" else oracle.DT_F16)
    Y = torch.full((g.n_rows, d + 4), -7.0, device="cuda")           # a pitch the 16-bit matrix path accepts
    hc.hcspmm_spmm(plan, Xd, Y[:, :d])
    torch.cuda.synchronize()
    got = Y.cpu().numpy().astype(np.float64)
    assert np.all(got[:, d:] == -7.0)
    if check_table and info["n_runs"] > 0:
        arrays = hc.hcspmm_plan_export(plan, with_ecol=False)
        table = hc.hcspmm_plan_export_runs(plan)
        ref = oracle.derive_runs(arrays["mfma_windows"], arrays["wptr"], arrays["wcols"])
        assert len(ref) == info["n_runs"] == table["run_nu"].shape[0]
        at = 0
        for r, nu in zip(ref, table["run_nu"]):
            assert nu == r["union"].shape[0]
            assert np.array_equal(table["ucols"][at:at + nu], r["union"])
            at += nu
            for w, sl in zip(r["windows"], r["slots"]):
                assert np.array_equal(table["wslot"][arrays["wptr"][w]:arrays["wptr"][w + 1]], sl)
        assert at == info["run_union_cols"]
        on_scalar = np.ones(arrays["wcols"].shape[0], bool)
        for w in arrays["mfma_windows"]:
            on_scalar[arrays["wptr"][w]:arrays["wptr"][w + 1]] = False
        assert np.all(table["wslot"][on_scalar] == -1)
    plan.destroy()
    ref = oracle.spmm_rows(None, g.rowptr, g.colind, g.vals, x_or, x_code)
    bound = oracle.spmm_rows(None, g.rowptr, g.colind, g.vals, x_or, x_code, use_abs=True)
    assert_close(got[:, :d], ref, bound, 1e-5 if kind == "f32" else 2e-2, "runs %s d=%d" % (kind, d))
    return info


@pytest.mark.parametrize("d", [4, 8, 20, 32, 64, 96, 128, 136, 256, 300])
def test_small_random_all_widths(d):
    g = tiny_random_csr(83, 70, 0.12, seed=100 + d)            # ragged last window and a run of fewer than four windows
    info = run_spmm(g, dense_normal(70, d, seed=200 + d))
    assert info["n_runs"] == (info["n_mfma_windows"] + 3) // 4 and info["n_run_slices"] >= info["n_runs"]


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("d", [8, 32, 64, 128, 136, 264])
def test_small_random_16bit(kind, d):
    g = tiny_random_csr(150, 333, 0.06, seed=300 + d)
    run_spmm(g, dense_normal(333, d, seed=400 + d), kind=kind)


def test_exact_integer_case_bit_for_bit():
    import torch
    import paper_2412_08902_amd.binding as hc
    g = tiny_random_csr(200, 333, 0.08, seed=5, integer_values=True)
    rng = np.random.default_rng(6)
    X = rng.integers(-8, 9, size=(333, 40)).astype(np.float32)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=ALL_MFMA, d_hint=40, matrix_kernels=hc.HCSPMM_MATRIX_RUNS)
    Y = torch.empty((200, 40), device="cuda")
    hc.hcspmm_spmm(plan, torch.from_numpy(X).cuda(), Y)
    torch.cuda.synchronize()
    plan.destroy()
    assert np.array_equal(Y.cpu().numpy().astype(np.float64), oracle.spmm(g.rowptr, g.colind, g.vals, X))


def test_wide_runs_are_cut_into_slices_with_duplicates_in_rows():
    # windows of thousands of condensed columns: several slices per run, partial tiles, starting cursors by search;
    # sorted rows with duplicate entries (summed)
    n, m = 100, 30000
    rng = np.random.default_rng(12)
    lens = np.full(n, 40)
    lens[[0, 17, 18, 50, 99]] = [8000, 513, 2049, 4500, 700]
    cols = [np.sort(rng.choice(m, size=l, replace=True)) for l in lens]
    rp = np.zeros(n + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    g = CSRGraph(n, m, rp, np.concatenate(cols).astype(np.int32), rng.standard_normal(int(lens.sum())).astype(np.float32))
    for d in (32, 128, 20):
        info = run_spmm(g, dense_normal(m, d, seed=13 + d))
        assert info["n_run_slices"] > info["n_runs"]
    run_spmm(g, dense_normal(m, 64, seed=99), kind="bf16")


def test_mixed_routing_keeps_scalar_windows_out_of_the_runs():
    g = sbm_graph(24, 64, 0.25, 4.0, seed=2)
    info = run_spmm(g, dense_normal(g.n_cols, 64, seed=4), mode=PER_WINDOW, sel_coef=[1, 0, -120])
    assert info["n_mfma_windows"] > 0 and info["n_csr_windows"] > 0 and info["n_runs"] > 0


def test_unsorted_rows_fall_back_to_the_per_window_kernels():
    g = tiny_random_csr(70, 50, 0.2, seed=9, sorted_rows=False, duplicates=True)
    info = run_spmm(g, dense_normal(50, 32, seed=10))
    assert info["n_runs"] == 0


@pytest.mark.parametrize("name,kind", [("C1", "f32"), ("C2", "f32"), ("C3", "f32"), ("C3", "bf16")])
def test_configs_full_size(name, kind):
    g, X, _ = make_config(name)
    info = run_spmm(g, X, kind=kind, check_table=(name != "C2"))
    assert info["n_runs"] > 0 and info["run_union_cols"] <= info["total_ncols"]
