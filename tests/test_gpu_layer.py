"""GPU parity of the dense update (MFMA GEMM) and the fused GCN layer against the CPU oracle."""
import numpy as np
import pytest

import oracle
from workloads import make_config, dense_normal, glorot_uniform, chung_lu_graph, gcn_normalise, tiny_random_csr
from gpu_util import device_graph, assert_close

pytestmark = pytest.mark.gpu
TOL_F32 = 1e-5


@pytest.mark.parametrize("pad", [3, 2])        # odd and even leading dimension of T: single and paired stores
@pytest.mark.parametrize("m,k,n", [(1, 1, 1), (130, 17, 5), (257, 602, 128), (128, 16, 128), (300, 64, 200),
                                   (1000, 33, 64), (64, 250, 130), (96, 0, 8),
                                   # 256 tall row tiles and a ragged tail of 32-row tiles; K with a partial last slab
                                   (32768 + 77, 40, 128), (2 * 32768 + 32 * 5, 24, 130), (32768, 32, 12),
                                   # narrow outputs with K a multiple of 16: the 16-row streaming route
                                   (257, 32, 32), (1000, 64, 16), (300, 256, 7), (5000, 128, 64), (15, 16, 1), (70001, 48, 33)])
def test_gemm(m, k, n, pad):
    import torch
    import paper_2412_08902_amd.binding as hc
    X, W = dense_normal(m, max(k, 1), seed=m + k)[:, :k], dense_normal(max(k, 1), n, seed=k + n)[:k]
    X, W = np.ascontiguousarray(X), np.ascontiguousarray(W)
    T = torch.full((m, n + pad), -5.0, device="cuda")
    hc.hcspmm_gemm_f32(torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(), T[:, :n])
    torch.cuda.synchronize()
    got = T.cpu().numpy().astype(np.float64)
    assert np.all(got[:, n:] == -5.0)
    ref = oracle.gemm(X, W)
    bound = oracle.gemm(X, W, use_abs=True)
    assert_close(got[:, :n], ref, bound, TOL_F32)


@pytest.mark.parametrize("m,k,n", [(700, 75, 132), (129, 602, 128), (33, 32, 4), (5, 38, 2)])
@pytest.mark.parametrize("xoff,ldx_extra", [(0, 1), (0, 0), (2, 1), (1, 0), (4, 1), (0, 3), (2, 3), (6, 7)])
def test_gemm_operand_alignment(m, k, n, xoff, ldx_extra):
    """X views whose base and leading dimension allow aligned 16-byte loads, 16-byte pieces around 8-byte aligned rows
    (base on or off a 16-byte boundary; the first and the last piece stick out of the matrix), or only 4-byte loads;
    W with an odd leading dimension.  X sits at the very start and end of its allocation's used range."""
    import torch
    import paper_2412_08902_amd.binding as hc
    X, W = dense_normal(m, k, seed=5), dense_normal(k, n, seed=6)
    ldx = k + ldx_extra
    flat = torch.full((xoff + (m - 1) * ldx + k,), float("nan"), device="cuda")       # nothing valid outside the view
    Xv = torch.as_strided(flat, (m, k), (ldx, 1), xoff)
    Xv.copy_(torch.from_numpy(X).cuda())
    if ldx_extra:
        pad = torch.as_strided(flat, (m - 1, ldx_extra), (ldx, 1), xoff + k)
        pad.fill_(float("nan"))
    Wbig = torch.zeros((k, n + (1 if ldx_extra % 2 else 0)), device="cuda")
    Wbig[:, :n] = torch.from_numpy(W).cuda()
    T = torch.full((m, n), -5.0, device="cuda")
    hc.hcspmm_gemm_f32(Xv, Wbig[:, :n], T)
    torch.cuda.synchronize()
    assert_close(T.cpu().numpy().astype(np.float64), oracle.gemm(X, W), oracle.gemm(X, W, use_abs=True), TOL_F32)


def test_gemm_random_shapes_and_alignments():
    """Random sizes, bases and leading dimensions of all three matrices (every load and store form of the kernel and
    the narrow-W route) against the oracle's fp64 loops.  HCSPMM_TEST_EXAMPLES=N runs N cases with a fresh seed."""
    import os
    import torch
    import paper_2412_08902_amd.binding as hc
    n_cases = int(os.environ.get("HCSPMM_TEST_EXAMPLES", "60"))
    rng = np.random.default_rng(None if "HCSPMM_TEST_EXAMPLES" in os.environ else 20250102)
    for case in range(n_cases):
        m = int(rng.choice([1, 7, 31, 33, 100, 129, 1000, 4097]))
        k, n = int(rng.integers(0, 300)), int(rng.integers(1, 200))
        xoff, xpad, wpad, tpad = (int(v) for v in rng.integers(0, 9, 4))
        X, W = dense_normal(m, max(k, 1), seed=case)[:, :k], dense_normal(max(k, 1), n, seed=case + 1)[:k]
        X, W = np.ascontiguousarray(X), np.ascontiguousarray(W)
        ldx = max(k + xpad, 1)
        flat = torch.full((xoff + (m - 1) * ldx + k + 1,), float("nan"), device="cuda")
        Xv = torch.as_strided(flat, (m, k), (ldx, 1), xoff)
        Xv.copy_(torch.from_numpy(X).cuda())
        Wb = torch.zeros((k, n + wpad), device="cuda")
        Wb[:, :n] = torch.from_numpy(W).cuda()
        T = torch.full((m, n + tpad), -5.0, device="cuda")
        hc.hcspmm_gemm_f32(Xv, Wb[:, :n], T[:, :n])
        torch.cuda.synchronize()
        got = T.cpu().numpy().astype(np.float64)
        assert np.all(got[:, n:] == -5.0), (case, m, k, n)
        assert_close(got[:, :n], oracle.gemm(X, W), oracle.gemm(X, W, use_abs=True), TOL_F32, str((case, m, k, n, xoff, xpad, wpad, tpad)))


def run_layer(g, X, W, mode, relu=True):
    import torch
    import paper_2412_08902_amd.binding as hc
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=W.shape[1])
    ws = torch.empty(hc.hcspmm_gcn_workspace_bytes(plan, X.shape[1], W.shape[1]), dtype=torch.uint8, device="cuda")
    Y = torch.full((g.n_rows, W.shape[1]), -3.0, device="cuda")
    hc.hcspmm_gcn_layer(plan, torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(), Y, ws, apply_relu=relu)
    torch.cuda.synchronize()
    out = Y.cpu().numpy().astype(np.float64)
    plan.destroy()
    return out


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("relu", [True, False])
def test_layer_small(mode, relu):
    g = gcn_normalise(chung_lu_graph(700, 9000, 2.0, seed=21))
    X, W = dense_normal(700, 50, seed=22), glorot_uniform(50, 24, seed=23)
    got = run_layer(g, X, W, mode, relu)
    ref = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W, relu=relu)
    bound = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W, use_abs=True)
    # two chained fp32 stages, still inside the single-stage gate (measured errors are a few unit roundoffs)
    assert_close(got, ref, bound, TOL_F32)
    if relu:
        assert got.min() >= 0.0 and (got == 0).any()


def test_layer_scaled_config5():
    g, X, W = make_config("C5", scale=0.01)
    got = run_layer(g, X, W, 0)
    ref = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W)
    bound = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W, use_abs=True)
    assert_close(got, ref, bound, TOL_F32)


def run_aggregate_update(g, X, W, mode, relu=True, x_bits=None, ldy_pad=0):
    import torch
    import paper_2412_08902_amd.binding as hc
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=X.shape[1],
                             mfma_dtype={None: 0, "bf16": 1, "f16": 2}[x_bits])
    ws = torch.empty(hc.hcspmm_aggregate_update_workspace_bytes(plan, X.shape[1], W.shape[1]), dtype=torch.uint8,
                     device="cuda")
    Y = torch.full((g.n_rows, W.shape[1] + ldy_pad), -3.0, device="cuda")
    if x_bits is None:
        Xd = torch.from_numpy(X).cuda()
    else:
        Xd = torch.from_numpy(X.view(np.int16)).cuda().view(torch.bfloat16 if x_bits == "bf16" else torch.float16)
    hc.hcspmm_aggregate_update(plan, Xd, torch.from_numpy(W).cuda(), Y[:, :W.shape[1]], ws, apply_relu=relu)
    torch.cuda.synchronize()
    out = Y.cpu().numpy().astype(np.float64)
    plan.destroy()
    assert np.all(out[:, W.shape[1]:] == -3.0)
    return out[:, :W.shape[1]]


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("relu", [True, False])
def test_aggregate_update_small(mode, relu):
    """Y = act((A X) W), the aggregate-then-update association, on all three routings."""
    g = gcn_normalise(chung_lu_graph(700, 9000, 2.0, seed=31))
    X, W = dense_normal(700, 40, seed=32), glorot_uniform(40, 56, seed=33)
    got = run_aggregate_update(g, X, W, mode, relu, ldy_pad=3)
    ref = oracle.aggregate_update(g.rowptr, g.colind, g.vals, X, W, relu=relu)
    bound = oracle.aggregate_update(g.rowptr, g.colind, g.vals, X, W, use_abs=True)
    assert_close(got, ref, bound, TOL_F32)
    if relu:
        assert got.min() >= 0.0 and (got == 0).any()


@pytest.mark.parametrize("din,dout", [(32, 32), (64, 16), (128, 128), (20, 7)])
def test_aggregate_update_widths(din, dout):
    from workloads import sbm_graph
    g = sbm_graph(24, 64, 0.4, 3.0, seed=41)
    X, W = dense_normal(g.n_cols, din, seed=42), glorot_uniform(din, dout, seed=43)
    got = run_aggregate_update(g, X, W, 0)
    ref = oracle.aggregate_update(g.rowptr, g.colind, g.vals, X, W)
    bound = oracle.aggregate_update(g.rowptr, g.colind, g.vals, X, W, use_abs=True)
    assert_close(got, ref, bound, TOL_F32)


def test_aggregate_update_bf16_x():
    from workloads import sbm_graph, to_bf16_bits
    g = sbm_graph(24, 64, 0.4, 3.0, seed=51)
    X, W = dense_normal(g.n_cols, 64, seed=52), glorot_uniform(64, 32, seed=53)
    Xb = to_bf16_bits(X)
    got = run_aggregate_update(g, Xb, W, 0, x_bits="bf16")
    ref = oracle.aggregate_update(g.rowptr, g.colind, g.vals, Xb, W, x_dtype=oracle.DT_BF16)
    bound = oracle.aggregate_update(g.rowptr, g.colind, g.vals, Xb, W, x_dtype=oracle.DT_BF16, use_abs=True)
    assert_close(got, ref, bound, 2e-2)


def test_aggregate_update_empty_and_errors():
    import torch
    import paper_2412_08902_amd.binding as hc
    g = tiny_random_csr(40, 40, 0.0, seed=3)          # no entries at all: Y = act(0 W) = 0
    X, W = dense_normal(40, 8, seed=4), glorot_uniform(8, 8, seed=5)
    got = run_aggregate_update(g, X, W, 0)
    assert np.all(got == 0.0)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va)
    Y = torch.empty(40, 8, device="cuda")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(hc.HcspmmError):
        hc.hcspmm_aggregate_update(plan, torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(), Y, small)
    plan.destroy()


def test_spmm_on_reformatted_layout():
    """Section V-B end to end: reorder the graph with the library's layout pass, run the hybrid SpMM on
    the reordered matrix with X permuted alike, and recover the original Y rows (Y' = P Y)."""
    import torch
    import paper_2412_08902_amd.binding as hc
    from workloads import sbm_graph, random_relabel, CSRGraph
    g = random_relabel(sbm_graph(40, 32, 0.5, 2.0, seed=61), seed=62)
    X = dense_normal(g.n_cols, 128, seed=63)
    order = hc.hcspmm_loa_order(g.n_rows, g.n_cols, g.rowptr, g.colind, 256)
    rp2, ci2, va2 = hc.hcspmm_permute_csr(g.n_rows, g.rowptr, g.colind, g.vals, order)
    g2 = CSRGraph(g.n_rows, g.n_cols, rp2, ci2, va2)
    rp, ci, va = device_graph(g2)
    plan = hc.hcspmm_prepare(g2.n_rows, g2.n_cols, rp, ci, va, d_hint=128)
    info = hc.hcspmm_plan_info(plan)
    Y2 = torch.empty(g.n_rows, 128, device="cuda")
    hc.hcspmm_spmm(plan, torch.from_numpy(X[order]).cuda(), Y2)
    torch.cuda.synchronize()
    plan.destroy()
    ref = oracle.spmm(g.rowptr, g.colind, g.vals, X)
    bound = oracle.spmm(g.rowptr, g.colind, g.vals, X, use_abs=True)
    assert_close(Y2.cpu().numpy().astype(np.float64), ref[order], bound[order], TOL_F32)
    # the scrambled layout has next to no shared columns; the reformatted one must have fewer condensed columns
    plan0 = hc.hcspmm_prepare(g.n_rows, g.n_cols, *device_graph(g), d_hint=128)
    info0 = hc.hcspmm_plan_info(plan0)
    plan0.destroy()
    assert info["total_ncols"] < 0.8 * info0["total_ncols"]
    assert info["n_mfma_windows"] >= info0["n_mfma_windows"]


@pytest.mark.parametrize("force", [False, True])
@pytest.mark.parametrize("mode", [0, 1, 2, 3])
@pytest.mark.parametrize("din,dout", [(16, 16), (32, 1), (48, 17), (64, 64), (128, 200), (256, 128), (112, 72)])
def test_aggregate_update_fused_shapes(mode, din, dout, force):
    """Widths the fused update covers (d_in a multiple of 16 up to 256), on a power-law graph whose hub rows
    and wide windows take the memory route, with a ragged last window and every routing.  `force` keeps the
    fused kernels on even where the library would judge the workspace rows too many to bother."""
    g = gcn_normalise(chung_lu_graph(3003, 150000, 2.0, seed=71, max_degree=2800))
    assert np.diff(g.rowptr).max() > 1024                    # a long row: several tiers are in play
    X, W = dense_normal(g.n_cols, din, seed=72), glorot_uniform(din, dout, seed=73)
    import paper_2412_08902_amd.binding as hc
    import torch
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=din,
                             sel_coef=[1, 0, -300] if mode == 3 else None,
                             update_fusion=hc.HCSPMM_UPDATE_FUSED if force else hc.HCSPMM_UPDATE_AUTO)
    ws = torch.empty(hc.hcspmm_aggregate_update_workspace_bytes(plan, din, dout), dtype=torch.uint8, device="cuda")
    Y = torch.full((g.n_rows, dout + 2), -3.0, device="cuda")
    hc.hcspmm_aggregate_update(plan, torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(), Y[:, :dout], ws,
                               apply_relu=(dout % 2 == 0))
    torch.cuda.synchronize()
    info = hc.hcspmm_plan_info(plan)
    plan.destroy()
    if mode == 3:
        assert info["n_mfma_windows"] > 0 and info["n_csr_windows"] > 0
    got = Y.cpu().numpy().astype(np.float64)
    assert np.all(got[:, dout:] == -3.0)
    ref = oracle.aggregate_update(g.rowptr, g.colind, g.vals, X, W, relu=(dout % 2 == 0))
    bound = oracle.aggregate_update(g.rowptr, g.colind, g.vals, X, W, use_abs=True)
    assert_close(got[:, :dout], ref, bound, TOL_F32)


def test_aggregate_update_fused_community_graph_with_empty_rows():
    from workloads import sbm_graph
    g = sbm_graph(30, 64, 0.3, 2.0, seed=81)
    # empty out a few rows and a whole window
    keep = np.ones(g.nnz, dtype=bool)
    for r in list(range(32, 48)) + [5, 77, 1900]:
        keep[g.rowptr[r]:g.rowptr[r + 1]] = False
    lens = np.add.reduceat(keep, g.rowptr[:-1]) * (np.diff(g.rowptr) > 0)
    rp = np.zeros(g.n_rows + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    from workloads import CSRGraph
    g = CSRGraph(g.n_rows, g.n_cols, rp, g.colind[keep], g.vals[keep])
    X, W = dense_normal(g.n_cols, 128, seed=82), glorot_uniform(128, 64, seed=83)
    for mode in (0, 1, 2):
        got = run_aggregate_update(g, X, W, mode, relu=False)
        ref = oracle.aggregate_update(g.rowptr, g.colind, g.vals, X, W, relu=False)
        bound = oracle.aggregate_update(g.rowptr, g.colind, g.vals, X, W, use_abs=True)
        assert_close(got, ref, bound, TOL_F32)
        assert np.all(got[32:48] == 0.0) and np.all(got[5] == 0.0)


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("mode", [0, 1, 2, 3])
@pytest.mark.parametrize("din,dout", [(32, 48), (64, 64), (128, 32), (256, 130), (80, 16)])
def test_aggregate_update_fused_16bit_x(kind, mode, din, dout):
    """16-bit X through the fused update (fp32 tile in LDS, fp32 update): scalar path exact widening, matrix
    path 16-bit products; hub rows and wide windows go through the workspace."""
    from workloads import to_bf16_bits, to_f16_bits
    g = gcn_normalise(chung_lu_graph(3003, 150000, 2.0, seed=171, max_degree=2800))
    X, W = dense_normal(g.n_cols, din, seed=172), glorot_uniform(din, dout, seed=173)
    Xb = to_bf16_bits(X) if kind == "bf16" else to_f16_bits(X)
    code = oracle.DT_BF16 if kind == "bf16" else oracle.DT_F16
    import paper_2412_08902_amd.binding as hc
    import torch
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=din,
                             mfma_dtype=1 if kind == "bf16" else 2, sel_coef=[1, 0, -300] if mode == 3 else None,
                             update_fusion=hc.HCSPMM_UPDATE_FUSED)
    ws = torch.empty(hc.hcspmm_aggregate_update_workspace_bytes(plan, din, dout), dtype=torch.uint8, device="cuda")
    Y = torch.full((g.n_rows, dout), -3.0, device="cuda")
    Xd = torch.from_numpy(Xb.view(np.int16)).cuda().view(torch.bfloat16 if kind == "bf16" else torch.float16)
    hc.hcspmm_aggregate_update(plan, Xd, torch.from_numpy(W).cuda(), Y, ws, apply_relu=False)
    torch.cuda.synchronize()
    plan.destroy()
    ref = oracle.aggregate_update(g.rowptr, g.colind, g.vals, Xb, W, relu=False, x_dtype=code)
    bound = oracle.aggregate_update(g.rowptr, g.colind, g.vals, Xb, W, x_dtype=code, use_abs=True)
    assert_close(Y.cpu().numpy().astype(np.float64), ref, bound, 2e-2 if mode != 1 else TOL_F32)


@pytest.mark.parametrize("kind,code", [("bf16", 1), ("f16", 2)])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_layer_with_16bit_intermediate(kind, code, mode):
    """Y = act(A (X W)) with X W stored in 16 bits: against the oracle that rounds the intermediate once."""
    import torch
    import paper_2412_08902_amd.binding as hc
    from workloads import sbm_graph
    g = sbm_graph(20, 64, 0.4, 3.0, seed=181) if mode == 2 else gcn_normalise(chung_lu_graph(2000, 40000, 2.0, seed=182, max_degree=900))
    X, W = dense_normal(g.n_cols, 70, seed=183), glorot_uniform(70, 64, seed=184)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=64, mfma_dtype=code)
    ws = torch.empty(hc.hcspmm_gcn_workspace_bytes(plan, 70, 64), dtype=torch.uint8, device="cuda")
    Y = torch.full((g.n_rows, 64), -3.0, device="cuda")
    hc.hcspmm_gcn_layer_ex(plan, torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(), Y, ws, t_dtype=code)
    torch.cuda.synchronize()
    plan.destroy()
    ocode = oracle.DT_BF16 if kind == "bf16" else oracle.DT_F16
    ref = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W, t_dtype=ocode)
    bound = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W, use_abs=True)
    # one 16-bit rounding of the intermediate (the device rounds its fp32 sums, the oracle its fp64 sums: they may
    # land on neighbouring 16-bit values) plus the 16-bit matrix path: the 2e-2 gate of the 16-bit paths
    assert_close(Y.cpu().numpy().astype(np.float64), ref, bound, 2e-2)
    # and it is not the fp32 layer in disguise: the rounding is visible
    exact = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W)
    assert np.abs(Y.cpu().numpy() - exact).max() > 1e-5 * np.abs(exact).max()
