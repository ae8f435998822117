"""GPU parity of the layer's backward pass (S = A G, dX = S W^T, dW = X^T S) against the CPU oracle."""
import numpy as np
import pytest

import oracle
from workloads import (make_config, dense_normal, glorot_uniform, chung_lu_graph, gcn_normalise, tiny_random_csr,
                       sbm_graph)
from gpu_util import device_graph, assert_close

pytestmark = pytest.mark.gpu
TOL_F32 = 1e-5


def run_backward(g, G, X, W, mode=0, Y_fwd=None, want_dx=True, want_dw=True, pad=0, sel_coef=None, mask_dx=False,
                 update_fusion=0):
    import torch
    import paper_2412_08902_amd.binding as hc
    rp, ci, va = device_graph(g)
    d_in, d_out = W.shape
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=d_out, sel_coef=sel_coef,
                             update_fusion=update_fusion)
    ws = torch.empty(hc.hcspmm_layer_backward_workspace_bytes(plan, d_in, d_out), dtype=torch.uint8, device="cuda")
    dX = torch.full((g.n_rows, d_in + pad), -3.0, device="cuda") if want_dx else None
    dW = torch.full((d_in, d_out + pad), -3.0, device="cuda") if want_dw else None
    hc.hcspmm_layer_backward(plan, torch.from_numpy(G).cuda(), torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(),
                             dX[:, :d_in] if want_dx else None, dW[:, :d_out] if want_dw else None, ws,
                             Y_fwd=None if Y_fwd is None else torch.from_numpy(Y_fwd).cuda(), mask_dx_by_x=mask_dx)
    torch.cuda.synchronize()
    S = ws[:g.n_rows * d_out * 4].view(torch.float32).reshape(g.n_rows, d_out).cpu().numpy().astype(np.float64)
    plan.destroy()
    out_dx = dX.cpu().numpy().astype(np.float64) if want_dx else None
    out_dw = dW.cpu().numpy().astype(np.float64) if want_dw else None
    if pad:
        assert out_dx is None or np.all(out_dx[:, d_in:] == -3.0)
        assert out_dw is None or np.all(out_dw[:, d_out:] == -3.0)
    return (None if out_dx is None else out_dx[:, :d_in]), (None if out_dw is None else out_dw[:, :d_out]), S


def check(g, G, X, W, dX, dW, S, Y_fwd=None, mask_dx=False):
    ref_dx, ref_dw = oracle.layer_backward(g.rowptr, g.colind, g.vals, G, X, W, Y_fwd=Y_fwd, mask_dx_by_x=mask_dx)
    if mask_dx and dX is not None:
        assert np.all(dX[X <= 0] == 0.0)
    b_dx, b_dw = oracle.layer_backward(g.rowptr, g.colind, g.vals, G, X, W, Y_fwd=Y_fwd, use_abs=True)
    Gm = G if Y_fwd is None else np.where(Y_fwd > 0, G, 0).astype(np.float32)
    ref_s = oracle.spmm(g.rowptr, g.colind, g.vals, Gm)
    b_s = oracle.spmm(g.rowptr, g.colind, g.vals, Gm, use_abs=True)
    if dW is not None or dX is None:
        assert_close(S, ref_s, b_s, TOL_F32, "S")
    # two chained fp32 stages, still inside the single-stage gate (measured errors are a few unit roundoffs)
    if dX is not None:
        assert_close(dX, ref_dx, b_dx, TOL_F32, "dX")
    if dW is not None:
        assert_close(dW, ref_dw, b_dw, TOL_F32, "dW")


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("relu", [False, True])
def test_backward_small(mode, relu):
    g = gcn_normalise(chung_lu_graph(700, 9000, 2.0, seed=21))
    X, W = dense_normal(700, 50, seed=22), glorot_uniform(50, 24, seed=23)
    G = dense_normal(700, 24, seed=24)
    Y = dense_normal(700, 24, seed=25) if relu else None
    if relu:
        Y[::7] = 0.0
    dX, dW, S = run_backward(g, G, X, W, mode, Y_fwd=Y, pad=3)
    check(g, G, X, W, dX, dW, S, Y_fwd=Y)


@pytest.mark.parametrize("force", [False, True])
@pytest.mark.parametrize("mode", [0, 1, 2, 3])
@pytest.mark.parametrize("din,dout", [(16, 16), (1, 32), (17, 48), (64, 64), (200, 128), (128, 256), (72, 112),
                                      (602, 128), (40, 300)])
def test_backward_shapes(mode, din, dout, force):
    """Widths in and out of the fused update's range (d_out a multiple of 16 up to 256), on a power-law graph whose
    hub rows and wide windows take the memory route, with a ragged last window and every routing."""
    g = gcn_normalise(chung_lu_graph(3003, 150000, 2.0, seed=71, max_degree=2800))
    X, W = dense_normal(g.n_rows, din, seed=72), glorot_uniform(din, dout, seed=73)
    G = dense_normal(g.n_cols, dout, seed=74)
    mask_dx = din % 2 == 0                                   # half of the shapes also mask dX by the layer's input
    dX, dW, S = run_backward(g, G, X, W, mode, pad=2, sel_coef=[1, 0, -300] if mode == 3 else None, mask_dx=mask_dx,
                             update_fusion=1 if force else 0)
    check(g, G, X, W, dX, dW, S, mask_dx=mask_dx)


def test_backward_matches_central_differences_of_the_forward_layer():
    """The forward layer on the GPU (hcspmm_gcn_layer) differentiated numerically in fp64 through the oracle is
    covered on the CPU; here the GPU backward is checked against the GPU forward by the bilinear identities
    <dW, W> = <G, A X W> = <dX, X> (no activation), which tie the two entry points together."""
    import torch
    import paper_2412_08902_amd.binding as hc
    g = gcn_normalise(chung_lu_graph(2000, 30000, 2.0, seed=5))
    X, W = dense_normal(2000, 64, seed=6), glorot_uniform(64, 32, seed=7)
    G = dense_normal(2000, 32, seed=8)
    dX, dW, _ = run_backward(g, G, X, W)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, d_hint=32)
    ws = torch.empty(hc.hcspmm_gcn_workspace_bytes(plan, 64, 32), dtype=torch.uint8, device="cuda")
    Y = torch.empty((2000, 32), device="cuda")
    hc.hcspmm_gcn_layer(plan, torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(), Y, ws, apply_relu=False)
    torch.cuda.synchronize()
    plan.destroy()
    L = float(np.sum(G.astype(np.float64) * Y.cpu().numpy().astype(np.float64)))
    scale = float(np.sum(np.abs(G) * oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W, use_abs=True)))
    assert abs(np.sum(dW * W) - L) <= 1e-5 * scale
    assert abs(np.sum(dX * X) - L) <= 1e-5 * scale


def test_backward_only_one_gradient():
    g = gcn_normalise(chung_lu_graph(900, 12000, 2.0, seed=31))
    X, W = dense_normal(900, 32, seed=32), glorot_uniform(32, 64, seed=33)
    G = dense_normal(900, 64, seed=34)
    dX, dW, S = run_backward(g, G, X, W, want_dw=False)
    assert dW is None
    check(g, G, X, W, dX, None, S)
    dX, dW, S = run_backward(g, G, X, W, want_dx=False)
    assert dX is None
    check(g, G, X, W, None, dW, S)


def test_backward_community_graph_with_empty_rows():
    from workloads import CSRGraph
    g = sbm_graph(30, 64, 0.3, 2.0, seed=81)
    keep = np.ones(g.nnz, dtype=bool)
    for r in list(range(32, 48)) + [5, 77, 1900]:
        keep[g.rowptr[r]:g.rowptr[r + 1]] = False
    lens = np.add.reduceat(keep, g.rowptr[:-1]) * (np.diff(g.rowptr) > 0)
    rp = np.zeros(g.n_rows + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    g = CSRGraph(g.n_rows, g.n_cols, rp, g.colind[keep], g.vals[keep])
    X, W = dense_normal(g.n_rows, 48, seed=82), glorot_uniform(48, 64, seed=83)
    G = dense_normal(g.n_cols, 64, seed=84)
    for mode in (0, 1, 2):
        dX, dW, S = run_backward(g, G, X, W, mode)
        check(g, G, X, W, dX, dW, S)
        assert np.all(dX[32:48] == 0.0) and np.all(S[5] == 0.0)


def test_backward_exact_on_integers():
    """0/1 adjacency, small-integer G, X and W: every partial sum is an integer below 2^24, so S, dX and dW must be
    bit-exact whatever the summation order."""
    rng = np.random.default_rng(3)
    g = tiny_random_csr(1500, 1500, 0.01, seed=9)
    g.vals[:] = 1.0
    G = rng.integers(-3, 4, size=(1500, 32)).astype(np.float32)
    X = rng.integers(-2, 3, size=(1500, 48)).astype(np.float32)
    W = rng.integers(-2, 3, size=(48, 32)).astype(np.float32)
    for mode in (0, 1, 2):
        dX, dW, S = run_backward(g, G, X, W, mode)
        ref_dx, ref_dw = oracle.layer_backward(g.rowptr, g.colind, g.vals, G, X, W)
        assert np.array_equal(dX, ref_dx) and np.array_equal(dW, ref_dw)


def test_backward_rectangular_and_errors():
    import torch
    import paper_2412_08902_amd.binding as hc
    # rectangular A (n_rows != n_cols): G has n_cols rows, X and dX have n_rows rows
    g = tiny_random_csr(333, 500, 0.03, seed=41)
    X, W = dense_normal(333, 24, seed=42), glorot_uniform(24, 32, seed=43)
    G = dense_normal(500, 32, seed=44)
    Y = dense_normal(500, 32, seed=45)
    dX, dW, S = run_backward(g, G, X, W, Y_fwd=Y)
    check(g, G, X, W, dX, dW, S, Y_fwd=Y)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, d_hint=32)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    dXt = torch.empty((333, 24), device="cuda")
    dWt = torch.empty((24, 32), device="cuda")
    with pytest.raises(hc.HcspmmError):
        hc.hcspmm_layer_backward(plan, torch.from_numpy(G).cuda(), torch.from_numpy(X).cuda(),
                                 torch.from_numpy(W).cuda(), dXt, dWt, small)
    plan.destroy()
    # a matrix with no entries: S, dX and dW are all zeros
    e = tiny_random_csr(40, 40, 0.0, seed=1)
    dX, dW, S = run_backward(e, dense_normal(40, 16, seed=2), dense_normal(40, 8, seed=3), glorot_uniform(8, 16, seed=4))
    assert np.all(dX == 0.0) and np.all(dW == 0.0) and np.all(S == 0.0)


def test_backward_scaled_config5():
    g, X, W = make_config("C5", scale=0.01)
    G = dense_normal(g.n_cols, W.shape[1], seed=91)
    ref_y = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W)
    Y = ref_y.astype(np.float32)
    dX, dW, S = run_backward(g, G, X, W, Y_fwd=Y)
    check(g, G, X, W, dX, dW, S, Y_fwd=Y)


def test_backward_is_deterministic():
    """dW is a sum over all rows: spans and their order are fixed, so two calls give the same bits."""
    g = gcn_normalise(chung_lu_graph(20000, 300000, 2.0, seed=51))
    X, W = dense_normal(20000, 64, seed=52), glorot_uniform(64, 64, seed=53)
    G = dense_normal(20000, 64, seed=54)
    a = run_backward(g, G, X, W)
    b = run_backward(g, G, X, W)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
    check(g, G, X, W, *a)


def test_layer_calls_replay_from_a_hip_graph():
    """Forward layer, fused aggregate-update and backward pass enqueue kernels only (after a first eager call that
    sizes the plan's lazily allocated buffers), so they can be captured; replays with new inputs written eagerly in
    between must reproduce the eager results bit for bit."""
    import torch
    import paper_2412_08902_amd.binding as hc
    g = gcn_normalise(chung_lu_graph(6000, 120000, 2.0, seed=61, max_degree=2500))
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, d_hint=32)
    d_in, d_out = 48, 32
    Xs = [torch.from_numpy(dense_normal(g.n_rows, d_in, seed=70 + i)).cuda() for i in range(2)]
    Gs = [torch.from_numpy(dense_normal(g.n_rows, d_out, seed=80 + i)).cuda() for i in range(2)]
    W = torch.from_numpy(glorot_uniform(d_in, d_out, seed=62)).cuda()
    W2 = torch.from_numpy(glorot_uniform(d_out, d_in, seed=63)).cuda()
    X, G = Xs[0].clone(), Gs[0].clone()
    Y = torch.empty((g.n_rows, d_out), device="cuda")
    Z = torch.empty((g.n_rows, d_in), device="cuda")
    dX = torch.empty((g.n_rows, d_in), device="cuda")
    dW = torch.empty((d_in, d_out), device="cuda")
    ws1 = torch.empty(hc.hcspmm_gcn_workspace_bytes(plan, d_in, d_out), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(hc.hcspmm_aggregate_update_workspace_bytes(plan, d_out, d_in), dtype=torch.uint8, device="cuda")
    ws3 = torch.empty(hc.hcspmm_layer_backward_workspace_bytes(plan, d_in, d_out), dtype=torch.uint8, device="cuda")

    def step():
        hc.hcspmm_gcn_layer(plan, X, W, Y, ws1)                       # Y = ReLU(A (X W))
        hc.hcspmm_aggregate_update(plan, G, W2, Z, ws2)               # Z = ReLU((A G) W2)
        hc.hcspmm_layer_backward(plan, G, X, W, dX, dW, ws3, Y_fwd=Y)

    eager = []
    for Xi, Gi in zip(Xs, Gs):
        X.copy_(Xi)
        G.copy_(Gi)
        step()
        torch.cuda.synchronize()
        eager.append([t.clone() for t in (Y, Z, dX, dW)])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in range(2):
        for i in range(2):
            X.copy_(Xs[i])
            G.copy_(Gs[i])
            for t in (Y, Z, dX, dW):
                t.fill_(-1.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for got, want, name in zip((Y, Z, dX, dW), eager[i], ("Y", "Z", "dX", "dW")):
                assert torch.equal(got, want), "replay %d, input %d: %s differs from the eager result" % (rep, i, name)
    del graph
    plan.destroy()


def test_two_layer_gcn_forward_and_backward_compose():
    """out = A (ReLU(A (X W1)) W2), L = <C, out>: both layers' forward and backward calls chained on the GPU against the
    same chain of oracle calls.  The hidden activations the GPU computed are handed to the oracle as they are (fp32),
    so the activation mask and the second layer's input are the same bits on both sides."""
    import torch
    import paper_2412_08902_amd.binding as hc
    g = gcn_normalise(chung_lu_graph(4000, 70000, 2.0, seed=91, max_degree=1500))
    n, d0, d1, d2 = g.n_rows, 40, 32, 16
    X, W1, W2 = dense_normal(n, d0, seed=92), glorot_uniform(d0, d1, seed=93), glorot_uniform(d1, d2, seed=94)
    C = dense_normal(n, d2, seed=95)
    rp, ci, va = device_graph(g)
    dev = lambda a: torch.from_numpy(a).cuda()
    Xd, W1d, W2d, Cd = dev(X), dev(W1), dev(W2), dev(C)
    H1 = torch.empty((n, d1), device="cuda")
    out = torch.empty((n, d2), device="cuda")
    dH1 = torch.empty((n, d1), device="cuda")
    dW2 = torch.empty((d1, d2), device="cuda")
    dX = torch.empty((n, d0), device="cuda")
    dW1 = torch.empty((d0, d1), device="cuda")
    plan1 = hc.hcspmm_prepare(n, n, rp, ci, va, d_hint=d1)
    plan2 = hc.hcspmm_prepare(n, n, rp, ci, va, d_hint=d2)
    ws = torch.empty(max(hc.hcspmm_gcn_workspace_bytes(plan1, d0, d1), hc.hcspmm_gcn_workspace_bytes(plan2, d1, d2),
                         hc.hcspmm_layer_backward_workspace_bytes(plan1, d0, d1),
                         hc.hcspmm_layer_backward_workspace_bytes(plan2, d1, d2)), dtype=torch.uint8, device="cuda")
    hc.hcspmm_gcn_layer(plan1, Xd, W1d, H1, ws, apply_relu=True)
    hc.hcspmm_gcn_layer(plan2, H1, W2d, out, ws, apply_relu=False)
    # layer 2 has no activation; its input H1 is layer 1's ReLU output, so dH1 is stored already masked by H1 > 0
    hc.hcspmm_layer_backward(plan2, Cd, H1, W2d, dH1, dW2, ws, mask_dx_by_x=True)
    hc.hcspmm_layer_backward(plan1, dH1, Xd, W1d, dX, dW1, ws)                    # layer 1: its G arrives masked
    torch.cuda.synchronize()
    plan1.destroy()
    plan2.destroy()
    f64 = lambda t: t.cpu().numpy().astype(np.float64)
    H1h = H1.cpu().numpy()
    a = (g.rowptr, g.colind, g.vals)
    # forward
    assert_close(f64(H1), oracle.gcn_layer(*a, X, W1), oracle.gcn_layer(*a, X, W1, use_abs=True), TOL_F32, "H1")
    assert_close(f64(out), oracle.gcn_layer(*a, H1h, W2, relu=False), oracle.gcn_layer(*a, H1h, W2, use_abs=True),
                 TOL_F32, "out")
    # backward, layer 2 then layer 1 (the oracle's layer-1 input gradient is its own fp64 dH1)
    r_dH1, r_dW2 = oracle.layer_backward(*a, C, H1h, W2, mask_dx_by_x=True)
    b_dH1, b_dW2 = oracle.layer_backward(*a, C, H1h, W2, use_abs=True)
    assert_close(f64(dH1), r_dH1, b_dH1, TOL_F32, "dH1")
    assert_close(f64(dW2), r_dW2, b_dW2, TOL_F32, "dW2")
    r_dX, r_dW1 = oracle.layer_backward(*a, r_dH1, X, W1)
    b_dX, b_dW1 = oracle.layer_backward(*a, b_dH1, X, W1, use_abs=True)
    assert_close(f64(dX), r_dX, b_dX, TOL_F32, "dX")
    assert_close(f64(dW1), r_dW1, b_dW1, TOL_F32, "dW1")
    # the bilinear identity of the last layer ties the loss to its weight gradient: <dW2, W2> = <C, out>
    L = float(np.sum(C.astype(np.float64) * f64(out)))
    assert abs(float(np.sum(f64(dW2) * W2)) - L) <= 1e-5 * float(np.sum(np.abs(C) * oracle.gcn_layer(*a, H1h, W2, use_abs=True)))


def test_backward_of_a_directed_graph_through_the_transposed_plan():
    """Forward with a non-symmetric matrix, backward with a plan of its transpose (hcspmm_transpose_csr): the GPU chain
    against the oracle chain, and <dW, W> = <G, forward output> ties the two plans together."""
    import torch
    import paper_2412_08902_amd.binding as hc
    g = tiny_random_csr(3000, 3000, 0.004, seed=71)             # no symmetry at all
    X, W = dense_normal(3000, 32, seed=72), glorot_uniform(32, 48, seed=73)
    G = dense_normal(3000, 48, seed=74)
    trp, tci, tva = hc.hcspmm_transpose_csr(g.n_rows, g.n_cols, g.rowptr, g.colind, g.vals)
    from workloads import CSRGraph
    gt = CSRGraph(g.n_cols, g.n_rows, trp, tci, tva)
    dX, dW, S = run_backward(gt, G, X, W)
    check(gt, G, X, W, dX, dW, S)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, d_hint=48)
    ws = torch.empty(hc.hcspmm_gcn_workspace_bytes(plan, 32, 48), dtype=torch.uint8, device="cuda")
    Y = torch.empty((3000, 48), device="cuda")
    hc.hcspmm_gcn_layer(plan, torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(), Y, ws, apply_relu=False)
    torch.cuda.synchronize()
    plan.destroy()
    L = float(np.sum(G.astype(np.float64) * Y.cpu().numpy().astype(np.float64)))
    scale = float(np.sum(np.abs(G) * oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W, use_abs=True)))
    assert abs(float(np.sum(dW * W)) - L) <= 1e-5 * scale
    assert abs(float(np.sum(dX * X)) - L) <= 1e-5 * scale
