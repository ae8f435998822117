"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest

import oracle
from workloads import (tiny_random_csr, make_config, dense_normal, dense_uniform, CSRGraph, chung_lu_graph,
                       gcn_normalise, sbm_graph)
from gpu_util import gpu_spmm, assert_close, oracle_pair, device_graph

pytestmark = pytest.mark.gpu

HYBRID, ALL_CSR, ALL_MFMA, PER_WINDOW = 0, 1, 2, 3
MODES = [HYBRID, ALL_CSR, ALL_MFMA]
TOL_F32 = 1e-5          # max error relative to |A||X|, fp32 path


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("d", [1, 2, 3, 4, 8, 16, 17, 32, 33, 48, 64, 96, 128, 130, 256, 300])
def test_small_random_all_widths(mode, d):
    g = tiny_random_csr(83, 70, 0.12, seed=100 + d)            # ragged last window, some empty rows
    X = dense_normal(70, d, seed=200 + d)
    Y, _ = gpu_spmm(g, X, mode, pad_x=(d % 3), pad_y=(d % 2))
    ref, bound = oracle_pair(g, X)
    assert_close(Y, ref, bound, TOL_F32, "d=%d mode=%d" % (d, mode))


@pytest.mark.parametrize("mode", MODES)
def test_exact_integer_case_bit_for_bit(mode):
    g = tiny_random_csr(200, 333, 0.08, seed=5, integer_values=True)
    rng = np.random.default_rng(6)
    X = rng.integers(-8, 9, size=(333, 40)).astype(np.float32)
    Y, _ = gpu_spmm(g, X, mode)
    ref, _ = oracle_pair(g, X)
    assert np.array_equal(Y, ref)


@pytest.mark.parametrize("mode", MODES)
def test_unsorted_rows_and_duplicates(mode):
    g = tiny_random_csr(70, 50, 0.2, seed=9, sorted_rows=False, duplicates=True)
    X = dense_normal(50, 32, seed=10)
    Y, _ = gpu_spmm(g, X, mode)
    ref, bound = oracle_pair(g, X)
    assert_close(Y, ref, bound, TOL_F32)


@pytest.mark.parametrize("mode", MODES)
def test_degenerate_shapes(mode):
    # one row; fewer than 16 rows; all rows empty; one dense row among empty ones; identity
    X = dense_normal(40, 32, seed=3)
    one = CSRGraph(1, 40, np.array([0, 3], np.int32), np.array([5, 7, 39], np.int32), np.array([1, 2, 3], np.float32))
    empty = CSRGraph(37, 40, np.zeros(38, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
    rp = np.zeros(34, np.int32)
    rp[18:] = 40
    hub = CSRGraph(33, 40, rp, np.arange(40, dtype=np.int32), np.linspace(-1, 1, 40).astype(np.float32))
    eye = CSRGraph(40, 40, np.arange(41, dtype=np.int32), np.arange(40, dtype=np.int32), np.ones(40, np.float32))
    for g in (one, empty, hub, eye):
        Y, _ = gpu_spmm(g, X, mode)
        ref, bound = oracle_pair(g, X)
        assert_close(Y, ref, bound, TOL_F32)
    Y, _ = gpu_spmm(eye, X, mode)
    assert np.array_equal(Y, X.astype(np.float64))


@pytest.mark.parametrize("mode", MODES)
def test_long_rows_and_wide_windows(mode):
    # rows longer than one segment, several segments, windows with thousands of distinct columns
    n, m = 100, 9000
    rng = np.random.default_rng(12)
    lens = np.full(n, 3)
    lens[[0, 17, 18, 50, 99]] = [8000, 513, 2049, 4500, 700]
    cols = [np.sort(rng.choice(m, size=l, replace=False)) for l in lens]
    rp = np.zeros(n + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    g = CSRGraph(n, m, rp, np.concatenate(cols).astype(np.int32),
                 rng.standard_normal(int(lens.sum())).astype(np.float32))
    for d in (32, 128, 20):
        X = dense_normal(m, d, seed=13 + d)
        Y, _ = gpu_spmm(g, X, mode)
        ref, bound = oracle_pair(g, X)
        assert_close(Y, ref, bound, TOL_F32, "d=%d" % d)


@pytest.mark.parametrize("mode", MODES)
def test_wide_windows_with_unsorted_rows(mode):
    # windows with thousands of condensed columns whose rows are NOT sorted by column
    n, m = 48, 20000
    rng = np.random.default_rng(77)
    lens = rng.integers(200, 1500, size=n)
    cols = [rng.choice(m, size=l, replace=False) for l in lens]          # random order inside each row
    rp = np.zeros(n + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    g = CSRGraph(n, m, rp, np.concatenate(cols).astype(np.int32),
                 rng.standard_normal(int(lens.sum())).astype(np.float32))
    X = dense_normal(m, 64, seed=78)
    Y, _ = gpu_spmm(g, X, mode)
    ref, bound = oracle_pair(g, X)
    assert_close(Y, ref, bound, TOL_F32)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_configs_full_size(name, mode):
    g, X, _ = make_config(name)
    Y, info = gpu_spmm(g, X, mode)
    ref, bound = oracle_pair(g, X)
    assert_close(Y, ref, bound, TOL_F32, "%s mode=%d" % (name, mode))
    if mode == ALL_CSR:
        assert info["n_mfma_windows"] == 0
    if mode == ALL_MFMA:
        assert info["n_csr_windows"] == int((np.add.reduceat(np.diff(g.rowptr), np.arange(0, g.n_rows, 16)) == 0).sum())


def test_routes_agree_and_rerun_is_deterministic():
    g, X, _ = make_config("C2", scale=0.05)
    ys = [gpu_spmm(g, X, mode)[0] for mode in MODES]
    ref, bound = oracle_pair(g, X)
    for y in ys:
        assert_close(y, ref, bound, TOL_F32)
    again = gpu_spmm(g, X, HYBRID)[0]
    assert np.array_equal(ys[0], again)


def test_custom_selector_mixes_both_paths():
    g = sbm_graph(24, 64, 0.25, 4.0, seed=2)
    X = dense_normal(g.n_cols, 64, seed=4)
    # z = ncols + 0*sparsity - 120 < 0  <=>  ncols < 120: some windows on each path
    Y, info = gpu_spmm(g, X, PER_WINDOW, sel_coef=[1, 0, -120])
    assert info["n_mfma_windows"] > 0 and info["n_csr_windows"] > 0
    ref, bound = oracle_pair(g, X)
    assert_close(Y, ref, bound, TOL_F32)
    # the hybrid mode may merge a small side into the other path; the values stay the same product
    Y, info = gpu_spmm(g, X, HYBRID, sel_coef=[1, 0, -120])
    assert_close(Y, ref, bound, TOL_F32)


def test_hip_graph_replays_match_eager():
    """hcspmm_spmm only enqueues kernels on the caller's stream, so it can be captured in a HIP graph.
    Each replay -- with new inputs written eagerly in between -- must reproduce the eager result bit for bit."""
    import torch
    import paper_2412_08902_amd.binding as hc
    g = sbm_graph(24, 64, 0.25, 4.0, seed=2)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=PER_WINDOW, d_hint=64, sel_coef=[1, 0, -120])
    info = hc.hcspmm_plan_info(plan)
    assert info["n_mfma_windows"] > 0 and info["n_csr_windows"] > 0
    Xs = [torch.from_numpy(dense_normal(g.n_cols, 64, seed=40 + i)).cuda() for i in range(3)]
    X = Xs[0].clone()
    Y = torch.empty(g.n_rows, 64, device="cuda")
    eager = []
    for Xi in Xs:
        hc.hcspmm_spmm(plan, Xi, Y)
        torch.cuda.synchronize()
        eager.append(Y.clone())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        hc.hcspmm_spmm(plan, X, Y)
    for rep in range(2):
        for i, Xi in enumerate(Xs):
            X.copy_(Xi)                                   # eager work between replays
            Y.fill_(-1.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(Y, eager[i]), "replay %d of input %d differs from the eager result" % (rep, i)
    ref, bound = oracle_pair(g, Xs[2].cpu().numpy())
    assert_close(Y.cpu().numpy().astype(np.float64), ref, bound, TOL_F32)
    del graph
    plan.destroy()


@pytest.mark.parametrize("mode", [PER_WINDOW, ALL_CSR, ALL_MFMA])
def test_values_may_change_in_place_under_a_plan(mode):
    """The plan is a function of the structure only: new edge values written into the borrowed array are
    picked up by the next call on both paths."""
    import torch
    import paper_2412_08902_amd.binding as hc
    g = sbm_graph(16, 64, 0.3, 3.0, seed=12)
    X = dense_normal(g.n_cols, 48, seed=13)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=48, sel_coef=[1, 0, -118])
    Xd = torch.from_numpy(X).cuda()
    Y = torch.empty(g.n_rows, 48, device="cuda")
    rng = np.random.default_rng(14)
    for rep in range(3):
        new_vals = rng.standard_normal(g.nnz).astype(np.float32)
        va.copy_(torch.from_numpy(new_vals).cuda())
        hc.hcspmm_spmm(plan, Xd, Y)
        torch.cuda.synchronize()
        g2 = CSRGraph(g.n_rows, g.n_cols, g.rowptr, g.colind, new_vals)
        ref, bound = oracle_pair(g2, X)
        assert_close(Y.cpu().numpy().astype(np.float64), ref, bound, TOL_F32, "values of round %d" % rep)
    plan.destroy()


def test_two_plans_on_two_streams():
    """Different plans are independent: two SpMMs enqueued on two streams at once both match the oracle,
    and a plan prepared with one width hint serves another width."""
    import torch
    import paper_2412_08902_amd.binding as hc
    ga = gcn_normalise(chung_lu_graph(3000, 60000, 2.0, seed=91, max_degree=1500))
    gb = sbm_graph(40, 64, 0.5, 3.0, seed=92)
    Xa, Xb = dense_normal(ga.n_cols, 96, seed=93), dense_normal(gb.n_cols, 128, seed=94)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    pa = hc.hcspmm_prepare(ga.n_rows, ga.n_cols, *device_graph(ga), d_hint=32)          # hint differs from the width used
    pb = hc.hcspmm_prepare(gb.n_rows, gb.n_cols, *device_graph(gb), d_hint=128)
    Xad, Xbd = torch.from_numpy(Xa).cuda(), torch.from_numpy(Xb).cuda()
    Ya = torch.empty(ga.n_rows, 96, device="cuda")
    Yb = torch.empty(gb.n_rows, 128, device="cuda")
    torch.cuda.synchronize()
    for _ in range(3):
        hc.hcspmm_spmm(pa, Xad, Ya, stream=sa)
        hc.hcspmm_spmm(pb, Xbd, Yb, stream=sb)
    sa.synchronize()
    sb.synchronize()
    ra, ba = oracle_pair(ga, Xa)
    rb, bb = oracle_pair(gb, Xb)
    assert_close(Ya.cpu().numpy().astype(np.float64), ra, ba, TOL_F32, "plan a")
    assert_close(Yb.cpu().numpy().astype(np.float64), rb, bb, TOL_F32, "plan b")
    pa.destroy()
    pb.destroy()


@pytest.mark.parametrize("mode", MODES)
def test_very_wide_dense_operand(mode):
    """d far beyond one pass of a lane group or one launch of the matrix-path kernels (several column chunks)."""
    g = gcn_normalise(chung_lu_graph(300, 4000, 2.1, seed=101))
    X = dense_normal(g.n_cols, 1030, seed=102)
    Y, _ = gpu_spmm(g, X, mode, pad_x=2, pad_y=6)
    ref, bound = oracle_pair(g, X)
    assert_close(Y, ref, bound, TOL_F32)


@pytest.mark.parametrize("mode", MODES)
def test_column_count_at_the_documented_limit(mode):
    """n_cols = 2^27 - 1 (the largest the packed per-non-zero index allows), entries spread over the whole range:
    exercises the bitmap passes of the big-window unique kernel and 64-bit addressing of X."""
    n_cols = (1 << 27) - 1
    rng = np.random.default_rng(111)
    n_rows = 40
    lens = np.full(n_rows, 6)
    lens[0:16] = 400                                   # window 0 beyond the LDS-sort capacity
    cols = [np.sort(rng.choice(n_cols, size=int(l), replace=False)) for l in lens]
    cols[17][-1] = n_cols - 1                          # the last column itself
    cols[18][0] = 0
    rp = np.zeros(n_rows + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    vals = rng.standard_normal(int(lens.sum())).astype(np.float32)
    g = CSRGraph(n_rows, n_cols, rp, np.concatenate(cols).astype(np.int32), vals)
    X = np.zeros((n_cols, 1), dtype=np.float32)        # 512 MiB; only the referenced rows carry values
    used = np.unique(g.colind)
    X[used, 0] = rng.standard_normal(used.shape[0]).astype(np.float32)
    Y, info = gpu_spmm(g, X, mode)
    ref, bound = oracle_pair(g, X)
    assert_close(Y, ref, bound, TOL_F32)
    assert info["n_cols"] == n_cols


@pytest.mark.parametrize("kind", ["f32", "bf16"])
@pytest.mark.parametrize("mode", MODES)
def test_row_offsets_beyond_2_to_the_31_elements(mode, kind):
    """Leading dimensions so large that row * ld exceeds 2^31 ELEMENTS for most rows of X and of Y (the kernels must
    form these offsets in 64 bits): X and Y live in device buffers with a pitch of 36,000 elements, the oracle
    works on the compact columns."""
    import torch
    import paper_2412_08902_amd.binding as hc
    from workloads import to_bf16_bits
    n, d, ld = 70000, 24, 36000                         # last row starts at element 2.52e9 > 2^31 (2.15e9)
    assert (n - 1) * ld > 2 ** 31
    rng = np.random.default_rng(321)
    lens = rng.integers(0, 9, size=n)
    lens[n - 16:] = 40                                  # a dense last window, beyond the 2^31 mark on both sides
    lens[5] = 3000                                      # one long row whose columns span the whole range
    cols = [np.sort(rng.choice(n, size=int(l), replace=False)) for l in lens]
    cols[n - 1][-1] = n - 1
    rp = np.zeros(n + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    g = CSRGraph(n, n, rp, np.concatenate(cols).astype(np.int32),
                 rng.standard_normal(int(lens.sum())).astype(np.float32))
    X = dense_normal(n, d, seed=322)
    dev = torch.device("cuda:0")
    if kind == "f32":
        Xbuf = torch.empty((n, ld), dtype=torch.float32, device=dev)            # 10 GB, uninitialised beyond column d
        Xbuf[:, :d] = torch.from_numpy(X).to(dev)
        x_or, code, tol = X, None, TOL_F32
    else:
        bits = to_bf16_bits(X)
        Xbuf = torch.empty((n, ld), dtype=torch.bfloat16, device=dev)
        Xbuf[:, :d] = torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
        x_or, code, tol = bits, oracle.DT_BF16, (2e-2 if mode != ALL_CSR else TOL_F32)
    Ybuf = torch.empty((n, ld), dtype=torch.float32, device=dev)
    Ybuf[:, :d + 1] = -777.0
    rpd, cid, vad = device_graph(g)
    plan = hc.hcspmm_prepare(n, n, rpd, cid, vad, route_mode=mode, d_hint=d, mfma_dtype=0 if kind == "f32" else 1)
    hc.hcspmm_spmm(plan, Xbuf, Ybuf, d=d)
    torch.cuda.synchronize()
    plan.destroy()
    Y = Ybuf[:, :d + 1].cpu().numpy().astype(np.float64)
    assert np.all(Y[:, d] == -777.0), "wrote outside the d output columns"
    ref = oracle.spmm_rows(None, g.rowptr, g.colind, g.vals, x_or, code)
    bound = oracle.spmm_rows(None, g.rowptr, g.colind, g.vals, x_or, code, use_abs=True)
    assert_close(Y[:, :d], ref, bound, tol, "mode %d %s" % (mode, kind))
