"""Pins for the numeric CPU oracle: every check compares it with something that
is not the oracle itself -- hand-computed numbers, a dense fp64 product,
mathematical identities, and independent library routines."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from workloads import (CSRGraph, tiny_random_csr, make_config, gcn_normalise, to_bf16_bits,
                       bf16_bits_to_f32, to_f16_bits, dense_normal, chung_lu_graph)


def dense_of(g: CSRGraph) -> np.ndarray:
    a = np.zeros((g.n_rows, g.n_cols), dtype=np.float64)
    for i in range(g.n_rows):
        for k in range(g.rowptr[i], g.rowptr[i + 1]):
            a[i, g.colind[k]] += float(g.vals[k])
    return a


def test_hand_computed_3x4():
    # A = [[2, 0, -1, 0], [0, 0, 0, 0], [0, 3, 0, 4]],  X = [[1, 2], [3, 4], [5, 6], [7, 8]]
    rowptr = np.array([0, 2, 2, 4], dtype=np.int32)
    colind = np.array([0, 2, 1, 3], dtype=np.int32)
    vals = np.array([2, -1, 3, 4], dtype=np.float32)
    X = np.array([[1, 2], [3, 4], [5, 6], [7, 8]], dtype=np.float32)
    Y = oracle.spmm(rowptr, colind, vals, X)
    # by hand: row0 = 2*[1,2] - [5,6] = [-3,-2]; row1 = 0; row2 = 3*[3,4] + 4*[7,8] = [37,44]
    assert Y.tolist() == [[-3.0, -2.0], [0.0, 0.0], [37.0, 44.0]]


def test_hand_computed_nonsquare_not_transposed():
    # 2 x 3 matrix times 3 x 1: a transposed operand or swapped index cannot give this
    rowptr = np.array([0, 1, 3], dtype=np.int32)
    colind = np.array([2, 0, 1], dtype=np.int32)
    vals = np.array([10, 1, 100], dtype=np.float32)
    X = np.array([[1], [2], [3]], dtype=np.float32)
    assert oracle.spmm(rowptr, colind, vals, X).tolist() == [[30.0], [201.0]]


@pytest.mark.parametrize("seed,n,m,d,dens", [(1, 17, 23, 5, 0.2), (2, 64, 64, 33, 0.1), (3, 40, 9, 1, 0.5),
                                             (4, 33, 50, 16, 0.02)])
def test_matches_dense_bruteforce(seed, n, m, d, dens):
    g = tiny_random_csr(n, m, dens, seed)
    X = dense_normal(m, d, seed + 50)
    ref = dense_of(g) @ X.astype(np.float64)
    got = oracle.spmm(g.rowptr, g.colind, g.vals, X)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-13)


def test_unsorted_rows_and_duplicates_are_summed():
    g = tiny_random_csr(30, 20, 0.3, 7, sorted_rows=False, duplicates=True)
    X = dense_normal(20, 6, 8)
    ref = dense_of(g) @ X.astype(np.float64)
    np.testing.assert_allclose(oracle.spmm(g.rowptr, g.colind, g.vals, X), ref, rtol=0, atol=1e-13)


def test_exact_integer_case_bit_for_bit():
    g = tiny_random_csr(50, 60, 0.2, 11, integer_values=True)
    rng = np.random.default_rng(5)
    X = rng.integers(-8, 9, size=(60, 24)).astype(np.float32)
    ref = dense_of(g).astype(np.int64) @ X.astype(np.int64)
    got = oracle.spmm(g.rowptr, g.colind, g.vals, X)
    assert np.array_equal(got, ref.astype(np.float64))


def test_identity_gives_x():
    n, d = 37, 9
    rowptr = np.arange(n + 1, dtype=np.int32)
    colind = np.arange(n, dtype=np.int32)
    vals = np.ones(n, dtype=np.float32)
    X = dense_normal(n, d, 3)
    assert np.array_equal(oracle.spmm(rowptr, colind, vals, X), X.astype(np.float64))


def test_ones_gives_row_sums_and_degree():
    g, _, _ = make_config("C1", with_dense=False)
    X = np.ones((g.n_cols, 3), dtype=np.float32)
    Y = oracle.spmm(g.rowptr, g.colind, g.vals, X)
    deg = np.diff(g.rowptr).astype(np.float64)
    assert np.array_equal(Y, np.repeat(deg[:, None], 3, axis=1))


def test_linearity():
    g = tiny_random_csr(45, 45, 0.15, 21)
    X1, X2 = dense_normal(45, 7, 1), dense_normal(45, 7, 2)
    a, b = 0.75, -2.5
    # a, b and the products by them are exact in fp64 only if X is kept fp64: feed fp64 inputs
    lhs = oracle.spmm(g.rowptr, g.colind, g.vals, a * X1.astype(np.float64) + b * X2.astype(np.float64))
    rhs = a * oracle.spmm(g.rowptr, g.colind, g.vals, X1) + b * oracle.spmm(g.rowptr, g.colind, g.vals, X2)
    np.testing.assert_allclose(lhs, rhs, rtol=0, atol=1e-12)


def test_permutation_equivariance():
    n = 48
    g = tiny_random_csr(n, n, 0.2, 31)
    X = dense_normal(n, 5, 32)
    rng = np.random.default_rng(0)
    perm = rng.permutation(n)                      # new id of old node i is perm[i]
    A = sp.csr_matrix((g.vals, g.colind, g.rowptr), shape=(n, n)).tocoo()
    Ap = sp.csr_matrix((A.data, (perm[A.row], perm[A.col])), shape=(n, n))
    Ap.sort_indices()
    Xp = np.empty_like(X)
    Xp[perm] = X
    Y = oracle.spmm(g.rowptr, g.colind, g.vals, X)
    Yp = oracle.spmm(Ap.indptr.astype(np.int32), Ap.indices.astype(np.int32), Ap.data.astype(np.float32), Xp)
    np.testing.assert_allclose(Yp[perm], Y, rtol=0, atol=1e-13)


def test_gcn_normalised_fixed_vector():
    # A_hat D^{1/2} 1 = D^{1/2} 1 for A_hat = D^{-1/2} (A + I) D^{-1/2}: closed form
    g = gcn_normalise(chung_lu_graph(500, 4000, 2.1, seed=9))
    sqrt_d = np.sqrt(np.diff(g.rowptr).astype(np.float64))[:, None]
    Y = oracle.spmm(g.rowptr, g.colind, g.vals, sqrt_d)
    np.testing.assert_allclose(Y, sqrt_d, rtol=5e-7)           # vals were rounded once to fp32


def test_library_witnesses_scipy_and_torch():
    g, X, _ = make_config("C1")
    Y = oracle.spmm(g.rowptr, g.colind, g.vals, X)
    m = sp.csr_matrix((g.vals.astype(np.float64), g.colind, g.rowptr), shape=(g.n_rows, g.n_cols))
    np.testing.assert_allclose(Y, m @ X.astype(np.float64), rtol=0, atol=1e-12)
    import torch
    t = torch.sparse_csr_tensor(torch.from_numpy(g.rowptr.astype(np.int64)), torch.from_numpy(g.colind.astype(np.int64)),
                                torch.from_numpy(g.vals.astype(np.float64)), size=(g.n_rows, g.n_cols))
    Yt = torch.sparse.mm(t, torch.from_numpy(X.astype(np.float64))).numpy()
    np.testing.assert_allclose(Y, Yt, rtol=0, atol=1e-12)


def test_sixteen_bit_inputs_are_widened_exactly():
    g = tiny_random_csr(20, 30, 0.3, 41)
    X = dense_normal(30, 8, 42)
    xb = to_bf16_bits(X)
    # bf16 -> fp32 is exact; compare with the fp32 path on the widened values
    ref = oracle.spmm(g.rowptr, g.colind, g.vals, bf16_bits_to_f32(xb))
    assert np.array_equal(oracle.spmm(g.rowptr, g.colind, g.vals, xb, oracle.DT_BF16), ref)
    xh = to_f16_bits(X)
    ref = oracle.spmm(g.rowptr, g.colind, g.vals, xh.view(np.float16).astype(np.float32))
    assert np.array_equal(oracle.spmm(g.rowptr, g.colind, g.vals, xh, oracle.DT_F16), ref)
    # fp16 subnormals, zero, max
    bits = np.array([[0x0001, 0x03FF, 0x0000, 0x7BFF, 0x8001, 0xFBFF]], dtype=np.uint16)
    rp = np.array([0, 1], dtype=np.int32)
    got = oracle.spmm(rp, np.array([0], dtype=np.int32), np.ones(1, dtype=np.float32), bits, oracle.DT_F16)
    assert np.array_equal(got, bits.view(np.float16).astype(np.float64))


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -3.0e38, 1e-40], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1+2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up to 1+2^-6
    assert to_bf16_bits(x)[:3].tolist() == [0x3F80, 0x3F80, 0x3F82]
    import torch
    tb = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(to_bf16_bits(x), tb)


def test_abs_bound_dominates():
    g = tiny_random_csr(25, 25, 0.3, 51)
    X = dense_normal(25, 4, 52)
    Y = oracle.spmm(g.rowptr, g.colind, g.vals, X)
    S = oracle.spmm(g.rowptr, g.colind, g.vals, X, use_abs=True)
    assert np.all(S >= np.abs(Y) - 1e-15)
    np.testing.assert_allclose(S, np.abs(dense_of(g)) @ np.abs(X.astype(np.float64)), atol=1e-13)


def test_rows_subset_matches_full():
    g, X, _ = make_config("C1")
    rows = np.array([0, 5, 2707, 1234, 16, 15])
    Y = oracle.spmm(g.rowptr, g.colind, g.vals, X)
    assert np.array_equal(oracle.spmm_rows(rows, g.rowptr, g.colind, g.vals, X), Y[rows])


# ---- dense product and fused layer ------------------------------------------------

def test_gemm_hand_and_numpy():
    X = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.float32)
    W = np.array([[1, 0], [0, 1], [2, -1]], dtype=np.float32)
    assert oracle.gemm(X, W).tolist() == [[7.0, -1.0], [16.0, -1.0]]
    A, B = dense_normal(19, 37, 1), dense_normal(37, 11, 2)
    np.testing.assert_allclose(oracle.gemm(A, B), A.astype(np.float64) @ B.astype(np.float64), atol=1e-12)


def test_layer_associativity_and_reductions():
    n, din, dout = 60, 13, 7
    g = gcn_normalise(chung_lu_graph(n, 300, 2.1, seed=4))
    X, W = dense_normal(n, din, 5), dense_normal(din, dout, 6)
    Y = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W)
    # other association: (A X) W
    other = np.maximum(oracle.spmm(g.rowptr, g.colind, g.vals, X) @ W.astype(np.float64), 0.0)
    np.testing.assert_allclose(Y, other, atol=1e-12)
    assert Y.min() >= 0.0 and (Y == 0).any() and (Y > 0).any()
    # W = I reduces to ReLU(A X)
    Wi = np.eye(din, dtype=np.float32)
    np.testing.assert_array_equal(oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, Wi),
                                  np.maximum(oracle.spmm(g.rowptr, g.colind, g.vals, X), 0.0))
    # A = I reduces to ReLU(X W)
    rp, ci, v = np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32), np.ones(n, dtype=np.float32)
    np.testing.assert_allclose(oracle.gcn_layer(rp, ci, v, X, W),
                               np.maximum(X.astype(np.float64) @ W.astype(np.float64), 0.0), atol=1e-12)
    # no activation
    np.testing.assert_allclose(oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W, relu=False),
                               oracle.spmm(g.rowptr, g.colind, g.vals, X) @ W.astype(np.float64), atol=1e-12)


def test_layer_rows_subset():
    n, din, dout = 80, 9, 5
    g = gcn_normalise(chung_lu_graph(n, 500, 2.1, seed=14))
    X, W = dense_normal(n, din, 15), dense_normal(din, dout, 16)
    rows = np.array([3, 79, 0, 40])
    full = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W)
    np.testing.assert_allclose(oracle.gcn_layer_rows(rows, g.rowptr, g.colind, g.vals, X, W), full[rows], atol=1e-13)


def test_aggregate_update_pins():
    """Y = ReLU((A X) W) against scipy/numpy dense algebra, its reductions and the other association."""
    n, din, dout = 70, 11, 6
    g = gcn_normalise(chung_lu_graph(n, 420, 2.1, seed=24))
    X, W = dense_normal(n, din, 25), dense_normal(din, dout, 26)
    A = sp.csr_matrix((g.vals.astype(np.float64), g.colind, g.rowptr), shape=(n, n)).toarray()
    dense = np.maximum((A @ X.astype(np.float64)) @ W.astype(np.float64), 0.0)
    Y = oracle.aggregate_update(g.rowptr, g.colind, g.vals, X, W)
    np.testing.assert_allclose(Y, dense, atol=1e-12)
    # same value as the update-then-aggregate oracle up to rounding order
    np.testing.assert_allclose(Y, oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W), atol=1e-12)
    # W = I: ReLU(A X) exactly; no activation: signs survive
    np.testing.assert_array_equal(oracle.aggregate_update(g.rowptr, g.colind, g.vals, X, np.eye(din, dtype=np.float32)),
                                  np.maximum(oracle.spmm(g.rowptr, g.colind, g.vals, X), 0.0))
    raw = oracle.aggregate_update(g.rowptr, g.colind, g.vals, X, W, relu=False)
    np.testing.assert_allclose(raw, (A @ X.astype(np.float64)) @ W.astype(np.float64), atol=1e-12)
    assert raw.min() < 0
    # a transposed W or a swapped operand order cannot pass: W is not square
    assert Y.shape == (n, dout)
    rows = np.array([5, 69, 0, 33])
    np.testing.assert_allclose(oracle.aggregate_update_rows(rows, g.rowptr, g.colind, g.vals, X, W), Y[rows], atol=1e-13)
    # 16-bit X is widened exactly before the sums
    Xb = to_bf16_bits(X)
    Yb = oracle.aggregate_update(g.rowptr, g.colind, g.vals, Xb, W, x_dtype=oracle.DT_BF16)
    from workloads import bf16_bits_to_f32
    np.testing.assert_allclose(Yb, np.maximum((A @ bf16_bits_to_f32(Xb).astype(np.float64)) @ W.astype(np.float64), 0.0),
                               atol=1e-12)


def test_layer_with_16bit_intermediate():
    """Rounding the intermediate once: the result differs from the exact layer by at most the 16-bit unit
    roundoff times the magnitude bound, and equals the exact layer when X W is representable."""
    n, din, dout = 64, 9, 6
    g = gcn_normalise(chung_lu_graph(n, 380, 2.1, seed=34))
    X, W = dense_normal(n, din, 35), dense_normal(din, dout, 36)
    exact = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W, relu=False)
    bound = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W, use_abs=True)
    for code, u in ((oracle.DT_BF16, 2.0 ** -8), (oracle.DT_F16, 2.0 ** -11)):
        got = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W, relu=False, t_dtype=code)
        assert np.all(np.abs(got - exact) <= 1.01 * u * bound) and np.any(got != exact)
    # small integers survive both 16-bit formats: no difference at all
    Xi = np.round(X * 2).astype(np.float32)
    Wi = np.round(W * 2).astype(np.float32)
    gi = chung_lu_graph(n, 380, 2.1, seed=34)            # values 1
    np.testing.assert_array_equal(oracle.gcn_layer(gi.rowptr, gi.colind, gi.vals, Xi, Wi, t_dtype=oracle.DT_BF16),
                                  oracle.gcn_layer(gi.rowptr, gi.colind, gi.vals, Xi, Wi))
    # the rounding itself: ties to even on the bf16 grid
    from oracle.numeric import round_to_16bit
    t = np.array([[1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -2.5, 0.0]], dtype=np.float64)
    assert round_to_16bit(t, oracle.DT_BF16).tolist() == [[0x3F80, 0x3F80, 0x3F82, 0xC020, 0x0000]]
