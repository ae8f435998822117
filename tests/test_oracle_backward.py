"""Pins for the backward-layer oracle (Eq. 3 and Eq. 4): hand-computed numbers, dense fp64 numpy
products, central differences of the forward layer, the bilinear form's Euler identities and
special cases.  None of them calls the oracle's own loops to produce the expected value."""
import numpy as np
import pytest

import oracle
from workloads import tiny_random_csr, dense_normal


def dense_of(g) -> np.ndarray:
    a = np.zeros((g.n_rows, g.n_cols), dtype=np.float64)
    for i in range(g.n_rows):
        for k in range(g.rowptr[i], g.rowptr[i + 1]):
            a[i, g.colind[k]] += float(g.vals[k])
    return a


def test_hand_computed_2x2():
    # A = [[1, 2], [0, 3]], G = [[1, 0], [0, 1]] (so S = A), X = [[1, 2, 3], [4, 5, 6]], W = [[1, 0], [0, 1], [2, 2]]
    rowptr = np.array([0, 2, 3], dtype=np.int32)
    colind = np.array([0, 1, 1], dtype=np.int32)
    vals = np.array([1, 2, 3], dtype=np.float32)
    G = np.eye(2, dtype=np.float32)
    X = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.float32)
    W = np.array([[1, 0], [0, 1], [2, 2]], dtype=np.float32)
    dX, dW = oracle.layer_backward(rowptr, colind, vals, G, X, W)
    # S = [[1, 2], [0, 3]];  dX = S W^T: row0 = [1, 2, 2+4], row1 = [0, 3, 6]
    assert dX.tolist() == [[1.0, 2.0, 6.0], [0.0, 3.0, 6.0]]
    # dW = X^T S: [[1*1+4*0, 1*2+4*3], [2*1+5*0, 2*2+5*3], [3*1+6*0, 3*2+6*3]]
    assert dW.tolist() == [[1.0, 14.0], [2.0, 19.0], [3.0, 24.0]]


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_matches_dense_numpy(seed):
    g = tiny_random_csr(37, 37, 0.15, seed=seed)
    d_in, d_out = 5, 7
    X = dense_normal(37, d_in, seed=seed + 10)
    W = dense_normal(d_in, d_out, seed=seed + 20)
    G = dense_normal(37, d_out, seed=seed + 30)
    A = dense_of(g)
    S = A @ G.astype(np.float64)
    dX, dW = oracle.layer_backward(g.rowptr, g.colind, g.vals, G, X, W)
    np.testing.assert_allclose(dX, S @ W.astype(np.float64).T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dW, X.astype(np.float64).T @ S, rtol=1e-12, atol=1e-12)
    assert dX.shape == (37, d_in) and dW.shape == (d_in, d_out)


def _forward_dense(A, X, W, relu):
    Y = A @ (X @ W)
    return np.maximum(Y, 0.0) if relu else Y


@pytest.mark.parametrize("relu", [False, True])
def test_central_differences_of_the_forward_layer(relu):
    """dL/dW and dL/dX of L = sum(C * act(A (X W))) by central differences, for symmetric A (the
    backward pass then multiplies by A itself, as Eq. 4 is written)."""
    rng = np.random.default_rng(5)
    n, d_in, d_out = 12, 4, 3
    B = (rng.random((n, n)) < 0.3) * rng.standard_normal((n, n))
    A = (B + B.T).astype(np.float32).astype(np.float64)
    rows, cols = np.nonzero(A)
    rowptr = np.zeros(n + 1, dtype=np.int32)
    np.cumsum(np.bincount(rows, minlength=n), out=rowptr[1:])
    colind = cols.astype(np.int32)
    vals = A[rows, cols].astype(np.float32)
    X = rng.standard_normal((n, d_in))
    W = rng.standard_normal((d_in, d_out))
    C = rng.standard_normal((n, d_out))
    Y = _forward_dense(A, X, W, relu)
    if relu:
        assert np.min(np.abs(A @ (X @ W))) > 1e-4          # no pre-activation sits on the kink
    dX, dW = oracle.layer_backward(rowptr, colind, vals, C, X, W, Y_fwd=Y if relu else None)
    h = 1e-6
    num_dW = np.zeros_like(W)
    for a in range(d_in):
        for b in range(d_out):
            Wp, Wm = W.copy(), W.copy()
            Wp[a, b] += h
            Wm[a, b] -= h
            num_dW[a, b] = (np.sum(C * _forward_dense(A, X, Wp, relu)) - np.sum(C * _forward_dense(A, X, Wm, relu))) / (2 * h)
    num_dX = np.zeros_like(X)
    for i in range(n):
        for a in range(d_in):
            Xp, Xm = X.copy(), X.copy()
            Xp[i, a] += h
            Xm[i, a] -= h
            num_dX[i, a] = (np.sum(C * _forward_dense(A, Xp, W, relu)) - np.sum(C * _forward_dense(A, Xm, W, relu))) / (2 * h)
    np.testing.assert_allclose(dW, num_dW, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(dX, num_dX, rtol=1e-6, atol=1e-7)


def test_euler_identities_of_the_bilinear_form():
    # without activation L = <G, A X W> is linear in X and in W: <dW, W> = L = <dX, X> when the plan's
    # matrix is the transpose of the forward one
    g = tiny_random_csr(29, 29, 0.2, seed=9)
    A = dense_of(g)
    X = dense_normal(29, 6, seed=1).astype(np.float64)
    W = dense_normal(6, 4, seed=2).astype(np.float64)
    G = dense_normal(29, 4, seed=3)
    L = np.sum(G * (A.T @ (X @ W)))                        # forward with A^T, backward multiplies by A
    dX, dW = oracle.layer_backward(g.rowptr, g.colind, g.vals, G, X, W)
    assert abs(np.sum(dW * W) - L) <= 1e-10 * max(1.0, abs(L))
    assert abs(np.sum(dX * X) - L) <= 1e-10 * max(1.0, abs(L))


def test_special_cases():
    n, d_in, d_out = 19, 3, 5
    X = dense_normal(n, d_in, seed=4)
    W = dense_normal(d_in, d_out, seed=5)
    G = dense_normal(n, d_out, seed=6)
    # A = I: dX = G W^T, dW = X^T G
    rowptr = np.arange(n + 1, dtype=np.int32)
    colind = np.arange(n, dtype=np.int32)
    vals = np.ones(n, dtype=np.float32)
    dX, dW = oracle.layer_backward(rowptr, colind, vals, G, X, W)
    np.testing.assert_allclose(dX, G.astype(np.float64) @ W.astype(np.float64).T, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(dW, X.astype(np.float64).T @ G.astype(np.float64), rtol=1e-13, atol=1e-13)
    # W = I (d_in = d_out): dX = A G
    g = tiny_random_csr(n, n, 0.25, seed=8)
    G2 = dense_normal(n, d_in, seed=7)
    dX2, _ = oracle.layer_backward(g.rowptr, g.colind, g.vals, G2, X, np.eye(d_in, dtype=np.float32))
    np.testing.assert_allclose(dX2, dense_of(g) @ G2.astype(np.float64), rtol=1e-12, atol=1e-12)


def test_activation_mask_zeroes_whole_entries():
    # Y_fwd <= 0 removes the entry of G before the aggregation, not after it
    g = tiny_random_csr(23, 23, 0.2, seed=12)
    X = dense_normal(23, 4, seed=1)
    W = dense_normal(4, 6, seed=2)
    G = dense_normal(23, 6, seed=3)
    Y = dense_normal(23, 6, seed=4)
    Y[::3] = 0.0                                           # exactly zero counts as inactive
    Gm = np.where(Y > 0, G, 0.0).astype(np.float64)
    S = dense_of(g) @ Gm
    dX, dW = oracle.layer_backward(g.rowptr, g.colind, g.vals, G, X, W, Y_fwd=Y)
    np.testing.assert_allclose(dX, S @ W.astype(np.float64).T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dW, X.astype(np.float64).T @ S, rtol=1e-12, atol=1e-12)


def test_equation_3_with_the_aggregated_matrix_transposed():
    # Eq. 3 as printed, W' = Z^T X' with Z = A X the aggregated matrix: the same reduction with the
    # roles of the two dense matrices exchanged gives its transpose
    g = tiny_random_csr(31, 31, 0.2, seed=15)
    Xk = dense_normal(31, 5, seed=1)
    Xp = dense_normal(31, 3, seed=2)                       # X' (gradient of the next layer's input)
    Z = dense_of(g) @ Xk.astype(np.float64)
    _, dW = oracle.layer_backward(g.rowptr, g.colind, g.vals, Xk, Xp, np.zeros((3, 5), dtype=np.float32))
    np.testing.assert_allclose(dW.T, Z.T @ Xp.astype(np.float64), rtol=1e-12, atol=1e-12)


def test_magnitude_bound_dominates():
    g = tiny_random_csr(27, 27, 0.2, seed=21)
    X = dense_normal(27, 4, seed=1)
    W = dense_normal(4, 5, seed=2)
    G = dense_normal(27, 5, seed=3)
    dX, dW = oracle.layer_backward(g.rowptr, g.colind, g.vals, G, X, W)
    bX, bW = oracle.layer_backward(g.rowptr, g.colind, g.vals, G, X, W, use_abs=True)
    A = np.abs(dense_of(g))
    np.testing.assert_allclose(bX, (A @ np.abs(G)) @ np.abs(W).T.astype(np.float64), rtol=1e-12)
    np.testing.assert_allclose(bW, np.abs(X).T.astype(np.float64) @ (A @ np.abs(G)), rtol=1e-12)
    assert np.all(np.abs(dX) <= bX + 1e-300) and np.all(np.abs(dW) <= bW + 1e-300)


def test_masked_input_gradient_chains_two_layers():
    """mask_dx_by_x hands the previous layer its gradient already masked: L = <C, A ReLU(A X W1) W2> differentiated by
    central differences (dense numpy) against layer 2's call with the flag followed by layer 1's call without a mask."""
    rng = np.random.default_rng(11)
    n, d0, d1, d2 = 10, 3, 4, 2
    B = (rng.random((n, n)) < 0.35) * rng.standard_normal((n, n))
    A = (B + B.T).astype(np.float32).astype(np.float64)
    rows, cols = np.nonzero(A)
    rowptr = np.zeros(n + 1, dtype=np.int32)
    np.cumsum(np.bincount(rows, minlength=n), out=rowptr[1:])
    colind, vals = cols.astype(np.int32), A[rows, cols].astype(np.float32)
    X = rng.standard_normal((n, d0))
    W1 = rng.standard_normal((d0, d1))
    W2 = rng.standard_normal((d1, d2))
    C = rng.standard_normal((n, d2))

    def loss(Xv, W1v):
        return float(np.sum(C * (A @ (np.maximum(A @ (Xv @ W1v), 0.0) @ W2))))

    pre = A @ (X @ W1)
    assert np.min(np.abs(pre)) > 1e-4
    H1 = np.maximum(pre, 0.0)
    dH1m, dW2 = oracle.layer_backward(rowptr, colind, vals, C, H1, W2, mask_dx_by_x=True)
    assert np.all(dH1m[H1 <= 0] == 0.0) and np.any(dH1m != 0.0)
    np.testing.assert_allclose(dW2, H1.T @ (A @ C), rtol=1e-12, atol=1e-12)
    dX, dW1 = oracle.layer_backward(rowptr, colind, vals, dH1m, X, W1)          # no mask pass: G arrives masked
    h = 1e-6
    num_dW1 = np.zeros_like(W1)
    for a in range(d0):
        for b in range(d1):
            Wp, Wm = W1.copy(), W1.copy()
            Wp[a, b] += h
            Wm[a, b] -= h
            num_dW1[a, b] = (loss(X, Wp) - loss(X, Wm)) / (2 * h)
    num_dX = np.zeros_like(X)
    for i in range(n):
        for a in range(d0):
            Xp, Xm = X.copy(), X.copy()
            Xp[i, a] += h
            Xm[i, a] -= h
            num_dX[i, a] = (loss(Xp, W1) - loss(Xm, W1)) / (2 * h)
    np.testing.assert_allclose(dW1, num_dW1, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(dX, num_dX, rtol=1e-6, atol=1e-7)
    # and the flag is exactly "mask afterwards"
    dH1, _ = oracle.layer_backward(rowptr, colind, vals, C, H1, W2)
    assert np.array_equal(dH1m, np.where(H1 > 0, dH1, 0.0))


def test_directed_graph_backward_uses_the_transpose():
    """For a non-symmetric forward matrix the backward aggregation multiplies by its transpose: central differences of
    L = <C, ReLU(A_f X W)> against the oracle called with A_f^T (built here with scipy)."""
    import scipy.sparse as sp
    rng = np.random.default_rng(21)
    n, d_in, d_out = 11, 3, 4
    Af = ((rng.random((n, n)) < 0.3) * rng.standard_normal((n, n))).astype(np.float32).astype(np.float64)
    assert np.abs(Af - Af.T).max() > 0.1
    At = sp.csr_matrix(Af.T)
    At.sort_indices()
    X = rng.standard_normal((n, d_in))
    W = rng.standard_normal((d_in, d_out))
    C = rng.standard_normal((n, d_out))
    pre = Af @ (X @ W)
    assert np.min(np.abs(pre)) > 1e-4
    Y = np.maximum(pre, 0.0)
    dX, dW = oracle.layer_backward(At.indptr.astype(np.int32), At.indices.astype(np.int32), At.data.astype(np.float32),
                                   C, X, W, Y_fwd=Y)
    loss = lambda Xv, Wv: float(np.sum(C * np.maximum(Af @ (Xv @ Wv), 0.0)))
    h = 1e-6
    for a in range(d_in):
        for b in range(d_out):
            Wp, Wm = W.copy(), W.copy()
            Wp[a, b] += h
            Wm[a, b] -= h
            assert abs((loss(X, Wp) - loss(X, Wm)) / (2 * h) - dW[a, b]) <= 1e-6 * max(1.0, abs(dW[a, b]))
    for i in range(n):
        for a in range(d_in):
            Xp, Xm = X.copy(), X.copy()
            Xp[i, a] += h
            Xm[i, a] -= h
            assert abs((loss(Xp, W) - loss(Xm, W)) / (2 * h) - dX[i, a]) <= 1e-6 * max(1.0, abs(dX[i, a]))
