"""ctypes front-end of the C oracle (``spmm_oracle.c``).  TEST INFRASTRUCTURE ONLY.

The arithmetic lives in the C file (straight loops, fp64).  This module compiles
it with gcc on first use, marshals numpy arrays, and composes the fused-layer
oracle ``ReLU(A (X W))`` (Eq. 1 + Eq. 2, update-then-aggregate association, ReLU
applied after the complete row sum) out of the two C loops.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

DT_F32, DT_BF16, DT_F16, DT_F64 = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spmm_oracle.c")
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None


def build_oracle_lib(force: bool = False) -> str:
    """Compile the C oracle (gcc -O2 -fopenmp).  Returns the path of the shared object."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _SO)
    return _SO


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle_lib())
        i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        lib.oracle_spmm.argtypes = [i64, vp, vp, vp, vp, vp, ctypes.c_int, i64, i32, vp, i64, ctypes.c_int]
        lib.oracle_spmm.restype = None
        lib.oracle_gemm.argtypes = [i64, vp, vp, ctypes.c_int, i64, i32, vp, ctypes.c_int, i64, i32, vp, i64,
                                    ctypes.c_int]
        lib.oracle_gemm.restype = None
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def _dense_arg(a: np.ndarray, dtype_code: Optional[int]):
    """Return (array kept alive, dtype code, leading dimension in elements)."""
    if dtype_code is None:
        if a.dtype == np.float32:
            dtype_code = DT_F32
        elif a.dtype == np.float64:
            dtype_code = DT_F64
        else:
            raise TypeError("give dtype_code for 16-bit bit patterns")
    want = {DT_F32: np.float32, DT_F64: np.float64, DT_BF16: np.uint16, DT_F16: np.uint16}[dtype_code]
    if a.dtype != want:
        raise TypeError(f"array dtype {a.dtype} does not match dtype code {dtype_code}")
    a = np.ascontiguousarray(a)
    assert a.ndim == 2
    return a, dtype_code, a.shape[1]


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def spmm_rows(rows, rowptr, colind, vals, X, x_dtype: Optional[int] = None, use_abs: bool = False) -> np.ndarray:
    """fp64 rows ``rows`` of A X (``rows`` None = all rows in order)."""
    lib = _load()
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colind = np.ascontiguousarray(colind, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    Xc, code, ldx = _dense_arg(X, x_dtype)
    d = Xc.shape[1]
    if colind.size:
        assert int(colind.min()) >= 0 and int(colind.max()) < Xc.shape[0]
    if rows is None:
        n_sel, rows_arr = rowptr.shape[0] - 1, None
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        n_sel = rows_arr.shape[0]
        if n_sel:
            assert rows_arr.min() >= 0 and rows_arr.max() < rowptr.shape[0] - 1
    Z = np.zeros((n_sel, d), dtype=np.float64)
    lib.oracle_spmm(n_sel, _p(rows_arr), _p(rowptr), _p(colind), _p(vals), _p(Xc), code, ldx, d,
                    _p(Z), d, int(use_abs))
    return Z


def spmm(rowptr, colind, vals, X, x_dtype: Optional[int] = None, use_abs: bool = False) -> np.ndarray:
    """fp64 Z = A X by the CSR triple loop (Alg. 1 / Eq. 1)."""
    return spmm_rows(None, rowptr, colind, vals, X, x_dtype, use_abs)


def gemm(X, W, rows=None, x_dtype: Optional[int] = None, w_dtype: Optional[int] = None,
         use_abs: bool = False) -> np.ndarray:
    """fp64 T = X W by the dense triple loop (Eq. 2), optionally only for ``rows`` of X."""
    lib = _load()
    Xc, xc, ldx = _dense_arg(X, x_dtype)
    Wc, wc, ldw = _dense_arg(W, w_dtype)
    assert Xc.shape[1] == Wc.shape[0]
    if rows is None:
        n_sel, rows_arr = Xc.shape[0], None
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        n_sel = rows_arr.shape[0]
    T = np.zeros((n_sel, Wc.shape[1]), dtype=np.float64)
    lib.oracle_gemm(n_sel, _p(rows_arr), _p(Xc), xc, ldx, Xc.shape[1], _p(Wc), wc, ldw, Wc.shape[1],
                    _p(T), Wc.shape[1], int(use_abs))
    return T


def round_to_16bit(T: np.ndarray, dtype_code: int) -> np.ndarray:
    """Bit patterns (uint16) of T rounded to bf16 / fp16, nearest even, through fp32 as the device does
    (its accumulators are fp32).  Finite inputs."""
    t32 = np.ascontiguousarray(T, dtype=np.float32)
    if dtype_code == DT_F16:
        return t32.astype(np.float16).view(np.uint16)
    assert dtype_code == DT_BF16
    u = t32.view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def gcn_layer(rowptr, colind, vals, X, W, relu: bool = True, use_abs: bool = False,
              t_dtype: Optional[int] = None) -> np.ndarray:
    """fp64 Y = ReLU(A (X W)): full dense product first, then the CSR loop, then max(0, .).

    t_dtype = DT_BF16 / DT_F16: the intermediate X W is rounded once to that type before the CSR loop
    (the layer variant that stores it in 16 bits); the magnitude bound (use_abs) is not rounded."""
    T = gemm(X, W, use_abs=use_abs)
    if t_dtype in (DT_BF16, DT_F16) and not use_abs:
        Y = spmm(rowptr, colind, vals, round_to_16bit(T, t_dtype), t_dtype, use_abs=use_abs)
    else:
        Y = spmm(rowptr, colind, vals, T, DT_F64, use_abs=use_abs)
    if relu and not use_abs:
        Y = np.maximum(Y, 0.0)
    return Y


def gcn_layer_rows(rows, rowptr, colind, vals, X, W, relu: bool = True, use_abs: bool = False) -> np.ndarray:
    """Rows ``rows`` of ReLU(A (X W)) computing only the rows of X W those rows reference."""
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colind = np.ascontiguousarray(colind, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    segs = [np.arange(rowptr[i], rowptr[i + 1], dtype=np.int64) for i in rows]
    ks = np.concatenate(segs) if segs else np.empty(0, dtype=np.int64)
    needed, inv = np.unique(colind[ks], return_inverse=True)
    T = gemm(X, W, rows=needed, use_abs=use_abs)
    # a small CSR over the compacted T rows: row r of it is matrix row rows[r]
    sub_ptr = np.zeros(rows.shape[0] + 1, dtype=np.int32)
    np.cumsum([s.shape[0] for s in segs], out=sub_ptr[1:])
    Y = spmm(sub_ptr, inv.astype(np.int32), vals[ks], T, DT_F64, use_abs=use_abs)
    if relu and not use_abs:
        Y = np.maximum(Y, 0.0)
    return Y


def aggregate_update(rowptr, colind, vals, X, W, relu: bool = True, x_dtype: Optional[int] = None,
                     use_abs: bool = False) -> np.ndarray:
    """fp64 Y = ReLU((A X) W): the CSR loop first (Eq. 1), then the dense product with W, then max(0, .).

    This is the aggregate-then-update association (GIN forward, GCN backward) whose coupled
    kernel Section V-A describes; Z = A X stays in fp64 between the two loops.
    """
    Z = spmm(rowptr, colind, vals, X, x_dtype, use_abs=use_abs)
    Y = gemm(Z, W, use_abs=use_abs)
    if relu and not use_abs:
        Y = np.maximum(Y, 0.0)
    return Y


def aggregate_update_rows(rows, rowptr, colind, vals, X, W, relu: bool = True, x_dtype: Optional[int] = None,
                          use_abs: bool = False) -> np.ndarray:
    """Rows ``rows`` of ReLU((A X) W)."""
    Z = spmm_rows(rows, rowptr, colind, vals, X, x_dtype, use_abs=use_abs)
    Y = gemm(Z, W, use_abs=use_abs)
    if relu and not use_abs:
        Y = np.maximum(Y, 0.0)
    return Y


def layer_backward(rowptr, colind, vals, G, X, W, Y_fwd=None, use_abs: bool = False, mask_dx_by_x: bool = False):
    """fp64 gradients of the layer X_next = act(A (X W)) given G = dL/dX_next (Eq. 3 and Eq. 4).

    In the backward pass of this layer the aggregation comes first and both products of the update
    follow it (Section V-A: the stage where the update follows the aggregation):
        Gm = G where Y_fwd > 0, else 0      (derivative of max(0, .); Y_fwd None: no activation)
        S  = A Gm                           (Eq. 4; A is the matrix the plan holds: the transpose of
                                             the forward one, itself when it is symmetric)
        dX = S W^T                          (second product of Eq. 3)
        dW = X^T S                          (first product of Eq. 3: the transposed operand is the
                                             dense matrix whose rows match the aggregated rows)
    mask_dx_by_x: dX is returned as 0 where X <= 0 -- the derivative of the max(0, .) that produced X when X is
    the previous layer's output, i.e. the masked gradient that layer's backward pass starts from.
    Returns (dX, dW).  use_abs gives the magnitude bounds |A| |Gm| |W|^T and |X|^T |A| |Gm|.
    """
    G64 = np.asarray(G, dtype=np.float64)
    if Y_fwd is not None:
        G64 = np.where(np.asarray(Y_fwd) > 0, G64, 0.0)
    S = spmm(rowptr, colind, vals, np.ascontiguousarray(G64), DT_F64, use_abs=use_abs)
    Wt = np.ascontiguousarray(np.asarray(W, dtype=np.float64).T)
    Xt = np.ascontiguousarray(np.asarray(X, dtype=np.float64).T)
    dX = gemm(S, Wt, x_dtype=DT_F64, w_dtype=DT_F64, use_abs=use_abs)
    dW = gemm(Xt, S, x_dtype=DT_F64, w_dtype=DT_F64, use_abs=use_abs)
    if mask_dx_by_x:
        dX = np.where(np.asarray(X) > 0, dX, 0.0)
    return dX, dW
