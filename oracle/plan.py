"""CPU re-derivation of the preprocessing plan.  TEST INFRASTRUCTURE ONLY.

Steps, in the paper's order (Section IV-A "Combination Strategy", Section IV-C
"Adaptive Core Selection"):

1. row windows: window w holds rows [H*w, min(H*w+H, N)); its non-zeros are the
   contiguous CSR slice rowptr[H*w] .. rowptr[min(H*w+H, N)]            (H = 16)
2. condensing: the window's distinct column ids, ascending, are its non-zero
   columns; ``ncols`` is their count (= |union of the rows' neighbour sets|,
   Section V-B); every non-zero gets its position in that list (``ecol``)
3. features: ``nnzw`` (non-zeros in the window) and
   ``sparsity = 1 - nnzw / (H * ncols)``   (pinned by the training-set recipe:
   c columns with c .. 15c non-zeros span sparsity 15/16 .. 1/16)
4. selection: the logistic model's linear form ``w1*ncols + w2*sparsity + b``;
   label 1 of the training set means the scalar cores were faster, and the
   stored flag is 0 = scalar path, 1 = matrix path.  Evaluated exactly in
   integers after multiplying by ``H*ncols > 0``:
       z = c0*H*ncols^2 + c1*(H*ncols - nnzw) + c2*H*ncols
       route = 1 (matrix path)  iff  z < 0 ;  an empty window gets route 0.
   The coefficients are inputs to this module (the paper does not print its
   own, they are fitted per GPU and precision).
4b. launch guard (a choice of this implementation, not of the paper, whose single kernel
   has no per-path launch cost): in hybrid mode, when both paths got work and the smaller
   side holds fewer than 2^18 non-zeros and less than 1/8 of all non-zeros, all its windows
   take the other path -- checked for the matrix side first, then for the scalar side.
   Mode ROUTE_PER_WINDOW skips this step.
5. the ascending lists of window ids per route.
6. runs (a launch table of this implementation's optional run kernel, not of the paper): the
   matrix path's window list is cut into runs of RUN_WINDOWS consecutive entries; a run's union
   is the ascending list of the distinct columns of its windows, and every window column gets
   its position in that union.

All arithmetic is Python / numpy integer arithmetic.
"""
from __future__ import annotations

from fractions import Fraction
from typing import Dict, Sequence

import numpy as np

ROUTE_HYBRID, ROUTE_ALL_CSR, ROUTE_ALL_MFMA, ROUTE_PER_WINDOW = 0, 1, 2, 3
GUARD_NNZ, GUARD_SHARE = 1 << 18, 8
RUN_WINDOWS = 4


def window_features(cols_in_window: np.ndarray):
    """(ncols, nnzw) of one window from the column ids of its non-zeros."""
    cols_in_window = np.asarray(cols_in_window)
    return int(np.unique(cols_in_window).shape[0]), int(cols_in_window.shape[0])


def sparsity(ncols: int, nnzw: int, H: int = 16) -> Fraction:
    """Exact sparsity of the condensed H x ncols window."""
    return 1 - Fraction(nnzw, H * ncols)


def computing_intensity(ncols: int, nnzw: int) -> Fraction:
    """#non-zero elements / #non-zero columns (Eq. 5)."""
    return Fraction(nnzw, ncols)


def select_route(ncols: int, nnzw: int, coef: Sequence[int], H: int = 16, mode: int = ROUTE_HYBRID) -> int:
    """0 = scalar (CSR) path, 1 = matrix (MFMA) path."""
    ncols, nnzw = int(ncols), int(nnzw)
    if ncols == 0:
        return 0
    if mode == ROUTE_ALL_CSR:
        return 0
    if mode == ROUTE_ALL_MFMA:
        return 1
    c0, c1, c2 = (int(c) for c in coef[:3])
    z = c0 * H * ncols * ncols + c1 * (H * ncols - nnzw) + c2 * H * ncols
    return 1 if z < 0 else 0


def launch_guard(route: np.ndarray, ncols: np.ndarray, nnzw: np.ndarray) -> np.ndarray:
    """Step 4b: returns the routes after the launch guard (integer arithmetic only)."""
    route = np.asarray(route).astype(np.uint8).copy()
    total = int(np.asarray(nnzw, dtype=np.int64).sum())
    on_matrix = int(np.asarray(nnzw, dtype=np.int64)[route == 1].sum())
    on_scalar = total - on_matrix
    if on_matrix > 0 and on_scalar > 0:
        if on_matrix < GUARD_NNZ and GUARD_SHARE * on_matrix < total:
            route[:] = 0
        elif on_scalar < GUARD_NNZ and GUARD_SHARE * on_scalar < total:
            route = (np.asarray(ncols) > 0).astype(np.uint8)
    return route


def derive_window(w: int, rowptr: np.ndarray, colind: np.ndarray, H: int = 16):
    """(wcols_w, ecol of the window's non-zeros in CSR order, nnzw) for window ``w``."""
    n = rowptr.shape[0] - 1
    s = int(rowptr[min(H * w, n)])
    e = int(rowptr[min(H * w + H, n)])
    sl = np.asarray(colind[s:e], dtype=np.int64)
    wcols = np.unique(sl)
    ecol = np.searchsorted(wcols, sl)
    return wcols.astype(np.int32), ecol.astype(np.int32), e - s


def derive_plan(rowptr: np.ndarray, colind: np.ndarray, coef: Sequence[int], H: int = 16,
                mode: int = ROUTE_HYBRID) -> Dict[str, np.ndarray]:
    """Window-by-window derivation (the reference reading; slow, for small inputs)."""
    rowptr = np.asarray(rowptr)
    n = rowptr.shape[0] - 1
    nnz = int(rowptr[-1])
    W = (n + H - 1) // H
    ncols = np.zeros(W, dtype=np.int32)
    nnzw = np.zeros(W, dtype=np.int32)
    route = np.zeros(W, dtype=np.uint8)
    wptr = np.zeros(W + 1, dtype=np.int64)
    wcols_parts = []
    ecol = np.zeros(nnz, dtype=np.int32)
    for w in range(W):
        wc, ec, cnt = derive_window(w, rowptr, colind, H)
        s = int(rowptr[min(H * w, n)])
        ecol[s:s + cnt] = ec
        ncols[w] = wc.shape[0]
        nnzw[w] = cnt
        wptr[w + 1] = wptr[w] + wc.shape[0]
        wcols_parts.append(wc)
        route[w] = select_route(wc.shape[0], cnt, coef, H, mode)
    if mode == ROUTE_HYBRID:
        route = launch_guard(route, ncols, nnzw)
    wcols = np.concatenate(wcols_parts).astype(np.int32) if wcols_parts else np.zeros(0, dtype=np.int32)
    ids = np.arange(W, dtype=np.int32)
    return dict(H=H, W=W, ncols=ncols, nnzw=nnzw, route=route, wptr=wptr, wcols=wcols, ecol=ecol,
                mfma_windows=ids[route == 1], csr_windows=ids[route == 0])


def derive_plan_vectorised(rowptr: np.ndarray, colind: np.ndarray, coef: Sequence[int], H: int = 16,
                           mode: int = ROUTE_HYBRID, n_cols: int = None) -> Dict[str, np.ndarray]:
    """Same result as :func:`derive_plan` in whole-array numpy operations (for large inputs)."""
    rowptr = np.asarray(rowptr).astype(np.int64)
    colind = np.asarray(colind).astype(np.int64)
    n = rowptr.shape[0] - 1
    W = (n + H - 1) // H
    if n_cols is None:
        n_cols = int(colind.max()) + 1 if colind.size else 1
    bounds = rowptr[np.minimum(np.arange(W + 1, dtype=np.int64) * H, n)]
    nnzw = np.diff(bounds)
    win_of_edge = np.repeat(np.arange(W, dtype=np.int64), nnzw)
    uniq, inv = np.unique(win_of_edge * n_cols + colind, return_inverse=True)
    ncols = np.bincount(uniq // n_cols, minlength=W).astype(np.int64)
    wptr = np.zeros(W + 1, dtype=np.int64)
    np.cumsum(ncols, out=wptr[1:])
    ecol = inv.reshape(-1) - wptr[win_of_edge]
    wcols = uniq % n_cols
    if mode == ROUTE_ALL_CSR:
        route = np.zeros(W, dtype=np.uint8)
    elif mode == ROUTE_ALL_MFMA:
        route = (ncols > 0).astype(np.uint8)
    else:
        c0, c1, c2 = (int(c) for c in coef[:3])
        # exact: Python-int arithmetic through object arrays would be slow; int64 is
        # enough while |c0|*H*ncols^2 < 2^63, which the assert checks
        assert abs(c0) * H * int(ncols.max(initial=0)) ** 2 < 2 ** 62
        assert (abs(c1) + abs(c2)) * H * int(max(ncols.max(initial=0), nnzw.max(initial=0))) < 2 ** 62
        z = c0 * H * ncols * ncols + c1 * (H * ncols - nnzw) + c2 * H * ncols
        route = ((z < 0) & (ncols > 0)).astype(np.uint8)
        if mode == ROUTE_HYBRID:
            route = launch_guard(route, ncols, nnzw)
    ids = np.arange(W, dtype=np.int32)
    return dict(H=H, W=W, ncols=ncols.astype(np.int32), nnzw=nnzw.astype(np.int32), route=route, wptr=wptr,
                wcols=wcols.astype(np.int32), ecol=ecol.astype(np.int32),
                mfma_windows=ids[route == 1], csr_windows=ids[route == 0])


def derive_runs(mfma_windows: Sequence[int], wptr: np.ndarray, wcols: np.ndarray, run_windows: int = RUN_WINDOWS):
    """Step 6: per run of ``run_windows`` consecutive entries of the matrix path's window list, the ascending
    union of the windows' column lists and, per window, the position of each of its columns in that union.

    Returns a list of dicts {first, windows, union, slots} with ``slots[i][k]`` = position of column k of
    window ``windows[i]`` in ``union``; plain Python set/sort per run."""
    out = []
    lst = [int(w) for w in mfma_windows]
    for first in range(0, len(lst), run_windows):
        wins = lst[first:first + run_windows]
        lists = [[int(c) for c in wcols[int(wptr[w]):int(wptr[w + 1])]] for w in wins]
        union = sorted(set(c for l in lists for c in l))
        pos = {c: i for i, c in enumerate(union)}
        out.append(dict(first=first, windows=wins, union=np.array(union, dtype=np.int64),
                        slots=[np.array([pos[c] for c in l], dtype=np.int64) for l in lists]))
    return out
