"""ctypes binding of ``libhcspmm.so``: same names as the C entry points, argument marshalling only.

torch is used for device memory and streams; tensors are passed to the library as raw device
pointers.  Nothing here computes anything.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

from ._build import LIB_PATH, build_library

HCSPMM_OK, HCSPMM_EINVAL, HCSPMM_EBADCSR, HCSPMM_EALLOC, HCSPMM_EHIP, HCSPMM_EUNSUPPORTED = range(6)
HCSPMM_F32, HCSPMM_BF16, HCSPMM_F16 = 0, 1, 2
HCSPMM_ROUTE_HYBRID, HCSPMM_ROUTE_ALL_CSR, HCSPMM_ROUTE_ALL_MFMA, HCSPMM_ROUTE_PER_WINDOW = 0, 1, 2, 3
HCSPMM_UPDATE_AUTO, HCSPMM_UPDATE_FUSED, HCSPMM_UPDATE_SPLIT = 0, 1, 2
HCSPMM_MATRIX_AUTO, HCSPMM_MATRIX_PER_WINDOW, HCSPMM_MATRIX_RUNS = 0, 1, 2

EXPORTED_SYMBOLS = [
    "hcspmm_default_options", "hcspmm_default_selector", "hcspmm_prepare", "hcspmm_plan_info",
    "hcspmm_plan_export", "hcspmm_plan_export_runs", "hcspmm_plan_update", "hcspmm_spmm", "hcspmm_spmm_noalloc", "hcspmm_spmm_noalloc_scratch_limit", "hcspmm_spmm_timed", "hcspmm_gcn_layer", "hcspmm_gcn_layer_ex", "hcspmm_gcn_workspace_bytes",
    "hcspmm_aggregate_update", "hcspmm_aggregate_update_workspace_bytes",
    "hcspmm_layer_backward", "hcspmm_layer_backward_workspace_bytes",
    "hcspmm_gemm_f32", "hcspmm_plan_set_update_fusion", "hcspmm_probe_gather", "hcspmm_probe_gather_out_bytes", "hcspmm_loa_order", "hcspmm_loa_order_checked", "hcspmm_permute_csr", "hcspmm_transpose_csr", "hcspmm_plan_destroy", "hcspmm_status_string", "hcspmm_last_error", "hcspmm_version",
]


class HcspmmOptions(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_int32), ("window_rows", ctypes.c_int32), ("route_mode", ctypes.c_int32),
                ("mfma_dtype", ctypes.c_int32), ("d_hint", ctypes.c_int32), ("use_custom_selector", ctypes.c_int32),
                ("sel_coef", ctypes.c_int64 * 3), ("update_fusion", ctypes.c_int32), ("matrix_kernels", ctypes.c_int32)]


class HcspmmPlanInfo(ctypes.Structure):
    _fields_ = [("window_rows", ctypes.c_int32), ("n_rows", ctypes.c_int32), ("n_cols", ctypes.c_int32),
                ("nnz", ctypes.c_int64), ("n_windows", ctypes.c_int32), ("total_ncols", ctypes.c_int64),
                ("n_mfma_windows", ctypes.c_int32), ("n_csr_windows", ctypes.c_int32), ("nnz_mfma", ctypes.c_int64),
                ("route_mode", ctypes.c_int32), ("mfma_dtype", ctypes.c_int32), ("d_hint", ctypes.c_int32),
                ("sel_coef", ctypes.c_int64 * 3), ("device_bytes", ctypes.c_int64),
                ("n_short_rows", ctypes.c_int32), ("n_mid_rows", ctypes.c_int32), ("n_long_rows", ctypes.c_int32), ("n_segments", ctypes.c_int32),
                ("nnz_long", ctypes.c_int64), ("n_mfma_small", ctypes.c_int32), ("n_mfma_big", ctypes.c_int32),
                ("n_runs", ctypes.c_int32), ("n_run_slices", ctypes.c_int32), ("run_union_cols", ctypes.c_int64)]


class HcspmmStageTimes(ctypes.Structure):
    _fields_ = [("ms_total", ctypes.c_float), ("ms_mfma_big", ctypes.c_float), ("ms_mfma_small", ctypes.c_float),
                ("ms_csr", ctypes.c_float), ("ms_csr_reduce", ctypes.c_float)]


class HcspmmError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("hcspmm status %d: %s" % (status, message))
        self.status = status


_lib = None


def load_library(build_if_missing: bool = True) -> ctypes.CDLL:
    """Load libhcspmm.so (building it first only when no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise ImportError("libhcspmm.so is not built (run __graft_entry__.build())")
        build_library()
    # torch ships its own HIP runtime under the same soname; load it first so that this library
    # and torch share one runtime (device pointers and streams cross the boundary)
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.hcspmm_default_options.argtypes = [ctypes.POINTER(HcspmmOptions)]
    lib.hcspmm_default_options.restype = None
    lib.hcspmm_default_selector.argtypes = [i32, i32, i64, ctypes.POINTER(i64)]
    lib.hcspmm_default_selector.restype = ctypes.c_int
    lib.hcspmm_prepare.argtypes = [i32, i32, i64, vp, vp, vp, ctypes.POINTER(HcspmmOptions), vp, ctypes.POINTER(vp)]
    lib.hcspmm_prepare.restype = ctypes.c_int
    lib.hcspmm_plan_info.argtypes = [vp, ctypes.POINTER(HcspmmPlanInfo)]
    lib.hcspmm_plan_info.restype = ctypes.c_int
    lib.hcspmm_plan_export.argtypes = [vp] + [vp] * 8
    lib.hcspmm_plan_export.restype = ctypes.c_int
    lib.hcspmm_plan_update.argtypes = [vp, i64, vp, vp, vp, vp, i32, vp]
    lib.hcspmm_plan_update.restype = ctypes.c_int
    lib.hcspmm_plan_export_runs.argtypes = [vp, vp, vp, vp]
    lib.hcspmm_plan_export_runs.restype = ctypes.c_int
    lib.hcspmm_spmm.argtypes = [vp, vp, i64, i32, i32, vp, i64, i32, vp]
    lib.hcspmm_spmm.restype = ctypes.c_int
    lib.hcspmm_spmm_noalloc.argtypes = [vp, vp, i64, i32, i32, vp, i64, i32, vp]
    lib.hcspmm_spmm_noalloc.restype = ctypes.c_int
    lib.hcspmm_spmm_noalloc_scratch_limit.argtypes = []
    lib.hcspmm_spmm_noalloc_scratch_limit.restype = ctypes.c_size_t
    lib.hcspmm_spmm_timed.argtypes = [vp, vp, i64, i32, i32, vp, i64, i32, vp, ctypes.POINTER(HcspmmStageTimes)]
    lib.hcspmm_spmm_timed.restype = ctypes.c_int
    lib.hcspmm_gcn_layer.argtypes = [vp, vp, i64, i32, vp, i64, i32, vp, i64, i32, vp, ctypes.c_size_t, vp]
    lib.hcspmm_gcn_layer.restype = ctypes.c_int
    lib.hcspmm_gcn_layer_ex.argtypes = [vp, vp, i64, i32, vp, i64, i32, vp, i64, i32, i32, i32, vp, ctypes.c_size_t, vp]
    lib.hcspmm_gcn_layer_ex.restype = ctypes.c_int
    lib.hcspmm_gcn_workspace_bytes.argtypes = [vp, i32, i32]
    lib.hcspmm_gcn_workspace_bytes.restype = ctypes.c_size_t
    lib.hcspmm_aggregate_update.argtypes = [vp, vp, i64, i32, i32, vp, i64, i32, vp, i64, i32, i32, vp, ctypes.c_size_t, vp]
    lib.hcspmm_aggregate_update.restype = ctypes.c_int
    lib.hcspmm_aggregate_update_workspace_bytes.argtypes = [vp, i32, i32]
    lib.hcspmm_aggregate_update_workspace_bytes.restype = ctypes.c_size_t
    lib.hcspmm_layer_backward.argtypes = [vp, vp, i64, i32, vp, i64, vp, i64, i32, vp, i64, vp, i64, vp, i64, i32, vp,
                                          ctypes.c_size_t, vp]
    lib.hcspmm_layer_backward.restype = ctypes.c_int
    lib.hcspmm_layer_backward_workspace_bytes.argtypes = [vp, i32, i32]
    lib.hcspmm_layer_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.hcspmm_loa_order.argtypes = [i32, i32, vp, vp, i32, i32, vp]
    lib.hcspmm_loa_order.restype = ctypes.c_int
    lib.hcspmm_loa_order_checked.argtypes = [i32, i32, vp, vp, i32, i32, vp, vp]
    lib.hcspmm_loa_order_checked.restype = ctypes.c_int
    lib.hcspmm_permute_csr.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp]
    lib.hcspmm_permute_csr.restype = ctypes.c_int
    lib.hcspmm_transpose_csr.argtypes = [i32, i32, vp, vp, vp, vp, vp, vp]
    lib.hcspmm_transpose_csr.restype = ctypes.c_int
    lib.hcspmm_gemm_f32.argtypes = [i64, i32, i32, vp, i64, vp, i64, vp, i64, vp]
    lib.hcspmm_gemm_f32.restype = ctypes.c_int
    lib.hcspmm_probe_gather.argtypes = [vp, i64, vp, i64, i32, i32, vp, ctypes.c_size_t, vp]
    lib.hcspmm_probe_gather.restype = ctypes.c_int
    lib.hcspmm_probe_gather_out_bytes.argtypes = [i64, i32]
    lib.hcspmm_probe_gather_out_bytes.restype = ctypes.c_size_t
    lib.hcspmm_plan_set_update_fusion.argtypes = [vp, i32]
    lib.hcspmm_plan_set_update_fusion.restype = ctypes.c_int
    lib.hcspmm_plan_destroy.argtypes = [vp]
    lib.hcspmm_plan_destroy.restype = None
    lib.hcspmm_status_string.argtypes = [ctypes.c_int]
    lib.hcspmm_status_string.restype = ctypes.c_char_p
    lib.hcspmm_last_error.argtypes = []
    lib.hcspmm_last_error.restype = ctypes.c_char_p
    lib.hcspmm_version.argtypes = []
    lib.hcspmm_version.restype = i32
    _lib = lib
    return lib


def _check(status: int):
    if status != HCSPMM_OK:
        lib = load_library()
        detail = lib.hcspmm_last_error().decode()
        raise HcspmmError(status, "%s: %s" % (lib.hcspmm_status_string(status).decode(), detail))


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream=None):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


_TORCH_DTYPE_CODE = None


def _dtype_code(t) -> int:
    import torch
    return {torch.float32: HCSPMM_F32, torch.bfloat16: HCSPMM_BF16, torch.float16: HCSPMM_F16}[t.dtype]


def hcspmm_default_options() -> HcspmmOptions:
    o = HcspmmOptions()
    load_library().hcspmm_default_options(ctypes.byref(o))
    return o


def hcspmm_default_selector(mfma_dtype: int = HCSPMM_F32, d_hint: int = 0, nnz: int = 0):
    c = (ctypes.c_int64 * 3)()
    _check(load_library().hcspmm_default_selector(mfma_dtype, d_hint, nnz, c))
    return [int(c[0]), int(c[1]), int(c[2])]


class Plan:
    """Owns a ``hcspmm_plan*`` and keeps the borrowed CSR tensors alive."""

    def __init__(self, handle, rowptr, colind, vals):
        self._h = handle
        self._keep = (rowptr, colind, vals)

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("plan was destroyed")
        return self._h

    def destroy(self):
        if self._h is not None:
            load_library().hcspmm_plan_destroy(self._h)
            self._h = None
            self._keep = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def hcspmm_prepare(n_rows: int, n_cols: int, rowptr, colind, vals, *, route_mode: int = HCSPMM_ROUTE_HYBRID,
                   mfma_dtype: int = HCSPMM_F32, d_hint: int = 0, sel_coef: Optional[Sequence[int]] = None,
                   stream=None, nnz: Optional[int] = None, update_fusion: int = HCSPMM_UPDATE_AUTO,
                   matrix_kernels: int = HCSPMM_MATRIX_AUTO) -> Plan:
    """rowptr/colind: int32 CUDA tensors, vals: float32 CUDA tensor (borrowed by the plan)."""
    lib = load_library()
    o = hcspmm_default_options()
    o.route_mode, o.mfma_dtype, o.d_hint, o.update_fusion = route_mode, mfma_dtype, d_hint, update_fusion
    o.matrix_kernels = matrix_kernels
    if sel_coef is not None:
        o.use_custom_selector = 1
        for i in range(3):
            o.sel_coef[i] = int(sel_coef[i])
    if nnz is None:
        nnz = int(colind.numel())
    out = ctypes.c_void_p()
    _check(lib.hcspmm_prepare(n_rows, n_cols, nnz, _ptr(rowptr), _ptr(colind), _ptr(vals), ctypes.byref(o),
                              _stream_ptr(stream), ctypes.byref(out)))
    return Plan(out, rowptr, colind, vals)


def hcspmm_probe_gather_out_bytes(n: int, d: int) -> int:
    return int(load_library().hcspmm_probe_gather_out_bytes(n, d))


def hcspmm_probe_gather(index, X, out, *, d: Optional[int] = None, stream=None):
    """Bare gather of the rows X[index[i]] (measurement aid); index int32 CUDA tensor, out a CUDA buffer."""
    assert X.dim() == 2 and X.stride(1) == 1
    if d is None:
        d = X.shape[1]
    _check(load_library().hcspmm_probe_gather(_ptr(index), index.numel(), _ptr(X), X.stride(0), d, X.shape[0], _ptr(out),
                                              out.numel() * out.element_size(), _stream_ptr(stream)))


def hcspmm_plan_update(plan: Plan, rowptr, colind, vals, changed_rows, *, stream=None, nnz: Optional[int] = None):
    """Re-prepare ``plan`` for new CSR tensors (same shape) given the rows whose entries changed (host int32 array)."""
    rows = np.ascontiguousarray(changed_rows, dtype=np.int32)
    if nnz is None:
        nnz = int(colind.numel())
    _check(load_library().hcspmm_plan_update(plan.handle, nnz, _ptr(rowptr), _ptr(colind), _ptr(vals), _host_ptr(rows),
                                             rows.shape[0], _stream_ptr(stream)))
    plan._keep = (rowptr, colind, vals)


def hcspmm_plan_set_update_fusion(plan: Plan, update_fusion: int):
    _check(load_library().hcspmm_plan_set_update_fusion(plan.handle, update_fusion))


def hcspmm_plan_info(plan: Plan) -> dict:
    info = HcspmmPlanInfo()
    _check(load_library().hcspmm_plan_info(plan.handle, ctypes.byref(info)))
    d = {name: getattr(info, name) for name, _ in HcspmmPlanInfo._fields_ if name != "sel_coef"}
    d["sel_coef"] = [int(info.sel_coef[i]) for i in range(3)]
    return d


def hcspmm_plan_export(plan: Plan, with_ecol: bool = True) -> dict:
    """Canonical plan arrays as numpy arrays (host)."""
    info = hcspmm_plan_info(plan)
    W = info["n_windows"]
    out = dict(H=info["window_rows"], W=W,
               ncols=np.zeros(W, np.int32), nnzw=np.zeros(W, np.int32), route=np.zeros(W, np.uint8),
               wptr=np.zeros(W + 1, np.int64), wcols=np.zeros(info["total_ncols"], np.int32),
               ecol=np.zeros(info["nnz"] if with_ecol else 0, np.int32),
               mfma_windows=np.zeros(info["n_mfma_windows"], np.int32),
               csr_windows=np.zeros(info["n_csr_windows"], np.int32))

    def p(name):
        a = out[name]
        return a.ctypes.data_as(ctypes.c_void_p) if a.size else None

    _check(load_library().hcspmm_plan_export(plan.handle, p("ncols"), p("nnzw"), p("route"),
                                             out["wptr"].ctypes.data_as(ctypes.c_void_p), p("wcols"),
                                             p("ecol") if with_ecol else None, p("mfma_windows"), p("csr_windows")))
    return out


def hcspmm_plan_export_runs(plan: Plan) -> dict:
    """Launch table of the run kernel as numpy arrays (host): run_nu, ucols (concatenated), wslot (indexed like wcols)."""
    info = hcspmm_plan_info(plan)
    out = dict(run_nu=np.zeros(info["n_runs"], np.int32), ucols=np.zeros(info["run_union_cols"], np.int32),
               wslot=np.zeros(info["total_ncols"], np.int32))

    def p(name):
        a = out[name]
        return a.ctypes.data_as(ctypes.c_void_p) if a.size else None

    _check(load_library().hcspmm_plan_export_runs(plan.handle, p("run_nu"), p("ucols"), p("wslot")))
    return out


def hcspmm_spmm(plan: Plan, X, Y, *, d: Optional[int] = None, stream=None):
    """Y[:, :d] = A X[:, :d]; X, Y are 2-D CUDA tensors (row-major, last stride 1)."""
    assert X.dim() == 2 and Y.dim() == 2 and X.stride(1) == 1 and Y.stride(1) == 1
    if d is None:
        d = X.shape[1]
    _check(load_library().hcspmm_spmm(plan.handle, _ptr(X), X.stride(0), d, _dtype_code(X), _ptr(Y), Y.stride(0),
                                      _dtype_code(Y), _stream_ptr(stream)))
    return Y


def hcspmm_spmm_noalloc(plan: Plan, X, Y, *, d: Optional[int] = None, stream=None):
    """hcspmm_spmm with the call's scratch in the library's fixed device array (allocates nothing)."""
    assert X.dim() == 2 and Y.dim() == 2 and X.stride(1) == 1 and Y.stride(1) == 1
    if d is None:
        d = X.shape[1]
    _check(load_library().hcspmm_spmm_noalloc(plan.handle, _ptr(X), X.stride(0), d, _dtype_code(X), _ptr(Y),
                                              Y.stride(0), _dtype_code(Y), _stream_ptr(stream)))
    return Y


def hcspmm_spmm_noalloc_scratch_limit() -> int:
    return int(load_library().hcspmm_spmm_noalloc_scratch_limit())


def hcspmm_spmm_timed(plan: Plan, X, Y, *, d: Optional[int] = None, stream=None) -> dict:
    """hcspmm_spmm with per-stage HIP-event timing; returns the stage times in milliseconds."""
    assert X.dim() == 2 and Y.dim() == 2 and X.stride(1) == 1 and Y.stride(1) == 1
    if d is None:
        d = X.shape[1]
    t = HcspmmStageTimes()
    _check(load_library().hcspmm_spmm_timed(plan.handle, _ptr(X), X.stride(0), d, _dtype_code(X), _ptr(Y),
                                            Y.stride(0), _dtype_code(Y), _stream_ptr(stream), ctypes.byref(t)))
    return {name: float(getattr(t, name)) for name, _ in HcspmmStageTimes._fields_}


def hcspmm_gcn_workspace_bytes(plan: Plan, d_in: int, d_out: int) -> int:
    return int(load_library().hcspmm_gcn_workspace_bytes(plan.handle, d_in, d_out))


def hcspmm_gcn_layer(plan: Plan, X, W, Y, workspace, *, apply_relu: bool = True, stream=None):
    """Y = act(A (X W)), all fp32; workspace: a uint8/float CUDA tensor of at least hcspmm_gcn_workspace_bytes bytes."""
    assert X.stride(1) == 1 and W.stride(1) == 1 and Y.stride(1) == 1 and _dtype_code(Y) == HCSPMM_F32
    _check(load_library().hcspmm_gcn_layer(plan.handle, _ptr(X), X.stride(0), X.shape[1], _ptr(W), W.stride(0),
                                           W.shape[1], _ptr(Y), Y.stride(0), 1 if apply_relu else 0, _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream_ptr(stream)))
    return Y


def hcspmm_aggregate_update_workspace_bytes(plan: Plan, d_in: int, d_out: int) -> int:
    return int(load_library().hcspmm_aggregate_update_workspace_bytes(plan.handle, d_in, d_out))


def hcspmm_aggregate_update(plan: Plan, X, W, Y, workspace, *, apply_relu: bool = True, stream=None):
    """Y = act((A X) W); workspace: a CUDA tensor of at least hcspmm_aggregate_update_workspace_bytes bytes."""
    assert X.stride(1) == 1 and W.stride(1) == 1 and Y.stride(1) == 1
    _check(load_library().hcspmm_aggregate_update(plan.handle, _ptr(X), X.stride(0), X.shape[1], _dtype_code(X),
                                                  _ptr(W), W.stride(0), W.shape[1], _ptr(Y), Y.stride(0), _dtype_code(Y),
                                                  1 if apply_relu else 0, _ptr(workspace),
                                                  workspace.numel() * workspace.element_size(), _stream_ptr(stream)))
    return Y


def hcspmm_layer_backward_workspace_bytes(plan: Plan, d_in: int, d_out: int) -> int:
    return int(load_library().hcspmm_layer_backward_workspace_bytes(plan.handle, d_in, d_out))


def hcspmm_layer_backward(plan: Plan, G, X, W, dX, dW, workspace, *, Y_fwd=None, mask_dx_by_x: bool = False, stream=None):
    """S = A (G masked by Y_fwd > 0), dX = S W^T (stored as 0 where X <= 0 with mask_dx_by_x), dW = X^T S;
    dX or dW may be None (not computed)."""
    assert G.stride(1) == 1 and X.stride(1) == 1 and W.stride(1) == 1
    assert dX is None or dX.stride(1) == 1
    assert dW is None or dW.stride(1) == 1
    assert Y_fwd is None or (Y_fwd.stride(1) == 1 and Y_fwd.shape == G.shape)
    assert W.shape == (X.shape[1], G.shape[1])
    _check(load_library().hcspmm_layer_backward(
        plan.handle, _ptr(G), G.stride(0), G.shape[1],
        _ptr(Y_fwd) if Y_fwd is not None else None, Y_fwd.stride(0) if Y_fwd is not None else 0,
        _ptr(X), X.stride(0), X.shape[1], _ptr(W), W.stride(0),
        _ptr(dX) if dX is not None else None, dX.stride(0) if dX is not None else 0,
        _ptr(dW) if dW is not None else None, dW.stride(0) if dW is not None else 0, 1 if mask_dx_by_x else 0,
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream_ptr(stream)))
    return dX, dW


def hcspmm_gcn_layer_ex(plan: Plan, X, W, Y, workspace, *, t_dtype: int = HCSPMM_F32, apply_relu: bool = True, stream=None):
    """Y = act(A (X W)) with the intermediate X W stored as t_dtype (HCSPMM_F32 / BF16 / F16)."""
    assert X.stride(1) == 1 and W.stride(1) == 1 and Y.stride(1) == 1
    _check(load_library().hcspmm_gcn_layer_ex(plan.handle, _ptr(X), X.stride(0), X.shape[1], _ptr(W), W.stride(0),
                                              W.shape[1], _ptr(Y), Y.stride(0), _dtype_code(Y), 1 if apply_relu else 0, t_dtype,
                                              _ptr(workspace), workspace.numel() * workspace.element_size(),
                                              _stream_ptr(stream)))
    return Y


def hcspmm_gemm_f32(X, W, T, *, stream=None):
    assert X.stride(1) == 1 and W.stride(1) == 1 and T.stride(1) == 1
    _check(load_library().hcspmm_gemm_f32(X.shape[0], X.shape[1], W.shape[1], _ptr(X), X.stride(0), _ptr(W),
                                          W.stride(0), _ptr(T), T.stride(0), _stream_ptr(stream)))
    return T


def _host_ptr(a):
    return ctypes.c_void_p(a.ctypes.data) if a.size else None


def hcspmm_loa_order(n_rows: int, n_cols: int, rowptr, colind, vw: int, window_rows: int = 16):
    """Layout reformatting on the host; rowptr/colind are int32 numpy arrays.  Returns the order (int32 numpy)."""
    import numpy as np
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colind = np.ascontiguousarray(colind, dtype=np.int32)
    assert rowptr.shape[0] == n_rows + 1
    order = np.empty(n_rows, dtype=np.int32)
    _check(load_library().hcspmm_loa_order(n_rows, n_cols, _host_ptr(rowptr), _host_ptr(colind), vw, window_rows,
                                           _host_ptr(order)))
    return order


def hcspmm_loa_order_checked(n_rows: int, n_cols: int, rowptr, colind, vw: int, window_rows: int = 16):
    """hcspmm_loa_order plus (total_ncols before, total_ncols after): apply the order only when the second is smaller."""
    import numpy as np
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colind = np.ascontiguousarray(colind, dtype=np.int32)
    assert rowptr.shape[0] == n_rows + 1
    order = np.empty(n_rows, dtype=np.int32)
    totals = np.zeros(2, dtype=np.int64)
    _check(load_library().hcspmm_loa_order_checked(n_rows, n_cols, _host_ptr(rowptr), _host_ptr(colind), vw, window_rows,
                                                   _host_ptr(order), ctypes.c_void_p(totals.ctypes.data)))
    return order, int(totals[0]), int(totals[1])


def hcspmm_permute_csr(n: int, rowptr, colind, vals, order):
    """P A P^T on the host for the vertex order ``order``; returns (rowptr, colind, vals) numpy arrays."""
    import numpy as np
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colind = np.ascontiguousarray(colind, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    order = np.ascontiguousarray(order, dtype=np.int32)
    assert rowptr.shape[0] == n + 1 and order.shape[0] == n
    out_rp, out_ci, out_va = np.empty_like(rowptr), np.empty_like(colind), np.empty_like(vals)
    _check(load_library().hcspmm_permute_csr(n, _host_ptr(rowptr), _host_ptr(colind), _host_ptr(vals),
                                             _host_ptr(order), _host_ptr(out_rp), _host_ptr(out_ci),
                                             _host_ptr(out_va)))
    return out_rp, out_ci, out_va


def hcspmm_transpose_csr(n_rows: int, n_cols: int, rowptr, colind, vals):
    """A^T on the host (n_cols x n_rows, ascending columns); returns (rowptr, colind, vals) numpy arrays."""
    import numpy as np
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colind = np.ascontiguousarray(colind, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    assert rowptr.shape[0] == n_rows + 1
    out_rp = np.empty(n_cols + 1, dtype=np.int32)
    out_ci, out_va = np.empty_like(colind), np.empty_like(vals)
    _check(load_library().hcspmm_transpose_csr(n_rows, n_cols, _host_ptr(rowptr), _host_ptr(colind), _host_ptr(vals),
                                               _host_ptr(out_rp), _host_ptr(out_ci), _host_ptr(out_va)))
    return out_rp, out_ci, out_va


def hcspmm_version() -> int:
    return int(load_library().hcspmm_version())
