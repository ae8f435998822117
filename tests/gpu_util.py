"""Helpers shared by the GPU parity tests (argument plumbing and the error criterion only)."""
import numpy as np

import oracle


def device_graph(g):
    import torch
    dev = torch.device("cuda:0")
    return (torch.from_numpy(np.ascontiguousarray(g.rowptr)).to(dev),
            torch.from_numpy(np.ascontiguousarray(g.colind)).to(dev),
            torch.from_numpy(np.ascontiguousarray(g.vals)).to(dev))


def gpu_spmm(g, X, mode, d_hint=None, sel_coef=None, pad_x=0, pad_y=0, dev_graph=None, x_bits=None, mfma_dtype=0):
    """Run prepare + spmm on the GPU through the C ABI; returns (Y numpy, plan info dict).

    x_bits = "bf16" / "f16": X is a uint16 array of bit patterns and is handed over as that 16-bit type."""
    import torch
    import paper_2412_08902_amd.binding as hc
    dev = torch.device("cuda:0")
    rp, ci, va = dev_graph if dev_graph is not None else device_graph(g)
    d = X.shape[1]
    if x_bits is None:
        Xd_full = torch.full((X.shape[0], d + pad_x), float("nan"), dtype=torch.float32, device=dev)
        Xd_full[:, :d] = torch.from_numpy(X).to(dev)
    else:
        tdt = torch.bfloat16 if x_bits == "bf16" else torch.float16
        Xd_full = torch.full((X.shape[0], d + pad_x), float("nan"), dtype=tdt, device=dev)
        Xd_full[:, :d] = torch.from_numpy(X.view(np.int16)).to(dev).view(tdt)
    Yd_full = torch.full((g.n_rows, d + pad_y), -777.0, dtype=torch.float32, device=dev)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode,
                             d_hint=d if d_hint is None else d_hint, sel_coef=sel_coef, mfma_dtype=mfma_dtype)
    info = hc.hcspmm_plan_info(plan)
    hc.hcspmm_spmm(plan, Xd_full, Yd_full, d=d)
    torch.cuda.synchronize()
    Y = Yd_full.cpu().numpy()
    plan.destroy()
    if pad_y:
        assert np.all(Y[:, d:] == -777.0), "wrote outside the d output columns"
    return Y[:, :d].astype(np.float64), info


def assert_close(Y, ref, bound, tol, what=""):
    """Componentwise criterion |Y - ref| <= tol * (|A| |X|): relative to the magnitude of the summed terms."""
    err = np.abs(Y - ref)
    lim = tol * bound
    bad = err > lim
    if bad.any():
        i, j = np.unravel_index(np.argmax(err - lim), err.shape)
        raise AssertionError("%s: %d entries beyond %g * bound; worst at (%d, %d): got %r want %r bound %r"
                             % (what, int(bad.sum()), tol, i, j, Y[i, j], ref[i, j], bound[i, j]))
    assert np.isfinite(Y).all(), what + ": non-finite output"
    if tol <= 1e-4:
        # fp32 paths: where the sum does not cancel (|ref| >= bound / 10) the plain relative error is well-posed
        # and must meet the same tolerance
        well = np.abs(ref) >= 0.1 * bound
        rel_bad = well & (err > tol * np.abs(ref))
        if rel_bad.any():
            i, j = np.argwhere(rel_bad)[0]
            raise AssertionError("%s: relative error beyond %g at (%d, %d): got %r want %r"
                                 % (what, tol, i, j, Y[i, j], ref[i, j]))


def oracle_pair(g, X, rows=None, x_dtype=None):
    ref = oracle.spmm_rows(rows, g.rowptr, g.colind, g.vals, X, x_dtype)
    bound = oracle.spmm_rows(rows, g.rowptr, g.colind, g.vals, X, x_dtype, use_abs=True)
    return ref, bound
