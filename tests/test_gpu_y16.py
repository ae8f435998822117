"""16-bit outputs: Y stored as bf16 / fp16 with one rounding of the fp32 result (hcspmm_spmm, hcspmm_gcn_layer_ex,
hcspmm_aggregate_update), and a chain of layers whose activations stay 16-bit with no conversion pass in between."""
import numpy as np
import pytest

import oracle
from workloads import (tiny_random_csr, make_config, dense_normal, glorot_uniform, chung_lu_graph, gcn_normalise,
                       to_bf16_bits, to_f16_bits, bf16_bits_to_f32)
from gpu_util import assert_close, device_graph

pytestmark = pytest.mark.gpu
U = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11}          # unit roundoff of the output type (half an ulp, relative)
TINY = {"bf16": 0.0, "f16": 2.0 ** -25}             # half the smallest fp16 subnormal: absolute floor of the rounding error


def widen(bits, kind):
    return (bf16_bits_to_f32(bits) if kind == "bf16" else bits.view(np.float16)).astype(np.float64)


def torch_16(kind):
    import torch
    return torch.bfloat16 if kind == "bf16" else torch.float16


def to_dev_16(bits, kind):
    import torch
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch_16(kind))


def from_dev_16(t):
    return t.view(__import__("torch").int16).cpu().numpy().view(np.uint16)


def close_16(Y, ref, bound, tol, kind, what):
    """|Y - ref| <= (tol + u) * bound (+ the fp16 subnormal floor): the path's own gate plus one output rounding."""
    assert_close(Y, ref, bound + TINY[kind] / (tol + U[kind]), tol + U[kind], what)


@pytest.mark.parametrize("ykind", ["bf16", "f16"])
@pytest.mark.parametrize("xkind", ["f32", "bf16"])
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("d", [4, 8, 20, 32, 64, 128, 136, 300])
def test_spmm_with_16bit_output(mode, d, xkind, ykind):
    import torch
    import paper_2412_08902_amd.binding as hc
    g = gcn_normalise(chung_lu_graph(1500, 60000, 2.0, seed=31, max_degree=1400))     # all row tiers, wide windows
    X = dense_normal(g.n_cols, d, seed=32 + d)
    rp, ci, va = device_graph(g)
    if xkind == "f32":
        Xd, x_or, code, tol = torch.from_numpy(X).cuda(), X, None, 1e-5
    else:
        bits = to_bf16_bits(X)
        Xd, x_or, code, tol = to_dev_16(bits, "bf16"), bits, oracle.DT_BF16, (1e-5 if mode == 1 else 2e-2)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=d, mfma_dtype=0 if xkind == "f32" else 1)
    Y = torch.full((g.n_rows, d + 4), 3.0, dtype=torch_16(ykind), device="cuda")
    hc.hcspmm_spmm(plan, Xd, Y[:, :d])
    torch.cuda.synchronize()
    plan.destroy()
    got = widen(from_dev_16(Y.contiguous()), ykind).reshape(g.n_rows, d + 4)
    assert np.all(got[:, d:] == 3.0), "wrote outside the d output columns"
    ref = oracle.spmm(g.rowptr, g.colind, g.vals, x_or, code)
    bound = oracle.spmm(g.rowptr, g.colind, g.vals, x_or, code, use_abs=True)
    close_16(got[:, :d], ref, bound, tol, ykind, "spmm y=%s x=%s mode=%d d=%d" % (ykind, xkind, mode, d))


@pytest.mark.parametrize("ykind", ["bf16", "f16"])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_exact_integer_case_is_bit_exact_in_16_bits(mode, ykind):
    """0/1 matrix, integer X in [-8, 8], row sums below 256 in magnitude: every result is an integer that both 16-bit
    types hold exactly, so the stored bits must equal the oracle's rounded bits on every path."""
    import torch
    import paper_2412_08902_amd.binding as hc
    g = tiny_random_csr(200, 333, 0.05, seed=5, integer_values=True)
    g.vals[:] = 1.0
    rng = np.random.default_rng(6)
    X = rng.integers(-8, 9, size=(333, 40)).astype(np.float32)
    ref = oracle.spmm(g.rowptr, g.colind, g.vals, X)
    assert np.abs(ref).max() < 256
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=40)
    Y = torch.empty((200, 40), dtype=torch_16(ykind), device="cuda")
    hc.hcspmm_spmm(plan, torch.from_numpy(X).cuda(), Y)
    torch.cuda.synchronize()
    plan.destroy()
    want = oracle.round_to_16bit(ref, oracle.DT_BF16 if ykind == "bf16" else oracle.DT_F16)
    got = from_dev_16(Y)
    # +0 and -0 are the same result
    assert np.array_equal(np.where(got == 0x8000, 0, got), np.where(want == 0x8000, 0, want))


@pytest.mark.parametrize("ykind", ["bf16", "f16"])
@pytest.mark.parametrize("fusion", [1, 2])
@pytest.mark.parametrize("mode", [0, 1, 2, 3])
@pytest.mark.parametrize("din,dout", [(32, 48), (64, 64), (128, 32), (80, 20)])
def test_aggregate_update_with_16bit_output(mode, din, dout, fusion, ykind):
    import torch
    import paper_2412_08902_amd.binding as hc
    g = gcn_normalise(chung_lu_graph(3003, 150000, 2.0, seed=171, max_degree=2800))
    X, W = dense_normal(g.n_cols, din, seed=172), glorot_uniform(din, dout, seed=173)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=din,
                             sel_coef=[1, 0, -300] if mode == 3 else None, update_fusion=fusion)
    ws = torch.empty(hc.hcspmm_aggregate_update_workspace_bytes(plan, din, dout), dtype=torch.uint8, device="cuda")
    Y = torch.full((g.n_rows, dout), 3.0, dtype=torch_16(ykind), device="cuda")
    hc.hcspmm_aggregate_update(plan, torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(), Y, ws, apply_relu=(dout % 3 == 0))
    torch.cuda.synchronize()
    plan.destroy()
    got = widen(from_dev_16(Y), ykind)
    ref = oracle.aggregate_update(g.rowptr, g.colind, g.vals, X, W, relu=(dout % 3 == 0))
    bound = oracle.aggregate_update(g.rowptr, g.colind, g.vals, X, W, use_abs=True)
    close_16(got, ref, bound, 1e-5, ykind, "aggregate-update")


@pytest.mark.parametrize("ykind,tkind", [("bf16", "bf16"), ("f16", "f32")])
@pytest.mark.parametrize("mode", [0, 2])
def test_gcn_layer_with_16bit_output(mode, ykind, tkind):
    import torch
    import paper_2412_08902_amd.binding as hc
    g = gcn_normalise(chung_lu_graph(2000, 80000, 2.0, seed=41, max_degree=1500))
    X, W = dense_normal(g.n_cols, 70, seed=42), glorot_uniform(70, 64, seed=43)
    tcode = {"f32": 0, "bf16": 1, "f16": 2}[tkind]
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=64, mfma_dtype=tcode)
    ws = torch.empty(hc.hcspmm_gcn_workspace_bytes(plan, 70, 64), dtype=torch.uint8, device="cuda")
    Y = torch.full((g.n_rows, 64), -3.0, dtype=torch_16(ykind), device="cuda")
    hc.hcspmm_gcn_layer_ex(plan, torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(), Y, ws, t_dtype=tcode)
    torch.cuda.synchronize()
    plan.destroy()
    got = widen(from_dev_16(Y), ykind)
    assert got.min() >= 0.0
    ref = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W, t_dtype=None if tkind == "f32" else tcode)
    bound = oracle.gcn_layer(g.rowptr, g.colind, g.vals, X, W, use_abs=True)
    close_16(got, ref, bound, 1e-5 if tkind == "f32" else 2e-2, ykind, "gcn layer")


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_two_layers_16bit_in_16bit_out_without_a_conversion_pass(mode, kind):
    """H1 = ReLU((A X) W1), out = (A H1) W2 with X, H1 and out all 16-bit: the first layer's output buffer IS the second
    layer's input.  The oracle runs the same chain (fp64 inside a layer, one rounding of its output to the 16-bit type);
    the second layer's gate adds what the first layer's admissible error can contribute."""
    import torch
    import paper_2412_08902_amd.binding as hc
    code = oracle.DT_BF16 if kind == "bf16" else oracle.DT_F16
    g = gcn_normalise(chung_lu_graph(4000, 120000, 2.1, seed=51, max_degree=1800))
    X = dense_normal(g.n_cols, 64, seed=52)
    W1, W2 = glorot_uniform(64, 64, seed=53), glorot_uniform(64, 32, seed=54)
    xb = to_bf16_bits(X) if kind == "bf16" else to_f16_bits(X)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=64, mfma_dtype=1 if kind == "bf16" else 2)
    ws = torch.empty(hc.hcspmm_aggregate_update_workspace_bytes(plan, 64, 64), dtype=torch.uint8, device="cuda")
    H1 = torch.empty((g.n_rows, 64), dtype=torch_16(kind), device="cuda")
    out = torch.empty((g.n_rows, 32), dtype=torch_16(kind), device="cuda")
    hc.hcspmm_aggregate_update(plan, to_dev_16(xb, kind), torch.from_numpy(W1).cuda(), H1, ws)
    hc.hcspmm_aggregate_update(plan, H1, torch.from_numpy(W2).cuda(), out, ws, apply_relu=False)
    torch.cuda.synchronize()
    plan.destroy()
    tol = (1e-5 if mode == 1 else 2e-2)
    a = (g.rowptr, g.colind, g.vals)
    r1 = oracle.aggregate_update(*a, xb, W1, x_dtype=code)
    b1 = oracle.aggregate_update(*a, xb, W1, x_dtype=code, use_abs=True)
    close_16(widen(from_dev_16(H1), kind), r1, b1, tol, kind, "layer 1")
    h1_bits = oracle.round_to_16bit(r1, code)
    r2 = oracle.aggregate_update(*a, h1_bits, W2, relu=False, x_dtype=code)
    b2 = oracle.aggregate_update(*a, h1_bits, W2, x_dtype=code, use_abs=True)
    # what an error of (tol + u) * b1 in the second layer's input can add to its output
    carried = oracle.aggregate_update(*a, np.ascontiguousarray(b1), np.abs(W2), x_dtype=oracle.DT_F64, use_abs=True)
    err = np.abs(widen(from_dev_16(out), kind) - r2)
    lim = (tol + U[kind]) * (b2 + carried) + TINY[kind]
    assert np.all(err <= lim), float((err / (lim + 1e-300)).max())
