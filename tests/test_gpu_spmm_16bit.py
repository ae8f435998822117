"""GPU parity with X in bf16 / fp16: the oracle reads the same 16-bit patterns (widened exactly);
the matrix path multiplies 16-bit operands with fp32 accumulation (gate 2e-2 of |A||X|), the scalar
path widens X to fp32 (gate 1e-5)."""
import numpy as np
import pytest

import oracle
from workloads import (tiny_random_csr, make_config, dense_normal, to_bf16_bits, to_f16_bits, CSRGraph, sbm_graph)
from gpu_util import gpu_spmm, assert_close

pytestmark = pytest.mark.gpu
HYBRID, ALL_CSR, ALL_MFMA = 0, 1, 2
TOL_16 = 2e-2
TOL_F32 = 1e-5
KINDS = [("bf16", to_bf16_bits, oracle.DT_BF16, 1), ("f16", to_f16_bits, oracle.DT_F16, 2)]


def pair(g, Xb, code):
    ref = oracle.spmm(g.rowptr, g.colind, g.vals, Xb, code)
    bound = oracle.spmm(g.rowptr, g.colind, g.vals, Xb, code, use_abs=True)
    return ref, bound


@pytest.mark.parametrize("kind", KINDS, ids=[k[0] for k in KINDS])
@pytest.mark.parametrize("mode", [HYBRID, ALL_CSR, ALL_MFMA])
@pytest.mark.parametrize("d", [4, 8, 32, 64, 72, 128, 192, 256, 320])
def test_small_random(kind, mode, d):
    name, conv, code, dt = kind
    g = tiny_random_csr(83, 70, 0.15, seed=300 + d)
    Xb = conv(dense_normal(70, d, seed=400 + d))
    Y, _ = gpu_spmm(g, Xb, mode, x_bits=name, mfma_dtype=dt, pad_x=4 * (d % 3), pad_y=4 * (d % 2))
    ref, bound = pair(g, Xb, code)
    assert_close(Y, ref, bound, TOL_F32 if mode == ALL_CSR else TOL_16, "%s d=%d mode=%d" % (name, d, mode))


@pytest.mark.parametrize("kind", KINDS, ids=[k[0] for k in KINDS])
def test_scalar_path_handles_any_width(kind):
    name, conv, code, dt = kind
    g = tiny_random_csr(50, 40, 0.2, seed=9)
    for d in (1, 3, 10, 33):
        Xb = conv(dense_normal(40, d, seed=d))
        Y, _ = gpu_spmm(g, Xb, ALL_CSR, x_bits=name, mfma_dtype=dt)
        ref, bound = pair(g, Xb, code)
        assert_close(Y, ref, bound, TOL_F32)


@pytest.mark.parametrize("kind", KINDS, ids=[k[0] for k in KINDS])
@pytest.mark.parametrize("mode", [ALL_CSR, ALL_MFMA])
def test_exact_small_integers(kind, mode):
    # A in {-3..3}, X integers in [-8, 8]: every product and partial sum is exact in 16-bit inputs / fp32 sums
    name, conv, code, dt = kind
    g = tiny_random_csr(120, 200, 0.1, seed=5, integer_values=True)
    X = np.random.default_rng(6).integers(-8, 9, size=(200, 64)).astype(np.float32)
    Xb = conv(X)
    Y, _ = gpu_spmm(g, Xb, mode, x_bits=name, mfma_dtype=dt)
    ref, _ = pair(g, Xb, code)
    assert np.array_equal(Y, ref)


@pytest.mark.parametrize("kind", KINDS, ids=[k[0] for k in KINDS])
@pytest.mark.parametrize("mode", [HYBRID, ALL_CSR, ALL_MFMA])
def test_wide_and_long(kind, mode):
    name, conv, code, dt = kind
    n, m = 64, 9000
    rng = np.random.default_rng(12)
    lens = np.full(n, 5)
    lens[[0, 17, 18, 50]] = [8000, 513, 2049, 4500]
    cols = [np.sort(rng.choice(m, size=l, replace=False)) for l in lens]
    rp = np.zeros(n + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    g = CSRGraph(n, m, rp, np.concatenate(cols).astype(np.int32), rng.standard_normal(int(lens.sum())).astype(np.float32))
    Xb = conv(dense_normal(m, 128, seed=13))
    Y, _ = gpu_spmm(g, Xb, mode, x_bits=name, mfma_dtype=dt)
    ref, bound = pair(g, Xb, code)
    assert_close(Y, ref, bound, TOL_F32 if mode == ALL_CSR else TOL_16)


@pytest.mark.parametrize("mode", [HYBRID, ALL_CSR, ALL_MFMA])
def test_config3_bf16_full_size(mode):
    g, X, _ = make_config("C3")
    Xb = to_bf16_bits(X)
    Y, info = gpu_spmm(g, Xb, mode, x_bits="bf16", mfma_dtype=1)
    ref, bound = pair(g, Xb, oracle.DT_BF16)
    assert_close(Y, ref, bound, TOL_F32 if mode == ALL_CSR else TOL_16, "C3 bf16 mode=%d" % mode)


def test_unsupported_shape_is_a_status_code():
    import torch
    import paper_2412_08902_amd.binding as hc
    from gpu_util import device_graph
    g = tiny_random_csr(40, 30, 0.5, seed=1)
    rp, ci, va = device_graph(g)
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=ALL_MFMA, mfma_dtype=1)
    X = torch.zeros((g.n_cols, 6), device="cuda", dtype=torch.bfloat16)
    Y = torch.zeros((g.n_rows, 6), device="cuda")
    with pytest.raises(hc.HcspmmError) as e:                      # d = 6 has no 16-bit matrix-path kernel
        hc.hcspmm_spmm(plan, X, Y)
    assert e.value.status == hc.HCSPMM_EUNSUPPORTED
    plan.destroy()
