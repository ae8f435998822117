"""hcspmm_spmm_noalloc (scratch in the library's fixed device array) against hcspmm_spmm and the oracle.

Runs last in the suite: it is the only test of the entry point whose scratch is shared by every
call on the GPU.
"""
import numpy as np
import pytest

from workloads import CSRGraph, dense_normal
from gpu_util import assert_close, oracle_pair, device_graph

pytestmark = pytest.mark.gpu

ALL_CSR, ALL_MFMA = 1, 2


def hub_graph(n, m, hubs, seed):
    """Short rows plus a few rows long enough to be cut into several segments / several column slices."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(0, 12, size=n)
    for r, l in hubs.items():
        lens[r] = l
    cols = [np.sort(rng.choice(m, size=l, replace=False)) for l in lens]
    rp = np.zeros(n + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    return CSRGraph(n, m, rp, np.concatenate(cols).astype(np.int32),
                    rng.standard_normal(int(lens.sum())).astype(np.float32))


def run_both(g, X, mode):
    import torch
    import paper_2412_08902_amd.binding as hc
    dev = torch.device("cuda:0")
    rp, ci, va = device_graph(g)
    Xd = torch.from_numpy(X).to(dev)
    d = X.shape[1]
    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=d)
    info = hc.hcspmm_plan_info(plan)
    Y0 = torch.full((g.n_rows, d), -3.0, dtype=torch.float32, device=dev)
    Y1 = torch.full((g.n_rows, d), -5.0, dtype=torch.float32, device=dev)
    hc.hcspmm_spmm(plan, Xd, Y0)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    hc.hcspmm_spmm_noalloc(plan, Xd, Y1)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, "device memory was allocated or freed during the call"
    out = Y0.cpu().numpy(), Y1.cpu().numpy(), info
    plan.destroy()
    return out


def check(g, X, mode, what):
    Y0, Y1, info = run_both(g, X, mode)
    assert np.array_equal(Y0, Y1), what + ": the two entry points differ"
    ref, bound = oracle_pair(g, X)
    assert_close(Y1.astype(np.float64), ref, bound, 1e-5, what)
    return info


def test_two_calls_in_a_row_second_one_smaller():
    # first call: rows of 8,000 / 4,500 / 2,049 non-zeros -> 4 + 3 + 2 partial rows on the scalar path, windows of
    # thousands of condensed columns -> several column slices with partial tiles on the matrix path
    big = hub_graph(300, 9000, {0: 8000, 50: 4500, 131: 2049, 299: 700}, seed=41)
    Xb = dense_normal(9000, 40, seed=42)
    # second call: a smaller matrix and a narrower X, so it reuses the front of what the first call left behind
    small = hub_graph(70, 5000, {3: 4100, 40: 2500}, seed=43)
    Xs = dense_normal(5000, 8, seed=44)
    for mode in (ALL_CSR, ALL_MFMA):
        info = check(big, Xb, mode, "first call, mode %d" % mode)
        if mode == ALL_CSR:
            assert info["n_segments"] >= 9 and info["n_long_rows"] >= 3      # the scratch path is really exercised
        else:
            assert info["n_mfma_big"] >= 3
        check(small, Xs, mode, "second call, mode %d" % mode)
    # and once more the large one after the small one
    check(big, Xb, ALL_CSR, "third call")


def test_sizes_beyond_the_static_scratch_are_rejected():
    import torch
    import paper_2412_08902_amd.binding as hc
    dev = torch.device("cuda:0")
    limit = hc.hcspmm_spmm_noalloc_scratch_limit()
    assert limit == 16 << 20
    # two rows of 4,097 entries (duplicates of 8 columns): 3 + 3 partial rows of d floats each
    n_rows, m, per_row = 2, 8, 4097
    rp = np.array([0, per_row, 2 * per_row], np.int32)
    ci = (np.arange(2 * per_row) % m).astype(np.int32)
    g = CSRGraph(n_rows, m, rp, ci, np.ones(2 * per_row, np.float32))
    d = 1 << 20                                     # 6 partial rows x 4 MiB = 24 MiB > 16 MiB
    rpd, cid, vad = device_graph(g)
    plan = hc.hcspmm_prepare(n_rows, m, rpd, cid, vad, route_mode=ALL_CSR, d_hint=d)
    X = torch.ones((m, d), dtype=torch.float32, device=dev)
    Y = torch.empty((n_rows, d), dtype=torch.float32, device=dev)
    with pytest.raises(hc.HcspmmError) as e:
        hc.hcspmm_spmm_noalloc(plan, X, Y)
    assert e.value.status == hc.HCSPMM_EUNSUPPORTED and "static scratch" in str(e.value)
    plan.destroy()
