"""Sanity of the seeded input generators (structure only; no SpMM arithmetic here)."""
import numpy as np

from workloads import make_config, CONFIGS, sbm_graph, random_relabel, chung_lu_graph


def _check_csr(g, symmetric=True):
    assert g.rowptr[0] == 0 and g.rowptr[-1] == g.colind.shape[0] == g.vals.shape[0]
    assert np.all(np.diff(g.rowptr) >= 0)
    assert g.colind.min() >= 0 and g.colind.max() < g.n_cols
    rows = np.repeat(np.arange(g.n_rows), np.diff(g.rowptr))
    key = rows.astype(np.int64) * g.n_cols + g.colind
    assert np.all(np.diff(key) > 0)                       # rows ascending, no duplicates
    if symmetric:
        tkey = np.sort(g.colind.astype(np.int64) * g.n_cols + rows)
        assert np.array_equal(tkey, key)


def test_config1_exact_counts_and_determinism():
    g, X, _ = make_config("C1")
    assert g.n_rows == 2708 and g.nnz == 10556 + 2708
    _check_csr(g)
    assert np.all(g.vals == 1.0) and X.shape == (2708, 32) and X.dtype == np.float32
    assert np.abs(X).max() <= 1.0
    g2, X2, _ = make_config("C1")
    assert np.array_equal(g.colind, g2.colind) and np.array_equal(X, X2)
    rows = np.repeat(np.arange(g.n_rows), np.diff(g.rowptr))
    assert np.count_nonzero(rows == g.colind) == 2708      # one self-loop per node
    deg = np.diff(g.rowptr)
    assert deg[:64].mean() > 4 * deg[-1024:].mean()        # ids in descending expected degree


def test_scaled_config2_is_gcn_normalised():
    g, X, _ = make_config("C2", scale=0.02)
    _check_csr(g)
    deg = np.diff(g.rowptr).astype(np.float64)
    rows = np.repeat(np.arange(g.n_rows), np.diff(g.rowptr))
    np.testing.assert_allclose(g.vals, 1.0 / np.sqrt(deg[rows] * deg[g.colind]), rtol=1e-6)
    assert X.shape[1] == CONFIGS["C2"]["d"]


def test_sbm_structure():
    g = sbm_graph(32, 64, 0.25, 4.0, seed=5)
    _check_csr(g)
    rows = np.repeat(np.arange(g.n_rows), np.diff(g.rowptr))
    assert not np.any(rows == g.colind)
    intra = (rows // 64) == (g.colind // 64)
    assert abs(intra.sum() / (32 * 64 * 63 * 0.25) - 1) < 0.1
    assert abs((~intra).sum() / (32 * 64 * 4.0) - 1) < 0.1


def test_random_relabel_keeps_the_graph():
    g = chung_lu_graph(300, 2000, 2.2, seed=3)
    h = random_relabel(g, seed=4)
    _check_csr(h)
    assert h.nnz == g.nnz
    assert sorted(np.diff(h.rowptr).tolist()) == sorted(np.diff(g.rowptr).tolist())


def test_mixed_config_is_a_disjoint_union():
    g, X, _ = make_config("C6", scale=0.02)
    _check_csr(g)
    c = CONFIGS["C6"]
    n_comm = max(2, int(round(c["n_blocks"] * 0.02))) * c["block"]
    rows = np.repeat(np.arange(g.n_rows), np.diff(g.rowptr))
    assert g.n_rows > n_comm and X.shape == (g.n_rows, c["d"])
    assert np.all((rows < n_comm) == (g.colind < n_comm))                 # no entry joins the two parts
    deg = np.diff(g.rowptr)
    assert deg[:n_comm].mean() > 3 * deg[n_comm:].mean()                  # dense communities, sparse power-law part
    assert not np.any((rows == g.colind) & (rows < n_comm))               # block model: no self-loops
    assert np.count_nonzero((rows == g.colind) & (rows >= n_comm)) == g.n_rows - n_comm
    np.testing.assert_allclose(g.vals, 1.0 / np.sqrt(deg[rows].astype(np.float64) * deg[g.colind]), rtol=1e-6)
