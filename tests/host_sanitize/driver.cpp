// Host-code sanitizer driver: exercises the library's host-only entry points (layout reformatting, permutation,
// transpose) and the C oracle on random inputs under -fsanitize=address,undefined.  Built and run by
// tests/test_host_sanitize.py; links no GPU code.  Exit status 0 = no sanitizer report and all invariants hold.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "hcspmm.h"

extern "C" {
// the C oracle (oracle/spmm_oracle.c)
void oracle_spmm(int64_t n_sel, const int64_t* rows, const int32_t* rowptr, const int32_t* colind, const float* vals,
                 const void* X, int x_dtype, int64_t ldx, int32_t d, double* Z, int64_t ldz, int use_abs);
void oracle_gemm(int64_t n_sel, const int64_t* rows, const void* X, int x_dtype, int64_t ldx, int32_t k_dim, const void* W,
                 int w_dtype, int64_t ldw, int32_t n_out, double* T, int64_t ldt, int use_abs);
}

// loa.cpp reports errors through this function of the GPU part of the library
namespace hcspmm { void set_error(const char*, ...) {} }

static int fail(const char* what) { std::fprintf(stderr, "FAILED: %s\n", what); return 1; }

int main()
{
    std::mt19937 rng(12345);
    for (int trial = 0; trial < 60; ++trial) {
        const int n = 1 + (int)(rng() % 300);
        const double dens = (trial % 5 == 0) ? 0.0 : 0.002 * (1 + rng() % 40);
        std::vector<int32_t> rp(n + 1, 0), ci;
        std::vector<float> va;
        for (int i = 0; i < n; ++i) {
            for (int j = 0; j < n; ++j)
                if ((rng() % 100000) < dens * 100000) { ci.push_back(j); va.push_back((float)(rng() % 17) - 8.f); }
            rp[i + 1] = (int32_t)ci.size();
        }
        const int64_t nnz = (int64_t)ci.size();
        // layout reformatting: the order is a permutation
        for (int vw : {0, 3, 64, 1000}) {
            std::vector<int32_t> order(n, -1);
            if (hcspmm_loa_order(n, n, rp.data(), ci.data(), vw, 16, order.data()) != HCSPMM_OK) return fail("loa_order status");
            std::vector<char> seen(n, 0);
            for (int v : order) { if (v < 0 || v >= n || seen[v]) return fail("loa_order is not a permutation"); seen[v] = 1; }
            // P A P^T keeps the number of entries and, applied with the inverse order, restores A
            std::vector<int32_t> rp2(n + 1), ci2(nnz ? nnz : 1), inv(n);
            std::vector<float> va2(nnz ? nnz : 1);
            if (hcspmm_permute_csr(n, rp.data(), ci.data(), va.data(), order.data(), rp2.data(), ci2.data(), va2.data()) != HCSPMM_OK)
                return fail("permute_csr status");
            if (rp2[n] != nnz) return fail("permute_csr lost entries");
            for (int i = 0; i < n; ++i) inv[order[i]] = i;
            std::vector<int32_t> rp3(n + 1), ci3(nnz ? nnz : 1);
            std::vector<float> va3(nnz ? nnz : 1);
            if (hcspmm_permute_csr(n, rp2.data(), ci2.data(), va2.data(), inv.data(), rp3.data(), ci3.data(), va3.data()) != HCSPMM_OK)
                return fail("permute_csr status (inverse)");
            for (int i = 0; i <= n; ++i) if (rp3[i] != rp[i]) return fail("permutation round trip: rowptr");
            for (int64_t k = 0; k < nnz; ++k) if (ci3[k] != ci[k] || va3[k] != va[k]) return fail("permutation round trip: entries");
        }
        // transpose twice restores the matrix (rows are generated with ascending columns)
        std::vector<int32_t> trp(n + 1), tci(nnz ? nnz : 1), rrp(n + 1), rci(nnz ? nnz : 1);
        std::vector<float> tva(nnz ? nnz : 1), rva(nnz ? nnz : 1);
        if (hcspmm_transpose_csr(n, n, rp.data(), ci.data(), va.data(), trp.data(), tci.data(), tva.data()) != HCSPMM_OK) return fail("transpose status");
        if (hcspmm_transpose_csr(n, n, trp.data(), tci.data(), tva.data(), rrp.data(), rci.data(), rva.data()) != HCSPMM_OK) return fail("transpose status 2");
        for (int i = 0; i <= n; ++i) if (rrp[i] != rp[i]) return fail("transpose round trip: rowptr");
        for (int64_t k = 0; k < nnz; ++k) if (rci[k] != ci[k] || rva[k] != va[k]) return fail("transpose round trip: entries");
        // the C oracle: A X with X = 1 gives the row sums; a row subset gives the same rows
        const int d = 1 + (int)(rng() % 9);
        std::vector<float> X((size_t)n * d, 1.f);
        std::vector<double> Y((size_t)n * d, -1.0);
        oracle_spmm(n, nullptr, rp.data(), ci.data(), va.data(), X.data(), 0, d, d, Y.data(), d, 0);
        for (int i = 0; i < n; ++i) {
            double sum = 0;
            for (int k = rp[i]; k < rp[i + 1]; ++k) sum += va[k];
            for (int j = 0; j < d; ++j) if (Y[(size_t)i * d + j] != sum) return fail("oracle row sums");
        }
        std::vector<int64_t> rows = {0, n - 1};
        std::vector<double> Ys(2 * (size_t)d, -1.0);
        oracle_spmm(2, rows.data(), rp.data(), ci.data(), va.data(), X.data(), 0, d, d, Ys.data(), d, 1);
        std::vector<double> T((size_t)n * 3, 0.0);
        std::vector<float> Wm((size_t)d * 3, 0.5f);
        oracle_gemm(n, nullptr, X.data(), 0, d, d, Wm.data(), 0, 3, 3, T.data(), 3, 0);
        for (int i = 0; i < n; ++i) if (T[(size_t)i * 3] != 0.5 * d) return fail("oracle gemm");
    }
    // error paths of the host entry points
    {
        int32_t rp_bad[3] = {0, 2, 1}, ci_bad[2] = {0, 5}, order[2];
        if (hcspmm_loa_order(2, 2, rp_bad, ci_bad, 4, 16, order) != HCSPMM_EBADCSR) return fail("bad CSR accepted");
        if (hcspmm_loa_order(2, 2, nullptr, ci_bad, 4, 16, order) == HCSPMM_OK) return fail("NULL accepted");
    }
    std::puts("host sanitize driver: ok");
    return 0;
}
