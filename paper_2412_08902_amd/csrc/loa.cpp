// Layout reformatting on the host (Section V-B): the optimised greedy algorithm (Alg. 6) that
// regroups vertices into row windows of higher computing intensity (Eq. 5), scoring a candidate
// with the incremental form (Eq. 6)
//     P(v) = (curEles + |N(v)|) / (curCols + |N(v)| - |N(v) ∩ allCols|).
//
// The intersection counts are kept per position of the vertices window only: a transposed copy
// of the graph, indexed by position in the sorted vertex list, lets a newly covered column bump
// exactly the candidates of the current vertices window (binary search for the window's first
// position, then a linear walk), so hub columns cost their share of the window, not their degree.
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <limits>
#include <new>
#include <numeric>
#include <thread>
#include <vector>

#include "common.hpp"

namespace {

struct Distinct {
    std::vector<int64_t> ptr;     // n + 1
    std::vector<int32_t> col;     // ascending, without repeats, per row
};

// N(v): ascending distinct columns of every row
bool distinct_neighbours(int32_t n_rows, int32_t n_cols, const int32_t* rowptr, const int32_t* colind, Distinct& out)
{
    out.ptr.assign((size_t)n_rows + 1, 0);
    out.col.clear();
    out.col.reserve((size_t)rowptr[n_rows]);
    std::vector<int32_t> tmp;
    for (int32_t v = 0; v < n_rows; ++v) {
        const int32_t s = rowptr[v], e = rowptr[v + 1];
        if (s < 0 || s > e || e > rowptr[n_rows]) return false;
        tmp.assign(colind + s, colind + e);
        for (int32_t c : tmp)
            if (c < 0 || c >= n_cols) return false;
        if (!std::is_sorted(tmp.begin(), tmp.end())) std::sort(tmp.begin(), tmp.end());
        tmp.erase(std::unique(tmp.begin(), tmp.end()), tmp.end());
        out.col.insert(out.col.end(), tmp.begin(), tmp.end());
        out.ptr[(size_t)v + 1] = (int64_t)out.col.size();
    }
    return true;
}

}  // namespace

extern "C" {

hcspmm_status hcspmm_loa_order(int32_t n_rows, int32_t n_cols, const int32_t* h_rowptr, const int32_t* h_colind,
                               int32_t vw, int32_t window_rows, int32_t* h_order)
{
    using hcspmm::set_error;
    if (n_rows < 0 || n_cols < 0) { set_error("n_rows, n_cols must be non-negative"); return HCSPMM_EINVAL; }
    if (vw < 0) { set_error("the vertices window must be non-negative"); return HCSPMM_EINVAL; }
    if (window_rows < 1) { set_error("window_rows must be at least 1"); return HCSPMM_EINVAL; }
    if (n_rows == 0) return HCSPMM_OK;
    if (!h_rowptr || !h_order) { set_error("rowptr or order is NULL"); return HCSPMM_EINVAL; }
    if (h_rowptr[0] != 0 || h_rowptr[n_rows] < 0 || (h_rowptr[n_rows] > 0 && !h_colind)) {
        set_error("invalid CSR: rowptr[0] != 0, negative nnz or colind is NULL");
        return HCSPMM_EBADCSR;
    }
    try {
        const int32_t n = n_rows;
        vw = std::min(vw, n);                               // positions beyond the list do not exist
        Distinct nb;
        if (!distinct_neighbours(n, n_cols, h_rowptr, h_colind, nb)) {
            set_error("invalid CSR: rowptr not monotone or a column index out of range");
            return HCSPMM_EBADCSR;
        }
        auto deg = [&](int32_t v) { return (int32_t)(nb.ptr[(size_t)v + 1] - nb.ptr[v]); };

        // sorted list: ascending smallest neighbour, vertices without neighbours last, stable in the id
        std::vector<int32_t> so((size_t)n);
        std::iota(so.begin(), so.end(), 0);
        std::vector<int32_t> key((size_t)n);
        for (int32_t v = 0; v < n; ++v) key[v] = deg(v) ? nb.col[(size_t)nb.ptr[v]] : std::numeric_limits<int32_t>::max();
        std::stable_sort(so.begin(), so.end(), [&](int32_t a, int32_t b) { return key[a] < key[b]; });

        // transposed graph in position space: for column u the ascending sorted-list positions of the rows holding u
        std::vector<int64_t> tptr((size_t)n_cols + 1, 0);
        for (int32_t c : nb.col) ++tptr[(size_t)c + 1];
        for (int32_t c = 0; c < n_cols; ++c) tptr[(size_t)c + 1] += tptr[c];
        std::vector<int32_t> tpos(nb.col.size());
        {
            std::vector<int64_t> fill(tptr.begin(), tptr.end() - 1);
            for (int32_t j = 0; j < n; ++j) {
                const int32_t v = so[j];
                for (int64_t k = nb.ptr[v]; k < nb.ptr[(size_t)v + 1]; ++k) tpos[(size_t)fill[nb.col[(size_t)k]]++] = j;
            }
        }

        std::vector<uint8_t> visited((size_t)n, 0);         // by position
        std::vector<int32_t> col_stamp((size_t)n_cols, -1);  // window id that last covered the column
        std::vector<int32_t> cns((size_t)vw + 1, 0);
        std::vector<int32_t> resi;
        int32_t first = 0, placed = 0, window_id = 0;

        while (placed < n) {
            while (visited[first]) ++first;
            const int32_t p0 = first;
            const int32_t hi = (int32_t)std::min<int64_t>((int64_t)p0 + vw, (int64_t)n - 1);
            std::fill(cns.begin(), cns.begin() + (hi - p0 + 1), 0);
            const int32_t v0 = so[p0];
            visited[p0] = 1;
            h_order[placed++] = v0;
            int64_t cur_eles = deg(v0), cur_cols = deg(v0);
            resi.assign(nb.col.begin() + nb.ptr[v0], nb.col.begin() + nb.ptr[(size_t)v0 + 1]);
            for (int32_t c : resi) col_stamp[c] = window_id;

            for (int32_t step = 1; step < window_rows && placed < n; ++step) {
                // newly covered columns raise the intersection count of every candidate that holds them
                for (int32_t u : resi) {
                    const int32_t* b = tpos.data() + tptr[u];
                    const int32_t* e = tpos.data() + tptr[(size_t)u + 1];
                    for (const int32_t* p = std::lower_bound(b, e, p0); p != e && *p <= hi; ++p) ++cns[*p - p0];
                }
                int32_t best = -1;
                int64_t best_num = 0, best_den = 1;
                int32_t best_deg = 0;
                for (int32_t j = p0 + 1; j <= hi; ++j) {
                    if (visited[j]) continue;
                    const int32_t dv = deg(so[j]);
                    int64_t num = cur_eles + dv, den = cur_cols + dv - cns[j - p0];
                    if (den == 0) { num = 0; den = 1; }          // nothing covered, nothing added
                    // P > maxP, ties to the higher degree, then to the earlier position (ascending scan)
                    const __int128 lhs = (__int128)num * best_den, rhs = (__int128)best_num * den;
                    if (best < 0 || lhs > rhs || (lhs == rhs && dv > best_deg)) {
                        best = j; best_num = num; best_den = den; best_deg = dv;
                    }
                }
                if (best < 0) {                                    // vertices window exhausted
                    best = hi + 1;
                    while (visited[best]) ++best;
                }
                const int32_t v = so[best];
                visited[best] = 1;
                h_order[placed++] = v;
                resi.clear();
                for (int64_t k = nb.ptr[v]; k < nb.ptr[(size_t)v + 1]; ++k) {
                    const int32_t c = nb.col[(size_t)k];
                    if (col_stamp[c] != window_id) { col_stamp[c] = window_id; resi.push_back(c); }
                }
                cur_eles += deg(v);
                cur_cols += (int64_t)resi.size();
            }
            ++window_id;
        }
    } catch (const std::bad_alloc&) {
        set_error("host allocation failed in layout reformatting");
        return HCSPMM_EALLOC;
    }
    return HCSPMM_OK;
}

// Sum over the row windows of the number of distinct columns, for the rows grouped as `order` lists them (NULL: as
// stored).  The windows are independent: worker threads take contiguous ranges of windows, each with its own stamp
// array over the columns.
static int64_t total_window_columns(int32_t n_rows, int32_t n_cols, const int32_t* rowptr, const int32_t* colind,
                                    const int32_t* order, int32_t window_rows)
{
    const int64_t n_win = ((int64_t)n_rows + window_rows - 1) / window_rows;
    unsigned n_thr = std::thread::hardware_concurrency();
    if (n_thr < 1) n_thr = 1;
    if (n_thr > 16) n_thr = 16;
    if ((int64_t)n_thr > n_win) n_thr = (unsigned)(n_win > 0 ? n_win : 1);
    std::vector<int64_t> part(n_thr, 0);
    auto work = [&](unsigned t) {
        std::vector<int32_t> stamp((size_t)n_cols, -1);
        const int64_t w0 = n_win * t / n_thr, w1 = n_win * (t + 1) / n_thr;
        int64_t sum = 0;
        for (int64_t w = w0; w < w1; ++w) {
            const int64_t r1 = std::min<int64_t>((w + 1) * window_rows, n_rows);
            for (int64_t i = w * window_rows; i < r1; ++i) {
                const int32_t v = order ? order[i] : (int32_t)i;
                for (int32_t k = rowptr[v]; k < rowptr[v + 1]; ++k) {
                    const int32_t c = colind[k];
                    if (stamp[c] != (int32_t)w) { stamp[c] = (int32_t)w; ++sum; }
                }
            }
        }
        part[t] = sum;
    };
    std::vector<std::thread> pool;
    for (unsigned t = 1; t < n_thr; ++t) pool.emplace_back(work, t);
    work(0);
    for (std::thread& th : pool) th.join();
    int64_t total = 0;
    for (int64_t v : part) total += v;
    return total;
}

hcspmm_status hcspmm_loa_order_checked(int32_t n_rows, int32_t n_cols, const int32_t* h_rowptr, const int32_t* h_colind,
                                       int32_t vw, int32_t window_rows, int32_t* h_order, int64_t* h_total_ncols)
{
    const hcspmm_status st = hcspmm_loa_order(n_rows, n_cols, h_rowptr, h_colind, vw, window_rows, h_order);
    if (st != HCSPMM_OK) return st;
    if (!h_total_ncols) { hcspmm::set_error("h_total_ncols is NULL"); return HCSPMM_EINVAL; }
    h_total_ncols[0] = h_total_ncols[1] = 0;
    if (n_rows == 0) return HCSPMM_OK;
    try {
        // hcspmm_loa_order has validated the arrays
        h_total_ncols[0] = total_window_columns(n_rows, n_cols, h_rowptr, h_colind, nullptr, window_rows);
        h_total_ncols[1] = total_window_columns(n_rows, n_cols, h_rowptr, h_colind, h_order, window_rows);
    } catch (const std::exception&) {
        hcspmm::set_error("host allocation or thread start failed while evaluating the layout");
        return HCSPMM_EALLOC;
    }
    return HCSPMM_OK;
}

hcspmm_status hcspmm_permute_csr(int32_t n, const int32_t* h_rowptr, const int32_t* h_colind, const float* h_vals,
                                 const int32_t* h_order, int32_t* h_out_rowptr, int32_t* h_out_colind,
                                 float* h_out_vals)
{
    using hcspmm::set_error;
    if (n < 0) { set_error("n must be non-negative"); return HCSPMM_EINVAL; }
    if (!h_rowptr || !h_out_rowptr || (n > 0 && !h_order)) { set_error("rowptr, out_rowptr or order is NULL"); return HCSPMM_EINVAL; }
    try {
        std::vector<int32_t> new_of_old((size_t)n, -1);
        for (int32_t i = 0; i < n; ++i) {
            const int32_t o = h_order[i];
            if (o < 0 || o >= n || new_of_old[o] != -1) { set_error("order is not a permutation of 0..n-1"); return HCSPMM_EINVAL; }
            new_of_old[o] = i;
        }
        if (h_rowptr[0] != 0) { set_error("invalid CSR: rowptr[0] != 0"); return HCSPMM_EBADCSR; }
        if (h_rowptr[n] > 0 && (!h_colind || !h_vals || !h_out_colind || !h_out_vals)) { set_error("an entry array is NULL"); return HCSPMM_EINVAL; }
        std::vector<std::pair<int32_t, float>> row;
        int32_t out = 0;
        h_out_rowptr[0] = 0;
        for (int32_t i = 0; i < n; ++i) {
            const int32_t o = h_order[i];
            const int32_t s = h_rowptr[o], e = h_rowptr[o + 1];
            if (s < 0 || s > e || e > h_rowptr[n]) { set_error("invalid CSR: rowptr not monotone"); return HCSPMM_EBADCSR; }
            row.clear();
            for (int32_t k = s; k < e; ++k) {
                const int32_t c = h_colind[k];
                if (c < 0 || c >= n) { set_error("invalid CSR: column index out of range (the matrix must be square)"); return HCSPMM_EBADCSR; }
                row.emplace_back(new_of_old[c], h_vals[k]);
            }
            std::stable_sort(row.begin(), row.end(), [](const auto& a, const auto& b) { return a.first < b.first; });
            for (const auto& p : row) { h_out_colind[out] = p.first; h_out_vals[out] = p.second; ++out; }
            h_out_rowptr[i + 1] = out;
        }
    } catch (const std::bad_alloc&) {
        set_error("host allocation failed in the CSR permutation");
        return HCSPMM_EALLOC;
    }
    return HCSPMM_OK;
}

// Transpose of a CSR matrix by a counting sort over the column indices; rows of the result are
// ascending in the column index and keep the input's row order among duplicates (stable).
hcspmm_status hcspmm_transpose_csr(int32_t n_rows, int32_t n_cols, const int32_t* h_rowptr, const int32_t* h_colind,
                                   const float* h_vals, int32_t* h_out_rowptr, int32_t* h_out_colind, float* h_out_vals)
{
    using hcspmm::set_error;
    if (n_rows < 0 || n_cols < 0) { set_error("sizes must be non-negative"); return HCSPMM_EINVAL; }
    if (!h_rowptr || !h_out_rowptr) { set_error("rowptr or out_rowptr is NULL"); return HCSPMM_EINVAL; }
    if (h_rowptr[0] != 0) { set_error("invalid CSR: rowptr[0] != 0"); return HCSPMM_EBADCSR; }
    const int32_t nnz = h_rowptr[n_rows];
    if (nnz < 0) { set_error("invalid CSR: negative entry count"); return HCSPMM_EBADCSR; }
    if (nnz > 0 && (!h_colind || !h_vals || !h_out_colind || !h_out_vals)) { set_error("an entry array is NULL"); return HCSPMM_EINVAL; }
    for (int32_t c = 0; c <= n_cols; ++c) h_out_rowptr[c] = 0;
    for (int32_t i = 0; i < n_rows; ++i) {
        const int32_t s = h_rowptr[i], e = h_rowptr[i + 1];
        if (s < 0 || s > e || e > nnz) { set_error("invalid CSR: rowptr not monotone"); return HCSPMM_EBADCSR; }
        for (int32_t k = s; k < e; ++k) {
            const int32_t c = h_colind[k];
            if (c < 0 || c >= n_cols) { set_error("invalid CSR: column index out of range"); return HCSPMM_EBADCSR; }
            ++h_out_rowptr[c + 1];
        }
    }
    for (int32_t c = 0; c < n_cols; ++c) h_out_rowptr[c + 1] += h_out_rowptr[c];
    try {
        std::vector<int32_t> cursor(h_out_rowptr, h_out_rowptr + n_cols);
        for (int32_t i = 0; i < n_rows; ++i)
            for (int32_t k = h_rowptr[i]; k < h_rowptr[i + 1]; ++k) {
                const int32_t p = cursor[h_colind[k]]++;
                h_out_colind[p] = i;
                h_out_vals[p] = h_vals[k];
            }
    } catch (const std::bad_alloc&) {
        set_error("host allocation failed in the CSR transpose");
        return HCSPMM_EALLOC;
    }
    return HCSPMM_OK;
}

}  // extern "C"
