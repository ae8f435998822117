// C-ABI entry points: argument checking, plan construction, launch sequencing.
#include "common.hpp"

#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <deque>
#include <mutex>
#include <new>
#include <vector>

// Device blocks kept for reuse instead of going back to the runtime (an allocation and its release cost the
// runtime 20-40 us each, a dozen of them per preparation).  Two uses:
//  * a plan that is updated (hcspmm_plan_update) keeps the scratch of its last update and the arrays of the plan it
//    replaced for the next update; a block that two updates in a row did not use is released; freed with the plan;
//  * one bounded cache per GPU for the whole process serves the preparations of small matrices (blocks of at most
//    16 MiB, 64 MiB in all; what does not fit is released at once).  It lives until the process ends.
struct BlockCache {
    struct Block { void* p; size_t n; int age; };
    std::vector<Block> blocks;
    std::mutex mu;
    size_t max_block = 0, cap = 0, held = 0;      // bounds of the per-GPU cache (0: none)
    // smallest cached block that holds n bytes without wasting more than half of itself (or 1 MiB)
    void* take(size_t n, size_t* got)
    {
        std::lock_guard<std::mutex> g(mu);
        int best = -1;
        for (int i = 0; i < (int)blocks.size(); ++i) {
            const size_t b = blocks[(size_t)i].n;
            if (b < n || b > n + (n / 2 > ((size_t)1 << 20) ? n / 2 : ((size_t)1 << 20))) continue;
            if (best < 0 || b < blocks[(size_t)best].n) best = i;
        }
        if (best < 0) return nullptr;
        void* q = blocks[(size_t)best].p;
        *got = blocks[(size_t)best].n;
        held -= *got;
        blocks.erase(blocks.begin() + best);
        return q;
    }
    void give(void* q, size_t n)
    {
        if (!q) return;
        {
            std::lock_guard<std::mutex> g(mu);
            if (!(max_block && n > max_block) && !(cap && held + n > cap)) {
                blocks.push_back(Block{q, n, 0});
                held += n;
                return;
            }
        }
        (void)hipFree(q);
    }
    void end_of_update()
    {
        std::lock_guard<std::mutex> g(mu);
        for (size_t i = 0; i < blocks.size();) {
            if (++blocks[i].age > 2) { held -= blocks[i].n; (void)hipFree(blocks[i].p); blocks.erase(blocks.begin() + (long)i); }
            else ++i;
        }
    }
    void clear()
    {
        std::lock_guard<std::mutex> g(mu);
        for (Block& b : blocks) (void)hipFree(b.p);
        blocks.clear();
        held = 0;
    }
};

// the process-wide cache of the given GPU (null for a device number beyond the table)
static BlockCache* small_block_cache(int device)
{
    constexpr int kMaxDevices = 64;
    static BlockCache caches[kMaxDevices];
    static std::once_flag once;
    std::call_once(once, [] {
        for (BlockCache& c : caches) { c.max_block = (size_t)16 << 20; c.cap = (size_t)64 << 20; }
    });
    return device >= 0 && device < kMaxDevices ? &caches[device] : nullptr;
}

namespace hcspmm {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

static int env_int(const char* name)
{
    const char* v = getenv(name);
    return v ? atoi(v) : -1;
}

const Tune& tune()
{
    static const Tune t = {env_int("HCSPMM_TUNE_MID_ROW"), env_int("HCSPMM_TUNE_LONG_ROW"), env_int("HCSPMM_TUNE_SLICE_COLS"),
                           getenv("HCSPMM_TUNE_SERIAL") ? 1 : 0, env_int("HCSPMM_TUNE_XCD_CHUNK"), env_int("HCSPMM_TUNE_RPG"),
                           env_int("HCSPMM_TUNE_TILES_PER_WAVE"), getenv("HCSPMM_TUNE_NO_ROWS16") ? 1 : 0,
                           getenv("HCSPMM_TUNE_RUNS") ? 1 : 0, env_int("HCSPMM_TUNE_RUN_SLICE"), env_int("HCSPMM_TUNE_SIDE_NNZ"), env_int("HCSPMM_TUNE_BANDS")};
    return t;
}

// Shipped selector coefficients (w1, w2, b) x 2^20 of  z = w1*ncols + w2*sparsity + b  (Section
// IV-C form; route = matrix path iff z < 0), one row per (precision, dense-width bucket).  Fitted
// on MI355X with the procedure of Section IV-C (synthetic 16-row windows, both deployed kernels
// timed; selector_fit.py) and then checked on community graphs of rising density -- the paper does
// not print its own values.  Read as
//     matrix path  iff  ncols / N0 + sparsity / S0 < 1 :
// N0 bounds the window width, S0 is the sparsity below which the matrix path pays.
//  * d > 64: the matrix path wins or ties from ~1.02 non-zeros per condensed column at every
//    width in the sweep and on the dense power-law graph of the benchmark set (-17 %); wide windows
//    are cut into column slices as far as parallelism needs, so no width limit (w1 = 0) and
//    S0 = 0.936 for large matrices.  On community graphs at d = 128 (blocks of 64, 128-column
//    windows) the scalar path with its XCD-local row order wins at sparsity 0.84 (76 vs 84 us) and
//    loses from 0.72 down (120 vs 96, 143 vs 106, 178 vs 118 us): S0 = 0.83 for smaller matrices.
//  * d <= 64: the sweep (whose windows share no columns with their neighbours) favours the
//    matrix path from ~1.3 non-zeros per column, but on community graphs, where neighbouring rows
//    and windows share columns, the scalar path gets the same reuse out of L1 and the two paths
//    tie within ~10 % up to fully dense blocks; a tie goes to the scalar path (S0 = 0.25: twelve
//    non-zeros per column, i.e. nearly full tiles only).
struct SelectorRow { int32_t dtype; int32_t d_max; int64_t nnz_min; int64_t c[3]; };
static const SelectorRow kSelectorTable[] = {
    // fp32 MFMA
    {HCSPMM_F32, 32, 0, {2048, 4194304, -1048576}},              // N0 = 512,  S0 = 0.25
    {HCSPMM_F32, 64, 0, {171, 4194304, -1048576}},               // N0 = 6144, S0 = 0.25
    // d > 64.  A workgroup-per-window launch has tens of microseconds of fixed latency per
    // workgroup, which only a large matrix amortises: below 16 M non-zeros windows wider than a
    // few hundred columns stay on the scalar path (N0 = 2048), above there is no width limit.
    {HCSPMM_F32, 1 << 30, 16000000, {0, 1120000, -1048576}},     // S0 = 0.936
    {HCSPMM_F32, 1 << 30, 0, {512, 1263344, -1048576}},          // N0 = 2048, S0 = 0.83
    // 16-bit X: the rows of fp32.  On the large dense power-law graph half the gather bytes make the
    // scalar path 2.2x faster than with fp32 X and the matrix path (whose 16-bit stages run three
    // ahead) 2.0x: all-matrix 2.63 ms, all-scalar 2.85 ms, this routing 2.64 ms.  Community graphs
    // at d = 128 favour the matrix path as in fp32 (49/64/91 vs 60/78/116 us), at d = 64 neither.
    {HCSPMM_BF16, 64, 0, {171, 4194304, -1048576}},
    {HCSPMM_BF16, 1 << 30, 16000000, {0, 1120000, -1048576}},    // S0 = 0.936
    {HCSPMM_BF16, 1 << 30, 0, {512, 1120000, -1048576}},
    {HCSPMM_F16, 64, 0, {171, 4194304, -1048576}},
    {HCSPMM_F16, 1 << 30, 16000000, {0, 1120000, -1048576}},
    {HCSPMM_F16, 1 << 30, 0, {512, 1120000, -1048576}},
};

static bool lookup_selector(int32_t dtype, int32_t d_hint, int64_t nnz, int64_t* coef)
{
    if (d_hint <= 0) d_hint = 64;
    for (const SelectorRow& r : kSelectorTable)
        if (r.dtype == dtype && d_hint <= r.d_max && nnz >= r.nnz_min) {
            coef[0] = r.c[0]; coef[1] = r.c[1]; coef[2] = r.c[2];
            return true;
        }
    return false;
}

struct DevAlloc {
    std::vector<void*> ptrs;
    std::vector<size_t> sizes;      // true size of every block in ptrs
    int64_t bytes = 0;
    ::BlockCache* cache = nullptr;  // optional: blocks come from / go back to a plan's cache
    char* arena = nullptr;          // optional: one allocation that get() carves up (scratch of known total size)
    size_t arena_size = 0, arena_used = 0;
    hipError_t raw(void** out, size_t n)
    {
        if (n == 0) n = 256;
        size_t got = n;
        void* q = cache ? cache->take(n, &got) : nullptr;
        if (!q) {
            const hipError_t e = hipMalloc(&q, n);
            if (e != hipSuccess) { *out = nullptr; return e; }
            got = n;
        }
        ptrs.push_back(q);
        sizes.push_back(got);
        *out = q;
        return hipSuccess;
    }
    hipError_t reserve(size_t total)
    {
        void* p = nullptr;
        const hipError_t e = raw(&p, total);
        if (e != hipSuccess) return e;
        arena = static_cast<char*>(p);
        arena_size = total;
        arena_used = 0;
        return hipSuccess;
    }
    size_t chunk_min = 0;           // > 0: arrays are carved out of chunks of at least this size (few device allocations)
    static size_t padded(size_t sz) { return (sz + 255) & ~(size_t)255; }
    template <class T> hipError_t get(T** out, size_t count)
    {
        size_t sz = count * sizeof(T);
        if (sz == 0) sz = sizeof(T) < 16 ? 16 : sizeof(T);
        if (chunk_min && 2 * padded(sz) < chunk_min && !(arena && arena_used + padded(sz) <= arena_size)) {
            const hipError_t e = reserve(chunk_min);            // small arrays share chunks; large ones get their own allocation below
            if (e != hipSuccess) { *out = nullptr; return e; }
        }
        if (!(chunk_min && 2 * padded(sz) >= chunk_min) && arena && arena_used + padded(sz) <= arena_size) {
            *out = reinterpret_cast<T*>(arena + arena_used);
            arena_used += padded(sz);
            bytes += (int64_t)sz;
            return hipSuccess;
        }
        void* q = nullptr;
        const hipError_t e = raw(&q, sz);
        if (e != hipSuccess) { *out = nullptr; return e; }
        bytes += (int64_t)sz;
        *out = static_cast<T*>(q);
        return hipSuccess;
    }
    void free_all()
    {
        for (size_t i = 0; i < ptrs.size(); ++i) {
            if (cache) cache->give(ptrs[i], sizes[i]);
            else (void)hipFree(ptrs[i]);
        }
        ptrs.clear();
        sizes.clear();
        arena = nullptr;
        arena_size = arena_used = 0;
    }
};

#define HC_ALLOC(alloc, ptr, count)                                                                \
    do {                                                                                           \
        if ((alloc).get(&(ptr), (size_t)(count)) != hipSuccess) {                                  \
            (void)hipGetLastError();                                                               \
            set_error("device allocation of %zu elements failed (%s:%d)", (size_t)(count), __FILE__, __LINE__); \
            st = HCSPMM_EALLOC;                                                                    \
            goto fail;                                                                             \
        }                                                                                          \
    } while (0)

#define HC_TRY(call)                                                                               \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) {                                                                    \
            set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__);  \
            st = HCSPMM_EHIP;                                                                      \
            goto fail;                                                                             \
        }                                                                                          \
    } while (0)

static void free_plan_arrays(hcspmm_plan* p)
{
    // the plan's arrays live in a few chunks; only the lazily sized buffers and arrays completed on export are separate
    BlockCache* to = p->cache ? p->cache : small_block_cache(p->device);
    for (int32_t i = 0; i < p->n_chunks; ++i) {
        if (to) to->give(p->chunks[i], p->chunk_bytes[i]);
        else (void)hipFree(p->chunks[i]);
    }
    p->n_chunks = 0;
    void* owned[] = {p->erc_own ? p->erc : nullptr, p->wcols_own ? p->wcols : nullptr, p->tile_partial, p->partial};
    for (void* q : owned)
        if (q) (void)hipFree(q);
}

// Completes what hcspmm_prepare leaves out because no kernel reads it: the window features (ncols,
// wptr, total_ncols) of a scalar-only plan, and -- unless features_only -- wcols / erc of the
// scalar-path windows.  The distinct-column lists are recomputed into scratch memory.  Default
// stream, synchronous.
static hcspmm_status complete_condensed(hcspmm_plan* p, bool features_only)
{
    hcspmm_status st = HCSPMM_OK;
    DevAlloc tmp;
    int32_t *tmp_cols = nullptr, *big_list = nullptr, *cnt = nullptr, *nc_tmp = nullptr, *nz_tmp = nullptr;
    int64_t* scan_tmp = nullptr;
    int32_t h_big = 0;
    const int32_t W = p->W;
    HC_ALLOC(tmp, tmp_cols, p->nnz);
    HC_ALLOC(tmp, big_list, W);
    HC_ALLOC(tmp, cnt, 2);
    HC_ALLOC(tmp, nc_tmp, W);
    HC_ALLOC(tmp, nz_tmp, W);
    HC_ALLOC(tmp, scan_tmp, scan_scratch_elems((int64_t)W + 1));
    HC_TRY(hipMemsetAsync(cnt, 0, 2 * sizeof(int32_t), nullptr));
    if (W > 0) {
        HC_TRY(launch_window_nnz(W, p->n_rows, p->rowptr, nz_tmp, big_list, cnt + 1, nullptr));
        HC_TRY(launch_unique_small(W, p->n_rows, p->rowptr, p->colind, tmp_cols, nc_tmp, nullptr, nullptr));
        HC_TRY(hipMemcpy(&h_big, cnt + 1, sizeof h_big, hipMemcpyDeviceToHost));
        HC_TRY(launch_unique_big(h_big, big_list, p->n_rows, p->n_cols, p->rowptr, p->colind, tmp_cols, nc_tmp, nullptr, nullptr));
    }
    if (!p->features_complete) {
        if (W > 0) HC_TRY(hipMemcpyAsync(p->ncols, nc_tmp, (size_t)W * sizeof(int32_t), hipMemcpyDeviceToDevice, nullptr));
        HC_TRY(exclusive_scan_i32_i64(p->ncols, W, p->wptr, scan_tmp, nullptr));
        HC_TRY(hipMemcpy(&p->total_ncols, p->wptr + W, sizeof(int64_t), hipMemcpyDeviceToHost));
        p->features_complete = 1;
    }
    if (!features_only && !p->condensed_complete) {
        if (!p->erc) {
            if (hipMalloc((void**)&p->erc, (size_t)(p->nnz > 0 ? p->nnz : 1) * sizeof(int32_t)) != hipSuccess) {
                (void)hipGetLastError(); p->erc = nullptr;
                set_error("device allocation failed while completing the condensed structure"); st = HCSPMM_EALLOC; goto fail;
            }
            p->erc_own = 1;
        }
        if (!p->wcols) {
            if (hipMalloc((void**)&p->wcols, (size_t)(p->total_ncols > 0 ? p->total_ncols : 1) * sizeof(int32_t)) != hipSuccess) {
                (void)hipGetLastError(); p->wcols = nullptr;
                set_error("device allocation failed while completing the condensed structure"); st = HCSPMM_EALLOC; goto fail;
            }
            p->wcols_own = 1;
        }
        if (W > 0)
            HC_TRY(launch_ecol(W, p->n_rows, p->rowptr, p->colind, tmp_cols, p->ncols, p->wptr, p->wcols, p->erc, cnt, p->route, 0,
                               0x7fffffff, nullptr));
        HC_TRY(hipDeviceSynchronize());
        p->condensed_complete = 1;
    }
    HC_TRY(hipDeviceSynchronize());
    tmp.free_all();
    return HCSPMM_OK;
fail:
    (void)hipDeviceSynchronize();
    tmp.free_all();
    return st;
}

// Small device-to-host read-backs of a preparation go through a page of pinned host memory: a copy into
// pageable memory costs the runtime tens of microseconds each, and a preparation makes five to eight of them.
// The pages are allocated on first use, handed out one per running preparation and kept until the process ends.
class PinnedPage {
public:
    static constexpr size_t kBytes = 4096;
    PinnedPage()
    {
        std::lock_guard<std::mutex> g(mu());
        for (Slot& sl : pool())
            if (!sl.busy) { sl.busy = true; slot_ = &sl; return; }
        void* q = nullptr;
        if (hipHostMalloc(&q, kBytes, hipHostMallocPortable) != hipSuccess) { (void)hipGetLastError(); return; }
        pool().push_back(Slot{q, true});
        slot_ = &pool().back();
    }
    ~PinnedPage()
    {
        if (!slot_) return;
        std::lock_guard<std::mutex> g(mu());
        slot_->busy = false;
    }
    PinnedPage(const PinnedPage&) = delete;
    PinnedPage& operator=(const PinnedPage&) = delete;
    char* ptr() const { return slot_ ? static_cast<char*>(slot_->p) : nullptr; }
private:
    struct Slot { void* p; bool busy; };
    static std::mutex& mu() { static std::mutex m; return m; }
    static std::deque<Slot>& pool() { static std::deque<Slot> v; return v; }   // (deque: growth keeps the slots in place)
    Slot* slot_ = nullptr;
};

// Read-backs queued on a stream into the pinned page, copied to their host destinations after the stream's next
// synchronisation.  Without a page (or for a block that does not fit) the copy goes straight to its destination.
struct Readback {
    char* page = nullptr;
    size_t used = 0;
    struct Pending { void* dst; size_t off, n; };
    Pending pend[16];
    int n_pend = 0;
    hipError_t add(void* dst, const void* src, size_t n, hipStream_t stream)
    {
        const size_t off = (used + 15) & ~(size_t)15;
        if (!page || n_pend == 16 || off + n > PinnedPage::kBytes) return hipMemcpyAsync(dst, src, n, hipMemcpyDeviceToHost, stream);
        pend[n_pend++] = Pending{dst, off, n};
        used = off + n;
        return hipMemcpyAsync(page + off, src, n, hipMemcpyDeviceToHost, stream);
    }
    hipError_t sync(hipStream_t stream)
    {
        const hipError_t e = hipStreamSynchronize(stream);
        if (e == hipSuccess)
            for (int i = 0; i < n_pend; ++i) memcpy(pend[i].dst, page + pend[i].off, pend[i].n);
        n_pend = 0;
        used = 0;
        return e;
    }
};

// What an incremental preparation carries over from the previous plan: the distinct-column counts of the windows
// that hold no changed row (device array of the old plan) and the list of windows that do (device, distinct ids).
struct PlanCarry {
    const int32_t* old_ncols; const int32_t* touched; int32_t n_touched;
    // the previous plan's condensed structure (matrix-path windows), when it has one whose rows were all sorted
    const uint8_t* old_route = nullptr; const int64_t* old_wptr = nullptr; const int32_t* old_nnzw = nullptr;
    const int32_t* old_wcols = nullptr; const int32_t* old_erc = nullptr;
};

static hcspmm_status build_plan(hcspmm_plan* p, hipStream_t stream, const PlanCarry* carry = nullptr)
{
    hcspmm_status st = HCSPMM_OK;
    DevAlloc tmp;      // scratch, freed on exit
    DevAlloc keep;     // plan-owned (chunks handed to the plan on success), freed on failure only
    PinnedPage pinned;
    Readback rb;
    rb.page = pinned.ptr();
    tmp.cache = keep.cache = p->cache ? p->cache : small_block_cache(p->device);
    const int32_t n_rows = p->n_rows, W = p->W;
    const int64_t nnz = p->nnz;
    keep.chunk_min = (size_t)1 << 20;      // small graphs: all plan arrays in one or two device allocations
    int32_t *err = nullptr, *big_list = nullptr, *huge_list = nullptr, *big_count = nullptr, *tmp_cols = nullptr;
    int32_t *f_mfma = nullptr, *f_csr = nullptr, *f_small = nullptr, *f_midw = nullptr, *f_big = nullptr, *nnz_if = nullptr;
    int32_t *f_short = nullptr, *f_mid = nullptr, *n_seg = nullptr, *f_multi = nullptr, *n_slot = nullptr, *len_long = nullptr;
    int64_t *scan_tmp = nullptr, *pos_a = nullptr, *pos_b = nullptr, *pos_c = nullptr, *pos_d = nullptr, *pos_e = nullptr, *pos_f = nullptr;
    int32_t* f_rest = nullptr;
    int32_t *t_small = nullptr, *t_mid = nullptr, *t_huge = nullptr, *t_counts = nullptr;
    int64_t *totals_dev = nullptr;
    int32_t h_err = 0, h_big = 0, h_cls[2] = {0, 0}, h_tc[3] = {0, 0, 0};
    int64_t h_tot[16];
    const int64_t scan_n = (int64_t)(n_rows > W ? n_rows : W) + 1;

    {
        // every scratch array of this function has a size known from (n_rows, W, nnz): one allocation
        const size_t i32 = sizeof(int32_t), i64 = sizeof(int64_t);
        size_t total = DevAlloc::padded(4 * i32) + DevAlloc::padded((size_t)nnz * i32) + 2 * DevAlloc::padded((size_t)W * i32) +
                       DevAlloc::padded((size_t)scan_multi_scratch_elems(scan_n) * i64) +
                       6 * DevAlloc::padded((size_t)(scan_n + 1) * i64) +
                       DevAlloc::padded(16 * i64) + 6 * DevAlloc::padded(((size_t)W + 1) * i32) +
                       7 * DevAlloc::padded(((size_t)n_rows + 1) * i32) + 64 * 256 +
                       (carry ? 3 * DevAlloc::padded((size_t)carry->n_touched * i32) + 256 : 0);
        if (tmp.reserve(total) != hipSuccess) {
            (void)hipGetLastError();
            set_error("device allocation of %zu scratch bytes failed", total);
            st = HCSPMM_EALLOC;
            goto fail;
        }
    }
    HC_ALLOC(tmp, err, 4);
    big_count = err + 1;                           // two counters: windows for the large hash set, for the bitmap
    HC_TRY(hipMemsetAsync(err, 0, 4 * sizeof(int32_t), stream));
    if (carry) {
        // the row offsets are checked in full (they all move when a row grows), the columns only where rows changed
        HC_ALLOC(tmp, t_small, carry->n_touched);
        HC_ALLOC(tmp, t_mid, carry->n_touched);
        HC_ALLOC(tmp, t_huge, carry->n_touched);
        HC_ALLOC(tmp, t_counts, 4);
        HC_TRY(hipMemsetAsync(t_counts, 0, 4 * sizeof(int32_t), stream));
        HC_TRY(launch_validate_rowptr(n_rows, nnz, p->rowptr, err, stream));
        HC_TRY(rb.add(&h_err, err, sizeof h_err, stream));
        HC_TRY(rb.sync(stream));
        if (!h_err) {           // the windows' spans are only meaningful with sound row offsets
            HC_TRY(launch_touched_classes(carry->n_touched, carry->touched, n_rows, p->n_cols, p->rowptr, p->colind, t_small,
                                          t_mid, t_huge, t_counts, err, stream));
            HC_TRY(rb.add(h_tc, t_counts, 3 * sizeof(int32_t), stream));
        }
    } else {
        HC_TRY(launch_validate(n_rows, p->n_cols, nnz, p->rowptr, p->colind, err, stream));
    }
    HC_TRY(rb.add(&h_err, err, sizeof h_err, stream));
    HC_TRY(rb.sync(stream));
    if (h_err) {
        set_error("invalid CSR: %s%s%s%s", (h_err & 1) ? "rowptr[0] != 0; " : "",
                  (h_err & 2) ? "rowptr[n_rows] != nnz; " : "", (h_err & 4) ? "rowptr not non-decreasing; " : "",
                  (h_err & 8) ? "column index out of range; " : "");
        st = HCSPMM_EBADCSR;
        goto fail;
    }

    HC_ALLOC(keep, p->ncols, W);
    HC_ALLOC(keep, p->nnzw, W);
    HC_ALLOC(keep, p->route, W);
    HC_ALLOC(keep, p->wptr, (size_t)W + 1);
    HC_ALLOC(tmp, tmp_cols, nnz);
    HC_ALLOC(tmp, big_list, W);
    HC_ALLOC(tmp, huge_list, W);
    HC_ALLOC(tmp, scan_tmp, scan_multi_scratch_elems(scan_n));
    HC_ALLOC(tmp, pos_a, scan_n + 1);
    HC_ALLOC(tmp, pos_b, scan_n + 1);
    HC_ALLOC(tmp, pos_c, scan_n + 1);
    HC_ALLOC(tmp, pos_d, scan_n + 1);
    HC_ALLOC(tmp, pos_e, scan_n + 1);
    HC_ALLOC(tmp, pos_f, scan_n + 1);
    HC_ALLOC(tmp, totals_dev, 16);

    // A scalar-only plan never reads the condensed structure (the paper has no preprocessing for its
    // scalar path either): its window features stay zero here and are computed when first asked for
    // (hcspmm_plan_info / hcspmm_plan_export), which makes prepare cheap for matrices that keep changing.
    p->features_complete = (p->opt.route_mode == HCSPMM_ROUTE_ALL_CSR && nnz > 0) ? 0 : 1;
    if (W > 0) {
        // windows, condensing (Section IV-A)
        // The selector needs the number of distinct columns of every window but the sorted lists only
        // for the windows it sends to the matrix path: count with LDS hash sets first (bitmap passes for
        // the few windows beyond the hash set's capacity, which leave their lists behind as well).
        HC_TRY(launch_window_classes(W, n_rows, p->rowptr, p->nnzw, big_list, huge_list, big_count, stream));
        if (p->features_complete && carry) {
            // counts of the untouched windows are the previous plan's; the touched ones are counted again
            HC_TRY(hipMemcpyAsync(p->ncols, carry->old_ncols, (size_t)W * sizeof(int32_t), hipMemcpyDeviceToDevice, stream));
            HC_TRY(rb.add(h_cls, big_count, sizeof h_cls, stream));
            HC_TRY(rb.sync(stream));
            h_big = h_cls[0];
            HC_TRY(launch_count_small_list(h_tc[0], t_small, n_rows, p->rowptr, p->colind, p->ncols, stream));
            HC_TRY(launch_count_mid(h_tc[1], t_mid, n_rows, p->rowptr, p->colind, p->ncols, stream));
            HC_TRY(launch_unique_big(h_tc[2], t_huge, n_rows, p->n_cols, p->rowptr, p->colind, tmp_cols, p->ncols, nullptr,
                                     stream));
        } else if (p->features_complete) {
            HC_TRY(launch_count_small(W, n_rows, p->rowptr, p->colind, p->ncols, stream));
            HC_TRY(rb.add(h_cls, big_count, sizeof h_cls, stream));
            HC_TRY(rb.sync(stream));
            h_big = h_cls[0];
            HC_TRY(launch_count_mid(h_big, big_list, n_rows, p->rowptr, p->colind, p->ncols, stream));
            HC_TRY(launch_unique_big(h_cls[1], huge_list, n_rows, p->n_cols, p->rowptr, p->colind, tmp_cols, p->ncols,
                                     nullptr, stream));
        } else {
            HC_TRY(hipMemsetAsync(p->ncols, 0, (size_t)W * sizeof(int32_t), stream));
        }
    }
    if (p->features_complete) {
        ScanMulti m{};
        m.k = 1;
        m.in[0] = p->ncols;
        m.out[0] = p->wptr;
        HC_TRY(exclusive_scan_multi(m, W, totals_dev + 8, scan_tmp, stream));     // the total is read back with the list sizes below
    } else {
        HC_TRY(hipMemsetAsync(p->wptr, 0, ((size_t)W + 1) * sizeof(int64_t), stream));
        HC_TRY(hipMemsetAsync(totals_dev + 8, 0, sizeof(int64_t), stream));
    }
    p->total_ncols = 0;
    p->rows_sorted = 1;

    // selection (Section IV-C) and the per-route window lists
    HC_ALLOC(tmp, f_mfma, (size_t)W + 1);
    HC_ALLOC(tmp, f_csr, (size_t)W + 1);
    HC_ALLOC(tmp, f_small, (size_t)W + 1);
    HC_ALLOC(tmp, f_midw, (size_t)W + 1);
    HC_ALLOC(tmp, f_big, (size_t)W + 1);
    HC_ALLOC(tmp, nnz_if, (size_t)W + 1);
    // Selection, then the positions of every window in its lists and the non-zeros on the matrix path: six scans in
    // one pass, their totals in one read-back.  Launch guard (hybrid mode): a path whose share cannot repay a kernel
    // launch of its own joins the other path -- decided from the same totals, so only a plan that is actually merged
    // pays a second selection pass.
    for (int32_t mode = p->opt.route_mode, pass = 0;; ++pass) {
        if (W > 0)
            HC_TRY(launch_select(W, p->ncols, p->nnzw, p->coef[0], p->coef[1], p->coef[2], mode, p->route, f_mfma, f_csr,
                                 f_small, f_midw, f_big, nnz_if, stream));
        ScanMulti m{};
        m.k = 6;
        m.in[0] = f_mfma;  m.out[0] = pos_a;
        m.in[1] = f_csr;   m.out[1] = pos_b;
        m.in[2] = f_small; m.out[2] = pos_c;
        m.in[3] = f_big;   m.out[3] = pos_d;
        m.in[4] = f_midw;  m.out[4] = pos_e;
        m.in[5] = nnz_if;  m.out[5] = nullptr;
        HC_TRY(exclusive_scan_multi(m, W, totals_dev, scan_tmp, stream));
        HC_TRY(rb.add(h_tot, totals_dev, 9 * sizeof(int64_t), stream));
        HC_TRY(rb.sync(stream));
        if (pass == 0 && p->opt.route_mode == HCSPMM_ROUTE_HYBRID) {
            const int64_t on_matrix = h_tot[5], on_scalar = p->nnz - on_matrix;
            int32_t forced = -1;
            if (on_matrix > 0 && on_scalar > 0) {
                if (on_matrix < kGuardNnz && kGuardShare * on_matrix < p->nnz) forced = HCSPMM_ROUTE_ALL_CSR;
                else if (on_scalar < kGuardNnz && kGuardShare * on_scalar < p->nnz) forced = HCSPMM_ROUTE_ALL_MFMA;
            }
            if (forced >= 0) { mode = forced; continue; }
        }
        break;
    }
    p->total_ncols = h_tot[8];
    p->n_mfma = (int32_t)h_tot[0];
    p->n_csr = W - p->n_mfma;
    p->n_mfma_small = (int32_t)h_tot[2];
    p->n_mfma_big = (int32_t)h_tot[3];
    p->n_mfma_mid = (int32_t)h_tot[4];
    p->nnz_mfma = h_tot[5];
    // condensed structure (column lists, condensed column of every non-zero) of the matrix-path
    // windows; scalar-path windows never read theirs at SpMM time and get it on export only, and a
    // plan without matrix-path windows does not even allocate the arrays
    p->condensed_complete = 0;
    if (p->n_mfma > 0) {
        HC_ALLOC(keep, p->erc, nnz);
        HC_ALLOC(keep, p->wcols, p->total_ncols);
        // err[0] is zero here (validation passed): reuse it as the "some row is unsorted" flag.
        // Windows up to kUniqueSmallCap non-zeros: sorted list by the LDS sort, positions by binary search in it.
        // Larger ones: list and positions together from bitmap ranks, unless the matrix is so wide that the
        // bitmap passes would cost more than searching (then the bitmap list + search route serves them too).
        const bool by_rank = p->n_cols <= kRankMaxCols;
        // After a structural change the untouched windows that were and are on the matrix path keep the previous
        // plan's lists and condensed columns (copied to their new offsets); only the others are condensed, through
        // a route array masked down to them.
        const uint8_t* todo_route = p->route;
        if (carry && carry->old_erc && carry->old_wcols) {
            uint8_t *carried = nullptr, *todo = nullptr;
            int64_t* old_start = nullptr;
            HC_ALLOC(tmp, carried, (size_t)W);
            HC_ALLOC(tmp, todo, (size_t)W);
            HC_ALLOC(tmp, old_start, (size_t)W + 1);
            HC_TRY(launch_carry_mask(W, carry->old_route, p->route, carry->n_touched, carry->touched, carried, todo, stream));
            HC_TRY(exclusive_scan_i32_i64(carry->old_nnzw, W, old_start, scan_tmp, stream));
            HC_TRY(launch_carry_copy(W, n_rows, carried, carry->old_wptr, p->wptr, carry->old_wcols, p->wcols, old_start,
                                     p->rowptr, carry->old_erc, p->erc, stream));
            todo_route = todo;
        }
        HC_TRY(launch_unique_small(W, n_rows, p->rowptr, p->colind, tmp_cols, p->ncols, todo_route, stream));
        if (by_rank) {
            HC_TRY(launch_condense_rank(h_big, big_list, n_rows, p->rowptr, p->colind, todo_route, p->wptr, p->wcols, p->erc,
                                        err, stream));
            HC_TRY(launch_condense_rank(h_cls[1], huge_list, n_rows, p->rowptr, p->colind, todo_route, p->wptr, p->wcols,
                                        p->erc, err, stream));
        } else {
            HC_TRY(launch_unique_big(h_big, big_list, n_rows, p->n_cols, p->rowptr, p->colind, tmp_cols, p->ncols, todo_route,
                                     stream));
        }
        HC_TRY(launch_ecol(W, n_rows, p->rowptr, p->colind, tmp_cols, p->ncols, p->wptr, p->wcols, p->erc, err, todo_route, 1,
                           by_rank ? kUniqueSmallCap : 0x7fffffff, stream));
        HC_TRY(rb.add(&h_err, err, sizeof h_err, stream));
        HC_TRY(rb.sync(stream));
        p->rows_sorted = h_err ? 0 : 1;
    } else if (nnz == 0) {
        p->condensed_complete = 1;
    }
    HC_ALLOC(keep, p->mfma_windows, p->n_mfma);
    HC_ALLOC(keep, p->csr_windows, p->n_csr);
    HC_ALLOC(keep, p->mfma_small, p->n_mfma_small);
    HC_ALLOC(keep, p->mfma_mid, p->n_mfma_mid);
    HC_ALLOC(keep, p->mfma_big, p->n_mfma_big);
    HC_TRY(launch_compact_ids(W, f_mfma, pos_a, p->mfma_windows, stream));
    HC_TRY(launch_compact_ids(W, f_csr, pos_b, p->csr_windows, stream));
    HC_TRY(launch_compact_ids(W, f_small, pos_c, p->mfma_small, stream));
    HC_TRY(launch_compact_ids(W, f_big, pos_d, p->mfma_big, stream));
    HC_TRY(launch_compact_ids(W, f_midw, pos_e, p->mfma_mid, stream));
    // Runs of matrix-path windows (kRunWindows consecutive list entries each): merged column lists and slots on the
    // device, the slice layout on the host from the union sizes (a few bytes per run cross the bus).
    p->runs_ok = 0;
    if (p->n_mfma > 0 && p->rows_sorted && p->n_cols <= kRankMaxCols && (p->opt.matrix_kernels == HCSPMM_MATRIX_RUNS || tune().runs)) {
        const int32_t n_runs = (p->n_mfma + kRunWindows - 1) / kRunWindows;
        HC_ALLOC(keep, p->ucols, p->total_ncols);
        HC_ALLOC(keep, p->wslot, p->total_ncols);
        HC_ALLOC(keep, p->runs, n_runs);
        HC_TRY(hipMemsetAsync(p->wslot, 0xff, (size_t)p->total_ncols * sizeof(int32_t), stream));   // -1 where no run owns the column
        HC_TRY(launch_run_union(n_runs, p->mfma_windows, p->n_mfma, p->ncols, p->wptr, p->wcols, p->ucols, p->wslot, p->runs,
                                stream));
        std::vector<RunDesc> h_runs((size_t)n_runs);
        std::vector<int32_t> h_list((size_t)p->n_mfma);
        HC_TRY(rb.add(h_runs.data(), p->runs, (size_t)n_runs * sizeof(RunDesc), stream));
        HC_TRY(rb.add(h_list.data(), p->mfma_windows, (size_t)p->n_mfma * sizeof(int32_t), stream));
        HC_TRY(rb.sync(stream));
        int64_t u_total = 0;
        for (const RunDesc& r : h_runs) u_total += r.nu;
        int64_t slice_u = (u_total / kRunTargetSlices + 63) / 64 * 64;
        if (slice_u < kRunMinSlice) slice_u = kRunMinSlice;
        if (tune().run_slice >= 64) slice_u = tune().run_slice / 64 * 64;
        std::vector<RunSlice> h_slices;
        std::vector<MultiRow> h_multi;
        int64_t slots = 0;
        for (int32_t r = 0; r < n_runs; ++r) {
            RunDesc& rd = h_runs[(size_t)r];
            const int32_t ns = (int32_t)((rd.nu + slice_u - 1) / slice_u);
            rd.n_slices = ns < 1 ? 1 : ns;
            rd.slot0 = 0;
            if (rd.n_slices > 1) {
                if (slots + (int64_t)rd.nw * rd.n_slices >= ((int64_t)1 << 27)) { set_error("too many partial tiles"); st = HCSPMM_EUNSUPPORTED; goto fail; }
                rd.slot0 = (int32_t)slots;
                for (int32_t i = 0; i < rd.nw; ++i)
                    h_multi.push_back(MultiRow{h_list[(size_t)rd.first + i], rd.slot0 + i * rd.n_slices, rd.n_slices, 0});
                slots += (int64_t)rd.nw * rd.n_slices;
            }
            for (int32_t q = 0; q < rd.n_slices; ++q) {
                const int64_t b = (int64_t)q * slice_u;
                h_slices.push_back(RunSlice{rd.up, r, (int32_t)b, (int32_t)(b + slice_u < rd.nu ? b + slice_u : rd.nu), q, rd.nw,
                                            rd.n_slices, rd.slot0, {0, 0, 0}});
            }
        }
        p->n_runs = n_runs;
        p->n_run_slices = (int32_t)h_slices.size();
        p->n_run_multi = (int32_t)h_multi.size();
        p->n_run_tile_slots = slots;
        p->run_union_cols = u_total;
        HC_ALLOC(keep, p->run_slices, h_slices.size());
        HC_ALLOC(keep, p->run_multi, h_multi.size());
        HC_TRY(hipMemcpyAsync(p->runs, h_runs.data(), (size_t)n_runs * sizeof(RunDesc), hipMemcpyHostToDevice, stream));
        HC_TRY(hipMemcpyAsync(p->run_slices, h_slices.data(), h_slices.size() * sizeof(RunSlice), hipMemcpyHostToDevice, stream));
        if (!h_multi.empty())
            HC_TRY(hipMemcpyAsync(p->run_multi, h_multi.data(), h_multi.size() * sizeof(MultiRow), hipMemcpyHostToDevice, stream));
        HC_ALLOC(keep, p->run_wins, h_slices.size() * kRunWindows);
        HC_TRY(launch_run_wins(p->n_run_slices, p->run_slices, p->runs, p->mfma_windows, p->ncols, p->wptr, n_rows, p->rowptr,
                               p->run_wins, stream));
        HC_TRY(rb.sync(stream));                    // the host vectors go out of scope
        p->runs_ok = 1;
    }
    if (W > 0) HC_TRY(launch_masked_copy(W, f_big, p->ncols, nnz_if, stream));     // nnz_if <- ncols of wide windows, else 0
    // workgroup slices: one per medium window, slice_cols condensed columns each for wide windows
    {
        int32_t* sc_n = f_mfma;      // the flag arrays are free again: reuse them as scratch (W + 1 ints each)
        int32_t* sc_multi = f_csr;
        int32_t* sc_slots = f_small;
        ScanMulti m{};
        m.k = 3;
        m.in[0] = sc_n;     m.out[0] = pos_a;
        m.in[1] = sc_multi; m.out[1] = pos_b;
        m.in[2] = sc_slots; m.out[2] = pos_d;
        HC_ALLOC(keep, p->mid_slices, p->n_mfma_mid);
        if (p->n_mfma_mid > 0) {
            HC_TRY(launch_slice_count(p->n_mfma_mid, p->mfma_mid, p->ncols, 0x40000000, sc_n, sc_multi, sc_slots, stream));
            HC_TRY(exclusive_scan_multi(m, p->n_mfma_mid, nullptr, scan_tmp, stream));
            HC_TRY(launch_slice_fill(p->n_mfma_mid, p->mfma_mid, p->ncols, 0x40000000, pos_a, pos_b, pos_d, p->mid_slices,
                                     nullptr, stream));
        }
        // Wide windows are cut into slices only as far as parallelism needs it (a slice loses the
        // alignment of concurrently running windows on the same hot low-numbered columns): aim
        // at ~4 workgroups per CU over the summed width of the wide windows.
        if (tune().slice_cols < 0 && p->n_mfma_big > 0) {
            HC_TRY(exclusive_scan_i32_i64(nnz_if, W, pos_a, scan_tmp, stream));     // nnz_if holds ncols of wide windows here
            int64_t wide_cols = 0;
            HC_TRY(rb.add(&wide_cols, pos_a + W, 8, stream));
            HC_TRY(rb.sync(stream));
            int64_t want = wide_cols / 1024;
            if (want < kKcBig) want = kKcBig;
            if (want > (1 << 27)) want = 1 << 27;
            p->slice_cols = (int32_t)((want + kKcBig - 1) / kKcBig * kKcBig);
        }
        h_tot[0] = h_tot[1] = h_tot[2] = 0;
        if (p->n_mfma_big > 0) {
            HC_TRY(launch_slice_count(p->n_mfma_big, p->mfma_big, p->ncols, p->slice_cols, sc_n, sc_multi, sc_slots, stream));
            HC_TRY(exclusive_scan_multi(m, p->n_mfma_big, totals_dev, scan_tmp, stream));
            HC_TRY(rb.add(h_tot, totals_dev, 3 * sizeof(int64_t), stream));
            HC_TRY(rb.sync(stream));
        }
        p->n_big_slices = (int32_t)h_tot[0];
        p->n_tile_multi = (int32_t)h_tot[1];
        p->n_tile_slots = h_tot[2];
        if (tune().bands > 0 && p->n_mfma_big > 0) {
            // Measurement aid (HCSPMM_TUNE_BANDS): wide windows are cut at the same global column boundaries and the
            // slices ordered band by band, so that all windows walk one band's X rows at about the same time.  Built on
            // the host from a copy of the column lists: slow, and only for the experiment that profiles/ reports.
            const int32_t Bc = tune().bands;
            std::vector<int32_t> h_list((size_t)p->n_mfma_big), h_nc((size_t)W), h_wc((size_t)p->total_ncols);
            std::vector<int64_t> h_wp((size_t)W + 1);
            HC_TRY(hipMemcpyAsync(h_list.data(), p->mfma_big, h_list.size() * 4, hipMemcpyDeviceToHost, stream));
            HC_TRY(hipMemcpyAsync(h_nc.data(), p->ncols, h_nc.size() * 4, hipMemcpyDeviceToHost, stream));
            HC_TRY(hipMemcpyAsync(h_wp.data(), p->wptr, h_wp.size() * 8, hipMemcpyDeviceToHost, stream));
            HC_TRY(hipMemcpyAsync(h_wc.data(), p->wcols, h_wc.size() * 4, hipMemcpyDeviceToHost, stream));
            HC_TRY(hipStreamSynchronize(stream));
            // HCSPMM_TUNE_BANDS_HOT=k: only the first k bands are cut; all columns behind them form one last band
            const int32_t hot = getenv("HCSPMM_TUNE_BANDS_HOT") ? atoi(getenv("HCSPMM_TUNE_BANDS_HOT")) : 0x7fffffff;
            const int32_t n_bands = std::min((p->n_cols + Bc - 1) / Bc, hot < 0x7fffffff ? hot + 1 : 0x7fffffff);
            std::vector<std::vector<WgSlice>> per_band((size_t)n_bands);
            std::vector<MultiRow> h_multi;
            int64_t slots = 0;
            for (int32_t w : h_list) {
                const int32_t* c0 = h_wc.data() + h_wp[(size_t)w];
                const int32_t nc = h_nc[(size_t)w];
                int32_t n_here = 0;
                const int64_t first = slots;
                int32_t kb = 0;
                while (kb < nc) {
                    const int32_t b = std::min(c0[kb] / Bc, n_bands - 1);
                    const int32_t ke = b == n_bands - 1 ? nc : (int32_t)(std::lower_bound(c0 + kb, c0 + nc, (b + 1) * Bc) - c0);
                    per_band[(size_t)b].push_back(WgSlice{w, kb, ke, (int32_t)(first + n_here)});
                    ++n_here;
                    kb = ke;
                }
                slots += n_here;
                h_multi.push_back(MultiRow{w, (int32_t)first, n_here, 0});
            }
            std::vector<WgSlice> h_sl;
            for (auto& v : per_band) h_sl.insert(h_sl.end(), v.begin(), v.end());
            p->n_big_slices = (int32_t)h_sl.size();
            p->n_tile_multi = (int32_t)h_multi.size();
            p->n_tile_slots = slots;
            HC_ALLOC(keep, p->big_slices, p->n_big_slices);
            HC_ALLOC(keep, p->tile_multi, p->n_tile_multi);
            HC_TRY(hipMemcpy(p->big_slices, h_sl.data(), h_sl.size() * sizeof(WgSlice), hipMemcpyHostToDevice));
            HC_TRY(hipMemcpy(p->tile_multi, h_multi.data(), h_multi.size() * sizeof(MultiRow), hipMemcpyHostToDevice));
        } else {
        HC_ALLOC(keep, p->big_slices, p->n_big_slices);
        HC_ALLOC(keep, p->tile_multi, p->n_tile_multi);
        if (p->n_mfma_big > 0)
            HC_TRY(launch_slice_fill(p->n_mfma_big, p->mfma_big, p->ncols, p->slice_cols, pos_a, pos_b, pos_d, p->big_slices,
                                     p->tile_multi, stream));
        }
        if (p->rows_sorted && p->n_big_slices > 0) {
            HC_ALLOC(keep, p->big_slice_rows, (size_t)p->n_big_slices * kH);
            HC_TRY(launch_slice_rows(p->n_big_slices, p->big_slices, n_rows, p->rowptr, p->erc, p->big_slice_rows,
                                     stream));
        }
    }
    HC_ALLOC(keep, p->mfma_small_desc, p->n_mfma_small);
    HC_TRY(launch_build_desc(p->n_mfma_small, p->mfma_small, n_rows, p->rowptr, p->ncols, p->wptr, p->mfma_small_desc,
                             stream));

    // scalar-path launch tables
    HC_ALLOC(tmp, f_short, (size_t)n_rows + 1);
    HC_ALLOC(tmp, f_mid, (size_t)n_rows + 1);
    HC_ALLOC(tmp, n_seg, (size_t)n_rows + 1);
    HC_ALLOC(tmp, f_multi, (size_t)n_rows + 1);
    HC_ALLOC(tmp, n_slot, (size_t)n_rows + 1);
    HC_ALLOC(tmp, len_long, (size_t)n_rows + 1);
    HC_ALLOC(tmp, f_rest, (size_t)n_rows + 1);
    HC_TRY(launch_row_class(n_rows, p->rowptr, p->route, p->mid_row, p->long_row, f_short, f_mid, n_seg, f_multi, n_slot, len_long, stream));
    // rows the fused update finishes through the workspace
    HC_TRY(launch_rest_flag(n_rows, p->rowptr, p->route, p->ncols, p->fused_mid_row, f_rest, stream));
    {
        // all row-level positions and counts in one pass and one read-back
        ScanMulti m{};
        m.k = 7;
        m.in[0] = len_long; m.out[0] = nullptr;
        m.in[1] = f_short;  m.out[1] = pos_a;
        m.in[2] = n_seg;    m.out[2] = pos_b;
        m.in[3] = f_multi;  m.out[3] = pos_c;
        m.in[4] = n_slot;   m.out[4] = pos_d;
        m.in[5] = f_mid;    m.out[5] = pos_e;
        m.in[6] = f_rest;   m.out[6] = pos_f;
        HC_TRY(exclusive_scan_multi(m, n_rows, totals_dev, scan_tmp, stream));
        HC_TRY(rb.add(h_tot, totals_dev, 7 * sizeof(int64_t), stream));
        HC_TRY(rb.sync(stream));
    }
    p->nnz_long = h_tot[0];
    p->n_short = (int32_t)h_tot[1];
    p->n_segs = (int32_t)h_tot[2];
    p->n_multi = (int32_t)h_tot[3];
    p->n_slots = h_tot[4];
    p->n_mid = (int32_t)h_tot[5];
    p->n_rest = (int32_t)h_tot[6];
    p->n_long_rows = (int32_t)(p->n_segs - p->n_slots + p->n_multi);   // single-segment rows + multi-segment rows
    HC_ALLOC(keep, p->segs, p->n_segs);
    HC_ALLOC(keep, p->multi, p->n_multi);
    if (p->n_segs > 0)
        HC_TRY(launch_build_segments(n_rows, p->rowptr, n_seg, pos_b, pos_c, pos_d, p->segs, p->multi, stream));
    // rows that get a whole wave
    HC_ALLOC(keep, p->mid_rows, p->n_mid);
    HC_TRY(launch_compact_ids(n_rows, f_mid, pos_e, p->mid_rows, stream));
    // Walking every row and skipping the ones another kernel owns is cheaper than an index list
    // while most rows are short scalar-path rows; otherwise keep the explicit list.
    if ((int64_t)p->n_short * 2 < n_rows) {
        HC_ALLOC(keep, p->short_rows, p->n_short);
        HC_TRY(launch_compact_ids(n_rows, f_short, pos_a, p->short_rows, stream));
    } else {
        p->short_rows = nullptr;
    }
    HC_ALLOC(keep, p->rest_rows, p->n_rest);
    HC_TRY(launch_compact_ids(n_rows, f_rest, pos_f, p->rest_rows, stream));
    HC_TRY(rb.sync(stream));
    p->device_bytes = keep.bytes;
    if (keep.ptrs.size() > sizeof p->chunks / sizeof p->chunks[0]) {
        set_error("internal: too many plan chunks");
        st = HCSPMM_EALLOC;
        goto fail;
    }
    p->n_chunks = (int32_t)keep.ptrs.size();
    for (size_t i = 0; i < keep.ptrs.size(); ++i) { p->chunks[i] = keep.ptrs[i]; p->chunk_bytes[i] = keep.sizes[i]; }
    tmp.free_all();
    return HCSPMM_OK;

fail:
    (void)hipStreamSynchronize(stream);
    tmp.free_all();
    keep.free_all();
    return st;
}

// partial tiles a call may need: the slices of wide windows, or of wide runs when the run kernel serves the matrix path
static int64_t tile_slots(const hcspmm_plan* p) { return p->n_tile_slots > p->n_run_tile_slots ? p->n_tile_slots : p->n_run_tile_slots; }

// Scratch of one SpMM call: partial rows of long rows cut into several segments, then partial tiles of
// wide windows cut into several slices (each part padded to 256 bytes).
static size_t spmm_scratch_bytes(const hcspmm_plan* p, int32_t d, size_t* tile_off)
{
    const size_t part = ((size_t)p->n_slots * (size_t)d * sizeof(float) + 255) & ~(size_t)255;
    const size_t tiles = ((size_t)tile_slots(p) * kH * (size_t)d * sizeof(float) + 255) & ~(size_t)255;
    if (tile_off) *tile_off = part;
    return part + tiles;
}

static hcspmm_status run_spmm(const hcspmm_plan* plan, const SpmmArgs& a, hipStream_t stream,
                              hipEvent_t* ev = nullptr /* 5 events when timing stages */,
                              const UpdateArgs* upd = nullptr /* fuse the update stage where a tile stays on chip */,
                              char* scratch_mem = nullptr /* device, spmm_scratch_bytes(): used instead of the plan's own lazily sized buffers */)
{
    hcspmm_plan* p = const_cast<hcspmm_plan*>(plan);
    float* partial = p->partial;
    float* tile_partial = p->tile_partial;
    if (scratch_mem) {
        size_t tile_off = 0;
        (void)spmm_scratch_bytes(p, a.d, &tile_off);
        partial = reinterpret_cast<float*>(scratch_mem);
        tile_partial = reinterpret_cast<float*>(scratch_mem + tile_off);
    }
    // long rows cut into several segments need one partial row per segment
    if (!scratch_mem && p->n_slots > 0 && p->partial_elems < p->n_slots * (int64_t)a.d) {
        if (p->partial) { HC_HIP(hipStreamSynchronize(stream)); (void)hipFree(p->partial); p->partial = nullptr; }
        const int64_t want = p->n_slots * (int64_t)a.d;
        if (hipMalloc((void**)&p->partial, (size_t)want * sizeof(float)) != hipSuccess) {
            (void)hipGetLastError();
            p->partial = nullptr;
            p->partial_elems = 0;
            set_error("allocation of %lld floats for long-row partial sums failed", (long long)want);
            return HCSPMM_EALLOC;
        }
        p->partial_elems = want;
        partial = p->partial;
    }
    if (!scratch_mem && tile_slots(p) > 0 && p->tile_partial_elems < tile_slots(p) * kH * (int64_t)a.d) {
        if (p->tile_partial) { HC_HIP(hipStreamSynchronize(stream)); (void)hipFree(p->tile_partial); p->tile_partial = nullptr; }
        const int64_t want = tile_slots(p) * kH * (int64_t)a.d;
        if (hipMalloc((void**)&p->tile_partial, (size_t)want * sizeof(float)) != hipSuccess) {
            (void)hipGetLastError();
            p->tile_partial = nullptr;
            p->tile_partial_elems = 0;
            set_error("allocation of %lld floats for wide-window partial tiles failed", (long long)want);
            return HCSPMM_EALLOC;
        }
        p->tile_partial_elems = want;
        tile_partial = p->tile_partial;
    }
    const bool use_runs = p->runs_ok && !upd && mfma_run_shape_supported(a);
    const bool has_wg = use_runs ? p->n_run_slices > 0 : (p->n_big_slices > 0 || p->n_mfma_mid > 0);
    const bool has_small = !use_runs && p->n_mfma_small > 0;
    const bool has_csr = p->n_segs > 0 || p->n_mid > 0 || p->n_short > 0;
    // The paths own disjoint rows of Y.  When more than one has work (and the stages are not being
    // timed one by one) they run side by side: the matrix-path kernels on the plan's two side
    // streams, forked from and joined back to the caller's stream with events.
    const bool side = !ev && p->side_ok && (int)has_wg + (int)has_small + (int)has_csr > 1;
    hipStream_t s_wg = stream, s_small = stream;
    if (side) {
        HC_HIP(hipEventRecord(p->ev_fork, stream));
        if (has_wg && has_csr) { s_wg = p->side[0]; HC_HIP(hipStreamWaitEvent(s_wg, p->ev_fork, 0)); }
        if (has_small && (has_csr || has_wg)) { s_small = p->side[1]; HC_HIP(hipStreamWaitEvent(s_small, p->ev_fork, 0)); }
    }
    if (ev) HC_HIP(hipEventRecord(ev[0], stream));
    if (use_runs) {
        // every matrix-path window through the run kernel: neighbouring windows share their gathered rows in LDS
        HC_HIP(launch_mfma_run(a, p->n_run_slices, p->run_slices, p->run_wins, p->ucols, p->wslot, p->erc, tile_partial, s_wg));
        HC_HIP(launch_reduce_tiles(a, p->n_run_multi, p->run_multi, tile_partial, s_wg));
        if (ev) { HC_HIP(hipEventRecord(ev[1], stream)); HC_HIP(hipEventRecord(ev[2], stream)); }
    } else {
        HC_HIP(launch_mfma_wg(a, p->n_big_slices, p->big_slices, p->ncols, p->wptr, p->wcols, p->erc, p->rows_sorted,
                              p->big_slice_rows, tile_partial, tune().bands <= 0 || getenv("HCSPMM_TUNE_BANDS_WIDE"), s_wg));
        HC_HIP(launch_reduce_tiles(a, p->n_tile_multi, p->tile_multi, tile_partial, s_wg));
        HC_HIP(launch_mfma_wg(a, p->n_mfma_mid, p->mid_slices, p->ncols, p->wptr, p->wcols, p->erc, p->rows_sorted,
                              nullptr, tile_partial, false, s_wg));
        if (ev) HC_HIP(hipEventRecord(ev[1], stream));
        HC_HIP(launch_mfma_small(a, p->n_mfma_small, p->mfma_small_desc, p->wcols, p->erc, s_small, upd));
        if (ev) HC_HIP(hipEventRecord(ev[2], stream));
    }
    if (upd)        // the fused launch walks every row: its tile tier also takes the shorter mid rows
        HC_HIP(launch_csr(a, p->n_segs, p->segs, partial, p->n_mid, p->mid_rows, p->n_csr > 0 ? p->n_rows : 0, nullptr,
                          p->route, p->fused_mid_row, stream, upd));
    else
        HC_HIP(launch_csr(a, p->n_segs, p->segs, partial, p->n_mid, p->mid_rows,
                          p->short_rows ? p->n_short : (p->n_short > 0 ? p->n_rows : 0), p->short_rows, p->route,
                          p->mid_row, stream));
    if (ev) HC_HIP(hipEventRecord(ev[3], stream));
    HC_HIP(launch_reduce_partials(a, p->n_multi, p->multi, partial, stream));
    if (ev) HC_HIP(hipEventRecord(ev[4], stream));
    if (s_wg != stream) {
        HC_HIP(hipEventRecord(p->ev_join[0], s_wg));
        HC_HIP(hipStreamWaitEvent(stream, p->ev_join[0], 0));
    }
    if (s_small != stream) {
        HC_HIP(hipEventRecord(p->ev_join[1], s_small));
        HC_HIP(hipStreamWaitEvent(stream, p->ev_join[1], 0));
    }
    // rows whose aggregation went to memory (long and mid rows, wide matrix-path windows)
    if (upd) HC_HIP(launch_update_rest(a, p->n_rest, p->rest_rows, *upd, stream));
    return HCSPMM_OK;
}

}  // namespace hcspmm

using namespace hcspmm;

// ---- scratch of the entry point that allocates nothing ------------------------------------------
// One array per GPU, part of the library's device image: it exists from the moment the library is loaded
// on a device until the process ends.  `scratch` itself is only the host-side handle of the symbol; the
// array's device address is looked up once per device and kept in g_scratch_ptr.
constexpr size_t kStaticScratchBytes = HCSPMM_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static char* g_scratch_ptr[kMaxDevices] = {};

// device address of the current GPU's copy of the array; the current device must be the plan's
static hcspmm_status static_scratch_ptr(const hcspmm_plan* plan, char** out)
{
    int dev = -1;
    HC_HIP(hipGetDevice(&dev));
    if (dev != plan->device) { set_error("the current device (%d) is not the plan's (%d)", dev, plan->device); return HCSPMM_EINVAL; }
    if (dev < 0 || dev >= kMaxDevices) { set_error("device index %d is beyond the %d devices supported", dev, kMaxDevices); return HCSPMM_EUNSUPPORTED; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        HC_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) { set_error("hipGetSymbolAddress returned no address for the static scratch array"); return HCSPMM_EHIP; }
        g_scratch_ptr[dev] = static_cast<char*>(ptr);
    }
    *out = g_scratch_ptr[dev];
    return HCSPMM_OK;
}

// everything of a plan that does not depend on the matrix's entries
static hcspmm_status init_plan_header(hcspmm_plan* p, int32_t n_rows, int32_t n_cols, int64_t nnz, const int32_t* d_rowptr,
                                      const int32_t* d_colind, const float* d_vals, const hcspmm_options& o)
{
    memset(p, 0, sizeof *p);
    p->H = kH; p->n_rows = n_rows; p->n_cols = n_cols; p->nnz = nnz;
    p->W = (int32_t)(((int64_t)n_rows + kH - 1) / kH);
    p->rowptr = d_rowptr; p->colind = d_colind; p->vals = d_vals;
    p->opt = o;
    p->mid_row = kMidRow;
    p->long_row = kLongRow;
    // tuning knobs for experiments (not part of the ABI): override the row-tier thresholds
    if (tune().mid_row >= 1) p->mid_row = tune().mid_row;
    if (tune().long_row >= p->mid_row) p->long_row = tune().long_row;
    if (p->long_row < p->mid_row) p->long_row = p->mid_row;
    p->fused_mid_row = kFusedMidRow < p->mid_row ? p->mid_row : (kFusedMidRow > p->long_row ? p->long_row : kFusedMidRow);
    p->slice_cols = kSliceCols;
    if (tune().slice_cols >= kKcBig) p->slice_cols = tune().slice_cols / kKcBig * kKcBig;
    if (o.use_custom_selector) {
        for (int i = 0; i < 3; ++i) {
            if (o.sel_coef[i] <= -((int64_t)1 << 40) || o.sel_coef[i] >= ((int64_t)1 << 40)) {
                set_error("selector coefficients must be below 2^40 in magnitude");
                return HCSPMM_EINVAL;
            }
            p->coef[i] = o.sel_coef[i];
        }
    } else {
        lookup_selector(o.mfma_dtype, o.d_hint, nnz, p->coef);
    }
    if (hipGetDevice(&p->device) != hipSuccess) { (void)hipGetLastError(); set_error("hipGetDevice failed"); return HCSPMM_EHIP; }
    // set-up of hcspmm_spmm_noalloc: this device's address of the static scratch array, looked up once per device
    char* unused = nullptr;
    return static_scratch_ptr(p, &unused);
}

// side streams (default priority) and events for running the paths side by side; optional
// (the fork/join costs ~20 us of launch latency, so only matrices with milliseconds of work use them)
constexpr int64_t kSideStreamNnz = 16000000;
static void setup_side_streams(hcspmm_plan* p)
{
    if (p->side_ok || p->side[0]) return;
    p->side_ok = 0;
    if (p->n_mfma > 0 && p->n_mfma < p->W && p->nnz >= (tune().side_nnz >= 0 ? tune().side_nnz : kSideStreamNnz) && !tune().serial) {
        bool ok = hipStreamCreateWithFlags(&p->side[0], hipStreamNonBlocking) == hipSuccess;
        ok = ok && hipStreamCreateWithFlags(&p->side[1], hipStreamNonBlocking) == hipSuccess;
        ok = ok && hipEventCreateWithFlags(&p->ev_fork, hipEventDisableTiming) == hipSuccess;
        ok = ok && hipEventCreateWithFlags(&p->ev_join[0], hipEventDisableTiming) == hipSuccess;
        ok = ok && hipEventCreateWithFlags(&p->ev_join[1], hipEventDisableTiming) == hipSuccess;
        if (!ok) (void)hipGetLastError();
        p->side_ok = ok ? 1 : 0;
    }
}

extern "C" {

void hcspmm_default_options(hcspmm_options* opt)
{
    if (!opt) return;
    memset(opt, 0, sizeof *opt);
    opt->struct_size = (int32_t)sizeof *opt;
    opt->window_rows = kH;
    opt->route_mode = HCSPMM_ROUTE_HYBRID;
    opt->mfma_dtype = HCSPMM_F32;
    opt->d_hint = 0;
    opt->use_custom_selector = 0;
}

hcspmm_status hcspmm_default_selector(int32_t mfma_dtype, int32_t d_hint, int64_t nnz, int64_t* coef)
{
    if (!coef) { set_error("coef is NULL"); return HCSPMM_EINVAL; }
    if (nnz < 0) { set_error("nnz is negative"); return HCSPMM_EINVAL; }
    if (!lookup_selector(mfma_dtype, d_hint, nnz, coef)) { set_error("unknown mfma_dtype %d", mfma_dtype); return HCSPMM_EINVAL; }
    return HCSPMM_OK;
}

hcspmm_status hcspmm_prepare(int32_t n_rows, int32_t n_cols, int64_t nnz, const int32_t* d_rowptr,
                             const int32_t* d_colind, const float* d_vals, const hcspmm_options* opt, void* stream,
                             hcspmm_plan** out_plan)
{
    if (!out_plan) { set_error("out_plan is NULL"); return HCSPMM_EINVAL; }
    *out_plan = nullptr;
    if (n_rows < 0 || n_cols < 1 || nnz < 0) { set_error("negative size or n_cols < 1"); return HCSPMM_EINVAL; }
    if (n_cols >= (1 << 27)) { set_error("n_cols must be below 2^27"); return HCSPMM_EUNSUPPORTED; }
    if (nnz >= ((int64_t)1 << 31)) { set_error("nnz must be below 2^31"); return HCSPMM_EUNSUPPORTED; }
    if (!d_rowptr || (nnz > 0 && (!d_colind || !d_vals))) { set_error("NULL CSR array"); return HCSPMM_EINVAL; }
    hcspmm_options o;
    hcspmm_default_options(&o);
    if (opt) {
        if (opt->struct_size != (int32_t)sizeof(hcspmm_options)) { set_error("options.struct_size mismatch"); return HCSPMM_EINVAL; }
        o = *opt;
    }
    if (o.window_rows != kH) { set_error("only window_rows = 16 is implemented"); return HCSPMM_EUNSUPPORTED; }
    if (o.route_mode < 0 || o.route_mode > 3) { set_error("bad route_mode"); return HCSPMM_EINVAL; }
    if (o.mfma_dtype < 0 || o.mfma_dtype > 2) { set_error("bad mfma_dtype"); return HCSPMM_EINVAL; }
    if (o.d_hint < 0) { set_error("bad d_hint"); return HCSPMM_EINVAL; }
    if (o.update_fusion < 0 || o.update_fusion > 2) { set_error("bad update_fusion"); return HCSPMM_EINVAL; }
    if (o.matrix_kernels < 0 || o.matrix_kernels > 2) { set_error("bad matrix_kernels"); return HCSPMM_EINVAL; }
    hcspmm_plan* p = new (std::nothrow) hcspmm_plan();
    if (!p) { set_error("host allocation failed"); return HCSPMM_EALLOC; }
    hcspmm_status st = init_plan_header(p, n_rows, n_cols, nnz, d_rowptr, d_colind, d_vals, o);
    if (st != HCSPMM_OK) { delete p; return st; }
    st = build_plan(p, static_cast<hipStream_t>(stream));
    if (st != HCSPMM_OK) { delete p; return st; }
    setup_side_streams(p);
    *out_plan = p;
    return HCSPMM_OK;
}

hcspmm_status hcspmm_plan_update(hcspmm_plan* plan, int64_t nnz, const int32_t* d_rowptr, const int32_t* d_colind,
                                 const float* d_vals, const int32_t* h_changed_rows, int32_t n_changed, void* stream)
{
    if (!plan) { set_error("plan is NULL"); return HCSPMM_EINVAL; }
    if (nnz < 0 || n_changed < 0 || (n_changed > 0 && !h_changed_rows)) { set_error("negative size or NULL row list"); return HCSPMM_EINVAL; }
    if (nnz >= ((int64_t)1 << 31)) { set_error("nnz must be below 2^31"); return HCSPMM_EUNSUPPORTED; }
    if (!d_rowptr || (nnz > 0 && (!d_colind || !d_vals))) { set_error("NULL CSR array"); return HCSPMM_EINVAL; }
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the windows that hold a changed row, ascending and distinct
    std::vector<int32_t> touched;
    {
        std::vector<uint8_t> mark((size_t)plan->W, 0);
        for (int32_t i = 0; i < n_changed; ++i) {
            const int32_t r = h_changed_rows[i];
            if (r < 0 || r >= plan->n_rows) { set_error("changed row %d is outside the matrix", r); return HCSPMM_EINVAL; }
            mark[(size_t)(r / kH)] = 1;
        }
        for (int32_t w = 0; w < plan->W; ++w)
            if (mark[(size_t)w]) touched.push_back(w);
    }
    HC_HIP(hipStreamSynchronize(s));                             // calls that still use the old arrays are done
    hcspmm_plan fresh;
    hcspmm_status st = init_plan_header(&fresh, plan->n_rows, plan->n_cols, nnz, d_rowptr, d_colind, d_vals, plan->opt);
    if (st != HCSPMM_OK) return st;
    // a plan that is updated keeps the device blocks of its updates (see BlockCache)
    if (!plan->cache) plan->cache = new (std::nothrow) BlockCache;
    fresh.cache = plan->cache;
    int32_t* d_touched = nullptr;
    size_t touched_bytes = 0;
    PlanCarry carry{plan->ncols, nullptr, (int32_t)touched.size()};
    // The counts of untouched windows are carried over whenever the old plan has them and fewer than an eighth of
    // the windows changed (beyond that the list-driven passes cost as much as the plain ones); otherwise this is a
    // preparation from scratch.
    const bool incremental = plan->features_complete && plan->nnz > 0 && !touched.empty() && 8 * (int64_t)touched.size() < plan->W &&
                             !(plan->opt.route_mode == HCSPMM_ROUTE_ALL_CSR);
    if (incremental) {
        touched_bytes = touched.size() * sizeof(int32_t);
        if (plan->cache) d_touched = static_cast<int32_t*>(plan->cache->take(touched_bytes, &touched_bytes));
        if (!d_touched && hipMalloc((void**)&d_touched, touched_bytes) != hipSuccess) {
            (void)hipGetLastError(); set_error("device allocation failed"); return HCSPMM_EALLOC;
        }
        if (hipMemcpyAsync(d_touched, touched.data(), touched.size() * sizeof(int32_t), hipMemcpyHostToDevice, s) != hipSuccess) {
            (void)hipGetLastError(); (void)hipFree(d_touched); set_error("copy of the window list failed"); return HCSPMM_EHIP;
        }
        carry.touched = d_touched;
        // (a plan with an unsorted row somewhere does not say where: its structure is not carried)
        if (plan->n_mfma > 0 && plan->erc && plan->wcols && plan->rows_sorted) {
            carry.old_route = plan->route; carry.old_wptr = plan->wptr; carry.old_nnzw = plan->nnzw;
            carry.old_wcols = plan->wcols; carry.old_erc = plan->erc;
        }
    }
    const bool nothing_changed = touched.empty() && nnz == plan->nnz && plan->features_complete;
    if (nothing_changed) {
        // same structure: only the borrowed pointers move
        plan->rowptr = d_rowptr; plan->colind = d_colind; plan->vals = d_vals;
        return HCSPMM_OK;
    }
    st = build_plan(&fresh, s, incremental ? &carry : nullptr);
    if (d_touched) {
        if (plan->cache) plan->cache->give(d_touched, touched_bytes);
        else (void)hipFree(d_touched);
    }
    if (st != HCSPMM_OK) return st;                              // the old plan is untouched and still valid for the old arrays
    // the new tables replace the old ones; streams, events and the lazily sized scratch buffers stay
    fresh.partial = plan->partial; fresh.partial_elems = plan->partial_elems;
    fresh.tile_partial = plan->tile_partial; fresh.tile_partial_elems = plan->tile_partial_elems;
    plan->partial = nullptr; plan->tile_partial = nullptr;
    free_plan_arrays(plan);
    fresh.side_ok = plan->side_ok;
    fresh.side[0] = plan->side[0]; fresh.side[1] = plan->side[1];
    fresh.ev_fork = plan->ev_fork; fresh.ev_join[0] = plan->ev_join[0]; fresh.ev_join[1] = plan->ev_join[1];
    *plan = fresh;
    setup_side_streams(plan);
    if (plan->cache) plan->cache->end_of_update();
    return HCSPMM_OK;
}

hcspmm_status hcspmm_plan_info(const hcspmm_plan* p, hcspmm_plan_info_t* info)
{
    if (!p || !info) { set_error("NULL argument"); return HCSPMM_EINVAL; }
    if (!p->features_complete) {
        const hcspmm_status st = complete_condensed(const_cast<hcspmm_plan*>(p), true);
        if (st != HCSPMM_OK) return st;
    }
    memset(info, 0, sizeof *info);
    info->window_rows = p->H; info->n_rows = p->n_rows; info->n_cols = p->n_cols; info->nnz = p->nnz;
    info->n_windows = p->W; info->total_ncols = p->total_ncols;
    info->n_mfma_windows = p->n_mfma; info->n_csr_windows = p->n_csr; info->nnz_mfma = p->nnz_mfma;
    info->route_mode = p->opt.route_mode; info->mfma_dtype = p->opt.mfma_dtype; info->d_hint = p->opt.d_hint;
    for (int i = 0; i < 3; ++i) info->sel_coef[i] = p->coef[i];
    info->device_bytes = p->device_bytes + (p->partial_elems + p->tile_partial_elems) * (int64_t)sizeof(float);
    info->n_short_rows = p->n_short; info->n_long_rows = p->n_long_rows; info->n_segments = p->n_segs;
    info->n_mid_rows = p->n_mid;
    info->nnz_long = p->nnz_long; info->n_mfma_small = p->n_mfma_small;
    info->n_mfma_big = p->n_mfma_mid + p->n_mfma_big;
    info->n_runs = p->runs_ok ? p->n_runs : 0;
    info->n_run_slices = p->runs_ok ? p->n_run_slices : 0;
    info->run_union_cols = p->runs_ok ? p->run_union_cols : 0;
    return HCSPMM_OK;
}

hcspmm_status hcspmm_plan_export(const hcspmm_plan* p, int32_t* ncols, int32_t* nnzw, uint8_t* route, int64_t* wptr,
                                 int32_t* wcols, int32_t* ecol, int32_t* mfma_windows, int32_t* csr_windows)
{
    if (!p) { set_error("plan is NULL"); return HCSPMM_EINVAL; }
    HC_HIP(hipDeviceSynchronize());
    if (!p->features_complete || ((wcols || ecol) && !p->condensed_complete)) {
        const hcspmm_status st = complete_condensed(const_cast<hcspmm_plan*>(p), !(wcols || ecol));
        if (st != HCSPMM_OK) return st;
    }
    const size_t W = (size_t)p->W;
    if (ncols && W) HC_HIP(hipMemcpy(ncols, p->ncols, W * 4, hipMemcpyDeviceToHost));
    if (nnzw && W) HC_HIP(hipMemcpy(nnzw, p->nnzw, W * 4, hipMemcpyDeviceToHost));
    if (route && W) HC_HIP(hipMemcpy(route, p->route, W, hipMemcpyDeviceToHost));
    if (wptr) HC_HIP(hipMemcpy(wptr, p->wptr, (W + 1) * 8, hipMemcpyDeviceToHost));
    if (wcols && p->total_ncols) HC_HIP(hipMemcpy(wcols, p->wcols, (size_t)p->total_ncols * 4, hipMemcpyDeviceToHost));
    if (ecol && p->nnz) {
        HC_HIP(hipMemcpy(ecol, p->erc, (size_t)p->nnz * 4, hipMemcpyDeviceToHost));
        for (int64_t k = 0; k < p->nnz; ++k) ecol[k] >>= 4;    // drop the packed row-in-window
    }
    if (mfma_windows && p->n_mfma) HC_HIP(hipMemcpy(mfma_windows, p->mfma_windows, (size_t)p->n_mfma * 4, hipMemcpyDeviceToHost));
    if (csr_windows && p->n_csr) HC_HIP(hipMemcpy(csr_windows, p->csr_windows, (size_t)p->n_csr * 4, hipMemcpyDeviceToHost));
    return HCSPMM_OK;
}

hcspmm_status hcspmm_plan_export_runs(const hcspmm_plan* p, int32_t* run_nu, int32_t* ucols, int32_t* wslot)
{
    if (!p) { set_error("plan is NULL"); return HCSPMM_EINVAL; }
    if (!p->runs_ok) { set_error("the plan has no run table (prepare with matrix_kernels = HCSPMM_MATRIX_RUNS)"); return HCSPMM_EINVAL; }
    HC_HIP(hipDeviceSynchronize());
    std::vector<RunDesc> h_runs((size_t)p->n_runs);
    HC_HIP(hipMemcpy(h_runs.data(), p->runs, h_runs.size() * sizeof(RunDesc), hipMemcpyDeviceToHost));
    int64_t at = 0;
    for (const RunDesc& r : h_runs) {
        if (run_nu) run_nu[&r - h_runs.data()] = r.nu;
        if (ucols && r.nu > 0) HC_HIP(hipMemcpy(ucols + at, p->ucols + r.up, (size_t)r.nu * sizeof(int32_t), hipMemcpyDeviceToHost));
        at += r.nu;
    }
    if (wslot && p->total_ncols > 0) HC_HIP(hipMemcpy(wslot, p->wslot, (size_t)p->total_ncols * sizeof(int32_t), hipMemcpyDeviceToHost));
    return HCSPMM_OK;
}

static hcspmm_status check_dense(const char* name, const void* ptr, int64_t ld, int32_t width)
{
    if (!ptr) { set_error("%s is NULL", name); return HCSPMM_EINVAL; }
    if (ld < width) { set_error("leading dimension of %s (%lld) is smaller than its width (%d)", name, (long long)ld, width); return HCSPMM_EINVAL; }
    return HCSPMM_OK;
}

static hcspmm_status spmm_impl(const hcspmm_plan* plan, const void* d_X, int64_t ldx, int32_t d, int32_t x_dtype,
                               void* d_Y, int64_t ldy, int32_t y_dtype, void* stream, hipEvent_t* ev,
                               bool static_scratch = false);

hcspmm_status hcspmm_spmm(const hcspmm_plan* plan, const void* d_X, int64_t ldx, int32_t d, int32_t x_dtype, void* d_Y,
                          int64_t ldy, int32_t y_dtype, void* stream)
{
    return spmm_impl(plan, d_X, ldx, d, x_dtype, d_Y, ldy, y_dtype, stream, nullptr);
}

hcspmm_status hcspmm_spmm_timed(const hcspmm_plan* plan, const void* d_X, int64_t ldx, int32_t d, int32_t x_dtype,
                                void* d_Y, int64_t ldy, int32_t y_dtype, void* stream, hcspmm_stage_times* times)
{
    if (!times) { set_error("times is NULL"); return HCSPMM_EINVAL; }
    memset(times, 0, sizeof *times);
    hipEvent_t ev[5];
    int made = 0;
    hcspmm_status st = HCSPMM_OK;
    for (; made < 5; ++made)
        if (hipEventCreate(&ev[made]) != hipSuccess) { (void)hipGetLastError(); set_error("hipEventCreate failed"); st = HCSPMM_EHIP; break; }
    if (st == HCSPMM_OK) st = spmm_impl(plan, d_X, ldx, d, x_dtype, d_Y, ldy, y_dtype, stream, ev);
    if (st == HCSPMM_OK && plan->n_rows > 0) {
        if (hipEventSynchronize(ev[4]) != hipSuccess) { (void)hipGetLastError(); set_error("hipEventSynchronize failed"); st = HCSPMM_EHIP; }
        else {
            float* out[4] = {&times->ms_mfma_big, &times->ms_mfma_small, &times->ms_csr, &times->ms_csr_reduce};
            for (int i = 0; i < 4; ++i) (void)hipEventElapsedTime(out[i], ev[i], ev[i + 1]);
            (void)hipEventElapsedTime(&times->ms_total, ev[0], ev[4]);
        }
    }
    for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
    return st;
}

static hcspmm_status spmm_impl(const hcspmm_plan* plan, const void* d_X, int64_t ldx, int32_t d, int32_t x_dtype,
                               void* d_Y, int64_t ldy, int32_t y_dtype, void* stream, hipEvent_t* ev, bool static_scratch)
{
    if (!plan) { set_error("plan is NULL"); return HCSPMM_EINVAL; }
    if (d < 1 || d > (1 << 20)) { set_error("d must be in [1, 2^20]"); return HCSPMM_EINVAL; }
    if (x_dtype < 0 || x_dtype > 2 || y_dtype < 0 || y_dtype > 2) { set_error("bad dtype"); return HCSPMM_EINVAL; }
    if (plan->n_rows == 0) return HCSPMM_OK;
    hcspmm_status st;
    if ((st = check_dense("X", d_X, ldx, d)) != HCSPMM_OK) return st;
    if ((st = check_dense("Y", d_Y, ldy, d)) != HCSPMM_OK) return st;
    SpmmArgs a{};
    a.n_rows = plan->n_rows; a.rowptr = plan->rowptr; a.colind = plan->colind; a.vals = plan->vals;
    a.X = d_X; a.ldx = ldx; a.d = d; a.x_dtype = x_dtype; a.Y = static_cast<float*>(d_Y); a.ldy = ldy; a.relu = 0;
    a.y_dtype = y_dtype;
    if (plan->n_mfma > 0 && !mfma_shape_supported(a)) {
        set_error("16-bit X on the matrix path needs d, ldx and ldy to be multiples of 4 and 8-byte aligned X, 16-byte aligned Y");
        return HCSPMM_EUNSUPPORTED;
    }
    char* scratch_mem = nullptr;
    if (static_scratch) {
        const size_t need = spmm_scratch_bytes(plan, d, nullptr);
        if (need > kStaticScratchBytes) {
            set_error("this plan needs %zu bytes of scratch at d = %d, the static scratch array holds %zu; use hcspmm_spmm",
                      need, d, kStaticScratchBytes);
            return HCSPMM_EUNSUPPORTED;
        }
        if ((st = static_scratch_ptr(plan, &scratch_mem)) != HCSPMM_OK) return st;
    }
    return run_spmm(plan, a, static_cast<hipStream_t>(stream), ev, nullptr, scratch_mem);
}

hcspmm_status hcspmm_spmm_noalloc(const hcspmm_plan* plan, const void* d_X, int64_t ldx, int32_t d, int32_t x_dtype,
                                  void* d_Y, int64_t ldy, int32_t y_dtype, void* stream)
{
    return spmm_impl(plan, d_X, ldx, d, x_dtype, d_Y, ldy, y_dtype, stream, nullptr, true);
}

size_t hcspmm_spmm_noalloc_scratch_limit(void) { return kStaticScratchBytes; }

size_t hcspmm_gcn_workspace_bytes(const hcspmm_plan* plan, int32_t d_in, int32_t d_out)
{
    (void)d_in;
    if (!plan || d_out < 1) return 0;
    size_t b = (size_t)plan->n_cols * (size_t)d_out * sizeof(float);
    return (b + 255) & ~(size_t)255;
}

hcspmm_status hcspmm_gemm_f32(int64_t m, int32_t k, int32_t n, const float* d_X, int64_t ldx, const float* d_W,
                              int64_t ldw, float* d_T, int64_t ldt, void* stream)
{
    if (m < 0 || k < 0 || n < 0) { set_error("negative size"); return HCSPMM_EINVAL; }
    if (m == 0 || n == 0) return HCSPMM_OK;
    hcspmm_status st;
    if (k > 0 && (st = check_dense("X", d_X, ldx, k)) != HCSPMM_OK) return st;
    if (k > 0 && (st = check_dense("W", d_W, ldw, n)) != HCSPMM_OK) return st;
    if ((st = check_dense("T", d_T, ldt, n)) != HCSPMM_OK) return st;
    HC_HIP(launch_gemm_f32(m, k, n, d_X, ldx, d_W, ldw, d_T, ldt, 0, static_cast<hipStream_t>(stream)));
    return HCSPMM_OK;
}

hcspmm_status hcspmm_gcn_layer(const hcspmm_plan* plan, const void* d_X, int64_t ldx, int32_t d_in, const void* d_W,
                               int64_t ldw, int32_t d_out, void* d_Y, int64_t ldy, int32_t apply_relu,
                               void* d_workspace, size_t workspace_bytes, void* stream)
{
    return hcspmm_gcn_layer_ex(plan, d_X, ldx, d_in, d_W, ldw, d_out, d_Y, ldy, HCSPMM_F32, apply_relu, HCSPMM_F32, d_workspace,
                               workspace_bytes, stream);
}

hcspmm_status hcspmm_gcn_layer_ex(const hcspmm_plan* plan, const void* d_X, int64_t ldx, int32_t d_in, const void* d_W,
                                  int64_t ldw, int32_t d_out, void* d_Y, int64_t ldy, int32_t y_dtype, int32_t apply_relu,
                                  int32_t t_dtype, void* d_workspace, size_t workspace_bytes, void* stream)
{
    if (!plan) { set_error("plan is NULL"); return HCSPMM_EINVAL; }
    if (y_dtype != HCSPMM_F32 && y_dtype != HCSPMM_BF16 && y_dtype != HCSPMM_F16) { set_error("y_dtype %d is not a dtype code", y_dtype); return HCSPMM_EINVAL; }
    if (d_in < 1 || d_out < 1 || d_in > (1 << 20) || d_out > (1 << 20)) { set_error("d_in, d_out must be in [1, 2^20]"); return HCSPMM_EINVAL; }
    if (t_dtype != HCSPMM_F32 && t_dtype != HCSPMM_BF16 && t_dtype != HCSPMM_F16) { set_error("t_dtype %d is not a dtype code", t_dtype); return HCSPMM_EINVAL; }
    hcspmm_status st;
    if ((st = check_dense("X", d_X, ldx, d_in)) != HCSPMM_OK) return st;
    if ((st = check_dense("W", d_W, ldw, d_out)) != HCSPMM_OK) return st;
    if ((st = check_dense("Y", d_Y, ldy, d_out)) != HCSPMM_OK) return st;
    const size_t need = hcspmm_gcn_workspace_bytes(plan, d_in, d_out);      // sized for fp32 T; 16-bit T uses half of it
    if (!d_workspace || workspace_bytes < need) { set_error("workspace too small: need %zu bytes", need); return HCSPMM_EINVAL; }
    if (((uintptr_t)d_workspace & 255) != 0) { set_error("workspace must be 256-byte aligned"); return HCSPMM_EINVAL; }
    hipStream_t s = static_cast<hipStream_t>(stream);
    SpmmArgs a{};
    a.n_rows = plan->n_rows; a.rowptr = plan->rowptr; a.colind = plan->colind; a.vals = plan->vals;
    a.X = d_workspace; a.ldx = d_out; a.d = d_out; a.x_dtype = t_dtype; a.Y = static_cast<float*>(d_Y); a.ldy = ldy;
    a.relu = apply_relu ? 1 : 0;
    a.y_dtype = y_dtype;
    if (t_dtype != HCSPMM_F32 && plan->n_mfma > 0 && !mfma_shape_supported(a)) {
        set_error("the matrix path with 16-bit T needs d_out a multiple of 4 and 16-byte aligned Y rows");
        return HCSPMM_EUNSUPPORTED;
    }
    HC_HIP(launch_gemm_f32_out(plan->n_cols, d_in, d_out, static_cast<const float*>(d_X), ldx,
                               static_cast<const float*>(d_W), ldw, d_workspace, d_out, t_dtype, 0, s));
    if (plan->n_rows == 0) return HCSPMM_OK;
    return run_spmm(plan, a, s);
}

// Where the separate update runs through the streaming 16-row kernel (narrow W, aggregated width 64 or 128) it
// measured 4-23 % ahead of the fused update on graphs large enough not to be launch-bound; everywhere else
// (aggregated width up to 32 or of 256, wide W, small graphs) the fused kernels are level or ahead.
static bool split_update_faster(int64_t n_rows, int32_t agg_width, int32_t out_width, const float* Z)
{
    return n_rows >= 32768 && agg_width > 32 && gemm_rows16_usable(n_rows, agg_width, out_width, Z, agg_width);
}

size_t hcspmm_aggregate_update_workspace_bytes(const hcspmm_plan* plan, int32_t d_in, int32_t d_out)
{
    (void)d_out;
    if (!plan || d_in < 1) return 0;
    size_t b = (size_t)plan->n_rows * (size_t)d_in * sizeof(float);
    return (b + 255) & ~(size_t)255;
}

hcspmm_status hcspmm_aggregate_update(const hcspmm_plan* plan, const void* d_X, int64_t ldx, int32_t d_in,
                                      int32_t x_dtype, const void* d_W, int64_t ldw, int32_t d_out, void* d_Y,
                                      int64_t ldy, int32_t y_dtype, int32_t apply_relu, void* d_workspace,
                                      size_t workspace_bytes, void* stream)
{
    if (!plan) { set_error("plan is NULL"); return HCSPMM_EINVAL; }
    if (y_dtype != HCSPMM_F32 && y_dtype != HCSPMM_BF16 && y_dtype != HCSPMM_F16) { set_error("y_dtype %d is not a dtype code", y_dtype); return HCSPMM_EINVAL; }
    if (d_in < 1 || d_out < 1 || d_in > (1 << 20) || d_out > (1 << 20)) { set_error("d_in, d_out must be in [1, 2^20]"); return HCSPMM_EINVAL; }
    if (x_dtype != HCSPMM_F32 && x_dtype != HCSPMM_BF16 && x_dtype != HCSPMM_F16) { set_error("x_dtype %d is not a dtype code", x_dtype); return HCSPMM_EINVAL; }
    hcspmm_status st;
    if ((st = check_dense("X", d_X, ldx, d_in)) != HCSPMM_OK) return st;
    if ((st = check_dense("W", d_W, ldw, d_out)) != HCSPMM_OK) return st;
    if ((st = check_dense("Y", d_Y, ldy, d_out)) != HCSPMM_OK) return st;
    const size_t need = hcspmm_aggregate_update_workspace_bytes(plan, d_in, d_out);
    if (!d_workspace || workspace_bytes < need) { set_error("workspace too small: need %zu bytes", need); return HCSPMM_EINVAL; }
    if (((uintptr_t)d_workspace & 255) != 0) { set_error("workspace must be 256-byte aligned"); return HCSPMM_EINVAL; }
    if (plan->n_rows == 0) return HCSPMM_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* Z = static_cast<float*>(d_workspace);
    SpmmArgs a{};
    a.n_rows = plan->n_rows; a.rowptr = plan->rowptr; a.colind = plan->colind; a.vals = plan->vals;
    a.X = d_X; a.ldx = ldx; a.d = d_in; a.x_dtype = x_dtype; a.Y = Z; a.ldy = d_in; a.relu = 0;
    // The fused update pays where most rows can keep their tile on chip; rows that go through the
    // workspace anyway (wide matrix-path windows, mid and long rows) are finished 16 at a time, which
    // a plain GEMM does better once they are a large share of the matrix.
    const bool worth = (4 * (int64_t)plan->n_rest < plan->n_rows &&
                        !(x_dtype == HCSPMM_F32 && split_update_faster(plan->n_rows, d_in, d_out, Z))) ||
                       plan->opt.update_fusion == HCSPMM_UPDATE_FUSED;
    if (update_fusable(a) && worth && plan->opt.update_fusion != HCSPMM_UPDATE_SPLIT) {
        const UpdateArgs u{static_cast<const float*>(d_W), ldw, d_out, static_cast<float*>(d_Y), ldy, apply_relu ? 1 : 0, 0,
                           nullptr, 0, y_dtype};
        return run_spmm(plan, a, s, nullptr, &u);
    }
    if ((st = run_spmm(plan, a, s)) != HCSPMM_OK) return st;
    HC_HIP(launch_gemm_f32_out(plan->n_rows, d_in, d_out, Z, d_in, static_cast<const float*>(d_W), ldw, d_Y, ldy, y_dtype,
                               apply_relu ? 1 : 0, s));
    return HCSPMM_OK;
}

static size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

// workspace of the backward pass: S | masked G | W^T | partial products of dW
struct BackwardLayout { size_t s_off, gm_off, wt_off, part_off, total; };

static BackwardLayout backward_layout(const hcspmm_plan* plan, int32_t d_in, int32_t d_out)
{
    BackwardLayout l;
    l.s_off = 0;
    l.gm_off = l.s_off + align256((size_t)plan->n_rows * d_out * sizeof(float));
    l.wt_off = l.gm_off + align256((size_t)plan->n_cols * d_out * sizeof(float));
    l.part_off = l.wt_off + align256((size_t)d_in * d_out * sizeof(float));
    l.total = l.part_off + align256((size_t)gemm_tn_spans(plan->n_rows, d_in, d_out) * d_in * d_out * sizeof(float));
    return l;
}

size_t hcspmm_layer_backward_workspace_bytes(const hcspmm_plan* plan, int32_t d_in, int32_t d_out)
{
    if (!plan || d_in < 1 || d_out < 1) return 0;
    return backward_layout(plan, d_in, d_out).total;
}

hcspmm_status hcspmm_layer_backward(const hcspmm_plan* plan, const void* d_G, int64_t ldg, int32_t d_out,
                                    const void* d_Yfwd, int64_t ldyf, const void* d_X, int64_t ldx, int32_t d_in,
                                    const void* d_W, int64_t ldw, void* d_dX, int64_t lddx, void* d_dW, int64_t lddw,
                                    int32_t mask_dx_by_x, void* d_workspace, size_t workspace_bytes, void* stream)
{
    if (!plan) { set_error("plan is NULL"); return HCSPMM_EINVAL; }
    if (d_in < 1 || d_out < 1 || d_in > (1 << 20) || d_out > (1 << 20)) { set_error("d_in, d_out must be in [1, 2^20]"); return HCSPMM_EINVAL; }
    hcspmm_status st;
    if (mask_dx_by_x && d_dX && (st = check_dense("X", d_X, ldx, d_in)) != HCSPMM_OK) return st;
    if ((st = check_dense("G", d_G, ldg, d_out)) != HCSPMM_OK) return st;
    if (d_Yfwd && (st = check_dense("Yfwd", d_Yfwd, ldyf, d_out)) != HCSPMM_OK) return st;
    if ((st = check_dense("W", d_W, ldw, d_out)) != HCSPMM_OK) return st;
    if (d_dX && (st = check_dense("dX", d_dX, lddx, d_in)) != HCSPMM_OK) return st;
    if (d_dW) {
        if ((st = check_dense("dW", d_dW, lddw, d_out)) != HCSPMM_OK) return st;
        if ((st = check_dense("X", d_X, ldx, d_in)) != HCSPMM_OK) return st;
    }
    const BackwardLayout l = backward_layout(plan, d_in, d_out);
    if (!d_workspace || workspace_bytes < l.total) { set_error("workspace too small: need %zu bytes", l.total); return HCSPMM_EINVAL; }
    if (((uintptr_t)d_workspace & 255) != 0) { set_error("workspace must be 256-byte aligned"); return HCSPMM_EINVAL; }
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(d_workspace);
    float* S = reinterpret_cast<float*>(ws + l.s_off);
    float* Gm = reinterpret_cast<float*>(ws + l.gm_off);
    float* Wt = reinterpret_cast<float*>(ws + l.wt_off);
    float* part = reinterpret_cast<float*>(ws + l.part_off);
    const float* G = static_cast<const float*>(d_G);
    int64_t g_ld = ldg;
    if (d_Yfwd && plan->n_cols > 0) {
        HC_HIP(launch_relu_mask(plan->n_cols, d_out, G, ldg, static_cast<const float*>(d_Yfwd), ldyf, Gm, d_out, s));
        G = Gm;
        g_ld = d_out;
    }
    if (plan->n_rows > 0) {
        SpmmArgs a{};
        a.n_rows = plan->n_rows; a.rowptr = plan->rowptr; a.colind = plan->colind; a.vals = plan->vals;
        a.X = G; a.ldx = g_ld; a.d = d_out; a.x_dtype = HCSPMM_F32; a.Y = S; a.ldy = d_out; a.relu = 0;
        if (d_dX) {
            HC_HIP(launch_transpose(d_in, d_out, static_cast<const float*>(d_W), ldw, Wt, s));
            // as in hcspmm_aggregate_update; when dW needs S in memory as well, the fused kernels store every
            // tile besides multiplying it, which measured faster than the separate GEMM only for narrow S
            const bool worth = (4 * (int64_t)plan->n_rest < plan->n_rows && (!d_dW || d_out <= 32) &&
                                !split_update_faster(plan->n_rows, d_out, d_in, S)) ||
                               plan->opt.update_fusion == HCSPMM_UPDATE_FUSED;
            if (update_fusable(a) && worth && plan->opt.update_fusion != HCSPMM_UPDATE_SPLIT) {
                // the next layer's activation mask (its output is this layer's input X) goes into the update's epilogue
                const UpdateArgs u{Wt, d_in, d_in, static_cast<float*>(d_dX), lddx, 0, d_dW ? 1 : 0,
                                   mask_dx_by_x ? static_cast<const float*>(d_X) : nullptr, ldx};
                if ((st = run_spmm(plan, a, s, nullptr, &u)) != HCSPMM_OK) return st;
            } else {
                if ((st = run_spmm(plan, a, s)) != HCSPMM_OK) return st;
                HC_HIP(launch_gemm_f32(plan->n_rows, d_out, d_in, S, d_out, Wt, d_in, static_cast<float*>(d_dX), lddx, 0, s));
                if (mask_dx_by_x)
                    HC_HIP(launch_relu_mask(plan->n_rows, d_in, static_cast<const float*>(d_dX), lddx,
                                            static_cast<const float*>(d_X), ldx, static_cast<float*>(d_dX), lddx, s));
            }
        } else if ((st = run_spmm(plan, a, s)) != HCSPMM_OK) {
            return st;
        }
    }
    if (d_dW)
        HC_HIP(launch_gemm_tn(plan->n_rows, static_cast<const float*>(d_X), ldx, d_in, S, d_out, d_out,
                              static_cast<float*>(d_dW), lddw, part, s));
    return HCSPMM_OK;
}

size_t hcspmm_probe_gather_out_bytes(int64_t n, int32_t d)
{
    if (n <= 0 || d < 1) return 256;
    return (size_t)probe_gather_blocks(n, d) * 256 * 4 * sizeof(float);
}

hcspmm_status hcspmm_probe_gather(const int32_t* d_index, int64_t n, const float* d_X, int64_t ldx, int32_t d,
                                  int32_t n_rows_x, float* d_out, size_t out_bytes, void* stream)
{
    if (n < 0 || n_rows_x < 1) { set_error("negative n or empty X"); return HCSPMM_EINVAL; }
    if (d < 4 || d > 256 || d % 4 != 0 || ldx % 4 != 0 || ((uintptr_t)d_X & 15) != 0) {
        set_error("the gather probe needs d a multiple of 4 in [4, 256] and 16-byte aligned X rows");
        return HCSPMM_EUNSUPPORTED;
    }
    hcspmm_status st;
    if ((st = check_dense("X", d_X, ldx, d)) != HCSPMM_OK) return st;
    if (n == 0) return HCSPMM_OK;
    if (!d_index || !d_out) { set_error("NULL argument"); return HCSPMM_EINVAL; }
    if (out_bytes < hcspmm_probe_gather_out_bytes(n, d)) { set_error("out buffer too small: need %zu bytes", hcspmm_probe_gather_out_bytes(n, d)); return HCSPMM_EINVAL; }
    if (((uintptr_t)d_out & 15) != 0) { set_error("out must be 16-byte aligned"); return HCSPMM_EINVAL; }
    HC_HIP(launch_probe_gather(d_index, n, d_X, ldx, d, n_rows_x, d_out, static_cast<hipStream_t>(stream)));
    return HCSPMM_OK;
}

hcspmm_status hcspmm_plan_set_update_fusion(hcspmm_plan* plan, int32_t update_fusion)
{
    if (!plan) { set_error("plan is NULL"); return HCSPMM_EINVAL; }
    if (update_fusion < 0 || update_fusion > 2) { set_error("bad update_fusion"); return HCSPMM_EINVAL; }
    plan->opt.update_fusion = update_fusion;
    return HCSPMM_OK;
}

void hcspmm_plan_destroy(hcspmm_plan* plan)
{
    if (!plan) return;
    (void)hipDeviceSynchronize();
    if (plan->side[0]) (void)hipStreamDestroy(plan->side[0]);
    if (plan->side[1]) (void)hipStreamDestroy(plan->side[1]);
    if (plan->ev_fork) (void)hipEventDestroy(plan->ev_fork);
    if (plan->ev_join[0]) (void)hipEventDestroy(plan->ev_join[0]);
    if (plan->ev_join[1]) (void)hipEventDestroy(plan->ev_join[1]);
    free_plan_arrays(plan);
    if (plan->cache) { plan->cache->clear(); delete plan->cache; }
    delete plan;
}

const char* hcspmm_status_string(hcspmm_status s)
{
    switch (s) {
        case HCSPMM_OK: return "ok";
        case HCSPMM_EINVAL: return "invalid argument";
        case HCSPMM_EBADCSR: return "invalid CSR";
        case HCSPMM_EALLOC: return "allocation failed";
        case HCSPMM_EHIP: return "HIP runtime error";
        case HCSPMM_EUNSUPPORTED: return "unsupported";
    }
    return "unknown status";
}

const char* hcspmm_last_error(void) { return g_err; }

int32_t hcspmm_version(void) { return 10100; }

}  // extern "C"
