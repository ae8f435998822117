// Preprocessing kernels: row windows, condensing, window features, selection, launch tables.
//
// Section IV-A: A is cut into windows of 16 rows and each window's non-zero columns are moved to
// the front.  Here "moved to the front" is materialised as (a) the ascending list of the
// window's distinct column ids and (b) for every non-zero the position of its column in that
// list.  Section IV-C: the per-window features (number of non-zero columns, sparsity) feed a
// three-parameter linear model whose sign picks the path; it is evaluated in exact integers.
#include "common.hpp"

namespace hcspmm {

// ------------------------------------------------------------------------------------------------
// block-wide exclusive scan of one int per thread (NT threads, NT a multiple of 64, NT <= 1024)
// ------------------------------------------------------------------------------------------------
template <int NT>
__device__ inline int block_exclusive_scan(int v, int* total, int* smem /* NT/64 + 1 ints */)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int t = __shfl_up(inc, off, 64);
        if (lane >= off) inc += t;
    }
    __syncthreads();                       // smem may still be in use by a previous call
    if (lane == 63) smem[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int i = 0; i < NT / 64; ++i) { int t = smem[i]; smem[i] = run; run += t; }
        smem[NT / 64] = run;
    }
    __syncthreads();
    *total = smem[NT / 64];
    return smem[wave] + inc - v;
}

// ------------------------------------------------------------------------------------------------
// generic device-wide exclusive scan  int32[n] -> int64[n+1]
// ------------------------------------------------------------------------------------------------
constexpr int kScanThreads = 256;
constexpr int kScanItems = 16;
constexpr int kScanTile = kScanThreads * kScanItems;

size_t scan_scratch_elems(int64_t n) { return (size_t)((n + kScanTile - 1) / kScanTile) + 2; }

__global__ __launch_bounds__(kScanThreads) void k_scan_tile_sums(const int32_t* __restrict__ in, int64_t n,
                                                                 int64_t* __restrict__ tile_sums)
{
    __shared__ long long part[kScanThreads / 64];
    const int64_t base = (int64_t)blockIdx.x * kScanTile;
    long long acc = 0;
    for (int i = 0; i < kScanItems; ++i) {
        int64_t idx = base + (int64_t)i * kScanThreads + threadIdx.x;
        if (idx < n) acc += in[idx];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        long long t = 0;
        for (int i = 0; i < kScanThreads / 64; ++i) t += part[i];
        tile_sums[blockIdx.x] = t;
    }
}

// one workgroup walks the tile sums in order (there are at most a few hundred thousand)
__global__ __launch_bounds__(256) void k_scan_tile_offsets(int64_t* __restrict__ tile_sums, int64_t n_tiles)
{
    __shared__ long long wsum[4];
    __shared__ long long carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int64_t base = 0; base < n_tiles; base += 256) {
        int64_t idx = base + threadIdx.x;
        long long v = idx < n_tiles ? tile_sums[idx] : 0;
        long long inc = v;
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            long long t = __shfl_up(inc, off, 64);
            if (lane >= off) inc += t;
        }
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        long long wave_off = 0;
        for (int i = 0; i < wave; ++i) wave_off += wsum[i];
        long long carry = carry_s;
        if (idx < n_tiles) tile_sums[idx] = carry + wave_off + inc - v;
        __syncthreads();
        if (threadIdx.x == 255) carry_s = carry + wave_off + inc;
        __syncthreads();
    }
    if (threadIdx.x == 0) tile_sums[n_tiles] = carry_s;
}

__global__ __launch_bounds__(kScanThreads) void k_scan_apply(const int32_t* __restrict__ in, int64_t n,
                                                             const int64_t* __restrict__ tile_offsets,
                                                             int64_t n_tiles, int64_t* __restrict__ out)
{
    __shared__ int smem[kScanThreads / 64 + 1];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    int v[kScanItems];
    int local = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        int64_t idx = base + i;
        v[i] = idx < n ? in[idx] : 0;
        local += v[i];
    }
    int total;
    // int suffices inside one tile: every array scanned here sums to less than 2^31 overall
    long long off = (long long)block_exclusive_scan<kScanThreads>(local, &total, smem);
    long long run = tile_offsets[blockIdx.x] + off;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        int64_t idx = base + i;
        if (idx < n) out[idx] = run;
        run += v[i];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) out[n] = tile_offsets[n_tiles];
}

hipError_t exclusive_scan_i32_i64(const int32_t* in, int64_t n, int64_t* out, int64_t* scratch, hipStream_t stream)
{
    if (n <= 0) return hipMemsetAsync(out, 0, sizeof(int64_t), stream);
    const int64_t n_tiles = (n + kScanTile - 1) / kScanTile;
    hipLaunchKernelGGL(k_scan_tile_sums, dim3((unsigned)n_tiles), dim3(kScanThreads), 0, stream, in, n, scratch);
    hipLaunchKernelGGL(k_scan_tile_offsets, dim3(1), dim3(256), 0, stream, scratch, n_tiles);
    hipLaunchKernelGGL(k_scan_apply, dim3((unsigned)n_tiles), dim3(kScanThreads), 0, stream, in, n, scratch, n_tiles,
                       out);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// several arrays of one length scanned by one three-kernel sequence (the preprocessing is bound by
// the number of its small launches and read-backs, not by their work)
// ------------------------------------------------------------------------------------------------
size_t scan_multi_scratch_elems(int64_t n) { return (size_t)kScanMaxArrays * scan_scratch_elems(n); }

__global__ __launch_bounds__(kScanThreads) void k_scan_tile_sums_m(ScanMulti m, int64_t n, int64_t stride,
                                                                   int64_t* __restrict__ tile_sums)
{
    __shared__ long long part[kScanThreads / 64];
    const int64_t base = (int64_t)blockIdx.x * kScanTile;
    for (int a = 0; a < m.k; ++a) {
        const int32_t* __restrict__ in = m.in[a];
        long long acc = 0;
        for (int i = 0; i < kScanItems; ++i) {
            const int64_t idx = base + (int64_t)i * kScanThreads + threadIdx.x;
            if (idx < n) acc += in[idx];
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
        __syncthreads();                                        // part[] of the previous array has been read
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
        __syncthreads();
        if (threadIdx.x == 0) {
            long long t = 0;
            for (int i = 0; i < kScanThreads / 64; ++i) t += part[i];
            tile_sums[a * stride + blockIdx.x] = t;
        }
    }
}

// workgroup a walks the tile sums of array a in order; totals[a] receives the array's sum
__global__ __launch_bounds__(256) void k_scan_tile_offsets_m(int64_t* __restrict__ tile_sums_all, int64_t n_tiles,
                                                             int64_t stride, int64_t* __restrict__ totals)
{
    __shared__ long long wsum[4];
    __shared__ long long carry_s;
    int64_t* __restrict__ tile_sums = tile_sums_all + blockIdx.x * stride;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int64_t base = 0; base < n_tiles; base += 256) {
        const int64_t idx = base + threadIdx.x;
        const long long v = idx < n_tiles ? tile_sums[idx] : 0;
        long long inc = v;
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const long long t = __shfl_up(inc, off, 64);
            if (lane >= off) inc += t;
        }
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        long long wave_off = 0;
        for (int i = 0; i < wave; ++i) wave_off += wsum[i];
        const long long carry = carry_s;
        if (idx < n_tiles) tile_sums[idx] = carry + wave_off + inc - v;
        __syncthreads();
        if (threadIdx.x == 255) carry_s = carry + wave_off + inc;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        tile_sums[n_tiles] = carry_s;
        if (totals) totals[blockIdx.x] = carry_s;
    }
}

__global__ __launch_bounds__(kScanThreads) void k_scan_apply_m(ScanMulti m, int64_t n, int64_t stride,
                                                               const int64_t* __restrict__ tile_offsets_all,
                                                               int64_t n_tiles)
{
    __shared__ int smem[kScanThreads / 64 + 1];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    for (int a = 0; a < m.k; ++a) {
        int64_t* __restrict__ out = m.out[a];
        if (!out) continue;                                     // only the total of this array was wanted
        const int32_t* __restrict__ in = m.in[a];
        const int64_t* __restrict__ tile_offsets = tile_offsets_all + a * stride;
        int v[kScanItems];
        int local = 0;
#pragma unroll
        for (int i = 0; i < kScanItems; ++i) {
            const int64_t idx = base + i;
            v[i] = idx < n ? in[idx] : 0;
            local += v[i];
        }
        int total;
        const long long off = (long long)block_exclusive_scan<kScanThreads>(local, &total, smem);
        long long run = tile_offsets[blockIdx.x] + off;
#pragma unroll
        for (int i = 0; i < kScanItems; ++i) {
            const int64_t idx = base + i;
            if (idx < n) out[idx] = run;
            run += v[i];
        }
        if (blockIdx.x == 0 && threadIdx.x == 0) out[n] = tile_offsets[n_tiles];
    }
}

hipError_t exclusive_scan_multi(const ScanMulti& m, int64_t n, int64_t* totals_dev, int64_t* scratch, hipStream_t stream)
{
    if (m.k < 1 || m.k > kScanMaxArrays) return hipErrorInvalidValue;
    if (n <= 0) {
        for (int a = 0; a < m.k; ++a)
            if (m.out[a]) { hipError_t e = hipMemsetAsync(m.out[a], 0, sizeof(int64_t), stream); if (e != hipSuccess) return e; }
        if (totals_dev) return hipMemsetAsync(totals_dev, 0, (size_t)m.k * sizeof(int64_t), stream);
        return hipSuccess;
    }
    const int64_t n_tiles = (n + kScanTile - 1) / kScanTile;
    const int64_t stride = (int64_t)scan_scratch_elems(n);
    hipLaunchKernelGGL(k_scan_tile_sums_m, dim3((unsigned)n_tiles), dim3(kScanThreads), 0, stream, m, n, stride, scratch);
    hipLaunchKernelGGL(k_scan_tile_offsets_m, dim3((unsigned)m.k), dim3(256), 0, stream, scratch, n_tiles, stride, totals_dev);
    hipLaunchKernelGGL(k_scan_apply_m, dim3((unsigned)n_tiles), dim3(kScanThreads), 0, stream, m, n, stride, scratch, n_tiles);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// CSR validation
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_validate_rowptr(int32_t n_rows, int64_t nnz, const int32_t* __restrict__ rowptr,
                                                         int32_t* __restrict__ err)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) {
        if (rowptr[0] != 0) atomicOr(err, 1);
        if ((int64_t)rowptr[n_rows] != nnz) atomicOr(err, 2);
    }
    if (i < n_rows) {
        int32_t a = rowptr[i], b = rowptr[i + 1];
        if (a < 0 || b < a) atomicOr(err, 4);
    }
}

__global__ __launch_bounds__(256) void k_validate_cols(int32_t n_cols, int64_t nnz, const int32_t* __restrict__ colind,
                                                       int32_t* __restrict__ err)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    bool bad = false;
    for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < nnz; k += stride) {
        int32_t c = colind[k];
        bad |= (c < 0 || c >= n_cols);
    }
    if (bad) atomicOr(err, 8);
}

hipError_t launch_validate(int32_t n_rows, int32_t n_cols, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                           int32_t* err_flag, hipStream_t s)
{
    unsigned g = (unsigned)(((int64_t)n_rows + 1 + 255) / 256);
    hipLaunchKernelGGL(k_validate_rowptr, dim3(g), dim3(256), 0, s, n_rows, nnz, rowptr, err_flag);
    if (nnz > 0) {
        int64_t blocks = (nnz + 256 * 8 - 1) / (256 * 8);
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(k_validate_cols, dim3((unsigned)blocks), dim3(256), 0, s, n_cols, nnz, colind, err_flag);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// per-window non-zero count, and the list of windows too large for the LDS sort
// ------------------------------------------------------------------------------------------------
__device__ inline void window_span(int32_t w, int32_t n_rows, const int32_t* __restrict__ rowptr, int32_t& s,
                                   int32_t& e)
{
    int64_t r0 = (int64_t)w * kH;
    int64_t r1 = r0 + kH;
    if (r1 > n_rows) r1 = n_rows;
    s = rowptr[r0];
    e = rowptr[r1];
}

__global__ __launch_bounds__(256) void k_window_nnz(int32_t W, int32_t n_rows, const int32_t* __restrict__ rowptr,
                                                    int32_t* __restrict__ nnzw, int32_t* __restrict__ big_list,
                                                    int32_t* __restrict__ big_count)
{
    int32_t w = blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= W) return;
    int32_t s, e;
    window_span(w, n_rows, rowptr, s, e);
    nnzw[w] = e - s;
    if (e - s > kUniqueSmallCap) big_list[atomicAdd(big_count, 1)] = w;
}

hipError_t launch_window_nnz(int32_t W, int32_t n_rows, const int32_t* rowptr, int32_t* nnzw, int32_t* big_list,
                             int32_t* big_count, hipStream_t s)
{
    hipLaunchKernelGGL(k_window_nnz, dim3((W + 255) / 256), dim3(256), 0, s, W, n_rows, rowptr, nnzw, big_list,
                       big_count);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// condensing, small windows: sort the window's column ids in LDS, keep the distinct ones
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_unique_small(int32_t W, int32_t n_rows, const int32_t* __restrict__ rowptr,
                                                      const int32_t* __restrict__ colind,
                                                      int32_t* __restrict__ tmp_cols, int32_t* __restrict__ ncols,
                                                      const uint8_t* __restrict__ route /* may be null: every window */)
{
    __shared__ int32_t keys[kUniqueSmallCap];
    __shared__ int smem[256 / 64 + 1];
    const int32_t w = blockIdx.x;
    if (route && route[w] == 0) return;          // only the matrix path's windows need the list
    int32_t s, e;
    window_span(w, n_rows, rowptr, s, e);
    const int32_t n = e - s;
    if (n > kUniqueSmallCap) return;             // handled by k_unique_big
    if (n == 0) {
        if (threadIdx.x == 0) ncols[w] = 0;
        return;
    }
    int P = 2;
    while (P < n) P <<= 1;
    for (int i = threadIdx.x; i < P; i += 256) keys[i] = i < n ? colind[s + i] : 0x7fffffff;
    __syncthreads();
    for (int k = 2; k <= P; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < (P >> 1); t += 256) {
                int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                int p = i | j;
                bool up = (i & k) == 0;
                int32_t a = keys[i], b = keys[p];
                if ((a > b) == up) { keys[i] = b; keys[p] = a; }
            }
            __syncthreads();
        }
    }
    // distinct values: thread t owns the contiguous slice [t*ipt, (t+1)*ipt)
    const int ipt = (P + 255) / 256;
    const int lo = threadIdx.x * ipt;
    int cnt = 0;
    for (int i = lo; i < lo + ipt && i < n; ++i) cnt += (i == 0 || keys[i] != keys[i - 1]) ? 1 : 0;
    int total;
    int off = block_exclusive_scan<256>(cnt, &total, smem);
    for (int i = lo; i < lo + ipt && i < n; ++i)
        if (i == 0 || keys[i] != keys[i - 1]) tmp_cols[(int64_t)s + off++] = keys[i];
    if (threadIdx.x == 0) ncols[w] = total;
}

hipError_t launch_unique_small(int32_t W, int32_t n_rows, const int32_t* rowptr, const int32_t* colind,
                               int32_t* tmp_cols, int32_t* ncols, const uint8_t* route, hipStream_t s)
{
    hipLaunchKernelGGL(k_unique_small, dim3(W), dim3(256), 0, s, W, n_rows, rowptr, colind, tmp_cols, ncols, route);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// condensing, large windows: an LDS bitmap over a range of 2^20 columns per pass
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_unique_big(const int32_t* __restrict__ big_list, int32_t n_rows,
                                                     int32_t n_cols, const int32_t* __restrict__ rowptr,
                                                     const int32_t* __restrict__ colind,
                                                     int32_t* __restrict__ tmp_cols, int32_t* __restrict__ ncols,
                                                     const uint8_t* __restrict__ route /* may be null: every listed window */)
{
    __shared__ uint32_t bm[kBitmapWords];
    __shared__ int smem[1024 / 64 + 1];
    constexpr int kBits = kBitmapWords * 32;
    constexpr int kWordsPerThread = kBitmapWords / 1024;
    const int32_t w = big_list[blockIdx.x];
    if (route && route[w] == 0) return;
    int32_t s, e;
    window_span(w, n_rows, rowptr, s, e);
    int32_t running = 0;
    for (int64_t base = 0; base < n_cols; base += kBits) {
        for (int i = threadIdx.x; i < kBitmapWords; i += 1024) bm[i] = 0u;
        __syncthreads();
        for (int32_t k = s + threadIdx.x; k < e; k += 1024) {
            int64_t c = (int64_t)colind[k] - base;
            if (c >= 0 && c < kBits) atomicOr(&bm[c >> 5], 1u << (c & 31));
        }
        __syncthreads();
        const int w0 = threadIdx.x * kWordsPerThread;
        int cnt = 0;
#pragma unroll 4
        for (int i = 0; i < kWordsPerThread; ++i) cnt += __popc(bm[w0 + i]);
        int total;
        int off = block_exclusive_scan<1024>(cnt, &total, smem);
        int32_t* out = tmp_cols + (int64_t)s + running + off;
        for (int i = 0; i < kWordsPerThread; ++i) {
            uint32_t bits = bm[w0 + i];
            while (bits) {
                int b = __ffs(bits) - 1;
                bits &= bits - 1;
                *out++ = (int32_t)(base + (int64_t)(w0 + i) * 32 + b);
            }
        }
        running += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) ncols[w] = running;
}

hipError_t launch_unique_big(int32_t n_big, const int32_t* big_list, int32_t n_rows, int32_t n_cols,
                             const int32_t* rowptr, const int32_t* colind, int32_t* tmp_cols, int32_t* ncols,
                             const uint8_t* route, hipStream_t s)
{
    if (n_big <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_unique_big, dim3(n_big), dim3(1024), 0, s, big_list, n_rows, n_cols, rowptr, colind, tmp_cols,
                       ncols, route);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// window features without the lists: the selector needs only the NUMBER of distinct columns, which
// an LDS hash set gives for a fraction of the sort's cost; the sorted lists are then built for the
// matrix path's windows alone
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_window_classes(int32_t W, int32_t n_rows, const int32_t* __restrict__ rowptr,
                                                        int32_t* __restrict__ nnzw, int32_t* __restrict__ mid_list,
                                                        int32_t* __restrict__ huge_list, int32_t* __restrict__ counts)
{
    int32_t w = blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= W) return;
    int32_t s, e;
    window_span(w, n_rows, rowptr, s, e);
    const int32_t n = e - s;
    nnzw[w] = n;
    if (n > kCountMidCap) huge_list[atomicAdd(counts + 1, 1)] = w;
    else if (n > kUniqueSmallCap) mid_list[atomicAdd(counts, 1)] = w;
}

hipError_t launch_window_classes(int32_t W, int32_t n_rows, const int32_t* rowptr, int32_t* nnzw, int32_t* mid_list,
                                 int32_t* huge_list, int32_t* counts, hipStream_t s)
{
    hipLaunchKernelGGL(k_window_classes, dim3((W + 255) / 256), dim3(256), 0, s, W, n_rows, rowptr, nnzw, mid_list,
                       huge_list, counts);
    return hipGetLastError();
}

// Inserts the window's column ids into an open-addressing set of SLOTS >= 2n entries (linear probing,
// empty = -1; ids are non-negative) and counts the insertions that found an empty slot.  The set is
// never more than half full, so every probe sequence ends.
template <int NT, int SLOTS>
__device__ inline void count_distinct_body(int32_t w, int32_t n_rows, const int32_t* __restrict__ rowptr,
                                           const int32_t* __restrict__ colind, int32_t* __restrict__ ncols,
                                           int32_t* table, int* smem)
{
    int32_t s, e;
    window_span(w, n_rows, rowptr, s, e);
    const int32_t n = e - s;
    if (n == 0) {
        if (threadIdx.x == 0) ncols[w] = 0;
        return;
    }
    int T = NT;                                   // power of two, at least twice the entries
    while (T < 2 * n) T <<= 1;
    const uint32_t mask = (uint32_t)T - 1;
    for (int i = threadIdx.x; i < T; i += NT) table[i] = -1;
    __syncthreads();
    int cnt = 0;
    for (int32_t k = s + threadIdx.x; k < e; k += NT) {
        const int32_t c = colind[k];
        uint32_t h = ((uint32_t)c * 0x9E3779B1u >> 12) & mask;
        for (;;) {
            const int32_t prev = atomicCAS(&table[h], -1, c);
            if (prev == -1) { ++cnt; break; }
            if (prev == c) break;
            h = (h + 1) & mask;
        }
    }
    int total;
    (void)block_exclusive_scan<NT>(cnt, &total, smem);
    if (threadIdx.x == 0) ncols[w] = total;
}

__global__ __launch_bounds__(256) void k_count_small(int32_t W, int32_t n_rows, const int32_t* __restrict__ rowptr,
                                                     const int32_t* __restrict__ colind, int32_t* __restrict__ ncols)
{
    __shared__ int32_t table[2 * kUniqueSmallCap];
    __shared__ int smem[256 / 64 + 1];
    const int32_t w = blockIdx.x;
    int32_t s, e;
    window_span(w, n_rows, rowptr, s, e);
    if (e - s > kUniqueSmallCap) return;          // listed for k_count_mid or the bitmap kernel
    count_distinct_body<256, 2 * kUniqueSmallCap>(w, n_rows, rowptr, colind, ncols, table, smem);
}

__global__ __launch_bounds__(1024) void k_count_mid(const int32_t* __restrict__ mid_list, int32_t n_rows,
                                                    const int32_t* __restrict__ rowptr,
                                                    const int32_t* __restrict__ colind, int32_t* __restrict__ ncols)
{
    __shared__ int32_t table[2 * kCountMidCap];
    __shared__ int smem[1024 / 64 + 1];
    count_distinct_body<1024, 2 * kCountMidCap>(mid_list[blockIdx.x], n_rows, rowptr, colind, ncols, table, smem);
}

// ---- incremental preparation: only the windows that hold a changed row are looked at again ------
// classes of the touched windows by size (which counting kernel serves them), and the range check of their columns
__global__ __launch_bounds__(256) void k_touched_classes(int32_t n_touched, const int32_t* __restrict__ touched,
                                                         int32_t n_rows, int32_t n_cols, const int32_t* __restrict__ rowptr,
                                                         const int32_t* __restrict__ colind, int32_t* __restrict__ t_small,
                                                         int32_t* __restrict__ t_mid, int32_t* __restrict__ t_huge,
                                                         int32_t* __restrict__ counts /* 3 */, int32_t* __restrict__ err)
{
    const int32_t w = touched[blockIdx.x];
    int32_t s, e;
    window_span(w, n_rows, rowptr, s, e);
    const int32_t n = e - s;
    if (threadIdx.x == 0) {
        if (n > kCountMidCap) t_huge[atomicAdd(counts + 2, 1)] = w;
        else if (n > kUniqueSmallCap) t_mid[atomicAdd(counts + 1, 1)] = w;
        else t_small[atomicAdd(counts, 1)] = w;
    }
    bool bad = false;
    for (int32_t k = s + threadIdx.x; k < e; k += 256) {
        const int32_t c = colind[k];
        bad |= (c < 0 || c >= n_cols);
    }
    if (bad) atomicOr(err, 8);
}

__global__ __launch_bounds__(256) void k_count_small_list(const int32_t* __restrict__ list, int32_t n_rows,
                                                          const int32_t* __restrict__ rowptr,
                                                          const int32_t* __restrict__ colind, int32_t* __restrict__ ncols)
{
    __shared__ int32_t table[2 * kUniqueSmallCap];
    __shared__ int smem[256 / 64 + 1];
    count_distinct_body<256, 2 * kUniqueSmallCap>(list[blockIdx.x], n_rows, rowptr, colind, ncols, table, smem);
}

// Which matrix-path windows keep the previous plan's condensed structure: on that path before and now, and not
// touched.  todo[w] is the route restricted to the windows that still have to be condensed.
__global__ __launch_bounds__(256) void k_carry_mask(int32_t W, const uint8_t* __restrict__ old_route,
                                                    const uint8_t* __restrict__ route, uint8_t* __restrict__ carried,
                                                    uint8_t* __restrict__ todo)
{
    const int32_t w = blockIdx.x * 256 + threadIdx.x;
    if (w >= W) return;
    const uint8_t c = (old_route[w] != 0 && route[w] != 0) ? 1 : 0;
    carried[w] = c;
    todo[w] = (route[w] != 0 && !c) ? 1 : 0;
}

__global__ __launch_bounds__(256) void k_carry_untouch(int32_t n_touched, const int32_t* __restrict__ touched,
                                                       const uint8_t* __restrict__ route, uint8_t* __restrict__ carried,
                                                       uint8_t* __restrict__ todo)
{
    const int32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n_touched) return;
    const int32_t w = touched[i];
    carried[w] = 0;
    todo[w] = route[w] != 0 ? 1 : 0;
}

// Copies a carried window's column list and the condensed columns of its non-zeros from the previous plan's arrays
// to their new places (both move when windows in front of it changed size).
__global__ __launch_bounds__(256) void k_carry_copy(int32_t n_rows, const uint8_t* __restrict__ carried,
                                                    const int64_t* __restrict__ old_wptr, const int64_t* __restrict__ wptr,
                                                    const int32_t* __restrict__ old_wcols, int32_t* __restrict__ wcols,
                                                    const int64_t* __restrict__ old_start, const int32_t* __restrict__ rowptr,
                                                    const int32_t* __restrict__ old_erc, int32_t* __restrict__ erc)
{
    const int32_t w = blockIdx.x;
    if (!carried[w]) return;
    const int64_t so = old_wptr[w], sn = wptr[w];
    const int32_t nc = (int32_t)(wptr[w + 1] - sn);
    for (int32_t i = threadIdx.x; i < nc; i += 256) wcols[sn + i] = old_wcols[so + i];
    int32_t s, e;
    window_span(w, n_rows, rowptr, s, e);
    const int64_t eo = old_start[w];
    for (int32_t k = threadIdx.x; k < e - s; k += 256) erc[s + k] = old_erc[eo + k];
}

hipError_t launch_carry_mask(int32_t W, const uint8_t* old_route, const uint8_t* route, int32_t n_touched,
                             const int32_t* touched, uint8_t* carried, uint8_t* todo, hipStream_t s)
{
    if (W <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_carry_mask, dim3((W + 255) / 256), dim3(256), 0, s, W, old_route, route, carried, todo);
    if (n_touched > 0)
        hipLaunchKernelGGL(k_carry_untouch, dim3((n_touched + 255) / 256), dim3(256), 0, s, n_touched, touched, route,
                           carried, todo);
    return hipGetLastError();
}

hipError_t launch_carry_copy(int32_t W, int32_t n_rows, const uint8_t* carried, const int64_t* old_wptr, const int64_t* wptr,
                             const int32_t* old_wcols, int32_t* wcols, const int64_t* old_start, const int32_t* rowptr,
                             const int32_t* old_erc, int32_t* erc, hipStream_t s)
{
    if (W <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_carry_copy, dim3(W), dim3(256), 0, s, n_rows, carried, old_wptr, wptr, old_wcols, wcols, old_start,
                       rowptr, old_erc, erc);
    return hipGetLastError();
}

hipError_t launch_touched_classes(int32_t n_touched, const int32_t* touched, int32_t n_rows, int32_t n_cols,
                                  const int32_t* rowptr, const int32_t* colind, int32_t* t_small, int32_t* t_mid,
                                  int32_t* t_huge, int32_t* counts, int32_t* err, hipStream_t s)
{
    if (n_touched <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_touched_classes, dim3(n_touched), dim3(256), 0, s, n_touched, touched, n_rows, n_cols, rowptr, colind,
                       t_small, t_mid, t_huge, counts, err);
    return hipGetLastError();
}

hipError_t launch_count_small_list(int32_t n_list, const int32_t* list, int32_t n_rows, const int32_t* rowptr,
                                   const int32_t* colind, int32_t* ncols, hipStream_t s)
{
    if (n_list <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_count_small_list, dim3(n_list), dim3(256), 0, s, list, n_rows, rowptr, colind, ncols);
    return hipGetLastError();
}

hipError_t launch_validate_rowptr(int32_t n_rows, int64_t nnz, const int32_t* rowptr, int32_t* err_flag, hipStream_t s)
{
    const unsigned g = (unsigned)(((int64_t)n_rows + 1 + 255) / 256);
    hipLaunchKernelGGL(k_validate_rowptr, dim3(g), dim3(256), 0, s, n_rows, nnz, rowptr, err_flag);
    return hipGetLastError();
}

hipError_t launch_count_small(int32_t W, int32_t n_rows, const int32_t* rowptr, const int32_t* colind, int32_t* ncols,
                              hipStream_t s)
{
    if (W <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_count_small, dim3(W), dim3(256), 0, s, W, n_rows, rowptr, colind, ncols);
    return hipGetLastError();
}

hipError_t launch_count_mid(int32_t n_mid, const int32_t* mid_list, int32_t n_rows, const int32_t* rowptr,
                            const int32_t* colind, int32_t* ncols, hipStream_t s)
{
    if (n_mid <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_count_mid, dim3(n_mid), dim3(1024), 0, s, mid_list, n_rows, rowptr, colind, ncols);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// compact the distinct-column lists and give every non-zero its condensed column
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_ecol(int32_t n_rows, const int32_t* __restrict__ rowptr,
                                              const int32_t* __restrict__ colind,
                                              const int32_t* __restrict__ tmp_cols, const int32_t* __restrict__ ncols,
                                              const int64_t* __restrict__ wptr, int32_t* __restrict__ wcols,
                                              int32_t* __restrict__ erc, int32_t* __restrict__ unsorted_flag,
                                              const uint8_t* __restrict__ route, int want, int32_t skip_above)
{
    __shared__ int32_t ucols[kEcolLdsCap];
    __shared__ int32_t rp[kH + 1];
    const int32_t w = blockIdx.x;
    if ((route[w] != 0) != (want != 0)) return;      // only the windows of one route
    int32_t s, e;
    window_span(w, n_rows, rowptr, s, e);
    if (e == s || e - s > skip_above) return;        // larger windows were condensed by k_condense_rank
    const int32_t nc = ncols[w];
    const int64_t wp = wptr[w];
    const int32_t* __restrict__ src = tmp_cols + (int64_t)s;
    if (threadIdx.x <= kH) {
        int64_t r = (int64_t)w * kH + threadIdx.x;
        if (r > n_rows) r = n_rows;
        rp[threadIdx.x] = rowptr[r];
    }
    const bool in_lds = nc <= kEcolLdsCap;
    for (int i = threadIdx.x; i < nc; i += 256) {
        int32_t c = src[i];
        wcols[wp + i] = c;
        if (in_lds) ucols[i] = c;
    }
    __syncthreads();
    for (int32_t k = s + threadIdx.x; k < e; k += 256) {
        const int32_t c = colind[k];
        int lo = 0, hi = nc - 1;               // c is in the list by construction
        if (in_lds) {
            while (lo < hi) { int mid = (lo + hi) >> 1; if (ucols[mid] < c) lo = mid + 1; else hi = mid; }
        } else {
            while (lo < hi) { int mid = (lo + hi) >> 1; if (src[mid] < c) lo = mid + 1; else hi = mid; }
        }
        int r = 0;                              // row of k inside the window: last r with rp[r] <= k
#pragma unroll
        for (int step = 8; step > 0; step >>= 1)
            if (r + step < kH && rp[r + step] <= k) r += step;
        erc[k] = (lo << 4) | r;
        // note rows whose column indices are not non-decreasing (the matrix path's cursor walk needs them sorted)
        if (k > rp[r] && colind[k - 1] > c) atomicOr(unsorted_flag, 1);
    }
}

hipError_t launch_ecol(int32_t W, int32_t n_rows, const int32_t* rowptr, const int32_t* colind,
                       const int32_t* tmp_cols, const int32_t* ncols, const int64_t* wptr, int32_t* wcols,
                       int32_t* erc, int32_t* unsorted_flag, const uint8_t* route, int want, int32_t skip_above,
                       hipStream_t s)
{
    hipLaunchKernelGGL(k_ecol, dim3(W), dim3(256), 0, s, n_rows, rowptr, colind, tmp_cols, ncols, wptr, wcols, erc,
                       unsorted_flag, route, want, skip_above);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// condensing of large matrix-path windows in one go: an LDS bitmap of the window's columns plus a
// prefix count per bitmap word gives the sorted list AND every non-zero's position in it (its rank)
// without a search; 2^19 columns per pass over the window's own column range
// ------------------------------------------------------------------------------------------------
constexpr int kRankWords = 16384;

__global__ __launch_bounds__(1024) void k_condense_rank(const int32_t* __restrict__ list, int32_t n_rows,
                                                        const int32_t* __restrict__ rowptr,
                                                        const int32_t* __restrict__ colind,
                                                        const uint8_t* __restrict__ route,
                                                        const int64_t* __restrict__ wptr, int32_t* __restrict__ wcols,
                                                        int32_t* __restrict__ erc, int32_t* __restrict__ unsorted_flag)
{
    __shared__ uint32_t bm[kRankWords];
    __shared__ int32_t pre[kRankWords];
    __shared__ int smem[1024 / 64 + 1];
    __shared__ int32_t rp[kH + 1];
    __shared__ int32_t span_lo, span_hi;
    constexpr int kBits = kRankWords * 32;
    const int32_t w = list[blockIdx.x];
    if (route[w] == 0) return;
    int32_t s, e;
    window_span(w, n_rows, rowptr, s, e);
    if (e == s) return;
    const int64_t wp = wptr[w];
    if (threadIdx.x <= kH) {
        int64_t r = (int64_t)w * kH + threadIdx.x;
        if (r > n_rows) r = n_rows;
        rp[threadIdx.x] = rowptr[r];
    }
    if (threadIdx.x == 0) { span_lo = 0x7fffffff; span_hi = -1; }
    __syncthreads();
    {
        int32_t lo = 0x7fffffff, hi = -1;
        for (int32_t k = s + threadIdx.x; k < e; k += 1024) {
            const int32_t c = colind[k];
            lo = min(lo, c);
            hi = max(hi, c);
        }
        if (hi >= 0) { atomicMin(&span_lo, lo); atomicMax(&span_hi, hi); }
    }
    __syncthreads();
    const int32_t cmax = span_hi;
    int32_t running = 0;
    for (int64_t base = span_lo & ~31; base <= cmax; base += kBits) {
        // words of this pass that can hold a column of the window, dealt to the threads in equal consecutive runs
        const int n_words = (int)min((int64_t)kRankWords, (cmax - base) / 32 + 1);
        const int wpt = (n_words + 1023) / 1024;
        const int w0 = threadIdx.x * wpt;
        for (int i = threadIdx.x; i < n_words; i += 1024) bm[i] = 0u;
        __syncthreads();
        for (int32_t k = s + threadIdx.x; k < e; k += 1024) {
            const int64_t c = (int64_t)colind[k] - base;
            if (c >= 0 && c < kBits) atomicOr(&bm[c >> 5], 1u << (c & 31));
        }
        __syncthreads();
        const int my_words = max(0, min(wpt, n_words - w0));
        int cnt = 0;
        for (int i = 0; i < my_words; ++i) cnt += __popc(bm[w0 + i]);
        int total;
        const int off = block_exclusive_scan<1024>(cnt, &total, smem);
        {
            int run = off;
            int32_t* out = wcols + wp + running + off;
            for (int i = 0; i < my_words; ++i) {
                uint32_t bits = bm[w0 + i];
                pre[w0 + i] = run;
                run += __popc(bits);
                while (bits) {
                    const int b = __ffs(bits) - 1;
                    bits &= bits - 1;
                    *out++ = (int32_t)(base + (int64_t)(w0 + i) * 32 + b);
                }
            }
        }
        __syncthreads();
        for (int32_t k = s + threadIdx.x; k < e; k += 1024) {
            const int32_t col = colind[k];
            const int64_t c = (int64_t)col - base;
            if (c < 0 || c >= kBits) continue;
            const int word = (int)(c >> 5);
            const int rank = running + pre[word] + __popc(bm[word] & ((1u << (c & 31)) - 1u));
            int r = 0;                              // row of k inside the window: last r with rp[r] <= k
#pragma unroll
            for (int step = 8; step > 0; step >>= 1)
                if (r + step < kH && rp[r + step] <= k) r += step;
            erc[k] = (rank << 4) | r;
            if (k > rp[r] && colind[k - 1] > col) atomicOr(unsorted_flag, 1);
        }
        running += total;
        __syncthreads();
    }
}

hipError_t launch_condense_rank(int32_t n_list, const int32_t* list, int32_t n_rows, const int32_t* rowptr,
                                const int32_t* colind, const uint8_t* route, const int64_t* wptr, int32_t* wcols,
                                int32_t* erc, int32_t* unsorted_flag, hipStream_t s)
{
    if (n_list <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_condense_rank, dim3(n_list), dim3(1024), 0, s, list, n_rows, rowptr, colind, route, wptr, wcols,
                       erc, unsorted_flag);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// runs of matrix-path windows: the union of the windows' column lists and every window column's
// position in it, by the same bitmap ranks (the lists are ascending, the union comes out ascending)
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_run_union(const int32_t* __restrict__ win_list, int32_t n_list,
                                                    const int32_t* __restrict__ ncols, const int64_t* __restrict__ wptr,
                                                    const int32_t* __restrict__ wcols, int32_t* __restrict__ ucols,
                                                    int32_t* __restrict__ wslot, RunDesc* __restrict__ runs)
{
    __shared__ uint32_t bm[kRankWords];
    __shared__ int32_t pre[kRankWords];
    __shared__ int smem[1024 / 64 + 1];
    constexpr int kBits = kRankWords * 32;
    constexpr int kWordsPerThread = kRankWords / 1024;
    const int32_t first = blockIdx.x * kRunWindows;
    const int nw = min(kRunWindows, n_list - first);
    int64_t wp[kRunWindows];
    int32_t nc[kRunWindows];
    int32_t lo = 0x7fffffff, hi = -1;
    for (int i = 0; i < nw; ++i) {
        const int32_t w = win_list[first + i];
        wp[i] = wptr[w];
        nc[i] = ncols[w];
        if (nc[i] > 0) {
            lo = min(lo, wcols[wp[i]]);
            hi = max(hi, wcols[wp[i] + nc[i] - 1]);
        }
    }
    const int64_t up = wp[0];                                  // the union is stored where the run's first window's list starts
    int32_t running = 0;
    const int w0 = threadIdx.x * kWordsPerThread;
    for (int64_t base = lo & ~31; base <= hi; base += kBits) {
        for (int i = threadIdx.x; i < kRankWords; i += 1024) bm[i] = 0u;
        __syncthreads();
        for (int i = 0; i < nw; ++i)
            for (int32_t k = threadIdx.x; k < nc[i]; k += 1024) {
                const int64_t c = (int64_t)wcols[wp[i] + k] - base;
                if (c >= 0 && c < kBits) atomicOr(&bm[c >> 5], 1u << (c & 31));
            }
        __syncthreads();
        int cnt = 0;
#pragma unroll 4
        for (int i = 0; i < kWordsPerThread; ++i) cnt += __popc(bm[w0 + i]);
        int total;
        const int off = block_exclusive_scan<1024>(cnt, &total, smem);
        {
            int run = off;
            int32_t* out = ucols + up + running + off;
            for (int i = 0; i < kWordsPerThread; ++i) {
                uint32_t bits = bm[w0 + i];
                pre[w0 + i] = run;
                run += __popc(bits);
                while (bits) {
                    const int b = __ffs(bits) - 1;
                    bits &= bits - 1;
                    *out++ = (int32_t)(base + (int64_t)(w0 + i) * 32 + b);
                }
            }
        }
        __syncthreads();
        for (int i = 0; i < nw; ++i)
            for (int32_t k = threadIdx.x; k < nc[i]; k += 1024) {
                const int64_t c = (int64_t)wcols[wp[i] + k] - base;
                if (c < 0 || c >= kBits) continue;
                const int word = (int)(c >> 5);
                wslot[wp[i] + k] = running + pre[word] + __popc(bm[word] & ((1u << (c & 31)) - 1u));
            }
        running += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        RunDesc rd;
        rd.up = up; rd.first = first; rd.nw = nw; rd.nu = running;
        rd.n_slices = 1; rd.slot0 = 0; rd.pad = 0;              // slices are laid out by the host from the union sizes
        runs[blockIdx.x] = rd;
    }
}

// per slice and wave: the window the wave owns, with what the kernel needs to start on it
__global__ __launch_bounds__(256) void k_run_wins(int32_t n_slices, const RunSlice* __restrict__ slices,
                                                  const RunDesc* __restrict__ runs, const int32_t* __restrict__ win_list,
                                                  const int32_t* __restrict__ ncols, const int64_t* __restrict__ wptr,
                                                  int32_t n_rows, const int32_t* __restrict__ rowptr, RunWin* __restrict__ wins)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)n_slices * kRunWindows) return;
    const RunDesc rd = runs[slices[t / kRunWindows].run];
    const int i = (int)(t % kRunWindows);
    const int32_t w = win_list[rd.first + (i < rd.nw ? i : 0)];
    RunWin rw;
    rw.w = w; rw.nc = ncols[w]; rw.wp = wptr[w]; rw.pad = 0;
    rw.k_last = rowptr[min((int64_t)w * kH + kH, (int64_t)n_rows)] - 1;
    wins[t] = rw;
}

hipError_t launch_run_wins(int32_t n_slices, const RunSlice* slices, const RunDesc* runs, const int32_t* win_list,
                           const int32_t* ncols, const int64_t* wptr, int32_t n_rows, const int32_t* rowptr, RunWin* wins,
                           hipStream_t s)
{
    if (n_slices <= 0) return hipSuccess;
    const int64_t n = (int64_t)n_slices * kRunWindows;
    hipLaunchKernelGGL(k_run_wins, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, n_slices, slices, runs, win_list, ncols,
                       wptr, n_rows, rowptr, wins);
    return hipGetLastError();
}

hipError_t launch_run_union(int32_t n_runs, const int32_t* win_list, int32_t n_list, const int32_t* ncols,
                            const int64_t* wptr, const int32_t* wcols, int32_t* ucols, int32_t* wslot, RunDesc* runs,
                            hipStream_t s)
{
    if (n_runs <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_run_union, dim3(n_runs), dim3(1024), 0, s, win_list, n_list, ncols, wptr, wcols, ucols, wslot,
                       runs);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// selection (Section IV-C): z' = c0*H*ncols^2 + c1*(H*ncols - nnzw) + c2*H*ncols ; matrix path iff z' < 0
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_select(int32_t W, const int32_t* __restrict__ ncols,
                                                const int32_t* __restrict__ nnzw, long long c0, long long c1,
                                                long long c2, int32_t mode, uint8_t* __restrict__ route,
                                                int32_t* __restrict__ f_mfma, int32_t* __restrict__ f_csr,
                                                int32_t* __restrict__ f_small, int32_t* __restrict__ f_mid,
                                                int32_t* __restrict__ f_big, int32_t* __restrict__ nnz_if_mfma)
{
    int32_t w = blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= W) return;
    const long long nc = ncols[w], nz = nnzw[w];
    int r = 0;
    if (nc > 0) {
        if (mode == HCSPMM_ROUTE_ALL_MFMA) r = 1;
        else if (mode == HCSPMM_ROUTE_HYBRID || mode == HCSPMM_ROUTE_PER_WINDOW) {
            // |c*| < 2^40 and H*ncols^2 < 2^58: 128-bit integers keep the sign exact
            const __int128 hn = (__int128)kH * nc;
            const __int128 z = (__int128)c0 * hn * nc + (__int128)c1 * (hn - nz) + (__int128)c2 * hn;
            r = z < 0 ? 1 : 0;
        }
    }
    route[w] = (uint8_t)r;
    f_mfma[w] = r;
    f_csr[w] = 1 - r;
    f_small[w] = (r && nc <= kMfmaSmallMaxCols) ? 1 : 0;
    f_mid[w] = (r && nc > kMfmaSmallMaxCols && nc <= kMfmaMidMaxCols) ? 1 : 0;
    f_big[w] = (r && nc > kMfmaMidMaxCols) ? 1 : 0;
    nnz_if_mfma[w] = r ? (int32_t)nz : 0;
}

hipError_t launch_select(int32_t W, const int32_t* ncols, const int32_t* nnzw, int64_t c0, int64_t c1, int64_t c2,
                         int32_t mode, uint8_t* route, int32_t* f_mfma, int32_t* f_csr, int32_t* f_small,
                         int32_t* f_mid, int32_t* f_big, int32_t* nnz_if_mfma, hipStream_t s)
{
    hipLaunchKernelGGL(k_select, dim3((W + 255) / 256), dim3(256), 0, s, W, ncols, nnzw, (long long)c0, (long long)c1,
                       (long long)c2, mode, route, f_mfma, f_csr, f_small, f_mid, f_big, nnz_if_mfma);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_compact_ids(int32_t n, const int32_t* __restrict__ flags,
                                                     const int64_t* __restrict__ pos, int32_t* __restrict__ out)
{
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n && flags[i]) out[pos[i]] = i;
}

__global__ __launch_bounds__(256) void k_masked_copy(int32_t n, const int32_t* __restrict__ flags,
                                                     const int32_t* __restrict__ src, int32_t* __restrict__ dst)
{
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = flags[i] ? src[i] : 0;
}

hipError_t launch_masked_copy(int32_t n, const int32_t* flags, const int32_t* src, int32_t* dst, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_masked_copy, dim3((n + 255) / 256), dim3(256), 0, s, n, flags, src, dst);
    return hipGetLastError();
}

hipError_t launch_compact_ids(int32_t n, const int32_t* flags, const int64_t* pos, int32_t* out, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_compact_ids, dim3((n + 255) / 256), dim3(256), 0, s, n, flags, pos, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// matrix-path launch table: one descriptor per wave-per-window item
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_build_desc(int32_t n_list, const int32_t* __restrict__ win_list,
                                                    int32_t n_rows, const int32_t* __restrict__ rowptr,
                                                    const int32_t* __restrict__ ncols,
                                                    const int64_t* __restrict__ wptr, WinDesc* __restrict__ desc)
{
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_list) return;
    WinDesc ds;
    ds.w = win_list[i];
    window_span(ds.w, n_rows, rowptr, ds.s, ds.e);
    ds.nc = ncols[ds.w];
    ds.wp = wptr[ds.w];
    ds.pad = 0;
    desc[i] = ds;
}

hipError_t launch_build_desc(int32_t n_list, const int32_t* win_list, int32_t n_rows, const int32_t* rowptr,
                             const int32_t* ncols, const int64_t* wptr, WinDesc* desc, hipStream_t s)
{
    if (n_list <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_build_desc, dim3((n_list + 255) / 256), dim3(256), 0, s, n_list, win_list, n_rows, rowptr,
                       ncols, wptr, desc);
    return hipGetLastError();
}

// matrix-path launch table: workgroup slices of medium and wide windows
__global__ __launch_bounds__(256) void k_slice_count(int32_t n_list, const int32_t* __restrict__ win_list,
                                                     const int32_t* __restrict__ ncols, int32_t slice_cols,
                                                     int32_t* __restrict__ n_slices, int32_t* __restrict__ f_multi,
                                                     int32_t* __restrict__ n_slots)
{
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_list) return;
    const int32_t nc = ncols[win_list[i]];
    const int32_t ns = (nc + slice_cols - 1) / slice_cols;
    n_slices[i] = ns;
    f_multi[i] = ns > 1 ? 1 : 0;
    n_slots[i] = ns > 1 ? ns : 0;
}

__global__ __launch_bounds__(256) void k_slice_fill(int32_t n_list, const int32_t* __restrict__ win_list,
                                                    const int32_t* __restrict__ ncols, int32_t slice_cols,
                                                    const int64_t* __restrict__ slice_pos,
                                                    const int64_t* __restrict__ multi_pos,
                                                    const int64_t* __restrict__ slot_pos, WgSlice* __restrict__ slices,
                                                    MultiRow* __restrict__ multi)
{
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_list) return;
    const int32_t w = win_list[i];
    const int32_t nc = ncols[w];
    const int32_t ns = (nc + slice_cols - 1) / slice_cols;
    const int32_t slot0 = ns > 1 ? (int32_t)slot_pos[i] : -1;
    for (int32_t q = 0; q < ns; ++q) {
        WgSlice sl;
        sl.w = w;
        sl.kc_begin = q * slice_cols;
        sl.kc_end = min(nc, sl.kc_begin + slice_cols);
        sl.slot = ns > 1 ? slot0 + q : -1;
        slices[slice_pos[i] + q] = sl;
    }
    if (ns > 1) {
        MultiRow m;
        m.row = w; m.first_slot = slot0; m.n_slots = ns; m.pad = 0;
        multi[multi_pos[i]] = m;
    }
}

// per slice and window row: the first non-zero of the row whose condensed column is inside the slice
// (rows with ascending columns only: their condensed columns ascend too)
__global__ __launch_bounds__(256) void k_slice_rows(int32_t n_slices, const WgSlice* __restrict__ slices,
                                                    int32_t n_rows, const int32_t* __restrict__ rowptr,
                                                    const int32_t* __restrict__ erc, int32_t* __restrict__ slice_rows)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)n_slices * kH) return;
    const WgSlice sl = slices[t / kH];
    const int64_t row = (int64_t)sl.w * kH + (t % kH);
    int32_t lo = rowptr[min(row, (int64_t)n_rows)], hi = rowptr[min(row + 1, (int64_t)n_rows)];
    while (lo < hi) {
        const int32_t mid = lo + ((hi - lo) >> 1);
        if ((erc[mid] >> 4) < sl.kc_begin) lo = mid + 1; else hi = mid;
    }
    slice_rows[t] = lo;
}

hipError_t launch_slice_rows(int32_t n_slices, const WgSlice* slices, int32_t n_rows, const int32_t* rowptr,
                             const int32_t* erc, int32_t* slice_rows, hipStream_t s)
{
    if (n_slices <= 0) return hipSuccess;
    const int64_t n = (int64_t)n_slices * kH;
    hipLaunchKernelGGL(k_slice_rows, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, n_slices, slices, n_rows,
                       rowptr, erc, slice_rows);
    return hipGetLastError();
}

hipError_t launch_slice_count(int32_t n_list, const int32_t* win_list, const int32_t* ncols, int32_t slice_cols,
                              int32_t* n_slices, int32_t* f_multi, int32_t* n_slots, hipStream_t s)
{
    if (n_list <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_slice_count, dim3((n_list + 255) / 256), dim3(256), 0, s, n_list, win_list, ncols, slice_cols,
                       n_slices, f_multi, n_slots);
    return hipGetLastError();
}

hipError_t launch_slice_fill(int32_t n_list, const int32_t* win_list, const int32_t* ncols, int32_t slice_cols,
                             const int64_t* slice_pos, const int64_t* multi_pos, const int64_t* slot_pos,
                             WgSlice* slices, MultiRow* multi, hipStream_t s)
{
    if (n_list <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_slice_fill, dim3((n_list + 255) / 256), dim3(256), 0, s, n_list, win_list, ncols, slice_cols,
                       slice_pos, multi_pos, slot_pos, slices, multi);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// scalar-path launch tables: short rows, and segments of long rows
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_row_class(int32_t n_rows, const int32_t* __restrict__ rowptr,
                                                   const uint8_t* __restrict__ route, int32_t mid_row,
                                                   int32_t long_row, int32_t* __restrict__ f_short,
                                                   int32_t* __restrict__ f_mid, int32_t* __restrict__ n_seg, int32_t* __restrict__ f_multi,
                                                   int32_t* __restrict__ n_slot, int32_t* __restrict__ len_long)
{
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_rows) return;
    const int32_t len = rowptr[i + 1] - rowptr[i];
    const bool csr = route[i / kH] == 0;
    const bool is_long = csr && len > long_row;
    const bool is_mid = csr && !is_long && len > mid_row;
    const int32_t ns = is_long ? (len + kSegLen - 1) / kSegLen : 0;
    f_short[i] = (csr && !is_long && !is_mid) ? 1 : 0;
    f_mid[i] = is_mid ? 1 : 0;
    n_seg[i] = ns;
    f_multi[i] = ns > 1 ? 1 : 0;
    n_slot[i] = ns > 1 ? ns : 0;
    len_long[i] = (is_long || is_mid) ? len : 0;
}

hipError_t launch_row_class(int32_t n_rows, const int32_t* rowptr, const uint8_t* route, int32_t mid_row,
                            int32_t long_row, int32_t* f_short,
                            int32_t* f_mid, int32_t* n_seg, int32_t* f_multi, int32_t* n_slot, int32_t* len_long,
                            hipStream_t s)
{
    if (n_rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_row_class, dim3((n_rows + 255) / 256), dim3(256), 0, s, n_rows, rowptr, route, mid_row, long_row,
                       f_short, f_mid,
                       n_seg, f_multi, n_slot, len_long);
    return hipGetLastError();
}

// rows whose aggregated values reach memory even when the update stage is fused into the SpMM
// kernels: scalar-path rows above the short tier and all rows of matrix-path windows too wide for
// the wave-per-window kernel
__global__ __launch_bounds__(256) void k_rest_flag(int32_t n_rows, const int32_t* __restrict__ rowptr,
                                                   const uint8_t* __restrict__ route, const int32_t* __restrict__ ncols,
                                                   int32_t mid_row, int32_t* __restrict__ flag)
{
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_rows) return;
    const int32_t w = i / kH;
    flag[i] = route[w] ? (ncols[w] > kMfmaSmallMaxCols ? 1 : 0) : (rowptr[i + 1] - rowptr[i] > mid_row ? 1 : 0);
}

hipError_t launch_rest_flag(int32_t n_rows, const int32_t* rowptr, const uint8_t* route, const int32_t* ncols,
                            int32_t mid_row, int32_t* flag, hipStream_t s)
{
    if (n_rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_rest_flag, dim3((n_rows + 255) / 256), dim3(256), 0, s, n_rows, rowptr, route, ncols, mid_row, flag);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_build_segments(int32_t n_rows, const int32_t* __restrict__ rowptr,
                                                        const int32_t* __restrict__ n_seg,
                                                        const int64_t* __restrict__ seg_pos,
                                                        const int64_t* __restrict__ multi_pos,
                                                        const int64_t* __restrict__ slot_pos,
                                                        Segment* __restrict__ segs, MultiRow* __restrict__ multi)
{
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_rows) return;
    const int32_t ns = n_seg[i];
    if (ns == 0) return;
    const int32_t s = rowptr[i], e = rowptr[i + 1];
    const int64_t sp = seg_pos[i];
    const int32_t slot0 = ns > 1 ? (int32_t)slot_pos[i] : -1;
    for (int32_t q = 0; q < ns; ++q) {
        Segment sg;
        sg.row = i;
        sg.k_begin = s + q * kSegLen;
        sg.k_end = min(e, sg.k_begin + kSegLen);
        sg.slot = ns > 1 ? slot0 + q : -1;
        segs[sp + q] = sg;
    }
    if (ns > 1) {
        MultiRow m;
        m.row = i; m.first_slot = slot0; m.n_slots = ns; m.pad = 0;
        multi[multi_pos[i]] = m;
    }
}

hipError_t launch_build_segments(int32_t n_rows, const int32_t* rowptr, const int32_t* n_seg, const int64_t* seg_pos,
                                 const int64_t* multi_pos, const int64_t* slot_pos, Segment* segs, MultiRow* multi,
                                 hipStream_t s)
{
    if (n_rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_build_segments, dim3((n_rows + 255) / 256), dim3(256), 0, s, n_rows, rowptr, n_seg, seg_pos,
                       multi_pos, slot_pos, segs, multi);
    return hipGetLastError();
}

}  // namespace hcspmm
