// Scalar path: SpMM straight from CSR for the windows the selector leaves on the vector ALUs
// (Alg. 1 gives the arithmetic, Alg. 3 the mapping idea: a group of lanes owns one output row and
// each lane one slice of the dense width, so X rows are read as whole contiguous segments).
//
// wave64 mapping: a group of LPR lanes owns a row, every lane holds VEC consecutive output
// columns; a 64-lane wave therefore works on 64/LPR rows (short rows) or on 64/LPR non-zeros of
// the same row (mid and long rows) per load instruction.  Column indices and values are fetched
// LPR at a time with one coalesced load per group and handed round with cross-lane reads; X is
// read directly from global memory / L2 (the paper found staging X in shared memory a loss on
// this path).  Three tiers by row length balance power-law degree distributions:
//   short rows  a lane group walks one to four consecutive rows in one flattened loop, and the
//               workgroups reach the XCDs in runs so that neighbouring rows share an L2;
//   mid rows    one wave per row, the groups stride over the row and combine with cross-lane adds;
//   long rows   one workgroup per segment of kSegLen non-zeros, combined through LDS in a fixed
//               order (and, for rows of several segments, through partial rows in memory).
#include <cstdlib>

#include "common.hpp"
#include "update_tile.hpp"

namespace hcspmm {

// XK: element kind of X -- 0 fp32, 1 bf16, 2 fp16.  16-bit elements are widened to fp32 on load;
// all arithmetic of this path is fp32.
template <int XK> struct XElem { static constexpr int size = XK == 0 ? 4 : 2; };

template <int VEC> __device__ inline void vzero(float (&a)[VEC])
{
#pragma unroll
    for (int i = 0; i < VEC; ++i) a[i] = 0.f;
}

__device__ inline float widen16(uint32_t bits, int xk)
{
    if (xk == 1) return __uint_as_float(bits << 16);
    const _Float16 h = __builtin_bit_cast(_Float16, (unsigned short)bits);
    return (float)h;
}

// reads VEC consecutive elements starting at byte address p (aligned to the vector size)
template <int VEC, int XK> __device__ inline void vload(const char* __restrict__ p, float (&x)[VEC])
{
    if constexpr (XK == 0) {
        static_assert(VEC == 4 || VEC == 2 || VEC == 1, "fp32 vectors are 1, 2 or 4 wide");
        if constexpr (VEC == 4) { const float4 v = *reinterpret_cast<const float4*>(p); x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w; }
        else if constexpr (VEC == 2) { const float2 v = *reinterpret_cast<const float2*>(p); x[0] = v.x; x[1] = v.y; }
        else { x[0] = *reinterpret_cast<const float*>(p); }
    } else {
        static_assert(VEC == 8 || VEC == 4 || VEC == 1, "16-bit vectors are 1, 4 or 8 wide");
        if constexpr (VEC == 8) {
            const uint4 v = *reinterpret_cast<const uint4*>(p);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) { x[2 * i] = widen16(w[i] & 0xffffu, XK); x[2 * i + 1] = widen16(w[i] >> 16, XK); }
        } else if constexpr (VEC == 4) {
            const uint2 v = *reinterpret_cast<const uint2*>(p);
            x[0] = widen16(v.x & 0xffffu, XK); x[1] = widen16(v.x >> 16, XK);
            x[2] = widen16(v.y & 0xffffu, XK); x[3] = widen16(v.y >> 16, XK);
        } else {
            x[0] = widen16(*reinterpret_cast<const unsigned short*>(p), XK);
        }
    }
}

template <int VEC> __device__ inline void vstore(float* __restrict__ p, const float (&x)[VEC], int relu)
{
    float y[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) y[i] = relu ? fmaxf(x[i], 0.f) : x[i];
    if constexpr (VEC == 8) {
        *reinterpret_cast<float4*>(p) = make_float4(y[0], y[1], y[2], y[3]);
        *reinterpret_cast<float4*>(p + 4) = make_float4(y[4], y[5], y[6], y[7]);
    } else if constexpr (VEC == 4) {
        *reinterpret_cast<float4*>(p) = make_float4(y[0], y[1], y[2], y[3]);
    } else if constexpr (VEC == 2) {
        *reinterpret_cast<float2*>(p) = make_float2(y[0], y[1]);
    } else {
        *p = y[0];
    }
}

// One batch: the group's lanes hold up to LPR (column, value) pairs; every lane accumulates
// val * X[col, c .. c+VEC) over the batch.  Slots past the end of the row carry the row's last
// column with value 0, so the loads carry no branches and all of them are in flight together.
// Xc already points at a valid column for every lane (lanes past the matrix width read column 0
// and never store).
template <int LPR, int VEC, int XK>
__device__ inline void batch_accumulate(int32_t mc, float mv, int cnt, const char* __restrict__ Xc,
                                        int64_t ldx /* bytes */, float (&acc)[VEC])
{
    constexpr int U = LPR < 8 ? LPR : 8;
#pragma unroll 1
    for (int t0 = 0; t0 < cnt; t0 += U) {
        float x[U][VEC];
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int32_t c = __shfl(mc, t0 + u, LPR);
            v[u] = __shfl(mv, t0 + u, LPR);
            vload<VEC, XK>(Xc + (int64_t)c * ldx, x[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = fmaf(v[u], x[u][i], acc[i]);
    }
}

// (column, value) of non-zero k of a row ending at e (k may run past the end: value 0, last column)
__device__ inline void fetch_entry(const int32_t* __restrict__ colind, const float* __restrict__ vals, int k, int e,
                                   int32_t& c, float& v)
{
    const int kc = min(k, e - 1);
    c = colind[kc];
    const float t = vals[kc];
    v = k < e ? t : 0.f;
}

// Accumulate a span [kb, ke) of one row taken LPR non-zeros at a time with stride `stride`
// (stride = LPR when one group owns the span, larger when several groups share it).
template <int LPR, int VEC, int XK>
__device__ inline void span_accumulate(int kb, int ke, int stride, int lig,
                                       const int32_t* __restrict__ colind, const float* __restrict__ vals,
                                       const char* __restrict__ Xc, int64_t ldx, float (&acc)[VEC])
{
    if (kb >= ke) return;
    int32_t mc, nc;
    float mv, nv;
    fetch_entry(colind, vals, kb + lig, ke, mc, mv);
    for (int k0 = kb; k0 < ke; k0 += stride) {
        // fetch the next batch's indices before this batch's X rows
        fetch_entry(colind, vals, k0 + stride + lig, ke, nc, nv);
        batch_accumulate<LPR, VEC, XK>(mc, mv, min(LPR, ke - k0), Xc, ldx, acc);
        mc = nc;
        mv = nv;
    }
}

// ---- short rows -----------------------------------------------------------------------------
// A group of LPR lanes walks rows_per_group (<= kRowsPerGroup) consecutive items (rows, or entries of row_list) in a
// single flattened loop: each trip either moves to the next row (storing the finished one) or
// consumes one batch of the current row, so groups of one wave stay busy on rows of unequal
// length.  The rows' extents are fetched up front, one per lane.
template <int LPR, int VEC, int XK>
__device__ inline void csr_short_body(int64_t block, int32_t n_items, const int32_t* __restrict__ row_list,
                                      const uint8_t* __restrict__ route, int rows_per_group, int mid_row,
                                      const SpmmArgs& a)
{
    static_assert(LPR >= kRowsPerGroup, "a group must be able to hold one row extent per lane");
    constexpr int GPB = 256 / LPR;
    const int64_t blk = block * GPB + threadIdx.x / LPR;
    const int lig = threadIdx.x % LPR;
    const int64_t i0 = blk * rows_per_group;
    if (i0 >= n_items) return;
    const int nr = (int)min((int64_t)rows_per_group, (int64_t)n_items - i0);
    int32_t my_row = -1, my_s = 0, my_e = 0;
    if (lig < nr) {
        my_row = row_list ? row_list[i0 + lig] : (int32_t)(i0 + lig);
        my_s = a.rowptr[my_row];
        my_e = a.rowptr[my_row + 1];
        // walking every row: skip rows owned by the matrix path or by the mid/long-row kernels
        if (!row_list && (route[my_row / kH] != 0 || my_e - my_s > mid_row)) my_row = -1;
    }
    const char* __restrict__ X = static_cast<const char*>(a.X);
    constexpr int ES = XElem<XK>::size;
    const int64_t ldxb = a.ldx * ES;
    for (int c0 = 0; c0 < a.d; c0 += LPR * VEC) {
        const int c = c0 + lig * VEC;
        const bool col_ok = c < a.d;
        float acc[VEC];
        vzero<VEC>(acc);
        int j = 0, k = 0, e = 0;
        int32_t row = -1;
        int32_t mc = 0;
        float mv = 0.f;
        for (;;) {
            if (k >= e) {
                if (row >= 0 && col_ok) out_store<VEC>(a.Y, a.y_dtype, (int64_t)row * a.ldy + c, acc, a.relu);
                row = -1;
                while (j < nr && row < 0) {
                    row = __shfl(my_row, j, LPR);
                    k = __shfl(my_s, j, LPR);
                    e = __shfl(my_e, j, LPR);
                    ++j;
                }
                if (row < 0) break;
                vzero<VEC>(acc);
                if (k < e) fetch_entry(a.colind, a.vals, k + lig, e, mc, mv);
                continue;                       // an empty row is stored (as zeros) on the next trip
            }
            int32_t nc;
            float nv;
            fetch_entry(a.colind, a.vals, k + LPR + lig, e, nc, nv);
            batch_accumulate<LPR, VEC, XK>(mc, mv, min(LPR, e - k), X + (col_ok ? c : 0) * ES, ldxb, acc);
            mc = nc;
            mv = nv;
            k += LPR;
        }
    }
}

// ---- short rows with the update stage fused in ------------------------------------------------
// Same walk as csr_short_body, but a workgroup covers exactly 16 (or, with 8-lane groups, 32) list
// entries and a finished row goes to a 16 x d tile in LDS instead of memory; after a barrier the
// four waves share the tile(s), each multiplying it by an interleaved quarter (half) of W's
// 16-column blocks on the matrix cores, and write act(Z W) for the rows the workgroup owns
// (Section V-A: the aggregation result of a window stays on chip for the update).
// The width d must fit one pass of the group (d <= LPR*VEC) and be a multiple of 16.
template <int LPR, int VEC> struct FusedShape {
    static constexpr int G = 64 / LPR;                          // lane groups per wave
    static constexpr int RPG = LPR / 16 > 1 ? LPR / 16 : 1;     // consecutive rows per group
    static constexpr int ROWS = 4 * G * RPG;                    // list entries per workgroup
    static constexpr int T = ROWS / 16;                         // 16-row tiles per workgroup
    static constexpr int LDZ = LPR * VEC + 4;
    static_assert(ROWS % 16 == 0 && (T == 1 || T == 2), "one or two tiles per workgroup");
};

template <int LPR, int VEC, int XK>
__device__ inline void csr_short_fused_body(int64_t block, int32_t n_items, const int32_t* __restrict__ row_list,
                                            const uint8_t* __restrict__ route, int mid_row, const SpmmArgs& a,
                                            const UpdateArgs& u, float* __restrict__ zt, int32_t* __restrict__ rows_s)
{
    using S = FusedShape<LPR, VEC>;
    constexpr int RPG = S::RPG, LDZ = S::LDZ;
    static_assert(LPR >= RPG, "a group must be able to hold one row extent per lane");
    const int64_t b0 = (int64_t)block * S::ROWS;                // first list entry of the workgroup
    if (b0 >= n_items) return;                                  // whole workgroup past the end
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int gw = threadIdx.x / LPR, lig = threadIdx.x % LPR;  // group within the workgroup
    const int64_t i0 = b0 + gw * RPG;
    const int nr = (int)max((int64_t)0, min((int64_t)RPG, (int64_t)n_items - i0));
    int32_t my_row = -1, my_s = 0, my_e = 0;
    if (lig < nr) {
        my_row = row_list ? row_list[i0 + lig] : (int32_t)(i0 + lig);
        my_s = a.rowptr[my_row];
        my_e = a.rowptr[my_row + 1];
        if (!row_list && (route[my_row / kH] != 0 || my_e - my_s > mid_row)) my_row = -1;
    }
    if (lig < RPG) rows_s[gw * RPG + lig] = my_row;
    const char* __restrict__ X = static_cast<const char*>(a.X);
    constexpr int ES = XElem<XK>::size;
    const int64_t ldxb = a.ldx * ES;
    const int c = lig * VEC;
    const bool col_ok = c < a.d;
    float acc[VEC];
    vzero<VEC>(acc);
    int j = 0, k = 0, e = 0, slot = 0;
    int32_t row = -1;
    int32_t mc = 0;
    float mv = 0.f;
    for (;;) {
        if (k >= e) {
            if (row >= 0 && col_ok) vstore<VEC>(zt + (gw * RPG + slot) * LDZ + c, acc, 0);
            row = -1;
            while (j < nr && row < 0) {
                row = __shfl(my_row, j, LPR);
                k = __shfl(my_s, j, LPR);
                e = __shfl(my_e, j, LPR);
                slot = j;
                ++j;
            }
            if (row < 0) break;
            vzero<VEC>(acc);
            if (k < e) fetch_entry(a.colind, a.vals, k + lig, e, mc, mv);
            continue;
        }
        int32_t nc;
        float nv;
        fetch_entry(a.colind, a.vals, k + LPR + lig, e, nc, nv);
        batch_accumulate<LPR, VEC, XK>(mc, mv, min(LPR, e - k), X + (col_ok ? c : 0) * ES, ldxb, acc);
        mc = nc;
        mv = nv;
        k += LPR;
    }
    __syncthreads();
    if (u.keep_z) store_tile_rows(zt, LDZ, rows_s, S::ROWS, a.d, a.Y, a.ldy, threadIdx.x, 256);
    constexpr int WPT = 4 / S::T;                               // waves sharing one tile
    const int tile = wave / WPT;
    update_tile16(zt + tile * 16 * LDZ, LDZ, rows_s + tile * 16, a.d, u, lane, wave % WPT, WPT);
}

// ---- mid rows: one wave per row -------------------------------------------------------------
template <int LPR, int VEC, int XK>
__device__ inline void csr_mid_body(int64_t block, int32_t n_mid, const int32_t* __restrict__ mid_rows,
                                    const SpmmArgs& a, int min_len = 0 /* rows this short belong to another tier */)
{
    constexpr int G = 64 / LPR;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t item = block * 4 + wave;
    if (item >= n_mid) return;
    const int32_t row = mid_rows[item];
    const int32_t s = a.rowptr[row], e = a.rowptr[row + 1];
    if (e - s <= min_len) return;
    const int g = lane / LPR, lig = lane % LPR;
    const char* __restrict__ X = static_cast<const char*>(a.X);
    constexpr int ES = XElem<XK>::size;
    const int64_t ldxb = a.ldx * ES;
    for (int c0 = 0; c0 < a.d; c0 += LPR * VEC) {
        const int c = c0 + lig * VEC;
        const bool col_ok = c < a.d;
        float acc[VEC];
        vzero<VEC>(acc);
        span_accumulate<LPR, VEC, XK>(s + g * LPR, e, G * LPR, lig, a.colind, a.vals, X + (col_ok ? c : 0) * ES, ldxb, acc);
        // butterfly over the G groups: same operation order on every run
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] += __shfl_xor(acc[i], off, 64);
        if (g == 0 && col_ok) out_store<VEC>(a.Y, a.y_dtype, (int64_t)row * a.ldy + c, acc, a.relu);
    }
}

// ---- long rows: one workgroup per segment of a row ------------------------------------------
template <int LPR, int VEC, int XK>
__device__ inline void csr_long_body(int64_t block, const Segment* __restrict__ segs, float* __restrict__ partial,
                                     float* __restrict__ red /* LDS, 256*VEC floats */, const SpmmArgs& a)
{
    constexpr int G = 256 / LPR;
    const Segment sg = segs[block];
    const int g = threadIdx.x / LPR, lig = threadIdx.x % LPR;
    const char* __restrict__ X = static_cast<const char*>(a.X);
    constexpr int ES = XElem<XK>::size;
    const int64_t ldxb = a.ldx * ES;
    for (int c0 = 0; c0 < a.d; c0 += LPR * VEC) {
        const int c = c0 + lig * VEC;
        const bool col_ok = c < a.d;
        float acc[VEC];
        vzero<VEC>(acc);
        span_accumulate<LPR, VEC, XK>(sg.k_begin + g * LPR, sg.k_end, G * LPR, lig, a.colind, a.vals,
                                      X + (col_ok ? c : 0) * ES, ldxb, acc);
        // fixed-order tree over the G groups: the result does not depend on scheduling
#pragma unroll
        for (int i = 0; i < VEC; ++i) red[(g * LPR + lig) * VEC + i] = acc[i];
        __syncthreads();
        for (int st = G / 2; st > 0; st >>= 1) {
            if (g < st) {
#pragma unroll
                for (int i = 0; i < VEC; ++i)
                    red[(g * LPR + lig) * VEC + i] += red[((g + st) * LPR + lig) * VEC + i];
            }
            __syncthreads();
        }
        if (g == 0 && col_ok) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = red[lig * VEC + i];
            if (sg.slot < 0) out_store<VEC>(a.Y, a.y_dtype, (int64_t)sg.row * a.ldy + c, acc, a.relu);
            else vstore<VEC>(partial + (int64_t)sg.slot * a.d + c, acc, 0);
        }
        __syncthreads();
    }
}

// ---- one launch for all three tiers ---------------------------------------------------------
// Workgroups are numbered heaviest first: long-row segments, then mid rows (four per workgroup),
// then the blocks of short rows, so the short rows fill the machine while the last long rows
// drain instead of each tier waiting for the previous one's tail.
struct CsrWork {
    int32_t n_segs;
    const Segment* segs;
    float* partial;
    int32_t n_mid;
    const int32_t* mid_rows;
    int32_t n_items;
    const int32_t* row_list;
    const uint8_t* route;
    int32_t rows_per_group;
    int32_t mid_row;
    int32_t xcd_chunk;          // short-row workgroups per XCD-local run (0: plain order)
    int64_t mid_blocks;         // workgroups of the mid tier (padded to whole rounds of runs when xcd_chunk_mid > 0)
    int32_t xcd_chunk_mid;
};

template <int LPR, int VEC, int XK>
__global__ __launch_bounds__(256) void k_csr(CsrWork wk, SpmmArgs a)
{
    __shared__ float red[256 * VEC];
    int64_t b = blockIdx.x;
    if (b < wk.n_segs) {
        csr_long_body<LPR, VEC, XK>(b, wk.segs, wk.partial, red, a);
        return;
    }
    b -= wk.n_segs;
    const int64_t mid_blocks = wk.mid_blocks;
    if (b < mid_blocks) {
        if (wk.xcd_chunk_mid > 0) {                              // same XCD-local runs as for the short rows below
            const int64_t x = blockIdx.x & 7, q = b >> 3;
            b = ((q / wk.xcd_chunk_mid) * 8 + x) * wk.xcd_chunk_mid + q % wk.xcd_chunk_mid;
        }
        csr_mid_body<LPR, VEC, XK>(b, wk.n_mid, wk.mid_rows, a);
        return;
    }
    b -= mid_blocks;
    if (wk.xcd_chunk > 0) {
        // Workgroups go to the eight XCDs round-robin by their linear id, and each XCD has an L2 of
        // its own.  Hand out the short rows in runs of xcd_chunk consecutive workgroups, run r to XCD
        // r % 8: neighbouring rows -- which share columns in graphs with any locality -- then meet in
        // one L2 close in time, while all XCDs still advance through the matrix side by side (rows
        // sorted by degree stay balanced).
        const int64_t x = blockIdx.x & 7, q = b >> 3;
        b = ((q / wk.xcd_chunk) * 8 + x) * wk.xcd_chunk + q % wk.xcd_chunk;
    }
    csr_short_body<LPR, VEC, XK>(b, wk.n_items, wk.row_list, wk.route, wk.rows_per_group, wk.mid_row, a);
}

// The same launch with the update stage fused into the short rows; long and mid rows write their
// aggregated rows to a.Y (the workspace Z) and are finished by k_update_rest.
template <int LPR, int VEC, int XK>
__global__ __launch_bounds__(256) void k_csr_fused(CsrWork wk, SpmmArgs a, UpdateArgs u)
{
    using S = FusedShape<LPR, VEC>;
    __shared__ float red[256 * VEC];
    __shared__ float zt[S::ROWS * S::LDZ];
    __shared__ int32_t rows16[S::ROWS];
    int64_t b = blockIdx.x;
    if (b < wk.n_segs) {
        csr_long_body<LPR, VEC, XK>(b, wk.segs, wk.partial, red, a);
        return;
    }
    b -= wk.n_segs;
    const int64_t mid_blocks = wk.mid_blocks;
    if (b < mid_blocks) {
        csr_mid_body<LPR, VEC, XK>(b, wk.n_mid, wk.mid_rows, a, wk.mid_row);   // the fused tier takes rows up to mid_row
        return;
    }
    b -= mid_blocks;
    if (wk.xcd_chunk > 0) {                                     // XCD-local runs, as in k_csr
        const int64_t x = blockIdx.x & 7, q = b >> 3;
        b = ((q / wk.xcd_chunk) * 8 + x) * wk.xcd_chunk + q % wk.xcd_chunk;
    }
    csr_short_fused_body<LPR, VEC, XK>(b, wk.n_items, wk.row_list, wk.route, wk.mid_row, a, u, zt, rows16);
}

// ---- rows the fused kernels did not finish: gather their aggregated rows and apply the update ---
// One wave per 16 entries of the plan's list of such rows (rows of matrix-path windows wider than
// the wave-per-window kernel handles, scalar-path rows above the short tier): they were written to
// Z, are read back as a 16-row tile and multiplied by W.
// NT: output columns per lane and pass (chosen on the host by update_tile_nt; a narrower NT needs fewer registers,
// which is what bounds the waves in flight of this streaming kernel).
template <int ZD, int NT>
__global__ __launch_bounds__(256) void k_update_rest(int32_t n_rest, const int32_t* __restrict__ rest_rows, int tiles_per_wave,
                                                     SpmmArgs a, UpdateArgs u)
{
    constexpr int ldz = ZD + 4;                                 // ZD >= d
    __shared__ float tiles[4 * 16 * ldz];
    __shared__ int32_t rows_s[2][64];                           // two row lists per wave, alternating between tiles
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t n_tiles = ((int64_t)n_rest + 15) / 16;
    const int64_t t_begin = ((int64_t)blockIdx.x * 4 + wave) * tiles_per_wave;
    const int64_t t_end = min(n_tiles, t_begin + tiles_per_wave);
    if (t_begin >= t_end) return;
    float* __restrict__ zt = tiles + wave * 16 * ldz;
    constexpr int kPerLane = 16 * ZD / 4 / 64;                  // float4 per lane for the widest tile
    const int per_row = a.d >> 2;
    float4 v[kPerLane];
    // A wave walks tiles_per_wave consecutive 16-row tiles.  The whole 16 x d tile is requested at once, all lanes busy;
    // the next tile's rows are requested as soon as the current tile is parked in LDS, so they arrive during its MFMAs.
    auto request = [&](int64_t tile, int32_t* __restrict__ rows16) {
        const int64_t i0 = tile * 16;
        if (lane < 16) rows16[lane] = i0 + lane < n_rest ? (rest_rows ? rest_rows[i0 + lane] : (int32_t)(i0 + lane)) : -1;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) {
            const int idx = lane + 64 * j;
            v[j] = make_float4(0.f, 0.f, 0.f, 0.f);             // tile rows past the list are zero and never stored
            if (idx < 16 * per_row) {
                const int32_t rr = rows16[idx / per_row];
                if (rr >= 0) v[j] = *reinterpret_cast<const float4*>(&a.Y[(int64_t)rr * a.ldy + (idx % per_row) * 4]);
            }
        }
    };
    request(t_begin, rows_s[0] + wave * 16);
    for (int64_t t = t_begin; t < t_end; ++t) {
        int32_t* __restrict__ rows16 = rows_s[(t - t_begin) & 1] + wave * 16;
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) {
            const int idx = lane + 64 * j;
            if (idx < 16 * per_row) *reinterpret_cast<float4*>(&zt[(idx / per_row) * ldz + (idx % per_row) * 4]) = v[j];
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (t + 1 < t_end) request(t + 1, rows_s[(t + 1 - t_begin) & 1] + wave * 16);
        update_tile16_nt<NT>(zt, ldz, rows16, a.d, u, lane, 0, 1);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the tile's LDS reads are done before it is overwritten
    }
}

// ---- rows cut into several segments: add the partial rows in segment order ------------------
__global__ __launch_bounds__(256) void k_reduce_partials(int32_t n_multi, const MultiRow* __restrict__ multi,
                                                         const float* __restrict__ partial, SpmmArgs a)
{
    const MultiRow m = multi[blockIdx.x];
    for (int c = threadIdx.x; c < a.d; c += 256) {
        float acc = 0.f;
        for (int q = 0; q < m.n_slots; ++q) acc += partial[(int64_t)(m.first_slot + q) * a.d + c];
        const float one[1] = {acc};
        out_store<1>(a.Y, a.y_dtype, (int64_t)m.row * a.ldy + c, one, a.relu);
    }
}

// ---- dispatch ---------------------------------------------------------------------------------
struct CsrShape { int lpr, vec; };

static CsrShape pick_shape(const SpmmArgs& a, const float* partial)
{
    int vec = 1;
    const uintptr_t px = (uintptr_t)a.X, py = (uintptr_t)a.Y, pp = (uintptr_t)partial;
    const bool y4 = a.ldy % 4 == 0 && py % 16 == 0 && pp % 16 == 0;
    if (a.x_dtype == HCSPMM_F32) {
        if (a.d % 4 == 0 && a.ldx % 4 == 0 && px % 16 == 0 && y4) vec = 4;
        else if (a.d % 2 == 0 && a.ldx % 2 == 0 && a.ldy % 2 == 0 && px % 8 == 0 && py % 8 == 0 && pp % 8 == 0) vec = 2;
    } else {
        if (a.d % 8 == 0 && a.ldx % 8 == 0 && px % 16 == 0 && y4) vec = 8;
        else if (a.d % 4 == 0 && a.ldx % 4 == 0 && px % 8 == 0 && y4) vec = 4;
    }
    // a group needs at least kRowsPerGroup lanes; narrow the vectors of narrow matrices instead of idling lanes
    const int min_vec = 1;
    while (vec > min_vec && (a.d + vec - 1) / vec < kRowsPerGroup) {
        vec >>= 1;
        if (a.x_dtype != HCSPMM_F32 && vec == 2) vec = 1;      // 16-bit inputs have no 2-wide variant
    }
    const int lanes = (a.d + vec - 1) / vec;       // lanes needed to cover the width once
    int lpr = kRowsPerGroup;
    while (lpr < 64 && lpr < lanes) lpr <<= 1;
    return {lpr, vec};
}

#define HC_CSR_CASES(FN, XK, V)                                                                    \
    switch (sh.lpr) {                                                                              \
        case 8: FN(8, V, XK); break;                                                               \
        case 16: FN(16, V, XK); break;                                                             \
        case 32: FN(32, V, XK); break;                                                             \
        default: FN(64, V, XK); break;                                                             \
    }

#define HC_CSR_DISPATCH(FN)                                                                        \
    if (a.x_dtype == HCSPMM_F32) {                                                                 \
        if (sh.vec == 4) { HC_CSR_CASES(FN, 0, 4) } else if (sh.vec == 2) { HC_CSR_CASES(FN, 0, 2) } else { HC_CSR_CASES(FN, 0, 1) } \
    } else if (a.x_dtype == HCSPMM_BF16) {                                                         \
        if (sh.vec == 8) { HC_CSR_CASES(FN, 1, 8) } else if (sh.vec == 4) { HC_CSR_CASES(FN, 1, 4) } else { HC_CSR_CASES(FN, 1, 1) } \
    } else {                                                                                       \
        if (sh.vec == 8) { HC_CSR_CASES(FN, 2, 8) } else if (sh.vec == 4) { HC_CSR_CASES(FN, 2, 4) } else { HC_CSR_CASES(FN, 2, 1) } \
    }

// The fused update needs the whole aggregated row in one pass of a lane group, fp32 X read as
// float4/float2 and a width that the update's K loop takes 16 at a time.
bool update_fusable(const SpmmArgs& a)
{
    if (a.d % 16 != 0 || a.d < 16 || a.d > 256) return false;
    const CsrShape sh = pick_shape(a, nullptr);
    const bool vec_ok = a.x_dtype == HCSPMM_F32 ? (sh.vec == 4 || sh.vec == 2) : (sh.vec == 8 || sh.vec == 4);
    return vec_ok && sh.lpr * sh.vec >= a.d && a.ldy % 4 == 0 && (uintptr_t)a.Y % 16 == 0 && mfma_update_fusable(a);
}

hipError_t launch_csr(const SpmmArgs& a, int32_t n_segs, const Segment* segs, float* partial, int32_t n_mid,
                      const int32_t* mid_rows, int32_t n_items, const int32_t* row_list, const uint8_t* route,
                      int32_t mid_row, hipStream_t s, const UpdateArgs* upd)
{
    const CsrShape sh = pick_shape(a, partial);
    // XCD-local runs (see k_csr): tiers of at least 1024 workgroups are padded to whole rounds of
    // eight runs; the surplus workgroups exit at once
    int run = 32;
    if (tune().xcd_chunk >= 0) run = tune().xcd_chunk;
    auto pad_runs = [run](int64_t n, int32_t& chunk) {
        chunk = 0;
        if (run <= 0 || n < 1024) return n;
        chunk = run;
        return (n + 8 * run - 1) / (8 * run) * (8 * (int64_t)run);
    };
    if (upd) {
        const int rows_per_wg = sh.lpr == 8 ? 32 : 16;          // FusedShape<LPR, VEC>::ROWS
        int32_t xcd_chunk = 0;
        const int64_t short_blocks = pad_runs(((int64_t)n_items + rows_per_wg - 1) / rows_per_wg, xcd_chunk);
        const int64_t blocks = (int64_t)n_segs + ((int64_t)n_mid + 3) / 4 + short_blocks;
        if (blocks <= 0) return hipSuccess;
        CsrWork wk{n_segs, segs, partial, n_mid, mid_rows, n_items, row_list, route, 0, mid_row, xcd_chunk, ((int64_t)n_mid + 3) / 4, 0};
#define HC_LAUNCH_CSRF(L, V, K) hipLaunchKernelGGL((k_csr_fused<L, V, K>), dim3((unsigned)blocks), dim3(256), 0, s, wk, a, *upd)
#define HC_CSRF_CASES(V, K)                                                                        \
    switch (sh.lpr) {                                                                              \
        case 8: HC_LAUNCH_CSRF(8, V, K); break;                                                    \
        case 16: HC_LAUNCH_CSRF(16, V, K); break;                                                  \
        case 32: HC_LAUNCH_CSRF(32, V, K); break;                                                  \
        default: HC_LAUNCH_CSRF(64, V, K); break;                                                  \
    }
        if (a.x_dtype == HCSPMM_F32) {
            if (sh.vec == 4) { HC_CSRF_CASES(4, 0) } else if (sh.vec == 2) { HC_CSRF_CASES(2, 0) } else return hipErrorInvalidValue;
        } else if (a.x_dtype == HCSPMM_BF16) {
            if (sh.vec == 8) { HC_CSRF_CASES(8, 1) } else if (sh.vec == 4) { HC_CSRF_CASES(4, 1) } else return hipErrorInvalidValue;
        } else {
            if (sh.vec == 8) { HC_CSRF_CASES(8, 2) } else if (sh.vec == 4) { HC_CSRF_CASES(4, 2) } else return hipErrorInvalidValue;
        }
#undef HC_CSRF_CASES
#undef HC_LAUNCH_CSRF
        return hipGetLastError();
    }
    // consecutive rows per lane group: measured best when a wave walks about four to eight rows in
    // all (one row per group for 8- and 16-lane groups, two for 32, four for 64) -- more rows per
    // group serialise dependent loads, fewer pay the per-row set-up too often -- and only while the
    // launch still has tens of thousands of waves to hide the rows' dependent-load latencies
    int rpg = sh.lpr / 16 > 1 ? sh.lpr / 16 : 1;
    while (rpg > 1 && ((int64_t)n_items / rpg) * sh.lpr / 64 < 32768) rpg >>= 1;
    if (tune().rpg >= 1 && tune().rpg <= kRowsPerGroup) rpg = tune().rpg;
    const int64_t n_groups = ((int64_t)n_items + rpg - 1) / rpg;
    const int gpb = 256 / sh.lpr;
    int32_t xcd_chunk = 0, xcd_chunk_mid = 0;
    const int64_t short_blocks = pad_runs((n_groups + gpb - 1) / gpb, xcd_chunk);
    const int64_t mid_blocks = pad_runs(((int64_t)n_mid + 3) / 4, xcd_chunk_mid);
    const int64_t blocks = (int64_t)n_segs + mid_blocks + short_blocks;
    if (blocks <= 0) return hipSuccess;
    CsrWork wk{n_segs, segs, partial, n_mid, mid_rows, n_items, row_list, route, rpg, mid_row, xcd_chunk, mid_blocks, xcd_chunk_mid};
#define HC_LAUNCH_CSR(L, V, K) hipLaunchKernelGGL((k_csr<L, V, K>), dim3((unsigned)blocks), dim3(256), 0, s, wk, a)
    HC_CSR_DISPATCH(HC_LAUNCH_CSR)
#undef HC_LAUNCH_CSR
    return hipGetLastError();
}

// The same kernel as a dense product for narrow outputs: T = act(X W) for X m x k (k a multiple of 16 up to 128, rows
// 16-byte aligned), every wave taking 16 consecutive rows.  A 128-column GEMM tile would spend most of its matrix work
// on padding when W has 64 columns or fewer; here the product streams X once and W stays in L1/L2.
bool gemm_rows16_usable(int64_t m, int32_t k, int32_t n, const float* X, int64_t ldx)
{
    return m < ((int64_t)1 << 31) && k % 16 == 0 && k >= 16 && k <= 128 && n <= 64 && ldx % 4 == 0 && (uintptr_t)X % 16 == 0;
}

hipError_t launch_gemm_rows16(int64_t m, int32_t k, int32_t n, const float* X, int64_t ldx, const float* W, int64_t ldw,
                              float* T, int64_t ldt, int relu, hipStream_t s, int32_t t_dtype)
{
    SpmmArgs a{};
    a.n_rows = (int32_t)m; a.d = k; a.Y = const_cast<float*>(X); a.ldy = ldx;      // the kernel only reads these rows
    const UpdateArgs u{W, ldw, n, T, ldt, relu ? 1 : 0, 0, nullptr, 0, t_dtype};
    return launch_update_rest(a, (int32_t)m, nullptr, u, s);
}

hipError_t launch_update_rest(const SpmmArgs& a, int32_t n_rest, const int32_t* rest_rows, const UpdateArgs& upd,
                              hipStream_t s)
{
    if (n_rest <= 0) return hipSuccess;
    // several consecutive tiles per wave once there are enough tiles to keep every CU supplied with waves
    const int64_t n_tiles = ((int64_t)n_rest + 15) / 16;
    int tpw = 1;
    while (tpw < 8 && n_tiles / (2 * tpw) >= 16384) tpw *= 2;
    if (tune().tiles_per_wave >= 1 && tune().tiles_per_wave <= 64) tpw = tune().tiles_per_wave;
    const dim3 grid((unsigned)((n_tiles + 4 * (int64_t)tpw - 1) / (4 * (int64_t)tpw)));
    const int nt = update_tile_nt(upd, 1);
#define HC_REST(ZD)                                                                                                   \
    {                                                                                                                 \
        if (nt == 4) hipLaunchKernelGGL((k_update_rest<ZD, 4>), grid, dim3(256), 0, s, n_rest, rest_rows, tpw, a, upd);      \
        else if (nt == 2) hipLaunchKernelGGL((k_update_rest<ZD, 2>), grid, dim3(256), 0, s, n_rest, rest_rows, tpw, a, upd); \
        else hipLaunchKernelGGL((k_update_rest<ZD, 1>), grid, dim3(256), 0, s, n_rest, rest_rows, tpw, a, upd);              \
    }
    if (a.d <= 64) HC_REST(64)
    else if (a.d <= 128) HC_REST(128)
    else if (a.d <= 256) HC_REST(256)
    else return hipErrorInvalidValue;
#undef HC_REST
    return hipGetLastError();
}

// ---- measurement aid: the bare gather ------------------------------------------------------------
// Reads row index[i] of X for every i and does nothing else a sparse product would do (no row
// structure, no values, no output rows): a lane group takes a contiguous run of indices, LPR at a
// time with one coalesced load, keeps eight row requests in flight like the scalar path, and adds
// what arrives into registers; one vector per lane is stored at the end so the loads stay live.
// Its duration is the floor of any kernel that fetches one X row per non-zero of the same stream.
template <int LPR>
__global__ __launch_bounds__(256) void k_probe_gather(const int32_t* __restrict__ index, int64_t n, int64_t per_group,
                                                      const float* __restrict__ X, int64_t ldx, int32_t d,
                                                      int32_t n_rows_x, float* __restrict__ out)
{
    // workgroups in XCD-local runs of 32, like the scalar path's short rows (the grid is padded to whole rounds)
    const int64_t x = blockIdx.x & 7, q = blockIdx.x >> 3;
    const int64_t blk = ((q / 32) * 8 + x) * 32 + q % 32;
    const int64_t grp = blk * (256 / LPR) + threadIdx.x / LPR;
    const int lig = threadIdx.x % LPR;
    const int64_t b = min(n, grp * per_group), e = min(n, b + per_group);
    const int c = 4 * lig < d ? 4 * lig : 0;
    const char* __restrict__ Xc = reinterpret_cast<const char*>(X + c);
    float acc[4];
    vzero<4>(acc);
    for (int64_t k0 = b; k0 < e; k0 += LPR) {                   // (a group past the end of the stream has b == e)
        const int64_t k = min(k0 + lig, e - 1);
        const int32_t mc = min(max(index[k], 0), n_rows_x - 1);       // whatever the stream holds, the read stays inside X
        batch_accumulate<LPR, 4, 0>(mc, 1.f, (int)min((int64_t)LPR, e - k0), Xc, ldx * 4, acc);
    }
    *reinterpret_cast<float4*>(out + ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4) = make_float4(acc[0], acc[1], acc[2], acc[3]);
}

// Launch shape of the probe: lanes per row from d like the scalar path; indices per lane group 512 (long enough
// to amortise the start-up) unless the stream is too short to give every CU some tens of workgroups that way --
// then fewer, down to 64.
static void probe_gather_shape(int64_t n, int32_t d, int& lpr, int64_t& per_group, int64_t& blocks)
{
    lpr = 8;
    while (lpr < 64 && lpr * 4 < d) lpr <<= 1;
    const int64_t groups_per_block = 256 / lpr;
    per_group = (n / (8192 * groups_per_block) + 63) / 64 * 64;
    per_group = per_group < 64 ? 64 : (per_group > 512 ? 512 : per_group);
    const int64_t groups = (n + per_group - 1) / per_group;
    blocks = (groups + groups_per_block - 1) / groups_per_block;
    blocks = (blocks + 255) / 256 * 256;                       // whole rounds of eight XCD-local runs of 32 workgroups
}

int64_t probe_gather_blocks(int64_t n, int32_t d)
{
    int lpr;
    int64_t per_group, blocks;
    probe_gather_shape(n, d, lpr, per_group, blocks);
    return blocks;
}

hipError_t launch_probe_gather(const int32_t* index, int64_t n, const float* X, int64_t ldx, int32_t d, int32_t n_rows_x,
                               float* out, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    int lpr;
    int64_t per_group, blocks;
    probe_gather_shape(n, d, lpr, per_group, blocks);
#define HC_PROBE(L) hipLaunchKernelGGL((k_probe_gather<L>), dim3((unsigned)blocks), dim3(256), 0, s, index, n, per_group, X, ldx, d, n_rows_x, out)
    switch (lpr) {
        case 8: HC_PROBE(8); break;
        case 16: HC_PROBE(16); break;
        case 32: HC_PROBE(32); break;
        default: HC_PROBE(64); break;
    }
#undef HC_PROBE
    return hipGetLastError();
}

hipError_t launch_reduce_partials(const SpmmArgs& a, int32_t n_multi, const MultiRow* multi, const float* partial,
                                  hipStream_t s)
{
    if (n_multi <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_reduce_partials, dim3(n_multi), dim3(256), 0, s, n_multi, multi, partial, a);
    return hipGetLastError();
}

}  // namespace hcspmm
