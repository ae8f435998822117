// Matrix path: a row window's condensed 16 x ncols tile times the gathered X rows on the MFMA
// units (Alg. 2 gives the scheme: densify a slice of the condensed window into on-chip memory,
// fetch the matching X rows, multiply on the matrix cores, accumulate in registers, store the
// 16 x d result; Alg. 4's cooperative loading becomes the lane mapping below).
//
// fp32 path: v_mfma_f32_16x16x4_f32, i.e. D(16x16) += A(16x4) * B(4x16) per wave, true fp32.
// Operand layout per lane l (0..63):  A: row l%16, k = l/16.   B: k = l/16, column l%16.
//                                      D: column l%16, rows 4*(l/16) + {0,1,2,3} in 4 registers.
// A K-step therefore consumes 4 condensed columns: the lanes with the same l/16 read the same X
// row, 16 lanes wide.  Every lane reads VW consecutive floats of that row, which spreads them
// over VW accumulator tiles (tile t holds the output columns  base + VW*(l%16) + t), so a whole
// 16*VW-float stretch of the X row is one contiguous, coalesced read and the results go back to Y
// as VW-wide vector stores.  Each distinct column of the window is fetched once per window.
//
// The condensed A tile is rebuilt on chip from the window's non-zeros (value, condensed column,
// row): a k-major LDS image  tile[k*16 + row], zeroed and then filled with LDS float adds, so
// duplicate entries accumulate.  Read back, lane l of K-step q needs tile[(4q + l/16)*16 + l%16]
// = tile[64q + l]: conflict-free.
//
// Like any dense-tile formulation (the paper's included) this path multiplies every gathered X
// row with explicit zeros, so X must be finite: a NaN or Inf in a gathered row reaches all 16
// rows of the window, not only the rows that reference it.
#include "common.hpp"

namespace hcspmm {

typedef float v4f __attribute__((ext_vector_type(4)));

template <int VW> struct XVec;
template <> struct XVec<4> { using type = float4; };
template <> struct XVec<2> { using type = float2; };
template <> struct XVec<1> { using type = float; };

template <int VW>
__device__ inline void load_x(const float* __restrict__ p, float (&x)[VW])
{
    using V = typename XVec<VW>::type;
    V v = *reinterpret_cast<const V*>(p);
    const float* f = reinterpret_cast<const float*>(&v);
#pragma unroll
    for (int i = 0; i < VW; ++i) x[i] = f[i];
}

// A run of up to 16*NCR K-steps (64*NCR condensed columns) for one wave, software-pipelined:
// the X rows of stage s+1 are requested before the MFMAs of stage s are issued, so the gather
// latency hides behind the matrix work of the same wave.
//   tile   : LDS image of the A columns of this run (k-major, tile[k*16 + row])
//   mycol  : the run's column ids, lane l of mycol[i] holds condensed column 64*i + l; slots past the
//            window's last column repeat that last column (their A entries are zero), so every load
//            is unconditional and a whole stage is in flight together
template <int VW, int NG> struct MfmaPipe {
    static constexpr int U = (NG * VW >= 8) ? 4 : 8;       // K-steps per pipeline stage
};

// requests the X rows of K-steps [st*U, st*U + U) of a run into buf
template <int VW, int NG, int NCR>
__device__ inline void mfma_stage_load(int st, const int32_t (&mycol)[NCR], int lane, const float* __restrict__ X,
                                       int64_t ldx, int d, float (&buf)[MfmaPipe<VW, NG>::U][NG][VW])
{
    constexpr int U = MfmaPipe<VW, NG>::U;
    const int j = lane & 15, kk = lane >> 4;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int q = st * U + u;
        const int32_t c = __shfl(mycol[q >> 4], 4 * (q & 15) + kk, 64);
        const float* __restrict__ xr = X + (int64_t)c * ldx;
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int col = g * 16 * VW + VW * j;           // columns past d read column 0 and are never stored
            load_x<VW>(xr + (col < d ? col : 0), buf[u][g]);
        }
    }
}

template <int VW, int NG>
__device__ inline void mfma_stage_compute(int st, const float* __restrict__ tile, int lane,
                                          const float (&buf)[MfmaPipe<VW, NG>::U][NG][VW], v4f (&acc)[NG][VW])
{
    constexpr int U = MfmaPipe<VW, NG>::U;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int q = st * U + u;
        const float av = tile[4 * q * 16 + lane];
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int t = 0; t < VW; ++t)
                acc[g][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, buf[u][g][t], acc[g][t], 0, 0, 0);
    }
}

// PRELOADED: stage 0 of the run is already in flight in xa[0] (requested by the caller before it
// built the A tile, so that the first gather overlaps the tile construction).
template <int VW, int NG, int NCR, bool PRELOADED>
__device__ inline void mfma_run(const float* __restrict__ tile, int nsteps, const int32_t (&mycol)[NCR], int lane,
                                const float* __restrict__ X, int64_t ldx, int d,
                                float (&xa)[2][MfmaPipe<VW, NG>::U][NG][VW], v4f (&acc)[NG][VW])
{
    constexpr int U = MfmaPipe<VW, NG>::U;
    constexpr int NST = 16 * NCR / U;
#pragma unroll
    for (int st = 0; st <= NST; ++st) {
        if (st < NST && st * U < nsteps && !(PRELOADED && st == 0))
            mfma_stage_load<VW, NG, NCR>(st, mycol, lane, X, ldx, d, xa[st & 1]);
        if (st >= 1 && (st - 1) * U < nsteps) mfma_stage_compute<VW, NG>(st - 1, tile, lane, xa[(st - 1) & 1], acc);
    }
}

template <int VW, int NG>
__device__ inline void store_tile(const v4f (&acc)[NG][VW], int lane, int32_t r0, int32_t n_rows, float* __restrict__ Y,
                                  int64_t ldy, int d, int relu)
{
    using V = typename XVec<VW>::type;
    const int j = lane & 15, kk = lane >> 4;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int col = g * 16 * VW + VW * j;
        if (col >= d) continue;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int32_t row = r0 + 4 * kk + r;
            if (row >= n_rows) continue;
            V v;
            float* f = reinterpret_cast<float*>(&v);
#pragma unroll
            for (int t = 0; t < VW; ++t) {
                float y = acc[g][t][r];
                f[t] = relu ? fmaxf(y, 0.f) : y;
            }
            *reinterpret_cast<V*>(Y + (int64_t)row * ldy + col) = v;
        }
    }
}

// ---- wave per window --------------------------------------------------------------------------
// Four independent waves per workgroup; each owns a private kKcSmall x 16 LDS tile and one window.
// No workgroup barrier: LDS traffic of a wave is issued and completed in program order.
// The dependent chain of a window is kept short: one descriptor read (scalar), then the column
// list and the first kEdgeRegs*64 non-zeros in one go, then the first X rows, and only then the
// LDS work that builds the A tile.
constexpr int kEdgeRegs = 6;

template <int VW, int NG>
__global__ __launch_bounds__(256) void k_mfma_small(int32_t n_list, const WinDesc* __restrict__ desc,
                                                    const int32_t* __restrict__ wcols,
                                                    const int32_t* __restrict__ erc, int col0, SpmmArgs a)
{
    __shared__ float tiles[4][kKcSmall * 16];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * 4 + wave;
    if (item >= n_list) return;
    const WinDesc ds = desc[item];
    const int32_t r0 = ds.w * kH, s = ds.s, e = ds.e, nc = ds.nc;
    const int64_t wp = ds.wp;
    float* __restrict__ tile = tiles[wave];
    const float* __restrict__ X = static_cast<const float*>(a.X) + col0;
    const int d = min(a.d - col0, NG * 16 * VW);
    constexpr int NCR = kKcSmall / 64;
    v4f acc[NG][VW];
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int t = 0; t < VW; ++t) acc[g][t] = (v4f){0.f, 0.f, 0.f, 0.f};
    float xa[2][MfmaPipe<VW, NG>::U][NG][VW];

    // first chunk: column list, non-zeros and first X rows requested back to back
    int32_t mycol[NCR];
#pragma unroll
    for (int i = 0; i < NCR; ++i) mycol[i] = wcols[wp + min(64 * i + lane, nc - 1)];
    int32_t pe[kEdgeRegs];
    float ve[kEdgeRegs];
#pragma unroll
    for (int q = 0; q < kEdgeRegs; ++q) {
        const int32_t k = min(s + 64 * q + lane, e - 1);
        pe[q] = erc[k];
        ve[q] = a.vals[k];
    }
    mfma_stage_load<VW, NG, NCR>(0, mycol, lane, X, a.ldx, d, xa[0]);
    for (int i = lane * 4; i < kKcSmall * 16; i += 256)
        *reinterpret_cast<float4*>(&tile[i]) = make_float4(0.f, 0.f, 0.f, 0.f);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
    for (int q = 0; q < kEdgeRegs; ++q) {
        const int32_t ec = pe[q] >> 4;
        if (s + 64 * q + lane < e && ec < kKcSmall) atomicAdd(&tile[ec * 16 + (pe[q] & 15)], ve[q]);
    }
    for (int32_t k = s + 64 * kEdgeRegs + lane; k < e; k += 64) {
        const int32_t p = erc[k];
        const int32_t ec = p >> 4;
        if (ec < kKcSmall) atomicAdd(&tile[ec * 16 + (p & 15)], a.vals[k]);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    mfma_run<VW, NG, NCR, true>(tile, (min(kKcSmall, nc) + 3) >> 2, mycol, lane, X, a.ldx, d, xa, acc);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

    // further chunks of wider windows
    for (int32_t kc0 = kKcSmall; kc0 < nc; kc0 += kKcSmall) {
        const int kend = min(kKcSmall, nc - kc0);
#pragma unroll
        for (int i = 0; i < NCR; ++i) mycol[i] = wcols[wp + min(kc0 + 64 * i + lane, nc - 1)];
        for (int i = lane * 4; i < kKcSmall * 16; i += 256)
            *reinterpret_cast<float4*>(&tile[i]) = make_float4(0.f, 0.f, 0.f, 0.f);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        for (int32_t k = s + lane; k < e; k += 64) {
            const int32_t p = erc[k];
            const int32_t ec = (p >> 4) - kc0;
            if (ec >= 0 && ec < kKcSmall) atomicAdd(&tile[ec * 16 + (p & 15)], a.vals[k]);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        mfma_run<VW, NG, NCR, false>(tile, (kend + 3) >> 2, mycol, lane, X, a.ldx, d, xa, acc);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
    store_tile<VW, NG>(acc, lane, r0, a.n_rows, a.Y + col0, a.ldy, d, a.relu);
}

// ---- workgroup per window ---------------------------------------------------------------------
// For windows with more condensed columns than one wave's tile holds: all four waves stage a
// KC-column chunk together, split its K-steps between them (blocks of 64 columns, round-robin)
// and add their partial tiles through LDS at the end, in wave order.  KC = kKcMid keeps the LDS
// footprint small for windows of a few hundred columns, KC = kKcBig serves the very wide ones.
// A workgroup owns one slice of a window's condensed columns: windows wider than kSliceCols are
// cut into several slices so that a hub window is not one workgroup's serial work; the slices'
// partial tiles go to memory and k_reduce_tiles adds them in slice order (deterministic).
template <int VW, int NG, int KC>
__global__ __launch_bounds__(256) void k_mfma_wg(const WgSlice* __restrict__ slices,
                                                  const int32_t* __restrict__ ncols, const int64_t* __restrict__ wptr,
                                                  const int32_t* __restrict__ wcols, const int32_t* __restrict__ erc,
                                                  int rows_sorted, const int32_t* __restrict__ slice_rows,
                                                  float* __restrict__ tile_partial, int col0, SpmmArgs a)
{
    constexpr int kAccFloats = NG * VW * 4 * 64;           // one wave's accumulators
    constexpr int kLdsFloats = KC * 16 > kAccFloats ? KC * 16 : kAccFloats;
    __shared__ float tile[kLdsFloats];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const WgSlice sl = slices[blockIdx.x];
    const int32_t w = sl.w;
    const int32_t r0 = w * kH;
    const int32_t s = a.rowptr[r0];
    const int32_t e = a.rowptr[min(r0 + kH, a.n_rows)];
    const int32_t nc = min(ncols[w], sl.kc_end);           // this workgroup owns condensed columns [kc_begin, nc)
    const int64_t wp = wptr[w];
    const float* __restrict__ X = static_cast<const float*>(a.X) + col0;
    const int d = min(a.d - col0, NG * 16 * VW);
    v4f acc[NG][VW];
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int t = 0; t < VW; ++t) acc[g][t] = (v4f){0.f, 0.f, 0.f, 0.f};

    float xa[2][MfmaPipe<VW, NG>::U][NG][VW];
    // When every row's columns ascend, so do its condensed columns: 16 threads per row keep a
    // cursor that only moves forward, and a chunk costs only the entries that fall into it.
    // Otherwise every chunk scans the whole window.
    const int my_r = threadIdx.x >> 4, l16 = threadIdx.x & 15;
    int32_t cur = a.rowptr[min(r0 + my_r, a.n_rows)];
    const int32_t row_e = a.rowptr[min(r0 + my_r + 1, a.n_rows)];
    // a later slice of a wide window starts each row at its first entry inside the slice (found at prepare time)
    if (rows_sorted && slice_rows) cur = slice_rows[(int64_t)blockIdx.x * kH + my_r];
    // Each wave owns the 64-column blocks wave, wave+4, ... of every chunk.  Its gather pipeline
    // runs across block and chunk boundaries: the next block's column ids are fetched one block
    // ahead and its first X rows are requested before the current block's last MFMAs -- for the
    // first block of a chunk that is before the chunk's A tile is even built.
    constexpr int U = MfmaPipe<VW, NG>::U;
    constexpr int NST = 16 / U;
    int32_t col_cur[1] = {0}, col_next[1] = {0};
    if (wave * 64 < min(KC, nc - sl.kc_begin)) {
        col_cur[0] = wcols[wp + min(sl.kc_begin + wave * 64 + lane, nc - 1)];
        mfma_stage_load<VW, NG, 1>(0, col_cur, lane, X, a.ldx, d, xa[0]);
    }
    for (int32_t kc0 = sl.kc_begin; kc0 < nc; kc0 += KC) {
        const int kend = min(KC, nc - kc0);
        for (int i = threadIdx.x * 4; i < KC * 16; i += 1024)
            *reinterpret_cast<float4*>(&tile[i]) = make_float4(0.f, 0.f, 0.f, 0.f);
        __syncthreads();
        if (rows_sorted) {
            const int32_t limit = kc0 + KC;
            for (;;) {
                const int32_t k = cur + l16;
                int32_t p = 0;
                bool take = false;
                if (k < row_e) {
                    p = erc[k];
                    take = (p >> 4) < limit;
                }
                if (take) atomicAdd(&tile[((p >> 4) - kc0) * 16 + my_r], a.vals[k]);
                const unsigned long long b = __ballot(take);
                const int n = __popc((unsigned)((b >> (16 * ((threadIdx.x & 63) >> 4))) & 0xffffu));
                cur += n;
                if (n < 16) break;
            }
        } else {
            for (int32_t k = s + threadIdx.x; k < e; k += 256) {
                const int32_t p = erc[k];
                const int32_t ec = (p >> 4) - kc0;
                if (ec >= 0 && ec < KC) atomicAdd(&tile[ec * 16 + (p & 15)], a.vals[k]);
            }
        }
        __syncthreads();
        for (int kb = wave * 64; kb < kend; kb += 256) {
            const int nsteps = (min(64, kend - kb) + 3) >> 2;
            int32_t nkc0 = kc0, nkb = kb + 256;
            if (nkb >= kend) { nkc0 = kc0 + KC; nkb = wave * 64; }
            const bool has_next = nkc0 < nc && nkb < min(KC, nc - nkc0);
            col_next[0] = has_next ? wcols[wp + min(nkc0 + nkb + lane, nc - 1)] : col_cur[0];
            const float* __restrict__ blk = tile + kb * 16;
#pragma unroll
            for (int st = 0; st < NST; ++st) {
                if (st + 1 < NST) {
                    if ((st + 1) * U < nsteps) mfma_stage_load<VW, NG, 1>(st + 1, col_cur, lane, X, a.ldx, d, xa[(st + 1) & 1]);
                } else if (has_next) {
                    mfma_stage_load<VW, NG, 1>(0, col_next, lane, X, a.ldx, d, xa[0]);
                }
                if (st * U < nsteps) mfma_stage_compute<VW, NG>(st, blk, lane, xa[st & 1], acc);
            }
            col_cur[0] = col_next[0];
        }
        __syncthreads();
    }
    // add the four waves' partial tiles in wave order: waves 1..3 park their registers in LDS one
    // after the other and wave 0 adds each in turn
    for (int v = 1; v < 4; ++v) {
        if (wave == v) {
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int t = 0; t < VW; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r) tile[((g * VW + t) * 4 + r) * 64 + lane] = acc[g][t][r];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int t = 0; t < VW; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[g][t][r] += tile[((g * VW + t) * 4 + r) * 64 + lane];
        }
        __syncthreads();
    }
    if (wave == 0) {
        if (sl.slot < 0) store_tile<VW, NG>(acc, lane, r0, a.n_rows, a.Y + col0, a.ldy, d, a.relu);
        else store_tile<VW, NG>(acc, lane, sl.slot * kH, 0x7fffffff, tile_partial + col0, a.d, d, 0);
    }
}

// windows cut into several column slices: add the slices' 16 x d partial tiles in slice order
__global__ __launch_bounds__(256) void k_reduce_tiles(const MultiRow* __restrict__ multi,
                                                      const float* __restrict__ tile_partial, SpmmArgs a)
{
    const MultiRow m = multi[blockIdx.x];                 // row = window id
    for (int i = threadIdx.x; i < kH * a.d; i += 256) {
        const int r = i / a.d, c = i - r * a.d;
        const int64_t row = (int64_t)m.row * kH + r;
        if (row >= a.n_rows) continue;
        float acc = 0.f;
        for (int q = 0; q < m.n_slots; ++q) acc += tile_partial[((int64_t)(m.first_slot + q) * kH + r) * a.d + c];
        a.Y[row * a.ldy + c] = a.relu ? fmaxf(acc, 0.f) : acc;
    }
}

// ---- dispatch ---------------------------------------------------------------------------------
struct MfmaShape { int vw, ng; };

static MfmaShape pick_mfma_shape(const SpmmArgs& a)
{
    const uintptr_t px = (uintptr_t)a.X, py = (uintptr_t)a.Y;
    int vw = 1;
    if (a.d % 4 == 0 && a.ldx % 4 == 0 && a.ldy % 4 == 0 && px % 16 == 0 && py % 16 == 0) vw = 4;
    else if (a.d % 2 == 0 && a.ldx % 2 == 0 && a.ldy % 2 == 0 && px % 8 == 0 && py % 8 == 0) vw = 2;
    // prefer the narrowest vector that still covers d in one 16-lane stretch (no idle lanes)
    while (vw > 1 && 16 * (vw / 2) >= a.d) vw >>= 1;
    const int groups = (a.d + 16 * vw - 1) / (16 * vw);
    int ng = groups >= 4 ? 4 : (groups >= 2 ? 2 : 1);
    return {vw, ng};
}

#define HC_MFMA_DISPATCH(FN)                                                                       \
    switch (sh.vw * 10 + sh.ng) {                                                                  \
        case 41: FN(4, 1); break;                                                                  \
        case 42: FN(4, 2); break;                                                                  \
        case 44: FN(4, 4); break;                                                                  \
        case 21: FN(2, 1); break;                                                                  \
        case 22: FN(2, 2); break;                                                                  \
        case 24: FN(2, 4); break;                                                                  \
        case 11: FN(1, 1); break;                                                                  \
        case 12: FN(1, 2); break;                                                                  \
        default: FN(1, 4); break;                                                                  \
    }

hipError_t launch_mfma_small(const SpmmArgs& a, int32_t n_list, const WinDesc* desc, const int32_t* wcols,
                             const int32_t* erc, hipStream_t s)
{
    if (n_list <= 0) return hipSuccess;
    const MfmaShape sh = pick_mfma_shape(a);
    const int span = sh.ng * 16 * sh.vw;                       // output columns per launch
    for (int col0 = 0; col0 < a.d; col0 += span) {
#define HC_LAUNCH_MS(V, G)                                                                         \
    hipLaunchKernelGGL((k_mfma_small<V, G>), dim3((unsigned)((n_list + 3) / 4)), dim3(256), 0, s, n_list, desc,      \
                       wcols, erc, col0, a)
        HC_MFMA_DISPATCH(HC_LAUNCH_MS)
#undef HC_LAUNCH_MS
    }
    return hipGetLastError();
}

hipError_t launch_mfma_wg(const SpmmArgs& a, int32_t n_list, const WgSlice* slices, const int32_t* ncols,
                          const int64_t* wptr, const int32_t* wcols, const int32_t* erc, int rows_sorted,
                          const int32_t* slice_rows, float* tile_partial, bool wide, hipStream_t s)
{
    if (n_list <= 0) return hipSuccess;
    const MfmaShape sh = pick_mfma_shape(a);
    const int span = sh.ng * 16 * sh.vw;
    for (int col0 = 0; col0 < a.d; col0 += span) {
#define HC_LAUNCH_MB(V, G)                                                                         \
    if (wide)                                                                                      \
        hipLaunchKernelGGL((k_mfma_wg<V, G, kKcBig>), dim3(n_list), dim3(256), 0, s, slices, ncols, wptr, wcols,     \
                           erc, rows_sorted, slice_rows, tile_partial, col0, a);                   \
    else                                                                                           \
        hipLaunchKernelGGL((k_mfma_wg<V, G, kKcMid>), dim3(n_list), dim3(256), 0, s, slices, ncols, wptr, wcols,     \
                           erc, rows_sorted, slice_rows, tile_partial, col0, a)
        HC_MFMA_DISPATCH(HC_LAUNCH_MB)
#undef HC_LAUNCH_MB
    }
    return hipGetLastError();
}

hipError_t launch_reduce_tiles(const SpmmArgs& a, int32_t n_multi, const MultiRow* multi, const float* tile_partial,
                               hipStream_t s)
{
    if (n_multi <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_reduce_tiles, dim3(n_multi), dim3(256), 0, s, multi, tile_partial, a);
    return hipGetLastError();
}

}  // namespace hcspmm
