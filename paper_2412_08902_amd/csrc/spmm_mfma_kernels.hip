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
// 16-bit path (X in bf16 or fp16): v_mfma_f32_16x16x16 with fp32 accumulation; a K-step is 16
// condensed columns, lane l supplies A(row l%16, k 4*(l/16)+{0..3}) and B(k 4*(l/16)+{0..3}, col
// l%16).  A lane reads VW consecutive 16-bit elements from each of its four X rows and transposes
// them in registers into VW B operands (one per accumulator tile), so the global reads are the
// same contiguous row stretches as on the fp32 path.  The A slice is accumulated in fp32 in LDS
// (layout [k/4][row][k%4], so a lane's four values are one 16-byte read) and rounded to the
// 16-bit type when it is read.
//
// Like any dense-tile formulation (the paper's included) this path multiplies every gathered X
// row with explicit zeros, so X must be finite: a NaN or Inf in a gathered row reaches all 16
// rows of the window, not only the rows that reference it.
#include <cstdlib>

#include "common.hpp"
#include "update_tile.hpp"

namespace hcspmm {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef short v4s __attribute__((ext_vector_type(4)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------------------
// Path policies.  A policy fixes, for one element kind XK (0 fp32, 1 bf16, 2 fp16), lane vector
// width VW and number of 16*VW-column groups NG:
//   SCOLS         condensed columns per pipeline stage (a 64-column block has 64/SCOLS stages)
//   Buf           registers of one stage's gathered X rows
//   load/compute  request a stage's X rows / issue its MFMAs
//   tidx          position of A(row r, condensed column k) in the LDS tile
// Column ids arrive as one register per 64-column block: lane l holds condensed column l of the
// block; slots past the window's last column repeat that last column (their A entries are zero),
// so every load is unconditional and a whole stage is in flight together.
// ------------------------------------------------------------------------------------------------
template <int XK, int VW, int NG> struct Path;

template <int VW, int NG> struct Path<0, VW, NG> {
    static constexpr int ES = 4;
    static constexpr int SCOLS = 16;
    static constexpr int U = SCOLS / 4;                        // K-steps (4 columns each) per stage
    struct Buf { float x[U][NG][VW]; };
    __device__ static inline int tidx(int k, int r) { return k * 16 + r; }
    // one K-step (4 condensed columns) of a stage
    __device__ static inline void load_step(int st, int u, int32_t mycol, int lane, const char* __restrict__ X,
                                            int64_t ldxb, int d, Buf& b)
    {
        const int j = lane & 15, kk = lane >> 4;
        const int q = st * U + u;                              // K-step inside the 64-column block
        const int32_t c = __shfl(mycol, 4 * q + kk, 64);
        const char* __restrict__ xr = X + (int64_t)c * ldxb;
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int col = g * 16 * VW + VW * j;              // columns past d read column 0 and are never stored
            const char* p = xr + (col < d ? col : 0) * ES;
            if constexpr (VW == 4) { const float4 v = *reinterpret_cast<const float4*>(p); b.x[u][g][0] = v.x; b.x[u][g][1] = v.y; b.x[u][g][2] = v.z; b.x[u][g][3] = v.w; }
            else if constexpr (VW == 2) { const float2 v = *reinterpret_cast<const float2*>(p); b.x[u][g][0] = v.x; b.x[u][g][1] = v.y; }
            else { b.x[u][g][0] = *reinterpret_cast<const float*>(p); }
        }
    }
    __device__ static inline void compute_step(int st, int u, const float* __restrict__ blk, int lane, const Buf& b,
                                               v4f (&acc)[NG][VW])
    {
        const int q = st * U + u;
        const float av = blk[64 * q + lane];                   // tidx(4q + lane/16, lane%16)
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int t = 0; t < VW; ++t)
                acc[g][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, b.x[u][g][t], acc[g][t], 0, 0, 0);
    }
    __device__ static inline void load(int st, int32_t mycol, int lane, const char* __restrict__ X, int64_t ldxb, int d,
                                       Buf& b)
    {
#pragma unroll
        for (int u = 0; u < U; ++u) load_step(st, u, mycol, lane, X, ldxb, d, b);
    }
    __device__ static inline void compute(int st, const float* __restrict__ blk, int lane, const Buf& b, v4f (&acc)[NG][VW])
    {
#pragma unroll
        for (int u = 0; u < U; ++u) compute_step(st, u, blk, lane, b, acc);
    }
};

__device__ inline uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);                           // round to nearest even (finite inputs)
    return u >> 16;
}

template <int XK, int VW, int NG> struct Path {
    static_assert(XK == 1 || XK == 2, "16-bit element kinds");
    static_assert(VW == 4 || VW == 8, "a lane reads 4 or 8 consecutive 16-bit elements");
    static constexpr int ES = 2;
    static constexpr int SCOLS = (NG * VW >= 8) ? 16 : 32;
    static constexpr int U = SCOLS / 16;                       // K-steps (16 columns each) per stage
    struct Buf { uint32_t w[U][NG][4][VW / 2]; };
    __device__ static inline int tidx(int k, int r) { return ((k >> 2) * 16 + r) * 4 + (k & 3); }
    __device__ static inline void load(int st, int32_t mycol, int lane, const char* __restrict__ X, int64_t ldxb, int d,
                                       Buf& b)
    {
        const int j = lane & 15, kg = lane >> 4;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int q = st * U + u;                          // K-step inside the 64-column block
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int32_t c = __shfl(mycol, 16 * q + 4 * kg + t, 64);
                const char* __restrict__ xr = X + (int64_t)c * ldxb;
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    const int col = g * 16 * VW + VW * j;
                    const char* p = xr + (col < d ? col : 0) * ES;
                    if constexpr (VW == 8) { const uint4 v = *reinterpret_cast<const uint4*>(p); b.w[u][g][t][0] = v.x; b.w[u][g][t][1] = v.y; b.w[u][g][t][2] = v.z; b.w[u][g][t][3] = v.w; }
                    else { const uint2 v = *reinterpret_cast<const uint2*>(p); b.w[u][g][t][0] = v.x; b.w[u][g][t][1] = v.y; }
                }
            }
        }
    }
    __device__ static inline void compute(int st, const float* __restrict__ blk, int lane, const Buf& b, v4f (&acc)[NG][VW])
    {
        const int i = lane & 15, kg = lane >> 4;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int q = st * U + u;
            // A(i, 16q + 4kg + {0..3}) accumulated in fp32, rounded here to the 16-bit type
            const float4 af = *reinterpret_cast<const float4*>(&blk[((4 * q + kg) * 16 + i) * 4]);
            uint32_t a_lo, a_hi;
            if constexpr (XK == 1) {
                a_lo = f32_to_bf16_bits(af.x) | (f32_to_bf16_bits(af.y) << 16);
                a_hi = f32_to_bf16_bits(af.z) | (f32_to_bf16_bits(af.w) << 16);
            } else {
                a_lo = (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)af.x) | ((uint32_t)__builtin_bit_cast(unsigned short, (_Float16)af.y) << 16);
                a_hi = (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)af.z) | ((uint32_t)__builtin_bit_cast(unsigned short, (_Float16)af.w) << 16);
            }
            const uint2 a2 = make_uint2(a_lo, a_hi);
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int m = 0; m < VW / 2; ++m) {
                    // transpose: element 2m / 2m+1 of the four rows -> the B operands of tiles 2m / 2m+1
                    const uint32_t w0 = b.w[u][g][0][m], w1 = b.w[u][g][1][m], w2 = b.w[u][g][2][m], w3 = b.w[u][g][3][m];
                    const uint2 be = make_uint2((w0 & 0xffffu) | (w1 << 16), (w2 & 0xffffu) | (w3 << 16));
                    const uint2 bo = make_uint2((w0 >> 16) | (w1 & 0xffff0000u), (w2 >> 16) | (w3 & 0xffff0000u));
                    if constexpr (XK == 1) {
                        acc[g][2 * m] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(v4s, a2), __builtin_bit_cast(v4s, be), acc[g][2 * m], 0, 0, 0);
                        acc[g][2 * m + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(v4s, a2), __builtin_bit_cast(v4s, bo), acc[g][2 * m + 1], 0, 0, 0);
                    } else {
                        acc[g][2 * m] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(v4h, a2), __builtin_bit_cast(v4h, be), acc[g][2 * m], 0, 0, 0);
                        acc[g][2 * m + 1] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(v4h, a2), __builtin_bit_cast(v4h, bo), acc[g][2 * m + 1], 0, 0, 0);
                    }
                }
        }
    }
};

// K-steps u, u+1, ... of a stage, each preceded by  s_waitcnt vmcnt(n)  with n = NG * (U-1-u) (capped at 15): the
// wave's n most recent requests may still be outstanding, all older ones must have returned.  (vmcnt below 16 sits in
// the low four bits of the operand; the expcnt and lgkmcnt fields are left at "no wait".)
template <class P, int NG, int VW, int u_>
__device__ inline void throttled_steps(int st, const float* __restrict__ blk, int lane, const typename P::Buf& b,
                                       v4f (&acc)[NG][VW])
{
    constexpr int kAllow = NG * (P::U - 1 - u_) > 15 ? 15 : NG * (P::U - 1 - u_);
    __builtin_amdgcn_s_waitcnt(0x0F70 | kAllow);
    P::compute_step(st, u_, blk, lane, b, acc);
    if constexpr (u_ + 1 < P::U) throttled_steps<P, NG, VW, u_ + 1>(st, blk, lane, b, acc);
}

// The stages of one 64-column block, software-pipelined: the X rows of stage s+1 -- or, after the
// block's last stage, of the next block's first stage -- are requested before the MFMAs of stage s
// are issued, so the gather latency hides behind the matrix work of the same wave.
//   blk       LDS image of the block's A columns;  ncols_blk: valid columns in the block (1..64)
//   xa        the two stage buffers; stage 0 of this block is already in flight in xa[0]
template <class P, int NG, int VW>
__device__ inline void block_stages(const float* __restrict__ blk, int ncols_blk, int32_t col_cur, bool has_next,
                                    int32_t col_next, int lane, const char* __restrict__ X, int64_t ldxb, int d,
                                    typename P::Buf (&xa)[2], v4f (&acc)[NG][VW])
{
    constexpr int NST = 64 / P::SCOLS;
    static_assert(NST % 2 == 0, "stage buffers alternate, a block must end on buffer 1");
    // Every request is unconditional (a stage past the block's last column, or a "next block" that does not exist,
    // re-reads valid rows: the column registers repeat the last column): requests inside branches would make the
    // compiler wait for ALL outstanding loads before a stage's MFMAs, which serialises gather and matrix work.
    (void)has_next;
#pragma unroll
    for (int st = 0; st < NST; ++st) {
        if constexpr (P::ES == 4) {
            // fp32: the requests of the next stage are throttled -- before K-step u of this stage all but the last
            // NG*(U-1-u) of them must have returned -- so a wave never has more than one stage of rows in flight
            // and that window shrinks to nothing by the end of the stage (measured: more rows in flight per wave
            // cost more in L2 hits on the shared columns than they hide in latency)
            if (st + 1 < NST) P::load(st + 1, col_cur, lane, X, ldxb, d, xa[(st + 1) & 1]);
            else P::load(0, col_next, lane, X, ldxb, d, xa[0]);
            if (st * P::SCOLS < ncols_blk) {
                throttled_steps<P, NG, VW, 0>(st, blk, lane, xa[st & 1], acc);
            }
        } else {
            if (st + 1 < NST) P::load(st + 1, col_cur, lane, X, ldxb, d, xa[(st + 1) & 1]);
            else P::load(0, col_next, lane, X, ldxb, d, xa[0]);
            if (st * P::SCOLS < ncols_blk) P::compute(st, blk, lane, xa[st & 1], acc);
        }
    }
}

// The same with the gathers three stages ahead of the MFMAs (four stage buffers in a ring), for
// paths whose 64-column block has four stages.  On entry the block's stages 0..2 are in flight in
// xa[0..2]; on exit, if there is a next block, its stages 0..2 are.  Stages past a block's last
// column still have valid column ids (they repeat the last column), so requesting them is harmless
// and the ring needs no per-stage bookkeeping.
template <class P, int NG, int VW>
__device__ inline void block_stages_deep(const float* __restrict__ blk, int ncols_blk, int32_t col_cur, bool has_next,
                                         int32_t col_next, int lane, const char* __restrict__ X, int64_t ldxb, int d,
                                         typename P::Buf (&xa)[4], v4f (&acc)[NG][VW])
{
    static_assert(64 / P::SCOLS == 4, "ring of four stage buffers");
    (void)has_next;                                             // requests are unconditional, see block_stages
    P::load(3, col_cur, lane, X, ldxb, d, xa[3]);
    P::compute(0, blk, lane, xa[0], acc);
    P::load(0, col_next, lane, X, ldxb, d, xa[0]);
    if (1 * P::SCOLS < ncols_blk) P::compute(1, blk, lane, xa[1], acc);
    P::load(1, col_next, lane, X, ldxb, d, xa[1]);
    if (2 * P::SCOLS < ncols_blk) P::compute(2, blk, lane, xa[2], acc);
    P::load(2, col_next, lane, X, ldxb, d, xa[2]);
    if (3 * P::SCOLS < ncols_blk) P::compute(3, blk, lane, xa[3], acc);
}

template <int VW, int NG>
__device__ inline void store_tile(const v4f (&acc)[NG][VW], int lane, int32_t r0, int32_t n_rows, float* __restrict__ Y,
                                  int64_t ldy, int col0, int d, int relu, int y_dtype = HCSPMM_F32)
{
    const int j = lane & 15, kk = lane >> 4;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int col = g * 16 * VW + VW * j;
        if (col >= d) continue;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int32_t row = r0 + 4 * kk + r;
            if (row >= n_rows) continue;
            float y[VW];
#pragma unroll
            for (int t = 0; t < VW; ++t) y[t] = acc[g][t][r];
            out_store<VW>(Y, y_dtype, (int64_t)row * ldy + col0 + col, y, relu);
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

// FUSE: instead of storing the window's 16 x d result, the wave parks it in its LDS region (the A
// tile is dead by then), multiplies it by W on the matrix cores and stores act(Z W): the update
// stage of the aggregate-then-update layer (Section V-A).  Needs d in one launch (col0 = 0).
template <int XK, int VW, int NG, bool FUSE = false>
__global__ __launch_bounds__(256) void k_mfma_small(int32_t n_list, const WinDesc* __restrict__ desc,
                                                    const int32_t* __restrict__ wcols,
                                                    const int32_t* __restrict__ erc, int col0, int xcd_chunk,
                                                    SpmmArgs a, UpdateArgs u)
{
    using P = Path<XK, VW, NG>;
    constexpr int kLdz = NG * 16 * VW + 4;
    constexpr int kRegion = (FUSE && 16 * kLdz > kKcSmall * 16) ? 16 * kLdz : kKcSmall * 16;
    __shared__ float tiles[4][kRegion];
    __shared__ int32_t rows_s[FUSE ? 64 : 1];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    int64_t blk = blockIdx.x;
    if (xcd_chunk > 0) {
        // runs of xcd_chunk consecutive workgroups (4 neighbouring windows each) go to one XCD, run r
        // to XCD r % 8, so that windows which share columns meet in one L2 close in time
        const int64_t x = blockIdx.x & 7, q = blk >> 3;
        blk = ((q / xcd_chunk) * 8 + x) * xcd_chunk + q % xcd_chunk;
    }
    const int64_t item = blk * 4 + wave;
    if (item >= n_list) return;
    const WinDesc ds = desc[item];
    const int32_t r0 = ds.w * kH, s = ds.s, e = ds.e, nc = ds.nc;
    const int64_t wp = ds.wp;
    float* __restrict__ tile = tiles[wave];
    const char* __restrict__ X = static_cast<const char*>(a.X) + (int64_t)col0 * P::ES;
    const int64_t ldxb = a.ldx * P::ES;
    const int d = min(a.d - col0, NG * 16 * VW);
    constexpr int NB = kKcSmall / 64;                          // 64-column blocks per chunk
    v4f acc[NG][VW];
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int t = 0; t < VW; ++t) acc[g][t] = (v4f){0.f, 0.f, 0.f, 0.f};
    typename P::Buf xa[2];

    // first chunk: column list, non-zeros and first X rows requested back to back
    int32_t mycol[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) mycol[i] = wcols[wp + min(64 * i + lane, nc - 1)];
    int32_t pe[kEdgeRegs];
    float ve[kEdgeRegs];
#pragma unroll
    for (int q = 0; q < kEdgeRegs; ++q) {
        const int32_t k = min(s + 64 * q + lane, e - 1);
        pe[q] = erc[k];
        ve[q] = a.vals[k];
    }
    P::load(0, mycol[0], lane, X, ldxb, d, xa[0]);
    for (int i = lane * 4; i < kKcSmall * 16; i += 256)
        *reinterpret_cast<float4*>(&tile[i]) = make_float4(0.f, 0.f, 0.f, 0.f);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
    for (int q = 0; q < kEdgeRegs; ++q) {
        const int32_t ec = pe[q] >> 4;
        if (s + 64 * q + lane < e && ec < kKcSmall) atomicAdd(&tile[P::tidx(ec, pe[q] & 15)], ve[q]);
    }
    for (int32_t k = s + 64 * kEdgeRegs + lane; k < e; k += 64) {
        const int32_t p = erc[k];
        const int32_t ec = p >> 4;
        if (ec < kKcSmall) atomicAdd(&tile[P::tidx(ec, p & 15)], a.vals[k]);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    for (int32_t kc0 = 0;;) {
        const int kend = min(kKcSmall, nc - kc0);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (64 * b < kend) {
                const bool has_next = b + 1 < NB && 64 * (b + 1) < kend;
                block_stages<P, NG, VW>(tile + 64 * b * 16, min(64, kend - 64 * b), mycol[b], has_next,
                                        mycol[b + 1 < NB ? b + 1 : b], lane, X, ldxb, d, xa, acc);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        // further chunks of wider windows: rebuild the tile from all the window's non-zeros
        kc0 += kKcSmall;
        if (kc0 >= nc) break;
#pragma unroll
        for (int i = 0; i < NB; ++i) mycol[i] = wcols[wp + min(kc0 + 64 * i + lane, nc - 1)];
        for (int i = lane * 4; i < kKcSmall * 16; i += 256)
            *reinterpret_cast<float4*>(&tile[i]) = make_float4(0.f, 0.f, 0.f, 0.f);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        P::load(0, mycol[0], lane, X, ldxb, d, xa[0]);
        for (int32_t k = s + lane; k < e; k += 64) {
            const int32_t p = erc[k];
            const int32_t ec = (p >> 4) - kc0;
            if (ec >= 0 && ec < kKcSmall) atomicAdd(&tile[P::tidx(ec, p & 15)], a.vals[k]);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
    if constexpr (FUSE) {
        int32_t* __restrict__ rows16 = rows_s + wave * 16;
        if (lane < 16) rows16[lane] = r0 + lane < a.n_rows ? r0 + lane : -1;
        const int j = lane & 15, kk = lane >> 4;
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int col = g * 16 * VW + VW * j;
            if (col >= d) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float* __restrict__ zp = tile + (4 * kk + r) * kLdz + col;
#pragma unroll
                for (int t = 0; t < VW; ++t) zp[t] = acc[g][t][r];
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (u.keep_z) store_tile_rows(tile, kLdz, rows16, 16, a.d, a.Y, a.ldy, lane, 64);
        update_tile16(tile, kLdz, rows16, a.d, u, lane);
    } else {
        store_tile<VW, NG>(acc, lane, r0, a.n_rows, a.Y, a.ldy, col0, d, a.relu, a.y_dtype);
    }
}

// ---- workgroup per window ---------------------------------------------------------------------
// For windows with more condensed columns than one wave's tile holds: all four waves stage a
// KC-column chunk together, split its K-steps between them (blocks of 64 columns, round-robin)
// and add their partial tiles through LDS at the end, in wave order.  KC = kKcMid keeps the LDS
// footprint small for windows of a few hundred columns, KC = kKcBig serves the very wide ones.
// A workgroup owns one slice of a window's condensed columns: windows wider than the plan's
// slice width are cut into several slices so that a hub window is not one workgroup's serial
// work; the slices' partial tiles go to memory and k_reduce_tiles adds them in slice order
// (deterministic).
template <int XK, int VW, int NG, int KC>
__global__ __launch_bounds__(256) void k_mfma_wg(const WgSlice* __restrict__ slices,
                                                  const int32_t* __restrict__ ncols, const int64_t* __restrict__ wptr,
                                                  const int32_t* __restrict__ wcols, const int32_t* __restrict__ erc,
                                                  int rows_sorted, const int32_t* __restrict__ slice_rows,
                                                  float* __restrict__ tile_partial, int col0, SpmmArgs a)
{
    using P = Path<XK, VW, NG>;
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
    const char* __restrict__ X = static_cast<const char*>(a.X) + (int64_t)col0 * P::ES;
    const int64_t ldxb = a.ldx * P::ES;
    const int d = min(a.d - col0, NG * 16 * VW);
    v4f acc[NG][VW];
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int t = 0; t < VW; ++t) acc[g][t] = (v4f){0.f, 0.f, 0.f, 0.f};
    constexpr bool kDeep = XK != 0 && 64 / P::SCOLS == 4;   // 16-bit X: gathers three stages ahead instead of one
    typename P::Buf xa[kDeep ? 4 : 2];

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
    int32_t col_cur = 0, col_next = 0;
    if (wave * 64 < min(KC, nc - sl.kc_begin)) {
        col_cur = wcols[wp + min(sl.kc_begin + wave * 64 + lane, nc - 1)];
        P::load(0, col_cur, lane, X, ldxb, d, xa[0]);
        if constexpr (kDeep) {
            P::load(1, col_cur, lane, X, ldxb, d, xa[1]);
            P::load(2, col_cur, lane, X, ldxb, d, xa[2]);
        }
    }
    for (int32_t kc0 = sl.kc_begin; kc0 < nc; kc0 += KC) {
        const int kend = min(KC, nc - kc0);
        // a row's 16 threads take its next kRound*16 entries per round: the round's loads are
        // independent (one memory latency per round, not per 16 entries) and the first round is
        // requested before the tile is cleared
        constexpr int kRound = 4;
        int32_t pr[kRound];
        float vr[kRound];
        auto fetch_round = [&]() {
#pragma unroll
            for (int j = 0; j < kRound; ++j) {
                const int32_t k = cur + 16 * j + l16;
                pr[j] = 0x7fffffff;                            // past the row's end: never taken
                vr[j] = 0.f;
                if (k < row_e) {
                    pr[j] = erc[k];
                    vr[j] = a.vals[k];
                }
            }
        };
        if (rows_sorted) fetch_round();
        for (int i = threadIdx.x * 4; i < KC * 16; i += 1024)
            *reinterpret_cast<float4*>(&tile[i]) = make_float4(0.f, 0.f, 0.f, 0.f);
        __syncthreads();
        if (rows_sorted) {
            const int32_t limit = min(kc0 + KC, nc);          // (entries from nc on belong to the window's next slice)
            const int shift = 16 * ((threadIdx.x & 63) >> 4);
            for (;;) {
                int n = 0;
#pragma unroll
                for (int j = 0; j < kRound; ++j) {
                    // entries ascend, so the ones taken are a prefix; 0x7fffffff is no packed entry (positions stay below 2^27 - 1)
                    const bool take = pr[j] != 0x7fffffff && (pr[j] >> 4) < limit;
                    if (take) atomicAdd(&tile[P::tidx((pr[j] >> 4) - kc0, my_r)], vr[j]);
                    const unsigned long long b = __ballot(take);
                    n += __popc((unsigned)((b >> shift) & 0xffffu));
                }
                cur += n;
                if (n < 16 * kRound) break;
                fetch_round();
            }
        } else {
            for (int32_t k = s + threadIdx.x; k < e; k += 256) {
                const int32_t p = erc[k];
                const int32_t ec = (p >> 4) - kc0;
                if (ec >= 0 && ec < kend) atomicAdd(&tile[P::tidx(ec, p & 15)], a.vals[k]);
            }
        }
        __syncthreads();
        for (int kb = wave * 64; kb < kend; kb += 256) {
            int32_t nkc0 = kc0, nkb = kb + 256;
            if (nkb >= kend) { nkc0 = kc0 + KC; nkb = wave * 64; }
            const bool has_next = nkc0 < nc && nkb < min(KC, nc - nkc0);
            col_next = has_next ? wcols[wp + min(nkc0 + nkb + lane, nc - 1)] : col_cur;
            if constexpr (kDeep)
                block_stages_deep<P, NG, VW>(tile + kb * 16, min(64, kend - kb), col_cur, has_next, col_next, lane, X, ldxb,
                                             d, xa, acc);
            else
                block_stages<P, NG, VW>(tile + kb * 16, min(64, kend - kb), col_cur, has_next, col_next, lane, X, ldxb, d,
                                        xa, acc);
            col_cur = col_next;
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
        if (sl.slot < 0) store_tile<VW, NG>(acc, lane, r0, a.n_rows, a.Y, a.ldy, col0, d, a.relu, a.y_dtype);
        else store_tile<VW, NG>(acc, lane, sl.slot * kH, 0x7fffffff, tile_partial, a.d, col0, d, 0);
    }
}

// ---- workgroup per run of windows: gathered X rows shared through LDS -------------------------
// Neighbouring windows share columns (a community's members, a power-law graph's hubs), and on the
// matrix path loading X is the larger part of the work (Section IV-B, Table I).  Here a workgroup owns a
// RUN of up to four consecutive matrix-path windows, one per wave.  Preprocessing merges the windows'
// column lists into the run's ascending UNION list and gives every condensed column of a window its
// position ("slot") in that union.  The workgroup walks the union in chunks of UC columns: all 256
// threads fetch the chunk's X rows ONCE into LDS (requests for chunk c+1 are in flight during the
// matrix work of chunk c; two LDS buffers alternate, one barrier per chunk), and every wave multiplies
// ITS OWN window's condensed columns that fall into the chunk -- a contiguous range of its list, since
// both lists ascend -- taking the B operands from the staged rows by slot.  The dense A tile is still
// the 16-row window's own (the MFMA work does not grow with the run), only the row fetches shrink to
// the union's.  The A slice of a chunk is rebuilt in the wave's private LDS tile from the rows'
// non-zeros with per-row cursors (rows are sorted, so a row's entries inside a column range are
// contiguous; four lanes per row).  Wide runs are cut into slices of the union; a slice's waves find
// their starting cursors by binary search and write partial tiles that k_reduce_tiles adds in slice order.
// staging of one chunk of union rows: piece i of this thread is bytes [soff[i], soff[i] + 16) of staged row srow[i];
// rows past the chunk's end repeat its last row, so every staged LDS row holds finite data
template <int NPT>
__device__ __forceinline__ void run_request(v4u (&stg)[NPT], const int (&srow)[NPT], const int (&soff)[NPT], int32_t uc_reg,
                                            int n_rows_chunk, const char* __restrict__ X, int64_t ldxb)
{
#pragma unroll
    for (int i = 0; i < NPT; ++i) {
        const int32_t c = __shfl(uc_reg, min(srow[i], n_rows_chunk - 1), 64);
        stg[i] = *reinterpret_cast<const v4u*>(X + (int64_t)c * ldxb + soff[i]);
    }
}

template <int NPT, int UC, int PITCH>
__device__ __forceinline__ void run_park(const v4u (&stg)[NPT], const int (&srow)[NPT], const int (&soff)[NPT],
                                         char* __restrict__ buf)
{
#pragma unroll
    for (int i = 0; i < NPT; ++i)
        if (srow[i] < UC) *reinterpret_cast<v4u*>(buf + srow[i] * PITCH + soff[i]) = stg[i];
}

struct RunCursor {
    int32_t k;          // wave: next condensed column of the window
    int32_t cur;        // lane: next non-zero of row lane/4
    int32_t row_e;      // lane: end of that row
};

// one K-step (four condensed columns) of a chunk on the fp32 path: B operands from the staged rows by slot
template <int VW, int NG> struct RunStepB { float x[NG][VW]; };

template <int VW, int NG, int PITCH>
__device__ __forceinline__ void run_load_step(int q, int32_t sloc, int lane, const char* __restrict__ xb, int d,
                                              RunStepB<VW, NG>& b)
{
    const int j = lane & 15, kk = lane >> 4;
    const int32_t c = __shfl(sloc, 4 * q + kk, 64);
    const char* __restrict__ xr = xb + c * PITCH;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int col = g * 16 * VW + VW * j;                  // columns past d read column 0 and are never stored
        const char* p = xr + (col < d ? col : 0) * 4;
        if constexpr (VW == 4) { const float4 v = *reinterpret_cast<const float4*>(p); b.x[g][0] = v.x; b.x[g][1] = v.y; b.x[g][2] = v.z; b.x[g][3] = v.w; }
        else if constexpr (VW == 2) { const float2 v = *reinterpret_cast<const float2*>(p); b.x[g][0] = v.x; b.x[g][1] = v.y; }
        else { b.x[g][0] = *reinterpret_cast<const float*>(p); }
    }
}

template <int VW, int NG>
__device__ __forceinline__ void run_compute_step(int q, const float* __restrict__ tile, int lane, const RunStepB<VW, NG>& b,
                                                 v4f (&acc)[NG][VW])
{
    const float av = tile[64 * q + lane];                      // A(row lane%16, column 4q + lane/16)
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int t = 0; t < VW; ++t) acc[g][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, b.x[g][t], acc[g][t], 0, 0, 0);
}

template <int XK, int VW, int NG, int UC>
__global__ __launch_bounds__(256) void k_mfma_run(const RunSlice* __restrict__ slices, const RunWin* __restrict__ wins,
                                                   const int32_t* __restrict__ ucols, const int32_t* __restrict__ wslot,
                                                   const int32_t* __restrict__ erc, float* __restrict__ tile_partial,
                                                   int col0, SpmmArgs a)
{
    using P = Path<XK, VW, NG>;
    constexpr int ES = P::ES;
    constexpr int SPANB = NG * 16 * VW * ES;                   // bytes of one X row's share of this launch
    constexpr int PITCH = SPANB + 16;                          // LDS row pitch: neighbouring rows start 4 banks apart
    constexpr int NPT = UC * SPANB / 16 / 256 > 0 ? UC * SPANB / 16 / 256 : 1;   // 16-byte pieces per thread and chunk
    constexpr int NST = UC / P::SCOLS;                         // pipeline stages per chunk (16-bit path)
    static_assert(UC % P::SCOLS == 0 && UC <= 64, "a chunk is a whole number of stages and fits one lane per column");
    __shared__ __align__(16) char xs[2][UC * PITCH];
    __shared__ __align__(16) float tiles[4][UC * 16];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    // everything a workgroup needs to start comes from two records read side by side: the slice, and this wave's window
    const RunSlice sl = slices[blockIdx.x];
    const RunWin wn = wins[(int64_t)blockIdx.x * kRunWindows + wave];
    const int32_t u_begin = sl.u_begin, u_end = sl.u_end;
    const int64_t up = sl.up;
    const char* __restrict__ X = static_cast<const char*>(a.X) + (int64_t)col0 * ES;
    const int64_t ldxb = a.ldx * ES;
    const int d = min(a.d - col0, NG * 16 * VW);
    const int ppr = (d * ES + 15) >> 4;                        // 16-byte pieces per staged row

    // Waves beyond the run's last window only help staging: their record repeats the run's first window and every
    // column is masked out, so that all waves execute the same straight-line sequence of loads (a load inside a
    // branch makes the compiler wait for ALL outstanding loads at the next join, the staged rows included).
    const bool has_win = wave < sl.nw;
    const int32_t nc = wn.nc, r0 = wn.w * kH, k_last = wn.k_last;
    const int64_t wp = wn.wp;

    // staging map of this thread: piece p = tid + 256 i of a chunk is bytes [soff, soff + 16) of staged row `srow`
    int srow[NPT], soff[NPT];
#pragma unroll
    for (int i = 0; i < NPT; ++i) {
        const int pidx = threadIdx.x + 256 * i;
        srow[i] = pidx / ppr;
        soff[i] = (pidx - srow[i] * ppr) * 16;
    }
    auto union_ids = [&](int32_t cb) { return ucols[up + min(cb + lane, u_end - 1)]; };
    // two chunks of rows are in flight: while chunk c is multiplied, chunk c+1 waits in registers for its LDS buffer
    // and chunk c+2 is on its way
    v4u stg_a[NPT], stg_b[NPT];
    const int32_t uc0 = union_ids(u_begin), uc1 = union_ids(u_begin + UC);
    int32_t uc_next = union_ids(u_begin + 2 * UC);
    run_request<NPT>(stg_a, srow, soff, uc0, min(UC, u_end - u_begin), X, ldxb);

    RunCursor cs{0, 0, 0};
    {
        const int32_t row = min(r0 + (lane >> 2), a.n_rows);
        cs.cur = a.rowptr[row];
        cs.row_e = a.rowptr[min(row + 1, a.n_rows)];
        if (u_begin > 0) {
            // first condensed column at or beyond the slice, then every row's first non-zero at or beyond it
            int32_t lo = 0, hi = nc;
            while (lo < hi) { const int32_t mid = (lo + hi) >> 1; if (wslot[wp + mid] < u_begin) lo = mid + 1; else hi = mid; }
            cs.k = lo;
            int32_t a0 = cs.cur, a1 = cs.row_e;
            while (a0 < a1) { const int32_t mid = a0 + ((a1 - a0) >> 1); if ((erc[mid] >> 4) < lo) a0 = mid + 1; else a1 = mid; }
            cs.cur = a0;
        }
    }
    float* __restrict__ tile = tiles[wave];
    v4f acc[NG][VW];
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int t = 0; t < VW; ++t) acc[g][t] = (v4f){0.f, 0.f, 0.f, 0.f};

    // the next kRound*4 non-zeros of every row, four lanes per row; slots past the row's end are marked, their loads
    // are clamped to a valid index and issued all the same
    constexpr int kRound = 2;
    int32_t pr[kRound];
    float vr[kRound];
    auto fetch_round = [&]() {
#pragma unroll
        for (int j = 0; j < kRound; ++j) {
            const int32_t k = cs.cur + 4 * j + (lane & 3);
            const int32_t kc = min(k, k_last);
            const int32_t pe = erc[kc];
            const float ve = a.vals[kc];
            pr[j] = k < cs.row_e ? pe : 0x7fffffff;
            vr[j] = ve;
        }
    };
    int32_t s_cur = wslot[wp + min(cs.k + lane, nc - 1)];
    fetch_round();
    run_request<NPT>(stg_b, srow, soff, uc1, max(1, min(UC, u_end - u_begin - UC)), X, ldxb);

    const int n_chunks = (u_end - u_begin + UC - 1) / UC;
    // one chunk: request the rows of chunk c+2 into `stg_req`, multiply chunk c out of xs[c & 1], then move chunk c+1
    // from `stg_park` into the other buffer
    auto chunk = [&](int c, v4u (&stg_req)[NPT], const v4u (&stg_park)[NPT]) {
        const int32_t cb = u_begin + c * UC, ce = min(cb + UC, u_end);
        // the window's columns inside this chunk: [k, k + n)
        const int n = has_win ? __popcll(__ballot(cs.k + lane < nc && s_cur < ce)) : 0;
        const int32_t sloc = min(max(s_cur - cb, 0), UC - 1);
        const int32_t limit = cs.k + n;
        if (n > 0) {
            const int nz = ((n + P::SCOLS - 1) / P::SCOLS) * P::SCOLS * 16;      // floats of the tile the K-steps will read
            for (int i = lane * 4; i < nz; i += 256)
                *reinterpret_cast<float4*>(&tile[i]) = make_float4(0.f, 0.f, 0.f, 0.f);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            const int shift = lane & ~3;
            bool more;
            {
                int taken = 0;
#pragma unroll
                for (int j = 0; j < kRound; ++j) {
                    const bool take = (pr[j] >> 4) < limit;             // marked slots compare as beyond every limit
                    const float vv = take ? vr[j] : 0.f;                // the value is consumed outside the masked store
                    if (take) atomicAdd(&tile[P::tidx((pr[j] >> 4) - cs.k, lane >> 2)], vv);
                    taken += __popcll((__ballot(take) >> shift) & 0xfull);
                }
                cs.cur += taken;
                more = taken == 4 * kRound;                             // the row may have further entries inside the range
            }
            while (__any(more)) {                                       // rare: a row with more than kRound*4 entries in one chunk
                int taken = 0;
#pragma unroll
                for (int j = 0; j < kRound; ++j) {
                    const int32_t k = cs.cur + 4 * j + (lane & 3);
                    const int32_t kc = min(k, k_last);
                    const int32_t pe = erc[kc];
                    const float ve = a.vals[kc];
                    const bool take = more && k < cs.row_e && (pe >> 4) < limit;
                    const float vv = take ? ve : 0.f;
                    if (take) atomicAdd(&tile[P::tidx((pe >> 4) - cs.k, lane >> 2)], vv);
                    taken += __popcll((__ballot(take) >> shift) & 0xfull);
                }
                cs.cur += taken;
                more = more && taken == 4 * kRound;
            }
        }
        cs.k = limit;
        // Requested before this chunk's matrix work, in this order (outstanding loads are counted in order of issue, so
        // whatever is needed first has to be requested first): the next chunk's slots and first round of non-zeros, the
        // union ids of chunk c+3, then the rows of chunk c+2, which stay in flight until the end of chunk c+1.
        const int32_t s_next = wslot[wp + min(cs.k + lane, nc - 1)];
        fetch_round();
        const int32_t uc_req = uc_next;
        uc_next = union_ids(cb + 3 * UC);
        run_request<NPT>(stg_req, srow, soff, uc_req, max(1, min(UC, u_end - cb - 2 * UC)), X, ldxb);
        if (n > 0) {
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            const char* __restrict__ xb = xs[c & 1];
            if constexpr (XK == 0) {
                // K-steps of four columns, only as many as the window has columns in this chunk
                const int nk = (n + 3) >> 2;
                RunStepB<VW, NG> b0, b1;
                run_load_step<VW, NG, PITCH>(0, sloc, lane, xb, d, b0);
                for (int q = 0; q < nk; q += 2) {
                    run_load_step<VW, NG, PITCH>(min(q + 1, nk - 1), sloc, lane, xb, d, b1);
                    run_compute_step<VW, NG>(q, tile, lane, b0, acc);
                    run_load_step<VW, NG, PITCH>(min(q + 2, nk - 1), sloc, lane, xb, d, b0);
                    if (q + 1 < nk) run_compute_step<VW, NG>(q + 1, tile, lane, b1, acc);
                }
            } else {
                typename P::Buf xa[2];
                P::load(0, sloc, lane, xb, PITCH, d, xa[0]);
#pragma unroll
                for (int st = 0; st < NST; ++st) {
                    if (st + 1 < NST) P::load(st + 1, sloc, lane, xb, PITCH, d, xa[(st + 1) & 1]);
                    if (st * P::SCOLS < n) P::compute(st, tile, lane, xa[st & 1], acc);
                }
            }
        }
        s_cur = s_next;
        run_park<NPT, UC, PITCH>(stg_park, srow, soff, xs[(c + 1) & 1]);
        __syncthreads();
    };
    run_park<NPT, UC, PITCH>(stg_a, srow, soff, xs[0]);
    __syncthreads();
    // chunks are taken in pairs (the register sets alternate); an odd count ends with one empty chunk rather than a
    // branch around the second half, whose loads would otherwise cost a full wait at the join
    for (int c = 0; c < n_chunks; c += 2) {
        chunk(c, stg_a, stg_b);
        chunk(c + 1, stg_b, stg_a);
    }
    if (has_win) {
        if (sl.n_slices == 1) store_tile<VW, NG>(acc, lane, r0, a.n_rows, a.Y, a.ldy, col0, d, a.relu, a.y_dtype);
        else store_tile<VW, NG>(acc, lane, (sl.slot0 + wave * sl.n_slices + sl.q) * kH, 0x7fffffff, tile_partial, a.d, col0, d, 0);
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
        const float one[1] = {acc};
        out_store<1>(a.Y, a.y_dtype, row * a.ldy + c, one, a.relu);
    }
}

// ---- dispatch ---------------------------------------------------------------------------------
struct MfmaShape { int vw, ng; };

// 0 when the matrix path has no kernel for this combination of width, leading dimensions and alignment
static bool pick_mfma_shape(const SpmmArgs& a, MfmaShape& sh)
{
    const uintptr_t px = (uintptr_t)a.X, py = (uintptr_t)a.Y;
    int vw = 1;
    if (a.x_dtype == HCSPMM_F32) {
        if (a.d % 4 == 0 && a.ldx % 4 == 0 && a.ldy % 4 == 0 && px % 16 == 0 && py % 16 == 0) vw = 4;
        else if (a.d % 2 == 0 && a.ldx % 2 == 0 && a.ldy % 2 == 0 && px % 8 == 0 && py % 8 == 0) vw = 2;
        // prefer the narrowest vector that still covers d in one 16-lane stretch (no idle lanes)
        while (vw > 1 && 16 * (vw / 2) >= a.d) vw >>= 1;
    } else {
        const bool y4 = a.ldy % 4 == 0 && py % 16 == 0 && a.d % 4 == 0;
        if (a.d % 8 == 0 && a.ldx % 8 == 0 && px % 16 == 0 && y4 && a.d > 64) vw = 8;
        else if (a.d % 4 == 0 && a.ldx % 4 == 0 && px % 8 == 0 && y4) vw = 4;
        else return false;
    }
    const int groups = (a.d + 16 * vw - 1) / (16 * vw);
    int ng = groups >= 4 ? 4 : (groups >= 2 ? 2 : 1);
    if (a.x_dtype != HCSPMM_F32 && vw == 8 && ng > 2) ng = 2;   // 16 accumulator tiles at most
    sh = {vw, ng};
    return true;
}

bool mfma_shape_supported(const SpmmArgs& a)
{
    MfmaShape sh;
    return pick_mfma_shape(a, sh);
}

// the fused update needs the whole aggregated width in one launch of the wave-per-window kernel
bool mfma_update_fusable(const SpmmArgs& a)
{
    MfmaShape sh;
    return pick_mfma_shape(a, sh) && sh.ng * 16 * sh.vw >= a.d;
}

#define HC_MFMA_DISPATCH(FN)                                                                       \
    if (a.x_dtype == HCSPMM_F32) {                                                                 \
        switch (sh.vw * 10 + sh.ng) {                                                              \
            case 41: FN(0, 4, 1); break;                                                           \
            case 42: FN(0, 4, 2); break;                                                           \
            case 44: FN(0, 4, 4); break;                                                           \
            case 21: FN(0, 2, 1); break;                                                           \
            case 22: FN(0, 2, 2); break;                                                           \
            case 24: FN(0, 2, 4); break;                                                           \
            case 11: FN(0, 1, 1); break;                                                           \
            case 12: FN(0, 1, 2); break;                                                           \
            default: FN(0, 1, 4); break;                                                           \
        }                                                                                          \
    } else if (a.x_dtype == HCSPMM_BF16) {                                                         \
        switch (sh.vw * 10 + sh.ng) {                                                              \
            case 41: FN(1, 4, 1); break;                                                           \
            case 42: FN(1, 4, 2); break;                                                           \
            case 44: FN(1, 4, 4); break;                                                           \
            case 81: FN(1, 8, 1); break;                                                           \
            default: FN(1, 8, 2); break;                                                           \
        }                                                                                          \
    } else {                                                                                       \
        switch (sh.vw * 10 + sh.ng) {                                                              \
            case 41: FN(2, 4, 1); break;                                                           \
            case 42: FN(2, 4, 2); break;                                                           \
            case 44: FN(2, 4, 4); break;                                                           \
            case 81: FN(2, 8, 1); break;                                                           \
            default: FN(2, 8, 2); break;                                                           \
        }                                                                                          \
    }

hipError_t launch_mfma_small(const SpmmArgs& a, int32_t n_list, const WinDesc* desc, const int32_t* wcols,
                             const int32_t* erc, hipStream_t s, const UpdateArgs* upd)
{
    if (n_list <= 0) return hipSuccess;
    MfmaShape sh;
    if (!pick_mfma_shape(a, sh)) return hipErrorInvalidValue;
    const int span = sh.ng * 16 * sh.vw;                       // output columns per launch
    int64_t n_blocks = ((int64_t)n_list + 3) / 4;
    int xcd_chunk = 0;
    if (n_blocks >= 1024) {                      // pad to whole rounds of eight runs; surplus workgroups exit at once
        xcd_chunk = 32;
        if (tune().xcd_chunk >= 0) xcd_chunk = tune().xcd_chunk;
        if (xcd_chunk > 0) n_blocks = (n_blocks + 8 * xcd_chunk - 1) / (8 * xcd_chunk) * (8 * xcd_chunk);
        else xcd_chunk = 0;
    }
    if (upd) {
        if (span < a.d) return hipErrorInvalidValue;
        const dim3 grid((unsigned)n_blocks);
#define HC_LAUNCH_MSF(K, V, G) hipLaunchKernelGGL((k_mfma_small<K, V, G, true>), grid, dim3(256), 0, s, n_list, desc, wcols, erc, 0, xcd_chunk, a, *upd)
        HC_MFMA_DISPATCH(HC_LAUNCH_MSF)
#undef HC_LAUNCH_MSF
        return hipGetLastError();
    }
    const UpdateArgs no_update{};
    for (int col0 = 0; col0 < a.d; col0 += span) {
#define HC_LAUNCH_MS(K, V, G)                                                                      \
    hipLaunchKernelGGL((k_mfma_small<K, V, G>), dim3((unsigned)n_blocks), dim3(256), 0, s, n_list, desc,   \
                       wcols, erc, col0, xcd_chunk, a, no_update)
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
    MfmaShape sh;
    if (!pick_mfma_shape(a, sh)) return hipErrorInvalidValue;
    const int span = sh.ng * 16 * sh.vw;
    for (int col0 = 0; col0 < a.d; col0 += span) {
#define HC_LAUNCH_MB(K, V, G)                                                                      \
    if (wide)                                                                                      \
        hipLaunchKernelGGL((k_mfma_wg<K, V, G, kKcBig>), dim3(n_list), dim3(256), 0, s, slices, ncols, wptr, wcols,  \
                           erc, rows_sorted, slice_rows, tile_partial, col0, a);                   \
    else                                                                                           \
        hipLaunchKernelGGL((k_mfma_wg<K, V, G, kKcMid>), dim3(n_list), dim3(256), 0, s, slices, ncols, wptr, wcols,  \
                           erc, rows_sorted, slice_rows, tile_partial, col0, a)
        HC_MFMA_DISPATCH(HC_LAUNCH_MB)
#undef HC_LAUNCH_MB
    }
    return hipGetLastError();
}

// The run kernel stages whole 16-byte pieces of X rows: fp32 rows in float4 steps, 16-bit rows in steps of 8 elements.
bool mfma_run_shape_supported(const SpmmArgs& a)
{
    MfmaShape sh;
    if (!pick_mfma_shape(a, sh)) return false;
    const uintptr_t px = (uintptr_t)a.X;
    if (a.x_dtype == HCSPMM_F32) return a.d % 4 == 0 && a.ldx % 4 == 0 && px % 16 == 0;
    return a.d % 8 == 0 && a.ldx % 8 == 0 && px % 16 == 0;
}

hipError_t launch_mfma_run(const SpmmArgs& a, int32_t n_slices, const RunSlice* slices, const RunWin* wins,
                           const int32_t* ucols, const int32_t* wslot, const int32_t* erc, float* tile_partial, hipStream_t s)
{
    if (n_slices <= 0) return hipSuccess;
    MfmaShape sh;
    if (!pick_mfma_shape(a, sh) || !mfma_run_shape_supported(a)) return hipErrorInvalidValue;
    const int span = sh.ng * 16 * sh.vw;
    for (int col0 = 0; col0 < a.d; col0 += span) {
        // chunk of the union staged per step: about 16 KiB of X rows
#define HC_LAUNCH_RUN(K, V, G)                                                                     \
    {                                                                                              \
        constexpr int kSpanB = G * 16 * V * (K == 0 ? 4 : 2);                                      \
        constexpr int kUC = kSpanB >= 1024 ? 16 : (kSpanB >= 512 ? 32 : 64);                       \
        hipLaunchKernelGGL((k_mfma_run<K, V, G, (kUC < Path<K, V, G>::SCOLS ? Path<K, V, G>::SCOLS : kUC)>),   \
                           dim3(n_slices), dim3(256), 0, s, slices, wins, ucols, wslot, erc, tile_partial, col0, a);   \
    }
        HC_MFMA_DISPATCH(HC_LAUNCH_RUN)
#undef HC_LAUNCH_RUN
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
