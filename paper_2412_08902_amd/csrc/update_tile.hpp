// Update stage of the aggregate-then-update layer (Section V-A: a window's aggregation result is
// kept on chip and multiplied by W on the matrix cores before anything is written back).
//
// A wave owns (or shares) a 16 x d_in tile Z of aggregated rows in LDS and computes act(Z W) with
// v_mfma_f32_16x16x4_f32 (true fp32).  Lane l = (c = l%16, q = l/16) supplies A(row c, k q) and
// B(k q, column c).  Two freedoms of the instruction are used to make every memory access wide:
//   - the contraction index is taken in the order that lets a lane read four consecutive Z values
//     with one 16-byte LDS read: in step s of block j the lane's k is j + 4q + s, so its A values
//     are Z[c][j+4q .. j+4q+3] and its B values come from row j+4q+s of W;
//   - a pass covers 16*NT consecutive output columns with NT accumulator tiles, tile t holding the
//     columns  base + NT*c + t, so a lane reads its NT B values of one W row as one NT-float vector
//     (16 lanes read one contiguous stretch of the row) and stores NT consecutive results per row.
// W is read from global memory (it is small and stays in L2/L1); the loads of the next block are
// requested before the MFMAs of the current one.
#pragma once
#include "common.hpp"

namespace hcspmm {

typedef float v4f_upd __attribute__((ext_vector_type(4)));

template <int NT> __device__ inline void upd_load(const float* __restrict__ p, float (&b)[NT])
{
    if constexpr (NT == 4) { const float4 v = *reinterpret_cast<const float4*>(p); b[0] = v.x; b[1] = v.y; b[2] = v.z; b[3] = v.w; }
    else if constexpr (NT == 2) { const float2 v = *reinterpret_cast<const float2*>(p); b[0] = v.x; b[1] = v.y; }
    else { b[0] = *p; }
}

// zt      LDS, row r of the tile at zt + r*ldz (ldz a multiple of 4 floats, rows 16-byte aligned)
// rows16  LDS, the 16 output row indices of the tile (-1: no output for that tile row)
// d_in    multiple of 16;  d_out a multiple of NT, W and Y rows aligned for NT-float vectors
// The wave computes the passes pass_first, pass_first + pass_step, ... (several waves may share one
// Z tile by taking interleaved passes).
template <int NT>
__device__ inline void update_tile16_nt(const float* zt, int ldz, const int32_t* rows16, int d_in, const UpdateArgs& u,
                                        int lane, int pass_first, int pass_step)
{
    const int c = lane & 15, q = lane >> 4;
    int32_t myrow[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) myrow[r] = rows16[4 * q + r];
    const int64_t ldw = u.ldw;
    for (int n0 = pass_first * 16 * NT; n0 < u.d_out; n0 += pass_step * 16 * NT) {
        const int col = n0 + NT * c;
        const bool col_ok = col < u.d_out;                      // whole vector in or out (d_out % NT == 0)
        const float* __restrict__ wp = u.W + (col_ok ? col : 0) + (int64_t)(4 * q) * ldw;
        v4f_upd acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = (v4f_upd){0.f, 0.f, 0.f, 0.f};
        float b0[4][NT], b1[4][NT];
        auto fetch = [&](int j, float (&b)[4][NT]) {
            const int jc = j < d_in ? j : d_in - 16;            // a fetch past the end repeats the last block (unused)
#pragma unroll
            for (int s = 0; s < 4; ++s) upd_load<NT>(wp + (int64_t)(jc + s) * ldw, b[s]);
        };
        auto block = [&](int j, const float (&b)[4][NT]) {
            const float4 av = *reinterpret_cast<const float4*>(&zt[c * ldz + j + 4 * q]);
            const float a4[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[s], b[s][t], acc[t], 0, 0, 0);
        };
        fetch(0, b0);
        for (int j = 0; j < d_in; j += 32) {
            fetch(j + 16, b1);
            block(j, b0);
            if (j + 16 >= d_in) break;
            fetch(j + 32, b0);
            block(j + 16, b1);
        }
        if (!col_ok) continue;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (myrow[r] < 0) continue;
            float y[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) y[t] = u.relu ? fmaxf(acc[t][r], 0.f) : acc[t][r];
            if (u.mask) {                                       // derivative of an activation applied to another matrix
                const float* __restrict__ mp = u.mask + (int64_t)myrow[r] * u.ldm + col;
#pragma unroll
                for (int t = 0; t < NT; ++t) y[t] = mp[t] > 0.f ? y[t] : 0.f;
            }
            out_store<NT>(u.Y, u.y_dtype, (int64_t)myrow[r] * u.ldy + col, y, 0);
        }
    }
}

// Copies the rows of an LDS tile that have an output row to Z (row pitch ldz_out, 16-byte aligned rows,
// d a multiple of 4); the nthreads callers share the work.
__device__ inline void store_tile_rows(const float* zt, int ldz, const int32_t* rows, int n_tile_rows, int d,
                                       float* __restrict__ Z, int64_t ldz_out, int tid, int nthreads)
{
    const int per_row = d >> 2;
    for (int idx = tid; idx < n_tile_rows * per_row; idx += nthreads) {
        const int r = idx / per_row, c = (idx % per_row) * 4;
        const int32_t row = rows[r];
        if (row >= 0)
            *reinterpret_cast<float4*>(Z + (int64_t)row * ldz_out + c) = *reinterpret_cast<const float4*>(&zt[r * ldz + c]);
    }
}

// Picks the widest vector the operands allow, narrowed until the waves sharing the tile all get a pass.
__host__ __device__ inline int update_tile_nt(const UpdateArgs& u, int pass_step)
{
    const uintptr_t pw = (uintptr_t)u.W, py = (uintptr_t)u.Y;
    int nt = 1;
    if (u.d_out % 4 == 0 && u.ldw % 4 == 0 && u.ldy % 4 == 0 && pw % 16 == 0 && py % 16 == 0) nt = 4;
    else if (u.d_out % 2 == 0 && u.ldw % 2 == 0 && u.ldy % 2 == 0 && pw % 8 == 0 && py % 8 == 0) nt = 2;
    while (nt > 1 && (u.d_out + 16 * nt - 1) / (16 * nt) < pass_step) nt >>= 1;
    while (nt > 1 && 16 * (nt / 2) >= u.d_out) nt >>= 1;      // no accumulator tiles that hold only padding columns
    return nt;
}

__device__ inline void update_tile16(const float* zt, int ldz, const int32_t* rows16, int d_in, const UpdateArgs& u,
                                     int lane, int pass_first = 0, int pass_step = 1)
{
    const int nt = update_tile_nt(u, pass_step);
    if (nt == 4) update_tile16_nt<4>(zt, ldz, rows16, d_in, u, lane, pass_first, pass_step);
    else if (nt == 2) update_tile16_nt<2>(zt, ldz, rows16, d_in, u, lane, pass_first, pass_step);
    else update_tile16_nt<1>(zt, ldz, rows16, d_in, u, lane, pass_first, pass_step);
}

}  // namespace hcspmm
