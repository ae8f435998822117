// Update stage of the aggregate-then-update layer (Section V-A: a window's aggregation result is
// kept on chip and multiplied by W on the matrix cores before anything is written back).
//
// One wave owns a 16 x d_in tile Z of aggregated rows in LDS and computes act(Z W) with
// v_mfma_f32_16x16x4_f32 (true fp32).  Lane l = (c = l%16, q = l/16) supplies A(row c, k q) and
// B(k q, column c).  The contraction index is taken in the order that lets a lane read four
// consecutive Z values with one 16-byte LDS read: in step s of block j the lane's k is
// j + 4q + s, so its A values are Z[c][j+4q .. j+4q+3] and its B values W[j+4q+s][column].
// W is read from global memory (it is small and stays in L2/L1); the loads of the next block are
// requested before the MFMAs of the current one.
#pragma once
#include "common.hpp"

namespace hcspmm {

typedef float v4f_upd __attribute__((ext_vector_type(4)));

// zt      LDS, row r of the tile at zt + r*ldz (ldz a multiple of 4 floats, rows 16-byte aligned)
// rows16  LDS, the 16 output row indices of the tile (-1: no output for that tile row)
// d_in    multiple of 16
__device__ inline void update_tile16(const float* zt, int ldz, const int32_t* rows16, int d_in, const UpdateArgs& u,
                                     int lane)
{
    const int c = lane & 15, q = lane >> 4;
    int32_t myrow[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) myrow[r] = rows16[4 * q + r];
    const float* __restrict__ W = u.W;
    const int64_t ldw = u.ldw;
    for (int n0 = 0; n0 < u.d_out; n0 += 64) {               // four 16-column output tiles per pass
        const int nt = min(4, (u.d_out - n0 + 15) / 16);
        v4f_upd acc[4];
        const float* wp[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            acc[t] = (v4f_upd){0.f, 0.f, 0.f, 0.f};
            const int col = n0 + 16 * t + c;
            wp[t] = W + (col < u.d_out ? col : 0) + (int64_t)(4 * q) * ldw;   // columns past d_out read column 0, never stored
        }
        float b0[4][4], b1[4][4];
        auto fetch = [&](int j, float (&b)[4][4]) {
            const int jc = j < d_in ? j : d_in - 16;            // a fetch past the end repeats the last block (unused)
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int t = 0; t < 4; ++t) b[s][t] = wp[t][(int64_t)(jc + s) * ldw];
        };
        auto block = [&](int j, const float (&b)[4][4]) {
            const float4 av = *reinterpret_cast<const float4*>(&zt[c * ldz + j + 4 * q]);
            const float a4[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    if (t < nt) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[s], b[s][t], acc[t], 0, 0, 0);
        };
        fetch(0, b0);
        for (int j = 0; j < d_in; j += 32) {
            fetch(j + 16, b1);
            block(j, b0);
            if (j + 16 >= d_in) break;
            fetch(j + 32, b0);
            block(j + 16, b1);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int col = n0 + 16 * t + c;
            if (col >= u.d_out) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (myrow[r] < 0) continue;
                const float y = acc[t][r];
                u.Y[(int64_t)myrow[r] * u.ldy + col] = u.relu ? fmaxf(y, 0.f) : y;
            }
        }
    }
}

}  // namespace hcspmm
