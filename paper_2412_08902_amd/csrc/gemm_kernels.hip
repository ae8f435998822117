// Dense update T = act(X W) (Eq. 2; the activation is optional) in true fp32 on the MFMA units: v_mfma_f32_32x32x2_f32.
//
// Operand layout per lane l: A: row l%32, k = l/32.  B: k = l/32, column l%32.
// D (32x32, 16 registers): column l%32, row 8*(v/4) + 4*(l/32) + v%4 for register v.
//
// Workgroup tile 128 x 128 with K advanced 32 at a time; four waves in a 2 x 2 grid, each computing a 64 x 64
// sub-tile as 2 x 2 MFMA tiles.  The X slab sits in LDS row-major (a lane's two k values of two consecutive MFMA
// steps are one 8-byte read), the W slab k-major, and a wave's two column tiles interleave (tile j holds the columns
// base + 2*(l%32) + j) so that its two B values are one 8-byte read as well and the results go back as column pairs.
// The global loads of the next slab are issued before the MFMAs of the current one (register double buffering).
//
// X rows that are only 8-byte aligned (ldx even but not a multiple of 4: 602 features, say) are still read with 16-byte
// loads: a row's slab is fetched as the nine aligned 16-byte pieces that cover it, and the 8-byte halves of those
// pieces that belong to the slab are stored where they belong (two floats to the left when the row starts in the
// middle of a piece), so the LDS image and its readers are the same as for aligned rows.
//
// The row tiles of a launch come in two heights.  As many 128-row tiles as fill whole rounds of the chip's 256 CUs,
// and the rows that are left as 32-row tiles (four waves side by side, one MFMA tile each): the last, partly filled
// round of tall tiles would otherwise leave most CUs idle for a whole tile's duration.
#include <cstdlib>

#include "common.hpp"

namespace hcspmm {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 32, BM_TAIL = 32;
constexpr int LDA_S = BK + 2;     // A image: rows 136 bytes apart, so the 8-byte reads of 16 consecutive rows fall into 16 different bank pairs
constexpr int LDB_S = BN + 4;     // B image: k rows 528 bytes apart (16-byte aligned for the vector stores)

// One row tile of height H (128 or 32).
//   XV  4: X and ldx allow aligned 16-byte loads; 1: 4-byte loads; 2: rows are 8-byte aligned, read as the aligned
//       16-byte pieces covering them (xoff = floats between the 16-byte boundary below X and X: 0 or 2)
//   WV  floats per global load of W (4 or 1)
// Rows past M re-read row M-1 and columns past N read column N-WV: what they produce is never stored.  Only k >= K is
// zeroed (in the last slab), in both operands.
template <int XV, int WV, int H>
__device__ inline void gemm_tile(int64_t m0, int n0, int64_t M, int32_t K, int32_t N, const float* __restrict__ X,
                                 int64_t ldx, const float* __restrict__ Wm, int64_t ldw, float* __restrict__ T,
                                 int64_t ldt, int32_t t_dtype, int relu, int pair_ok, int xoff, float* __restrict__ As,
                                 float* __restrict__ Bs)
{
    constexpr bool SHIFT = XV == 2;
    constexpr int MI = H == BM ? 2 : 1, NJ = H == BM ? 2 : 1;        // MFMA tiles per wave
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = H == BM ? (wave >> 1) * 64 : 0;
    const int wn = H == BM ? (wave & 1) * 64 : wave * 32;

    // global -> register staging maps.  X slab: H rows x 32 k, thread -> (row, k piece); W slab: 32 k x 128 columns
    constexpr int XL = SHIFT ? 4 : XV;            // floats per load
    constexpr int LPRW = BK / XL;                 // loads per row (the shifted form adds one piece per row, see below)
    constexpr int ROWS_PER_IT = 256 / LPRW;
    constexpr int A_ITERS = H / ROWS_PER_IT;
    static_assert(A_ITERS >= 1, "a 32-row slab is at least one load per thread");
    constexpr int A_REGS = A_ITERS + (SHIFT ? 1 : 0);
    const int a_row = tid / LPRW, a_k = (tid % LPRW) * XL;
    constexpr int B_TPR = BN / WV;                // threads per k row
    constexpr int B_KPI = 256 / B_TPR;            // k rows per iteration
    constexpr int B_ITERS = BK / B_KPI;
    const int b_k = tid / B_TPR, b_col = (tid % B_TPR) * WV;
    const int b_cc = min(n0 + b_col, N - WV);     // (N >= WV: WV = 4 needs N % 4 == 0)

    float a_reg[A_REGS][XL];
    float b_reg[B_ITERS][WV];

    // Loads only: nothing here touches a loaded value, so the requests stay in flight behind the MFMAs of the
    // current slab.  k >= K is zeroed when the slab goes to LDS.
    const float* __restrict__ Xa = X - xoff;                        // (xoff = 0 unless SHIFT)
    const int64_t last = xoff + (M - 1) * ldx + K - 1;              // last float of the matrix, from Xa
    // piece c of tile row r: the four floats at the 16-byte boundary at or below the row's k0, plus 4c.  The guarded
    // form is for pieces that may stick out of the matrix (in front of its first float or behind its last one).
    auto piece = [&](int k0, int r, int c, bool guard, float (&dst)[4]) {
        const int64_t e = min(m0 + r, M - 1) * ldx + xoff;          // the row's first float, from Xa
        const int64_t b = ((e + k0) & ~(int64_t)3) + 4 * c;
        if (!guard) {
            const float4 v = *reinterpret_cast<const float4*>(Xa + b);
            dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)      // (volatile: keeps these rare loads apart from the 16-byte one above)
                dst[i] = *static_cast<const volatile float*>(Xa + min(max(b + i, (int64_t)xoff), last));
        }
    };
    constexpr int NP = LPRW + (SHIFT ? 1 : 0);                      // pieces per row
    const int64_t e_max = min(m0 + H - 1, M - 1) * ldx + xoff;      // first float of the tile's last row
    auto load_slab = [&](int k0) {
        if constexpr (XL == 4) {
            // uniform: can a piece of this tile and slab reach past the matrix?  (the tile that holds the last row, in
            // its last slabs; the first tile's first slab when X starts off a 16-byte boundary)
            const bool guard = e_max + k0 + 4 * NP + 3 > last || (xoff > 0 && m0 == 0 && k0 == 0);
#pragma unroll
            for (int it = 0; it < A_ITERS; ++it) piece(k0, a_row + it * ROWS_PER_IT, tid % LPRW, guard, a_reg[it]);
            if constexpr (SHIFT) {
                if (tid < H) piece(k0, tid, LPRW, guard, a_reg[A_ITERS]);
            }
        } else {
#pragma unroll
            for (int it = 0; it < A_ITERS; ++it)
                a_reg[it][0] = X[min(m0 + a_row + it * ROWS_PER_IT, M - 1) * ldx + min(k0 + a_k, K - 1)];
        }
#pragma unroll
        for (int it = 0; it < B_ITERS; ++it) {
            const float* __restrict__ p = Wm + (int64_t)min(k0 + b_k + it * B_KPI, K - 1) * ldw + b_cc;
            if constexpr (WV == 4) {
                const float4 v = *reinterpret_cast<const float4*>(p);
                b_reg[it][0] = v.x; b_reg[it][1] = v.y; b_reg[it][2] = v.z; b_reg[it][3] = v.w;
            } else {
                b_reg[it][0] = *p;
            }
        }
    };
    // half h of piece c holds the row's slab floats 4c + 2h - shift .. + 1 (shift = 0 or 2; always 0 for aligned rows):
    // the halves in front of the slab and behind it are dropped
    auto put = [&](int k0, bool full, int r, int c, float (&src)[4]) {
        const int shift = SHIFT ? (int)((min(m0 + r, M - 1) * ldx + xoff) & 3) : 0;
        const int t = 4 * c - shift;
        if (!full) {
#pragma unroll
            for (int i = 0; i < 4; ++i) src[i] = k0 + t + i < K ? src[i] : 0.f;
        }
        float* __restrict__ q = &As[r * LDA_S + t];
        if (t >= 0 && t < BK) *reinterpret_cast<float2*>(q) = make_float2(src[0], src[1]);
        if (t + 2 < BK) *reinterpret_cast<float2*>(q + 2) = make_float2(src[2], src[3]);
    };
    auto store_slab = [&](int k0) {
        const bool full = k0 + BK <= K;           // uniform
        if constexpr (XL == 4) {
#pragma unroll
            for (int it = 0; it < A_ITERS; ++it) put(k0, full, a_row + it * ROWS_PER_IT, tid % LPRW, a_reg[it]);
            if constexpr (SHIFT) {
                if (tid < H) put(k0, full, tid, LPRW, a_reg[A_ITERS]);
            }
        } else {
#pragma unroll
            for (int it = 0; it < A_ITERS; ++it)
                As[(a_row + it * ROWS_PER_IT) * LDA_S + a_k] = (full || k0 + a_k < K) ? a_reg[it][0] : 0.f;
        }
#pragma unroll
        for (int it = 0; it < B_ITERS; ++it) {
            const bool live = full || k0 + b_k + it * B_KPI < K;
            float* __restrict__ q = &Bs[(b_k + it * B_KPI) * LDB_S + b_col];
            if constexpr (WV == 4)
                *reinterpret_cast<float4*>(q) = live ? make_float4(b_reg[it][0], b_reg[it][1], b_reg[it][2], b_reg[it][3])
                                                     : make_float4(0.f, 0.f, 0.f, 0.f);
            else
                *q = live ? b_reg[it][0] : 0.f;
        }
    };

    v16f acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int li = lane & 31, lk = lane >> 5;
    if (K > 0) load_slab(0);                 // (K = 0: the product is all zeros)
    for (int k0 = 0; k0 < K; k0 += BK) {
        __syncthreads();                     // previous slab fully consumed
        store_slab(k0);
        __syncthreads();
        if (k0 + BK < K) load_slab(k0 + BK);
        // four k per step: the lane's A pair is k = 4s + 2*lk + {0, 1}; the first MFMA takes k = 4s + 2*lk from both
        // operands, the second k = 4s + 2*lk + 1
#pragma unroll
        for (int s = 0; s < BK / 4; ++s) {
            float2 av[MI];
#pragma unroll
            for (int i = 0; i < MI; ++i) av[i] = *reinterpret_cast<const float2*>(&As[(wm + 32 * i + li) * LDA_S + 4 * s + 2 * lk]);
            float b0[NJ], b1[NJ];
            if constexpr (NJ == 2) {
                const float2 u0 = *reinterpret_cast<const float2*>(&Bs[(4 * s + 2 * lk) * LDB_S + wn + 2 * li]);
                const float2 u1 = *reinterpret_cast<const float2*>(&Bs[(4 * s + 2 * lk + 1) * LDB_S + wn + 2 * li]);
                b0[0] = u0.x; b0[1] = u0.y; b1[0] = u1.x; b1[1] = u1.y;
            } else {
                b0[0] = Bs[(4 * s + 2 * lk) * LDB_S + wn + li];
                b1[0] = Bs[(4 * s + 2 * lk + 1) * LDB_S + wn + li];
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i].x, b0[j], acc[i][j], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i].y, b1[j], acc[i][j], 0, 0, 0);
        }
    }

#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t row = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * lk + (v & 3);
            if (row >= M) continue;
            if constexpr (NJ == 2) {
                const int col = n0 + wn + 2 * li;
                if (col >= N) continue;
                if (pair_ok) {                   // N is even then: col + 1 < N
                    const float y[2] = {acc[i][0][v], acc[i][1][v]};
                    out_store<2>(T, t_dtype, row * ldt + col, y, relu);
                } else {
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        if (col + j >= N) continue;
                        const float y[1] = {acc[i][j][v]};
                        out_store<1>(T, t_dtype, row * ldt + col + j, y, relu);
                    }
                }
            } else {
                const int col = n0 + wn + li;
                if (col >= N) continue;
                const float y[1] = {acc[i][0][v]};
                out_store<1>(T, t_dtype, row * ldt + col, y, relu);
            }
        }
}

// Row tiles 0 .. n_tall-1 are 128 rows tall; the rows from n_tall*128 on are cut into 32-row tiles.
template <int XV, int WV>
__global__ __launch_bounds__(256) void k_gemm_f32(int64_t M, int32_t K, int32_t N, const float* __restrict__ X,
                                                  int64_t ldx, const float* __restrict__ Wm, int64_t ldw,
                                                  float* __restrict__ T, int64_t ldt, int32_t t_dtype, int relu,
                                                  int pair_ok, int xoff, int64_t n_tall)
{
    __shared__ __attribute__((aligned(16))) float As[BM * LDA_S];
    __shared__ __attribute__((aligned(16))) float Bs[BK * LDB_S];
    const int n0 = blockIdx.y * BN;
    const int64_t bx = blockIdx.x;
    if (bx < n_tall)
        gemm_tile<XV, WV, BM>(bx * BM, n0, M, K, N, X, ldx, Wm, ldw, T, ldt, t_dtype, relu, pair_ok, xoff, As, Bs);
    else
        gemm_tile<XV, WV, BM_TAIL>(n_tall * BM + (bx - n_tall) * BM_TAIL, n0, M, K, N, X, ldx, Wm, ldw, T, ldt, t_dtype,
                                   relu, pair_ok, xoff, As, Bs);
}

hipError_t launch_gemm_f32(int64_t m, int32_t k, int32_t n, const float* X, int64_t ldx, const float* W, int64_t ldw,
                           float* T, int64_t ldt, int relu, hipStream_t s)
{
    return launch_gemm_f32_out(m, k, n, X, ldx, W, ldw, T, ldt, HCSPMM_F32, relu, s);
}

hipError_t launch_gemm_f32_out(int64_t m, int32_t k, int32_t n, const float* X, int64_t ldx, const float* W, int64_t ldw,
                               void* T, int64_t ldt, int32_t t_dtype, int relu, hipStream_t s)
{
    if (m <= 0 || n <= 0) return hipSuccess;
    if (t_dtype != HCSPMM_F32 && t_dtype != HCSPMM_BF16 && t_dtype != HCSPMM_F16) return hipErrorInvalidValue;
    if (gemm_rows16_usable(m, k, n, X, ldx) && !tune().no_rows16)
        return launch_gemm_rows16(m, k, n, X, ldx, W, ldw, static_cast<float*>(T), ldt, relu, s, t_dtype);
    // tall tiles for whole rounds of the 256 CUs, 32-row tiles for what is left
    const int64_t tall_all = m / BM;
    const int64_t n_tall = tall_all / 256 * 256;
    const int64_t rest = m - n_tall * BM;
    const int64_t n_tail = (rest + BM_TAIL - 1) / BM_TAIL;
    dim3 grid((unsigned)(n_tall + n_tail), (unsigned)((n + BN - 1) / BN));
    const uintptr_t px = (uintptr_t)X, pw = (uintptr_t)W, pt = (uintptr_t)T;
    // 4: aligned 16-byte loads; 2: rows 8-byte aligned, read through the aligned pieces that cover them; 1: the rest
    const int xv = (ldx % 4 == 0 && px % 16 == 0) ? 4 : ((ldx % 2 == 0 && px % 8 == 0 && k >= BK) ? 2 : 1);
    const int xoff = (int)((px % 16) / 4);
    const int wv = (n % 4 == 0 && ldw % 4 == 0 && pw % 16 == 0) ? 4 : 1;
    const size_t es = t_dtype == HCSPMM_F32 ? 4 : 2;
    const int pair_ok = (n % 2 == 0 && ldt % 2 == 0 && pt % (2 * es) == 0) ? 1 : 0;
    float* Tf = static_cast<float*>(T);
#define HC_LAUNCH_GEMM(V, WVV) hipLaunchKernelGGL((k_gemm_f32<V, WVV>), grid, dim3(256), 0, s, m, k, n, X, ldx, W, ldw, Tf, ldt, t_dtype, relu, pair_ok, xoff, n_tall)
    if (wv == 4) { if (xv == 4) HC_LAUNCH_GEMM(4, 4); else if (xv == 2) HC_LAUNCH_GEMM(2, 4); else HC_LAUNCH_GEMM(1, 4); }
    else { if (xv == 4) HC_LAUNCH_GEMM(4, 1); else if (xv == 2) HC_LAUNCH_GEMM(2, 1); else HC_LAUNCH_GEMM(1, 1); }
#undef HC_LAUNCH_GEMM
    return hipGetLastError();
}

}  // namespace hcspmm
