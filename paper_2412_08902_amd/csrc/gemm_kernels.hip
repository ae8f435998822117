// Dense update T = act(X W) (Eq. 2; the activation is optional) in true fp32 on the MFMA units: v_mfma_f32_32x32x2_f32.
//
// Operand layout per lane l: A: row l%32, k = l/32.  B: k = l/32, column l%32.
// D (32x32, 16 registers): column l%32, row 8*(v/4) + 4*(l/32) + v%4 for register v.
//
// Workgroup tile 128 x 128, K advanced 16 at a time; four waves in a 2 x 2 grid, each computing
// a 64 x 64 sub-tile as 2 x 2 MFMA tiles.  Both operands are staged k-major in LDS so that the
// per-lane operand reads are unit-stride; the global loads of the next K slab are issued before
// the MFMAs of the current one (register double buffering).
#include <cstdlib>

#include "common.hpp"

namespace hcspmm {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 16;
constexpr int LDA_S = BM + 4;     // padded leading dimensions of the LDS images
constexpr int LDB_S = BN + 4;

// XV: floats per global load of X (4, 2 or 1, by alignment of ldx); W rows are read one float at a
// time per lane and 64 lanes wide (always coalesced).
// TK: element kind of the output -- 0 fp32, 1 bf16 (round to nearest even), 2 fp16.
template <int XV, int TK = 0>
__global__ __launch_bounds__(256) void k_gemm_f32(int64_t M, int32_t K, int32_t N, const float* __restrict__ X,
                                                  int64_t ldx, const float* __restrict__ Wm, int64_t ldw,
                                                  void* __restrict__ Tv, int64_t ldt, int relu)
{
    __shared__ float As[BK * LDA_S];
    __shared__ float Bs[BK * LDB_S];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;

    // global -> register staging maps
    // X slab: 128 rows x 16 k.  With XV floats per load a row needs 16/XV loads; thread -> (row, kq)
    constexpr int LPRW = BK / XV;                 // loads per row
    constexpr int ROWS_PER_IT = 256 / LPRW;
    constexpr int A_ITERS = BM / ROWS_PER_IT;
    const int a_row = tid / LPRW, a_kq = (tid % LPRW) * XV;
    // W slab: 16 k x 128 columns: thread -> (k = tid/128 + 2*it, col = tid%128)
    constexpr int B_ITERS = BK * BN / 256;
    const int b_col = tid & 127, b_k = tid >> 7;

    float a_reg[A_ITERS][XV];
    float b_reg[B_ITERS];

    auto load_slab = [&](int k0) {
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it) {
            const int64_t row = m0 + a_row + it * ROWS_PER_IT;
            const int k = k0 + a_kq;
            const float* p = X + row * ldx + k;
            if (row < M && k + XV <= K) {
                if constexpr (XV == 4) { float4 v = *reinterpret_cast<const float4*>(p); a_reg[it][0] = v.x; a_reg[it][1] = v.y; a_reg[it][2] = v.z; a_reg[it][3] = v.w; }
                else if constexpr (XV == 2) { float2 v = *reinterpret_cast<const float2*>(p); a_reg[it][0] = v.x; a_reg[it][1] = v.y; }
                else { a_reg[it][0] = *p; }
            } else {
#pragma unroll
                for (int i = 0; i < XV; ++i) a_reg[it][i] = (row < M && k + i < K) ? p[i] : 0.f;
            }
        }
#pragma unroll
        for (int it = 0; it < B_ITERS; ++it) {
            const int k = k0 + b_k + 2 * it;
            const int col = n0 + b_col;
            b_reg[it] = (k < K && col < N) ? Wm[(int64_t)k * ldw + col] : 0.f;
        }
    };
    auto store_slab = [&]() {
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it)
#pragma unroll
            for (int i = 0; i < XV; ++i) As[(a_kq + i) * LDA_S + a_row + it * ROWS_PER_IT] = a_reg[it][i];
#pragma unroll
        for (int it = 0; it < B_ITERS; ++it) Bs[(b_k + 2 * it) * LDB_S + b_col] = b_reg[it];
    };

    v16f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int li = lane & 31, lk = lane >> 5;
    load_slab(0);
    for (int k0 = 0; k0 < K; k0 += BK) {
        __syncthreads();                     // previous slab fully consumed
        store_slab();
        __syncthreads();
        if (k0 + BK < K) load_slab(k0 + BK);
#pragma unroll
        for (int ks = 0; ks < BK; ks += 2) {
            float av[2], bv[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) av[i] = As[(ks + lk) * LDA_S + wm + 32 * i + li];
#pragma unroll
            for (int j = 0; j < 2; ++j) bv[j] = Bs[(ks + lk) * LDB_S + wn + 32 * j + li];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn + 32 * j + li;
            if (col >= N) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * lk + (v & 3);
                if (row >= M) continue;
                const float y = relu ? fmaxf(acc[i][j][v], 0.f) : acc[i][j][v];
                if constexpr (TK == 0) {
                    static_cast<float*>(Tv)[row * ldt + col] = y;
                } else if constexpr (TK == 1) {
                    uint32_t u = __float_as_uint(y);
                    u += 0x7fffu + ((u >> 16) & 1u);                 // round to nearest even (finite values)
                    static_cast<unsigned short*>(Tv)[row * ldt + col] = (unsigned short)(u >> 16);
                } else {
                    static_cast<_Float16*>(Tv)[row * ldt + col] = (_Float16)y;
                }
            }
        }
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
    if (gemm_rows16_usable(m, k, n, X, ldx) && !tune().no_rows16)
        return launch_gemm_rows16(m, k, n, X, ldx, W, ldw, static_cast<float*>(T), ldt, relu, s, t_dtype);
    dim3 grid((unsigned)((m + BM - 1) / BM), (unsigned)((n + BN - 1) / BN));
    const uintptr_t px = (uintptr_t)X;
    const int xv = (ldx % 4 == 0 && px % 16 == 0) ? 4 : ((ldx % 2 == 0 && px % 8 == 0) ? 2 : 1);
#define HC_LAUNCH_GEMM(V, TK) hipLaunchKernelGGL((k_gemm_f32<V, TK>), grid, dim3(256), 0, s, m, k, n, X, ldx, W, ldw, T, ldt, relu)
#define HC_GEMM_XV(TK) if (xv == 4) HC_LAUNCH_GEMM(4, TK); else if (xv == 2) HC_LAUNCH_GEMM(2, TK); else HC_LAUNCH_GEMM(1, TK)
    if (t_dtype == HCSPMM_F32) { HC_GEMM_XV(0); }
    else if (t_dtype == HCSPMM_BF16) { HC_GEMM_XV(1); }
    else if (t_dtype == HCSPMM_F16) { HC_GEMM_XV(2); }
    else return hipErrorInvalidValue;
#undef HC_GEMM_XV
#undef HC_LAUNCH_GEMM
    return hipGetLastError();
}

}  // namespace hcspmm
